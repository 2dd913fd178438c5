"""Layer-shape tables of the two CNNs the paper trains (Table 3: AlexNet, 227x227
input, 62 M parameters; ResNet-50, 224x224 input, 25 M parameters, 4 GFLOPs).

Pure bookkeeping: no arithmetic of the training method lives here, so both the
HIP path's callers and the CPU oracle's tests may use it.
"""
from dataclasses import dataclass
from typing import List, Tuple


@dataclass(frozen=True)
class ConvShape:
    name: str
    H: int          # input height = width
    C: int
    K: int
    R: int          # filter height = width
    stride: int
    pad: int
    first: bool = False   # first layer of the net: its input needs no gradient

    @property
    def P(self) -> int:
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    def macs(self, N: int) -> int:
        return N * self.P * self.P * self.K * self.R * self.R * self.C

    def weight_count(self) -> int:
        return self.K * self.R * self.R * self.C


@dataclass(frozen=True)
class FcShape:
    name: str
    I: int
    O: int

    def macs(self, N: int) -> int:
        return N * self.I * self.O

    def weight_count(self) -> int:
        return self.I * self.O


def resnet50_convs(variant: str = "v1", image: int = 224) -> List[ConvShape]:
    """The 53 convolutions of ResNet-50 in forward order.

    v1 (He et al. 2016, the network the paper cites) puts the stride-2 step of
    stages 3-5 on the first 1x1 of the first bottleneck; "v1.5" moves it to
    the 3x3.  Each bottleneck lists a (1x1), b (3x3), c (1x1), then the 1x1
    projection shortcut when the block has one.  image (a multiple of 32) is the
    input height = width; the paper's is 224, smaller ones serve tests.
    """
    assert variant in ("v1", "v1.5") and image % 32 == 0 and image >= 32
    L = [ConvShape("stem", image, 3, 64, 7, 2, 3, first=True)]
    h, cin = image // 4, 64   # after the 3x3/2 max-pool
    for stage, (width, blocks) in enumerate(((64, 3), (128, 4), (256, 6), (512, 3)), start=2):
        cout = 4 * width
        for b in range(blocks):
            st = 2 if (b == 0 and stage > 2) else 1
            sa, sb = (st, 1) if variant == "v1" else (1, st)
            nm = "s%db%d" % (stage, b + 1)
            L.append(ConvShape(nm + "a", h, cin, width, 1, sa, 0))
            hb = h // sa
            L.append(ConvShape(nm + "b", hb, width, width, 3, sb, 1))
            hc = hb // sb
            L.append(ConvShape(nm + "c", hc, width, cout, 1, 1, 0))
            if b == 0:
                L.append(ConvShape(nm + "p", h, cin, cout, 1, st, 0))
            h, cin = hc, cout
    assert len(L) == 53
    return L


RESNET50_FC = FcShape("fc", 2048, 1000)


def alexnet_convs() -> List[ConvShape]:
    """The five convolutions of AlexNet, ungrouped, 227x227 input."""
    return [
        ConvShape("conv1", 227, 3, 96, 11, 4, 0, first=True),
        ConvShape("conv2", 27, 96, 256, 5, 1, 2),
        ConvShape("conv3", 13, 256, 384, 3, 1, 1),
        ConvShape("conv4", 13, 384, 384, 3, 1, 1),
        ConvShape("conv5", 13, 384, 256, 3, 1, 1),
    ]


ALEXNET_FCS = [FcShape("fc6", 9216, 4096), FcShape("fc7", 4096, 4096), FcShape("fc8", 4096, 1000)]

# per-tensor flag bits of the fused flat parameter set
FLAG_WEIGHT_DECAY = 1   # Section 4.2: only affine weights are regularised
FLAG_LARS = 2           # Eq. 1: layer-wise local rate


def resnet50_param_tensors(variant: str = "v1") -> List[Tuple[str, Tuple[int, ...], str, int]]:
    """(name, shape, kind, flags) of the 161 trainable tensors in fused-buffer order:
    per convolution its filter, then the batch-norm gamma and beta that follow it;
    last the classifier weight and bias.  kind in {"conv","gamma","beta","fc","bias"}.
    Weight decay only on filters and the classifier weight; LARS on every tensor.
    """
    out = []
    for cs in resnet50_convs(variant):
        out.append((cs.name + ".w", (cs.K, cs.R, cs.R, cs.C), "conv", FLAG_WEIGHT_DECAY | FLAG_LARS))
        out.append((cs.name + ".gamma", (cs.K,), "gamma", FLAG_LARS))
        out.append((cs.name + ".beta", (cs.K,), "beta", FLAG_LARS))
    out.append(("fc.w", (RESNET50_FC.O, RESNET50_FC.I), "fc", FLAG_WEIGHT_DECAY | FLAG_LARS))
    out.append(("fc.b", (RESNET50_FC.O,), "bias", FLAG_LARS))
    return out


def offsets_of(tensors) -> List[int]:
    off = [0]
    for _, shape, _, _ in tensors:
        n = 1
        for s in shape:
            n *= s
        off.append(off[-1] + n)
    return off
