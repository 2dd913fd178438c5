"""Pins for the oracle's own binary16 conversion: the format definition, the paper's
2^-24 underflow remark (Section 5.2) and an independent library (numpy)."""
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))


def test_all_bit_patterns_widen_like_numpy(orc):
    bits = np.arange(65536, dtype=np.uint16)
    mine = orc.half_to_double(bits)
    ref = bits.view(np.float16).astype(np.float64)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(mine), nan)
    assert np.array_equal(mine[~nan], ref[~nan])
    assert np.array_equal(np.signbit(mine[~nan]), np.signbit(ref[~nan]))


def test_round_trip_every_non_nan_pattern(orc):
    bits = np.arange(65536, dtype=np.uint16)
    vals = orc.half_to_double(bits)
    ok = ~np.isnan(vals)
    back = orc.round_to_half(vals)
    assert np.array_equal(back[ok], bits[ok])
    assert np.all((back[~ok] & 0x7c00) == 0x7c00) and np.all((back[~ok] & 0x03ff) != 0)


def test_golden_facts(orc):
    rows = []
    with open(os.path.join(HERE, "golden", "fp16_facts.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                rows.append((float.fromhex(line[0]), int(line[1], 16)))
    assert len(rows) >= 12
    got = orc.round_to_half(np.array([r[0] for r in rows]))
    for (v, want), g in zip(rows, got):
        assert int(g) == want, (v.hex(), hex(int(g)), hex(want))


def test_every_midpoint_ties_to_even_and_neighbours_round_correctly(orc):
    # all adjacent finite non-negative pairs (a,b): exact midpoint, and one fp64 ulp either side of it
    bits = np.arange(0, 0x7bff, dtype=np.uint16)
    a = orc.half_to_double(bits)
    b = orc.half_to_double(bits + 1)
    mid = 0.5 * (a + b)                       # exact in fp64
    even = np.where(bits % 2 == 0, bits, bits + 1)
    assert np.array_equal(orc.round_to_half(mid), even)
    assert np.array_equal(orc.round_to_half(np.nextafter(mid, np.inf)), bits + 1)
    assert np.array_equal(orc.round_to_half(np.nextafter(mid, -np.inf)), bits)
    # negative side mirrors it
    assert np.array_equal(orc.round_to_half(-mid), even | 0x8000)


def test_overflow_and_specials(orc):
    v = np.array([65504.0, 65519.999, 65520.0, 1e9, -65520.0, np.inf, -np.inf, 0.0, -0.0])
    want = [0x7bff, 0x7bff, 0x7c00, 0x7c00, 0xfc00, 0x7c00, 0xfc00, 0x0000, 0x8000]
    assert [int(t) for t in orc.round_to_half(v)] == want
    n = int(orc.round_to_half(np.array([np.nan]))[0])
    assert (n & 0x7c00) == 0x7c00 and (n & 0x3ff) != 0


def test_random_doubles_match_numpy_rounding(orc):
    rng = np.random.default_rng(5)
    v = np.concatenate([rng.standard_normal(200000) * s for s in (1e-7, 1e-4, 1.0, 300.0, 4e4)])
    mine = orc.round_to_half(v)
    ref = v.astype(np.float16).view(np.uint16)   # numpy converts fp64->fp16 with a single rounding
    assert np.array_equal(mine, ref)
    # and from fp32 values (what the fp32 master -> fp16 cast-back sees)
    f = v.astype(np.float32)
    assert np.array_equal(orc.round_to_half(f.astype(np.float64)), f.astype(np.float16).view(np.uint16))
