// Forward convolution of a small-channel strided layer (the 3-channel stems: 7x7 stride 2, 11x11 stride 4; Jia et al.
// 2018, Section 4.1: FP16 operands, FP32 accumulation) out of an input patch that sits in LDS.
//
// The general implicit-GEMM kernel gathers, for every output pixel and filter row, one run of 4*S halves of the padded
// 4-channel copy xp[N][Hp][Wp][4]: neighbouring pixels' runs overlap (a 7x7 stride-2 window shares 5/7 of its columns
// and rows with the next one), every workgroup re-reads the whole filter, and the layer ends up bound by the bytes
// brought into LDS (13x the input for the ResNet-50 stem, 10x for the 11x11 one) at a tenth to a quarter of its
// roofline.  Here a workgroup owns MB consecutive output pixels of one image (all output channels), brings the input
// rows they touch into LDS once as one contiguous copy of xp, keeps the whole repacked filter in LDS for all the
// blocks it works through, and the MFMA operands are read straight out of the patch: with 4 channels and an even
// stride, the 8 halves a lane needs for k step `ks` of filter row r and pixel (p, q) are the 16 aligned bytes at
//     patch[(p - p_first) sh + r][q sw + 2 ks' ...]      (two taps of four channels each)
// so no im2col copy exists anywhere.  Filter layout in the workspace and in LDS: wq[r][c8][k][8 halves] with
// c8 = (4 s + c) / 8, so that the 32 lanes of an operand read 512 consecutive bytes.  "Taps" beyond S (the run is
// rounded up to 16 halves) multiply zeros of wq with real, finite neighbouring pixels.
//
// One wavefront owns TM tiles of 32 pixels x all NT tiles of 32 channels; results are staged per tile through LDS
// (the patch's space) and stored as whole 16-byte pieces of NHWC rows.
#include <hip/hip_runtime.h>

#include "jz_conv_plan.h"

namespace {
using namespace jz;

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) unsigned char lds_byte;

// every wavefront has finished its LDS accesses up to here, and none starts one from behind this point before all have
// arrived (no wait for outstanding global stores, which __syncthreads would add)
__device__ __forceinline__ void lds_barrier() {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
#endif
}

template <int NT, int TM, int NKS, int WPE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(WPE, WPE))) void stem_fwd_kernel(StemArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int K = NT * 32;          // output channels (a multiple of 32)
  constexpr int MB = 4 * TM * 32;     // pixels per block
  constexpr int SP = K * 2 + 16;      // staging row pitch: 32 pixels x K halves, rows 16 bytes apart in banks
  constexpr int CH = K / 8;           // 16-byte pieces of an output row
  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, hi = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  lds_byte* const lds_w = (lds_byte*)smem;
  lds_byte* const lds_p = lds_w + a.lds_w_bytes;
  const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void*)a.wq, 0, (int)a.wq_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_x = __builtin_amdgcn_make_buffer_rsrc((void*)a.xp, 0, (int)a.xp_bytes, 0x00020000);
  const unsigned pitch = (unsigned)a.Wp * 8u;
  const int PQ = a.P * a.Q;

  // the filter, once per workgroup (lanes past its end receive zeros and write them into the region's padding)
  for (unsigned off = 0; off < a.wq_bytes; off += 4096)
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_w, lds_w + off + wave * 1024, 16, (int)(off + tid * 16), 0, 0, 0);

  const unsigned woff = (unsigned)((hi * K + l32) * 16);
  lds_byte* const stage = lds_p + wave * (32 * SP);

  for (int b = blockIdx.x; b < a.total_blocks; b += gridDim.x) {
    const int n = b / a.blocks_per_image, bi = b - n * a.blocks_per_image;
    const int pix0 = bi * MB;
    const int pix_end = pix0 + MB < PQ ? pix0 + MB : PQ;
    const int p_first = pix0 / a.Q, p_last = (pix_end - 1) / a.Q;
    const unsigned bytes = (unsigned)((p_last - p_first) * a.sh + a.R) * pitch;
    const unsigned gbase = (unsigned)((n * a.Hp + p_first * a.sh) * a.Wp) * 8u;
    lds_barrier();  // every wavefront has left the previous block's patch and staging rows
    for (unsigned off = 0; off < bytes; off += 4096)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_x, lds_p + off + wave * 1024, 16, (int)(gbase + off + tid * 16), 0, 0, 0);

    unsigned aoff[TM];
#pragma unroll
    for (int t = 0; t < TM; ++t) {
      int pix = pix0 + (wave * TM + t) * 32 + l32;
      if (pix > pix_end - 1) pix = pix_end - 1;  // rows of a ragged last tile: computed on a real pixel, never stored
      const int p = pix / a.Q, q = pix - p * a.Q;
      aoff[t] = (unsigned)((p - p_first) * a.sh) * pitch + (unsigned)(q * a.sw) * 8u + (unsigned)hi * 16u;
    }
    f32x16 acc[TM][NT];
#pragma unroll
    for (int t = 0; t < TM; ++t)
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][j][e] = 0.f;

    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    lds_barrier();  // filter and patch have landed for every wavefront

    // steps (r, ks) in order, two sets of operand registers: the reads of step s + 1 are issued in front of the MFMAs of
    // step s.  offB / offA: where the next step to be read starts in the filter / in a patch row.
    const int T = a.R * NKS;
    unsigned offA = 0, offB = 0;
    int ks_next = 0;
    half8 fb0[NT], fa0[TM], fb1[NT], fa1[TM];
    auto read_step = [&](half8 (&fb)[NT], half8 (&fa)[TM]) {
#pragma unroll
      for (int j = 0; j < NT; ++j) fb[j] = *reinterpret_cast<const __attribute__((address_space(3))) half8*>(lds_w + woff + offB + j * 512);
#pragma unroll
      for (int t = 0; t < TM; ++t) fa[t] = *reinterpret_cast<const __attribute__((address_space(3))) half8*>(lds_p + aoff[t] + offA);
      offB += 2 * K * 16;
      if (++ks_next == NKS) {
        ks_next = 0;
        offA += pitch - (NKS - 1) * 32;
      } else {
        offA += 32;
      }
    };
    auto mma_step = [&](const half8 (&fb)[NT], const half8 (&fa)[TM]) {
#pragma unroll
      for (int t = 0; t < TM; ++t)
#pragma unroll
        for (int j = 0; j < NT; ++j) acc[t][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[j], fa[t], acc[t][j], 0, 0, 0);
    };
    read_step(fb0, fa0);
    int s = 0;
    for (; s + 2 <= T; s += 2) {
      read_step(fb1, fa1);
      mma_step(fb0, fa0);
      if (s + 2 < T) read_step(fb0, fa0);
      mma_step(fb1, fa1);
    }
    if (s < T) mma_step(fb0, fa0);
    lds_barrier();  // the patch is free: its space now stages the results

    // lane (pixel l32, half hi) holds, per channel tile j and register group v4, channels j 32 + v4 8 + hi 4 .. + 4
    unsigned short* const yb = a.y + ((size_t)n * PQ + pix0) * K;
#pragma unroll
    for (int t = 0; t < TM; ++t) {
      const int tile0 = (wave * TM + t) * 32;  // first pixel of the tile, relative to pix0
      if (pix0 + tile0 >= pix_end) break;      // wave-uniform
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
          half4 h;
#pragma unroll
          for (int e = 0; e < 4; ++e) h[e] = (_Float16)acc[t][j][v4 * 4 + e];  // round to nearest even
          *reinterpret_cast<__attribute__((address_space(3))) half4*>(stage + l32 * SP + (j * 32 + v4 * 8 + hi * 4) * 2) = h;
        }
      // 32 CH = 4 K pieces, a multiple of 64: every lane has one in every pass
      half8 v[CH / 2];
#pragma unroll
      for (int it = 0; it < CH / 2; ++it) {
        const int id = it * 64 + lane;
        const int px = id / CH, c = id - px * CH;
        v[it] = *reinterpret_cast<const __attribute__((address_space(3))) half8*>(stage + px * SP + c * 16);
      }
#pragma unroll
      for (int it = 0; it < CH / 2; ++it) {
        const int id = it * 64 + lane;
        const int px = id / CH, c = id - px * CH;
        if (pix0 + tile0 + px < pix_end) *reinterpret_cast<half8*>(yb + (size_t)(tile0 + px) * K + c * 8) = v[it];
      }
    }
  }
}

template <int NT, int TM, int NKS, int WPE>
int launch_stem(const StemArgs& a, hipStream_t st) {
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&stem_fwd_kernel<NT, TM, NKS, WPE>), hipFuncAttributeMaxDynamicSharedMemorySize,
                            160 * 1024) != hipSuccess)
      return JZ_ERR_LAUNCH;
    attr_set = true;
  }
  hipLaunchKernelGGL((stem_fwd_kernel<NT, TM, NKS, WPE>), dim3((unsigned)a.grid), dim3(256), a.lds_w_bytes + a.lds_p_bytes, st, a);
  return jz::launch_status();
}

}  // namespace

// Instances: (channel tiles, pixel tiles per wavefront, workgroups per compute unit the register budget is set for).
// 64 channels: blocks of 256 pixels and three workgroups per compute unit measured 34 us against 37 us for 512 pixels
// and two (ResNet-50 stem, N = 64); 96 channels: the filter alone takes 101 KB of LDS, one workgroup per compute unit.
int jz::stem_fwd_tm(int NT) { return NT == 1 ? 6 : NT == 2 ? 2 : NT == 3 ? 2 : NT == 4 ? 2 : 0; }
int jz::stem_fwd_wgs(int NT) { return NT == 2 ? 3 : 2; }

template <int NKS>
static int launch_stem_nks(const StemArgs& a, hipStream_t st) {
  if (a.NT == 1) return launch_stem<1, 6, NKS, 2>(a, st);
  if (a.NT == 2) return launch_stem<2, 2, NKS, 3>(a, st);
  if (a.NT == 3) return launch_stem<3, 2, NKS, 2>(a, st);
  if (a.NT == 4) return launch_stem<4, 2, NKS, 2>(a, st);
  return JZ_ERR_UNSUPPORTED;
}

int jz::launch_stem_fwd(const StemArgs& a, hipStream_t st) {
  if (a.NKS == 1) return launch_stem_nks<1>(a, st);
  if (a.NKS == 2) return launch_stem_nks<2>(a, st);
  if (a.NKS == 3) return launch_stem_nks<3>(a, st);
  if (a.NKS == 4) return launch_stem_nks<4>(a, st);
  return JZ_ERR_UNSUPPORTED;
}
