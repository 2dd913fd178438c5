// What the planner hands to the kernel launchers of the implicit-GEMM family: the GEMM view of one convolution /
// fully connected operation with the kernel variant chosen for it.  The launchers live in one translation unit per
// operation (jz_conv_fwd.hip, jz_conv_fwd_stats.hip, jz_conv_bwd_data.hip, jz_conv_bwd_data_stats.hip, jz_conv_bwd_data_block_end.hip, jz_conv_bwd_weight.hip) so that they
// compile in parallel; the planner and the entry points are in jz_conv.hip.
#pragma once
#include "jz_igemm.h"
#include "jz_internal.h"

namespace jz {

struct Plan {
  int op = 0;
  bool fast = false;    // vector (16-byte) operand access possible
  bool packed = false;  // small-channel layer run on a 4-channel padded copy
  bool gen = false;     // gather with per-load tap arithmetic (more than 32 taps, strided multi-tap backward-data)
  bool classes = false; // strided multi-tap backward-data as one unit-stride launch per parity class of the stride
  bool stem = false;    // packed forward layer that runs on the patch kernel (jz_conv_stem.hip) unless column sums are asked for
  bool rt_forced = false;  // the variant comes from jz_conv2d_tune_set (the patch kernel then steps aside)
  int BM = 128, BN = 128;
  int bk = 64;  // k tile depth of the kernel that will run
  int waves = 4, nst = 4;  // wavefronts per workgroup and ring depth (large tiles come in several variants)
  GemmArgs args{};
  size_t ws_bytes = 0;       // total workspace
  size_t part_offset = 0;    // where the split-K partial sums start inside it
  size_t bytesA = 0, bytesB = 0, bytesD = 0;  // caller's operand sizes in bytes, for the overlap checks
  // packed mode
  int Hp = 0, Wp = 0, KT = 0;
  size_t xp_bytes = 0, wp_bytes = 0;
};

// Small-channel forward layer on the patch kernel: the padded 4-channel copy, the filter repacked as
// wq[R][NKS * 2][K][8 halves], blocks of 128 * TM consecutive output pixels of one image.
struct StemArgs {
  const unsigned short* xp = nullptr;
  const unsigned short* wq = nullptr;
  unsigned short* y = nullptr;
  unsigned xp_bytes = 0, wq_bytes = 0;
  int N = 0, Hp = 0, Wp = 0, P = 0, Q = 0, R = 0, sh = 0, sw = 0;
  int NT = 0;   // output channels / 32
  int NKS = 0;  // MFMA k steps per filter row: ceil(4 S / 16)
  int blocks_per_image = 0, total_blocks = 0, grid = 0;
  unsigned lds_w_bytes = 0, lds_p_bytes = 0;  // filter region, patch / staging region (multiples of 4096)
};
int stem_fwd_tm(int NT);  // 32-pixel tiles per wavefront of the instance for NT channel tiles (0: none)
int stem_fwd_wgs(int NT); // workgroups of that instance a compute unit's registers hold
int launch_stem_fwd(const StemArgs& a, hipStream_t st);

// Launch the kernel variant `pl` names on `st`; JZ_OK, JZ_ERR_UNSUPPORTED (no such variant) or JZ_ERR_LAUNCH.
int launch_fwd(const Plan& pl, hipStream_t st);
int launch_fwd_stats(const Plan& pl, hipStream_t st);  // forward that also leaves per-tile column sums
int launch_bwd_data_stats(const Plan& pl, hipStream_t st);  // backward-data that also leaves batch-norm backward sums
int launch_bwd_data_block_end(const Plan& pl, hipStream_t st);  // ... of the block-end gradient it forms from its tile
int launch_bwd_data(const Plan& pl, hipStream_t st);
int launch_bwd_weight(const Plan& pl, hipStream_t st);

}  // namespace jz
