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

// Launch the kernel variant `pl` names on `st`; JZ_OK, JZ_ERR_UNSUPPORTED (no such variant) or JZ_ERR_LAUNCH.
int launch_fwd(const Plan& pl, hipStream_t st);
int launch_fwd_stats(const Plan& pl, hipStream_t st);  // forward that also leaves per-tile column sums
int launch_bwd_data_stats(const Plan& pl, hipStream_t st);  // backward-data that also leaves batch-norm backward sums
int launch_bwd_data_block_end(const Plan& pl, hipStream_t st);  // ... of the block-end gradient it forms from its tile
int launch_bwd_data(const Plan& pl, hipStream_t st);
int launch_bwd_weight(const Plan& pl, hipStream_t st);

}  // namespace jz
