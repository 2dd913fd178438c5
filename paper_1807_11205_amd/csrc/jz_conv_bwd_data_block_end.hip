// Kernel instantiations and variant dispatch of one implicit-GEMM operation (a translation unit of its own so that
// the operations compile in parallel).
#include "jz_igemm_kernels.h"

int jz::launch_bwd_data_block_end(const Plan& pl, hipStream_t st) { return launch_op<OP_BWD_DATA_BLOCK_END>(pl, st); }
