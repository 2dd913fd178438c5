#include "jz_internal.h"
extern "C" int jz_conv2d_workspace_bytes(int, const jz_conv_desc*, size_t*) { return JZ_ERR_UNSUPPORTED; }
extern "C" int jz_conv2d_fwd(const jz_conv_desc*, const void*, const void*, void*, void*, size_t, void*) { return JZ_ERR_UNSUPPORTED; }
extern "C" int jz_conv2d_bwd_data(const jz_conv_desc*, const void*, const void*, void*, void*, size_t, void*) { return JZ_ERR_UNSUPPORTED; }
extern "C" int jz_conv2d_bwd_weight(const jz_conv_desc*, const void*, const void*, void*, void*, size_t, void*) { return JZ_ERR_UNSUPPORTED; }
extern "C" int jz_gemm_fc_workspace_bytes(int, int, int, int, size_t*) { return JZ_ERR_UNSUPPORTED; }
extern "C" int jz_gemm_fc(int, int, int, int, const void*, const void*, void*, void*, size_t, void*) { return JZ_ERR_UNSUPPORTED; }
