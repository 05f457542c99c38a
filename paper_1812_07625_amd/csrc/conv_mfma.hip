// bf16 MFMA implicit-GEMM convolution kernels (placeholder: no shape is taken yet).
#include "common.h"
namespace w2l {
bool conv_fwd_mfma_ok(int, int, int, int, int, int) { return false; }
int conv_fwd_mfma(const void*, const void*, const float*, void*, int, int, int, int, int, int, int, hipStream_t) { return W2L_ERR_SHAPE; }
bool conv_dgrad_mfma_ok(int, int, int, int, int, int) { return false; }
int conv_dgrad_mfma(const void*, const void*, void*, int, int, int, int, int, int, hipStream_t) { return W2L_ERR_SHAPE; }
bool conv_wgrad_mfma_ok(int, int, int, int, int, int) { return false; }
size_t conv_wgrad_mfma_workspace(int, int, int, int, int, int) { return 0; }
int conv_wgrad_mfma(const void*, const void*, float*, int, int, int, int, int, int, int, void*, hipStream_t) { return W2L_ERR_SHAPE; }
}  // namespace w2l
