#include "kernels_mfma.h"
namespace mc {
bool skinny_linear_supported(int, int, int) { return false; }
int skinny_linear_splits(int, int, int) { return 1; }
int launch_linear_skinny(hipStream_t, int, int, int, const void *, const void *, const void *, float *, void *, int) { MC_FAIL(MC_ERR_UNSUPPORTED, "not built"); }
bool gemm_supported(int, int, int) { return false; }
int launch_gemm_mfma(hipStream_t, int, int, int, const void *, const void *, const void *, float *, void *) { MC_FAIL(MC_ERR_UNSUPPORTED, "not built"); }
bool decode_attention_mfma_supported(const DecodeAttnArgs &) { return false; }
size_t decode_attention_mfma_ws_bytes(int, int, int, int, int, int, int) { return 0; }
int launch_attention_decode_mfma(hipStream_t, const DecodeAttnArgs &) { MC_FAIL(MC_ERR_UNSUPPORTED, "not built"); }
}
