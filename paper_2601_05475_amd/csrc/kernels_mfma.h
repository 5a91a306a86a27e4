// bf16 MFMA kernels (gfx950): weight-streaming linear layers for few rows, tiled GEMM for many
// rows, split-K shared-prefix decode attention.
#pragma once
#include "common.h"

namespace mc {

// All operands of these linear kernels are in the tiled layout (see tiled_offset).
// Few-row linear layer (M <= 64): out = a w^T streamed once over the weights.
// w2 != nullptr selects the SwiGLU form (out_t = silu(a wg^T) * (a wu^T), bf16, tiled).
bool skinny_linear_supported(int M, int N, int K);
int skinny_linear_splits(int M, int N, int K);
int launch_linear_skinny(hipStream_t st, int M, int N, int K, const void *a, const void *w,
                         const void *w2, float *out, void *out_t, int n_splits);

// Many-row GEMM: 1 split; fp32 out, or the SwiGLU form with bf16 out.
bool gemm_supported(int M, int N, int K);
int launch_gemm_mfma(hipStream_t st, int M, int N, int K, const void *a, const void *w,
                     const void *w2, float *out, void *out_t);

bool decode_attention_mfma_supported(const DecodeAttnArgs &a);
size_t decode_attention_mfma_ws_bytes(int n_cands, int Hq, int Hkv, int hd, int prefix_len,
                                      int suffix_len, int page_tokens);
int launch_attention_decode_mfma(hipStream_t st, const DecodeAttnArgs &a);

}  // namespace mc
