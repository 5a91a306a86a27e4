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
// rope != nullptr: the fused QKV layer (one K split): w has the rows of every query / key head
// interleaved (launch_pack_tiled), and the result goes where *rope says instead of to `out`.
int launch_linear_skinny(hipStream_t st, int M, int N, int K, const void *a, const void *w,
                         const void *w2, float *out, void *out_t, int n_splits,
                         const RopeOut *rope = nullptr);

// Many-row GEMM: 1 split; fp32 out, or the SwiGLU form with bf16 out.
bool gemm_supported(int M, int N, int K);
int launch_gemm_mfma(hipStream_t st, int M, int N, int K, const void *a, const void *w,
                     const void *w2, float *out, void *out_t);

// The same for shapes that fill 256-row tiles (N % 256 == 0, or N % 128 == 0 in the SwiGLU form):
// 256 x 256 output tile per workgroup, double-buffered LDS, XCD-aware tile order.
bool gemm256_supported(int M, int N, int K, bool swiglu);
int launch_gemm256(hipStream_t st, int M, int N, int K, const void *a, const void *w,
                   const void *w2, float *out, void *out_t);

// Streaming-read probe over `bytes` of device memory (a multiple of 64 MiB); out: one word.
int launch_read_probe(hipStream_t st, const void *buf, size_t bytes, uint32_t *out);

// MFMA-only probe: n_workgroups * 256 threads, each with 6 x 16 bytes of bf16 operands.
int launch_mfma_probe(hipStream_t st, const void *operands, float *out, int n_workgroups, int iters);

// Causal attention over many rows.  items[i] = (first row, rows <= 64, position of the first
// row, page-table row or -1): up to 64 consecutive positions of one sequence.  Keys at positions
// < prefix_len come from the prefix pages, later ones from the sequence's suffix pages.
struct PrefillAttnArgs {
  const void *q;                 // bf16 [rows][Hq][hd]
  const void *k_prefix, *v_prefix, *k_suffix, *v_suffix;
  const int4 *items;             // device
  int32_t n_items;
  const int32_t *page_table;
  int32_t table_stride;
  int32_t n_q_heads, n_kv_heads, head_dim, page_tokens, prefix_len;
  void *out;                     // bf16 [rows][Hq*hd], row-major or tiled
  int32_t out_tiled;
};
bool prefill_attention_mfma_supported(int page_tokens, int head_dim, int Hq, int Hkv);
int launch_attention_prefill_mfma(hipStream_t st, const PrefillAttnArgs &a);

bool decode_attention_mfma_supported(const DecodeAttnArgs &a);
size_t decode_attention_mfma_ws_bytes(int n_cands, int Hq, int Hkv, int hd, int prefix_len,
                                      int suffix_len, int page_tokens);
int launch_attention_decode_mfma(hipStream_t st, const DecodeAttnArgs &a);
int decode_attention_plan(const DecodeAttnArgs &a, int32_t out[8]);

}  // namespace mc
