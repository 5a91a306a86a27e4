// bf16 MFMA kernels (gfx950): weight-streaming linear layers for few rows, tiled GEMM for many
// rows, split-K shared-prefix decode attention.
#pragma once
#include "common.h"

namespace mc {

// Attention kernels: a lane's sum of 16 probabilities above this means the reference maximum of
// the online softmax lags too far behind (or does not exist yet) and has to be moved.  2^20:
// far from overflow even after thousands of keys, and reached only when a score exceeds the
// reference by more than 16 in base-2 units.
constexpr float kSoftmaxSumLimit = 1048576.0f;

// maximum of the 16 values of an accumulator tile
template <typename V16>
__device__ inline float max16f(const V16 &s) {
  float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
#pragma unroll
  for (int r = 4; r < 16; r += 4) mx = fmaxf(mx, fmaxf(fmaxf(s[r], s[r + 1]), fmaxf(s[r + 2], s[r + 3])));
  return mx;
}

// x of lane (l ^ 32).  `addr` = ((l ^ 32) << 2), computed once by the caller: __shfl_xor would
// rebuild it (six vector instructions) at every use.
__device__ inline float swap_halves(float x, int addr) {
  return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(addr, __builtin_bit_cast(int, x)));
}

// All operands of these linear kernels are in the tiled layout (see tiled_offset).
// Few-row linear layer (M <= 64): out = a w^T streamed once over the weights.
// w2 != nullptr selects the SwiGLU form (out_t = silu(a wg^T) * (a wu^T), bf16, tiled).
bool skinny_linear_supported(int M, int N, int K);
int skinny_linear_splits(int M, int N, int K);
// rope != nullptr: the fused QKV layer (one K split): w has the rows of every query / key head
// interleaved (launch_pack_tiled), and the result goes where *rope says instead of to `out`.
// top_out != nullptr (plain sums of a layer with >= 2048 weight tiles, the LM head): besides the
// sums, for every row m and every group g of 64 consecutive outputs the kTopPerGroup largest
// (value, id) pairs under (value descending, id ascending), top_out[(m * N / 64 + g) * kTopPerGroup
// + t] = {float bits, id}: what the sampler needs of a row, 1 / 16 of its size.
constexpr int kTopPerGroup = 4;
bool skinny_top_lists_supported(int M, int N, int K);
int launch_linear_skinny(hipStream_t st, int M, int N, int K, const void *a, const void *w,
                         const void *w2, float *out, void *out_t, int n_splits,
                         const RopeOut *rope = nullptr, void *top_out = nullptr);

// Epilogue of the fused QKV layer for one row m and four consecutive outputs n .. n + 3 of the
// interleaved weight layout, i.e. coordinates (i, i + hd/2, i + 1, i + 1 + hd/2) of one query or
// key head (i = (n % hd) / 2), or four consecutive coordinates of a value head: rotate by the
// row's position (double, from the table) and store the query row-major, the key / value in its
// page slot.  In two steps, so that a caller with several quads can have all their loads in
// flight before the first store (stores may alias later loads as far as the compiler knows).
struct RopeQuad {
  double2 t0, t1;      // cos / sin of coordinates i and i + 1 at the row's position
  int32_t key, page;   // slot of the row in its KV page
};

__device__ inline RopeQuad rope_load_quad(const RopeOut &ro, int m, int n) {
  RopeQuad r;
  const int hd = ro.hd, head = n / hd, i = (n % hd) >> 1;
  r.key = ro.row_off[m];
  r.page = ro.row_page[m];
  if (head < ro.Hq + ro.Hkv) {
    const double2 *tp = ro.table + (size_t)ro.row_pos[m] * (hd >> 1) + i;
    r.t0 = tp[0];
    r.t1 = tp[1];
  } else {
    r.t0 = r.t1 = double2{1.0, 0.0};
  }
  return r;
}

__device__ inline void rope_store_quad(const RopeOut &ro, int m, int n, float4 s, const RopeQuad &r) {
  const int hd = ro.hd, half = hd >> 1, head = n / hd, jp = n % hd;
  const size_t pelems = (size_t)ro.Hkv * hd * ro.pg;
  if (head < ro.Hq + ro.Hkv) {
    const int i = jp >> 1;
    const double lo0 = s.x, hi0 = s.y, lo1 = s.z, hi1 = s.w;
    const uint32_t lo = (uint32_t)f32_to_bf16((float)(lo0 * r.t0.x - hi0 * r.t0.y)) |
                        ((uint32_t)f32_to_bf16((float)(lo1 * r.t1.x - hi1 * r.t1.y)) << 16);
    const uint32_t hi = (uint32_t)f32_to_bf16((float)(hi0 * r.t0.x + lo0 * r.t0.y)) |
                        ((uint32_t)f32_to_bf16((float)(hi1 * r.t1.x + lo1 * r.t1.y)) << 16);
    if (head < ro.Hq) {
      bf16_t *q = (bf16_t *)ro.q_out + ((size_t)m * ro.Hq + head) * hd;
      *(uint32_t *)(q + i) = lo;
      *(uint32_t *)(q + i + half) = hi;
    } else {
      bf16_t *k = (bf16_t *)ro.k_pages + (size_t)r.page * pelems + (size_t)(head - ro.Hq) * ro.pg * hd;
      *(uint32_t *)(k + k_elem_offset(r.key, i, ro.pg, hd)) = lo;          // i is even: i, i + 1 are adjacent
      *(uint32_t *)(k + k_elem_offset(r.key, i + half, ro.pg, hd)) = hi;
    }
  } else {
    bf16_t *v = (bf16_t *)ro.v_pages + (size_t)r.page * pelems + (size_t)(head - ro.Hq - ro.Hkv) * ro.pg * hd;
    v[v_elem_offset(r.key, jp, ro.pg, hd)] = f32_to_bf16(s.x);
    v[v_elem_offset(r.key, jp + 1, ro.pg, hd)] = f32_to_bf16(s.y);
    v[v_elem_offset(r.key, jp + 2, ro.pg, hd)] = f32_to_bf16(s.z);
    v[v_elem_offset(r.key, jp + 3, ro.pg, hd)] = f32_to_bf16(s.w);
  }
}

// Many-row GEMM (more than 64 rows): fp32 out, or the SwiGLU form with bf16 tiled out.  N % 128
// == 0, K % 64 == 0.  256 x 128 output tile per workgroup (256 x 64 of each weight matrix in the
// SwiGLU form), XCD-aware tile order.
bool gemm256_supported(int M, int N, int K, bool swiglu);
// rope != nullptr: the fused QKV layer as in launch_linear_skinny (N = (Hq + 2 Hkv) hd, hd % 4 == 0).
// accumulate: out[m][n] += the product (the residual stream updated in place) instead of a store.
int launch_gemm256(hipStream_t st, int M, int N, int K, const void *a, const void *w,
                   const void *w2, float *out, void *out_t, const RopeOut *rope = nullptr,
                   int accumulate = 0);

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
int decode_attention_plan(const DecodeAttnArgs &a, int32_t out[9]);

}  // namespace mc
