// Shared declarations of the library's translation units (HIP, gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "mc.h"

namespace mc {

typedef unsigned short bf16_t;   // bfloat16 bit pattern

__host__ __device__ inline float bf16_to_f32(bf16_t b) {
  union { uint32_t u; float f; } v;
  v.u = (uint32_t)b << 16;
  return v.f;
}

// round to nearest, ties to even; NaN stays NaN
__host__ __device__ inline bf16_t f32_to_bf16(float f) {
  union { uint32_t u; float f; } v;
  v.f = f;
  if ((v.u & 0x7FFFFFFFu) > 0x7F800000u) return (bf16_t)((v.u >> 16) | 0x40u);
  uint32_t lsb = (v.u >> 16) & 1u;
  return (bf16_t)((v.u + 0x7FFFu + lsb) >> 16);
}

template <typename T> struct Cvt;
template <> struct Cvt<float> {
  __host__ __device__ static float to_f32(float v) { return v; }
  __host__ __device__ static float from_f32(float v) { return v; }
};
template <> struct Cvt<bf16_t> {
  __host__ __device__ static float to_f32(bf16_t v) { return bf16_to_f32(v); }
  __host__ __device__ static bf16_t from_f32(float v) { return f32_to_bf16(v); }
};

// ---- error plumbing -----------------------------------------------------------------
void set_error(const char *fmt, ...);
#define MC_FAIL(code, ...)            \
  do {                                \
    ::mc::set_error(__VA_ARGS__);     \
    return (code);                    \
  } while (0)
#define MC_HIP(expr)                                                              \
  do {                                                                            \
    hipError_t e__ = (expr);                                                      \
    if (e__ != hipSuccess)                                                        \
      MC_FAIL(MC_ERR_DEVICE, "%s failed: %s", #expr, hipGetErrorString(e__));     \
  } while (0)
#define MC_TRY(expr)                  \
  do {                                \
    int s__ = (expr);                 \
    if (s__ != MC_OK) return s__;     \
  } while (0)

// Raise a kernel's limit of dynamic LDS to `bytes`, once per (kernel, device); safe to call from
// several threads and with several devices in one process.
int raise_dynamic_lds_limit(const void *kernel, int bytes);

// ---- geometry of one KV page ---------------------------------------------------------
// A page holds page_tokens keys of every KV head; head kvh owns elements
// [kvh * page_tokens * hd, (kvh + 1) * page_tokens * hd) of the K page and of the V page.
inline size_t page_elems(int n_kv_heads, int head_dim, int page_tokens) {
  return (size_t)n_kv_heads * head_dim * page_tokens;
}
// Inside a head's region there are two layouts.
//   plain (page_tokens % 32 != 0 or hd % 32 != 0): K as [key][hd], V transposed as [hd][key].
//   fragment order (otherwise): blocks of 32 keys, 32 * hd elements each.  A block is a run of
//     1 KB fragments, fragment f holding for lane l = 0..63 eight consecutive elements at
//     (f * 64 + l) * 8, exactly what one 32x32x16 MFMA reads as its A operand:
//       K fragment c (d = 16c..16c+15): lane l has key l % 32, d = 16c + 8 (l / 32) + 0..7;
//       V fragment 2 dt + sl: lane l has d = 32 dt + l % 32 and the eight keys
//         16 sl + 4 (l / 32) + {0,1,2,3, 8,9,10,11}, the order in which the transposed score
//         accumulator of the same MFMA holds its keys.
//     A wave then loads an operand with one fully coalesced 16-byte-per-lane instruction.
__host__ __device__ inline bool kv_fragment_layout(int page_tokens, int hd) {
  return page_tokens % 32 == 0 && hd % 32 == 0;
}
// element offset of K[key][d] / V[key][d] inside one head's region of a page
__host__ __device__ inline size_t k_elem_offset(int key, int d, int page_tokens, int hd) {
  if (!kv_fragment_layout(page_tokens, hd)) return (size_t)key * hd + d;
  const int lane = (key & 31) + 32 * ((d >> 3) & 1);
  return (size_t)(key >> 5) * 32 * hd + (size_t)((d >> 4) * 64 + lane) * 8 + (d & 7);
}
__host__ __device__ inline size_t v_elem_offset(int key, int d, int page_tokens, int hd) {
  if (!kv_fragment_layout(page_tokens, hd)) return (size_t)d * page_tokens + key;
  const int k16 = key & 15, sl = (key >> 4) & 1;
  const int lane = (d & 31) + 32 * ((k16 >> 2) & 1);
  const int j = 4 * (k16 >> 3) + (k16 & 3);
  return (size_t)(key >> 5) * 32 * hd + (size_t)(((d >> 5) * 2 + sl) * 64 + lane) * 8 + j;
}

// ---- tiled operand layout of the bf16 MFMA kernels --------------------------------------
// A [rows][K] matrix (rows padded to a multiple of 32, K % 64 == 0) is kept as 4 KB blocks;
// block (row / 32, k / 64) holds, as chunk c = (k % 32) / 8 of lane l = row % 32 + 32 ((k % 64) / 32),
// the 8 elements k - k % 8 .. +7.  This is the element offset of (row, k).
__host__ __device__ inline size_t tiled_offset(int row, int k, int K) {
  const int U = K >> 6;
  return ((size_t)(row >> 5) * U + (k >> 6)) * 2048 +
         (size_t)(((k & 31) >> 3) * 64 + (row & 31) + 32 * ((k & 63) >> 5)) * 8 + (k & 7);
}

// ---- kernel launchers (defined in kernels_*.hip) -----------------------------------
// Every launcher validates nothing: callers (runtime.cpp, ops.cpp) check shapes first.

struct AttnArgs {
  const void *q;                 // (T)[rows][Hq][hd]
  const void *k_prefix, *v_prefix, *k_suffix, *v_suffix;   // page pools of this layer
  const int32_t *row_pos;        // [rows] absolute position of each query row
  const int32_t *row_tab;        // [rows] page-table row of the query's sequence (unused if no suffix)
  const int32_t *page_table;     // [*][table_stride] suffix page ids
  int32_t table_stride;
  int32_t rows, n_q_heads, n_kv_heads, head_dim, page_tokens;
  int32_t prefix_len;            // keys at positions < prefix_len live in prefix pages pos / page_tokens
  void *out;                     // (T)[rows][Hq][hd], or the tiled [rows][Hq*hd] layout
  int32_t out_tiled;
};

struct DecodeAttnArgs {
  const void *q;                 // (T)[B][Hq][hd]
  const void *k_prefix, *v_prefix, *k_suffix, *v_suffix;
  const int32_t *page_table;
  int32_t table_stride;
  const int32_t *row_cand = nullptr;   // device: page-table row of each candidate row (nullptr: row r uses table row r)
  int32_t n_cands, n_q_heads, n_kv_heads, head_dim, page_tokens;
  int32_t prefix_len, suffix_len;
  // device, or nullptr: suffix keys of each candidate row (values outside 1..suffix_len are
  // clamped); nullptr = suffix_len for every row (lock-step)
  const int32_t *row_len = nullptr;
  int32_t prefix_splits;         // 0 = automatic
  void *workspace;
  size_t workspace_bytes;
  void *out;
  int32_t out_tiled;
};

int launch_embed(hipStream_t st, int dtype, int rows, int d, const int32_t *tokens,
                 const void *table, float *x);
int launch_add_rmsnorm(hipStream_t st, int dtype, int rows, int d, float *x, const float *partials,
                       int n_partials, const void *gain, float eps, void *h_out, int h_tiled);
int launch_gather_rows(hipStream_t st, int rows, int d, const float *x, const int32_t *idx,
                       float *out);
// tiled != 0: a, w (and the SwiGLU output) are in the tiled layout; bf16 only
// top_out != nullptr (tiled few-row layers with >= 2048 weight tiles only, see
// linear_top_lists_supported): also leave per-group top lists of every output row
bool linear_top_lists_supported(int dtype, int M, int N, int K, int tiled);
int launch_linear(hipStream_t st, int dtype, int M, int N, int K, const void *a, const void *w,
                  float *out, int n_splits, int tiled, void *top_out = nullptr);
int launch_linear_swiglu(hipStream_t st, int dtype, int M, int N, int K, const void *a,
                         const void *wg, const void *wu, void *out, int tiled);
// interleave_hd > 0: within every group of interleave_hd rows, destination row 2i takes source
// row i and destination row 2i + 1 source row i + interleave_hd / 2 (the two members of a rotary
// pair become neighbours)
int launch_pack_tiled(hipStream_t st, int rows, int K, const void *src, void *dst, int interleave_hd = 0);

// cos / sin of pos * base^(-2i/hd) in double for pos < n_pos, i < hd / 2: table[pos * hd/2 + i]
int launch_rope_table(hipStream_t st, int n_pos, int hd, double rope_base, double2 *table);

// Where the fused QKV layer puts its result (few-row bf16 path): rotated queries, and keys /
// values straight into their page slots.
struct RopeOut {
  const int32_t *row_pos, *row_page, *row_off;   // device, per row
  void *q_out, *k_pages, *v_pages;
  const double2 *table;                          // launch_rope_table
  int32_t Hq, Hkv, hd, pg;
};
// Events a profiling scope hands to the next launcher that knows how to attach them to its
// kernels (hipExtLaunchKernelGGL: the events then carry the kernel's own begin / end times, with
// no barrier packets around the launch).  A launcher takes them (which clears them); start goes to
// its first kernel, stop to its last.
struct LaunchEvents {
  hipEvent_t start = nullptr, stop = nullptr;
};
void offer_launch_events(hipEvent_t start, hipEvent_t stop);
LaunchEvents take_launch_events();
bool tiled_shapes_ok(int M, int N, int K);
// Tiled bf16 layers that finish their outputs themselves.  The fused QKV layer (rotation and
// query / key / value stores in the epilogue, w with interleaved query / key rows) exists for few
// rows and for products large enough for the 256-row-tile GEMM; x += a w^T for the latter only.
bool linear_qkv_rope_fused(int M, int N, int K);
int launch_linear_qkv_rope(hipStream_t st, int M, int N, int K, const void *a, const void *w, const RopeOut &ro);
bool linear_accumulate_fused(int M, int N, int K);
int launch_linear_accumulate(hipStream_t st, int M, int N, int K, const void *a, const void *w, float *x);
int launch_rope_kv(hipStream_t st, int dtype, int rows, int Hq, int Hkv, int hd, int page_tokens,
                   double rope_base, const float *qkv, int n_splits, const int32_t *row_pos,
                   const int32_t *row_page, const int32_t *row_off, void *q_out, void *k_pages,
                   void *v_pages, const double2 *table = nullptr, int qk_interleaved = 0);
int launch_attention_generic(hipStream_t st, int dtype, const AttnArgs &a);
size_t decode_attention_ws_bytes(int n_cands, int Hq, int Hkv, int hd, int prefix_len,
                                 int suffix_len, int page_tokens);
int launch_attention_decode(hipStream_t st, int dtype, const DecodeAttnArgs &a);
// top_lists != nullptr: the LM head's per-group top lists of the same rows ([row][n_groups][4]
// pairs of {float bits, id}, row stride top_stride pairs; 0 = every candidate reads row 0), which
// the selection uses instead of the rows where that is conclusive (see sample_kernel)
int launch_sample(hipStream_t st, int n_cands, int vocab, const float *logits, size_t row_stride,
                  float temperature, int top_k, const float *uniforms, int32_t *out_tokens,
                  int32_t *out_topk, const void *top_lists = nullptr, size_t top_stride = 0,
                  int n_groups = 0);
int launch_reward_score(hipStream_t st, int n_cands, int vocab, const float *logits,
                        const int32_t *reward_ids, const float *reward_values, int n_reward,
                        float score_temperature, float *out_logprobs, float *out_scores,
                        int32_t *out_rank);

// number of K-axis splits the linear kernels use for an [M x N x K] product
int linear_auto_splits(int dtype, int M, int N, int K, int tiled);

}  // namespace mc
