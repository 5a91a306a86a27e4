// Single-operation entry points of the C ABI (device pointers in, device pointers out) and the
// dispatch between the generic ALU kernels and the bf16 MFMA kernels.
#include <math.h>

#include <algorithm>
#include <mutex>
#include <set>
#include <utility>

#include "common.h"
#include "kernels_mfma.h"

namespace mc {

int launch_linear_generic(hipStream_t st, int dtype, int M, int N, int K, const void *a,
                          const void *w, float *out, int n_splits);
int launch_linear_swiglu_generic(hipStream_t st, int dtype, int M, int N, int K, const void *a,
                                 const void *wg, const void *wu, void *out);

// Shapes the tiled bf16 kernels cover for every row count: few rows go to the weight-streaming
// kernel (K % 256), many rows to the tiled GEMM (N % 128).
static thread_local LaunchEvents tl_launch_events;
void offer_launch_events(hipEvent_t start, hipEvent_t stop) {
  tl_launch_events.start = start;
  tl_launch_events.stop = stop;
}
LaunchEvents take_launch_events() {
  const LaunchEvents e = tl_launch_events;
  tl_launch_events = LaunchEvents{};
  return e;
}

int raise_dynamic_lds_limit(const void *kernel, int bytes) {
  static std::mutex mu;
  static std::set<std::pair<const void *, int>> done;
  int dev = 0;
  MC_HIP(hipGetDevice(&dev));
  std::lock_guard<std::mutex> lock(mu);
  if (done.count({kernel, dev})) return MC_OK;
  MC_HIP(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
  done.insert({kernel, dev});
  return MC_OK;
}

bool tiled_shapes_ok(int M, int N, int K) {
  (void)M;
  return N % 128 == 0 && K % 256 == 0;
}

// Many-row products on tiled operands all go to the one MFMA GEMM (it beats a 128 x 128-tile
// kernel from 128 rows up, measured).
static bool use_gemm256(int M, int N, int K, bool swiglu) { return M > 64 && gemm256_supported(M, N, K, swiglu); }

int linear_auto_splits(int dtype, int M, int N, int K, int tiled) {
  if (tiled) return (dtype == MC_BF16 && M <= 64) ? skinny_linear_splits(M, N, K) : 1;
  if (M > 64) return 1;
  // generic kernel, few rows: aim at >= 256 workgroups while keeping >= 256 of K per split
  const int tiles = (N + 63) / 64;
  int s = 1;
  while (tiles * s < 256 && K / (s * 2) >= 256 && s < 16) s *= 2;
  return s;
}

bool linear_top_lists_supported(int dtype, int M, int N, int K, int tiled) {
  return tiled && dtype == MC_BF16 && M <= 64 && tiled_shapes_ok(M, N, K) && skinny_top_lists_supported(M, N, K);
}

int launch_linear(hipStream_t st, int dtype, int M, int N, int K, const void *a, const void *w,
                  float *out, int n_splits, int tiled, void *top_out) {
  if (top_out && !(n_splits == 1 && linear_top_lists_supported(dtype, M, N, K, tiled)))
    MC_FAIL(MC_ERR_UNSUPPORTED, "per-group top lists: M=%d N=%d K=%d not covered", M, N, K);
  if (!tiled) return launch_linear_generic(st, dtype, M, N, K, a, w, out, n_splits);
  if (dtype != MC_BF16 || !tiled_shapes_ok(M, N, K))
    MC_FAIL(MC_ERR_UNSUPPORTED, "tiled linear layer: bf16 with N %% 128 == 0 and K %% 256 == 0 only");
  if (M <= 64) return launch_linear_skinny(st, M, N, K, a, w, nullptr, out, nullptr, n_splits, nullptr, top_out);
  if (n_splits != 1) MC_FAIL(MC_ERR_UNSUPPORTED, "the many-row GEMM does not split K");
  return launch_gemm256(st, M, N, K, a, w, nullptr, out, nullptr);
}

bool linear_qkv_rope_fused(int M, int N, int K) {
  if (!tiled_shapes_ok(M, N, K)) return false;
  return M <= 64 ? skinny_linear_supported(M, N, K) : use_gemm256(M, N, K, false);
}

int launch_linear_qkv_rope(hipStream_t st, int M, int N, int K, const void *a, const void *w, const RopeOut &ro) {
  if (!linear_qkv_rope_fused(M, N, K)) MC_FAIL(MC_ERR_UNSUPPORTED, "fused QKV layer: M=%d N=%d K=%d not covered", M, N, K);
  if (M <= 64) return launch_linear_skinny(st, M, N, K, a, w, nullptr, nullptr, nullptr, 1, &ro);
  return launch_gemm256(st, M, N, K, a, w, nullptr, nullptr, nullptr, &ro, 0);
}

bool linear_accumulate_fused(int M, int N, int K) {
  return tiled_shapes_ok(M, N, K) && M > 64 && use_gemm256(M, N, K, false);
}

int launch_linear_accumulate(hipStream_t st, int M, int N, int K, const void *a, const void *w, float *x) {
  if (!linear_accumulate_fused(M, N, K)) MC_FAIL(MC_ERR_UNSUPPORTED, "accumulating linear layer: M=%d N=%d K=%d not covered", M, N, K);
  return launch_gemm256(st, M, N, K, a, w, nullptr, x, nullptr, nullptr, 1);
}

int launch_linear_swiglu(hipStream_t st, int dtype, int M, int N, int K, const void *a,
                         const void *wg, const void *wu, void *out, int tiled) {
  if (!tiled) return launch_linear_swiglu_generic(st, dtype, M, N, K, a, wg, wu, out);
  if (dtype != MC_BF16 || !tiled_shapes_ok(M, N, K))
    MC_FAIL(MC_ERR_UNSUPPORTED, "tiled linear layer: bf16 with N %% 128 == 0 and K %% 256 == 0 only");
  if (M <= 64) return launch_linear_skinny(st, M, N, K, a, wg, wu, nullptr, out, 1);
  return launch_gemm256(st, M, N, K, a, wg, wu, nullptr, out);
}

// ---- decode attention: MFMA split-K kernel when the shape allows, else the generic kernel ---
__global__ void fill_decode_rows_kernel(int B, int prefix_len, int suffix_len,
                                        const int32_t *__restrict__ row_len,
                                        const int32_t *__restrict__ row_cand,
                                        int32_t *row_pos, int32_t *row_tab) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < B) {
    const int len = (row_len && suffix_len) ? min(max(row_len[b], 1), suffix_len) : suffix_len;
    row_pos[b] = prefix_len + len - 1;          // the row sees the keys at positions <= this one
    row_tab[b] = row_cand ? row_cand[b] : b;
  }
}

size_t decode_attention_ws_bytes(int n_cands, int Hq, int Hkv, int hd, int prefix_len,
                                 int suffix_len, int page_tokens) {
  size_t generic = (size_t)n_cands * 2 * sizeof(int32_t) + 256;
  size_t tuned = decode_attention_mfma_ws_bytes(n_cands, Hq, Hkv, hd, prefix_len, suffix_len, page_tokens);
  return std::max(generic, tuned);
}

int launch_attention_decode(hipStream_t st, int dtype, const DecodeAttnArgs &a) {
  if (a.n_cands <= 0) return MC_OK;
  if (dtype == MC_BF16 && decode_attention_mfma_supported(a))
    return launch_attention_decode_mfma(st, a);
  if (a.workspace_bytes < (size_t)a.n_cands * 2 * sizeof(int32_t))
    MC_FAIL(MC_ERR_INVALID, "attention workspace too small");
  int32_t *row_pos = (int32_t *)a.workspace, *row_tab = row_pos + a.n_cands;
  fill_decode_rows_kernel<<<(a.n_cands + 63) / 64, 64, 0, st>>>(
      a.n_cands, a.prefix_len, a.suffix_len, a.row_len, a.row_cand, row_pos, row_tab);
  MC_HIP(hipGetLastError());
  AttnArgs g;
  g.q = a.q; g.k_prefix = a.k_prefix; g.v_prefix = a.v_prefix; g.k_suffix = a.k_suffix;
  g.v_suffix = a.v_suffix; g.row_pos = row_pos; g.row_tab = row_tab; g.page_table = a.page_table;
  g.table_stride = a.table_stride; g.rows = a.n_cands; g.n_q_heads = a.n_q_heads;
  g.n_kv_heads = a.n_kv_heads; g.head_dim = a.head_dim; g.page_tokens = a.page_tokens;
  g.prefix_len = a.prefix_len; g.out = a.out; g.out_tiled = a.out_tiled;
  return launch_attention_generic(st, dtype, g);
}

static int check_dtype(int dtype) {
  if (dtype != MC_F32 && dtype != MC_BF16) MC_FAIL(MC_ERR_INVALID, "unknown dtype %d", dtype);
  return MC_OK;
}

static int check_tiled(int dtype, int tiled, int K) {
  if (tiled != 0 && tiled != 1) MC_FAIL(MC_ERR_INVALID, "tiled must be 0 or 1");
  if (tiled && (dtype != MC_BF16 || K % 64)) MC_FAIL(MC_ERR_UNSUPPORTED, "the tiled layout is bf16 with K %% 64 == 0");
  return MC_OK;
}

}  // namespace mc

using namespace mc;

extern "C" size_t mc_op_tiled_bytes(int32_t rows, int32_t K) {
  if (rows < 1 || K < 64 || K % 64) return 0;
  return (size_t)((rows + 31) / 32 * 32) * K * 2;
}

extern "C" int mc_op_pack_tiled(void *stream, int32_t rows, int32_t K, const void *src, void *dst) {
  if (rows < 0 || K < 64 || K % 64) MC_FAIL(MC_ERR_INVALID, "bad sizes (K must be a multiple of 64)");
  if (!src || !dst) MC_FAIL(MC_ERR_INVALID, "a pointer is NULL");
  return launch_pack_tiled((hipStream_t)stream, rows, K, src, dst);
}

extern "C" int mc_op_add_rmsnorm(void *stream, int32_t dtype, int32_t rows, int32_t d, float *x,
                                 const float *partials, int32_t n_partials, const void *gain,
                                 float eps, void *h_out, int32_t h_tiled) {
  MC_TRY(check_dtype(dtype));
  if (rows < 0 || d < 1 || n_partials < 0) MC_FAIL(MC_ERR_INVALID, "bad sizes");
  if (!x || !gain || !h_out || (n_partials && !partials)) MC_FAIL(MC_ERR_INVALID, "a pointer is NULL");
  MC_TRY(check_tiled(dtype, h_tiled, d));
  return launch_add_rmsnorm((hipStream_t)stream, dtype, rows, d, x, partials, n_partials, gain, eps, h_out, h_tiled);
}

extern "C" int mc_op_linear(void *stream, int32_t dtype, int32_t M, int32_t N, int32_t K,
                            const void *a, const void *w, float *out, int32_t n_splits,
                            int32_t tiled) {
  MC_TRY(check_dtype(dtype));
  if (M < 0 || N < 1 || K < 1 || n_splits < 1 || n_splits > K) MC_FAIL(MC_ERR_INVALID, "bad sizes");
  if (!a || !w || !out) MC_FAIL(MC_ERR_INVALID, "a pointer is NULL");
  MC_TRY(check_tiled(dtype, tiled, K));
  return launch_linear((hipStream_t)stream, dtype, M, N, K, a, w, out, n_splits, tiled);
}

extern "C" int mc_op_linear_accumulate(void *stream, int32_t M, int32_t N, int32_t K, const void *a,
                                       const void *w, float *x) {
  if (M < 1 || N < 1 || K < 1) MC_FAIL(MC_ERR_INVALID, "bad sizes");
  if (!a || !w || !x) MC_FAIL(MC_ERR_INVALID, "a pointer is NULL");
  return launch_linear_accumulate((hipStream_t)stream, M, N, K, a, w, x);
}

extern "C" int mc_op_linear_qkv_rope(void *stream, int32_t rows, int32_t n_q_heads, int32_t n_kv_heads,
                                     int32_t head_dim, int32_t page_tokens, int32_t K, float rope_base,
                                     int32_t n_pos, const void *a, const void *wqkv,
                                     const int32_t *row_pos, const int32_t *row_page,
                                     const int32_t *row_off, void *table, void *q_out, void *k_pages,
                                     void *v_pages) {
  if (rows < 1 || n_q_heads < 1 || n_kv_heads < 1 || head_dim < 4 || head_dim % 4 || page_tokens < 1 ||
      K < 1 || n_pos < 1 || !(rope_base > 0.f))
    MC_FAIL(MC_ERR_INVALID, "bad sizes");
  if (!a || !wqkv || !row_pos || !row_page || !row_off || !table || !q_out || !k_pages || !v_pages)
    MC_FAIL(MC_ERR_INVALID, "a pointer is NULL");
  hipStream_t st = (hipStream_t)stream;
  MC_TRY(launch_rope_table(st, n_pos, head_dim, (double)rope_base, (double2 *)table));
  RopeOut ro;
  ro.row_pos = row_pos; ro.row_page = row_page; ro.row_off = row_off;
  ro.q_out = q_out; ro.k_pages = k_pages; ro.v_pages = v_pages; ro.table = (const double2 *)table;
  ro.Hq = n_q_heads; ro.Hkv = n_kv_heads; ro.hd = head_dim; ro.pg = page_tokens;
  return launch_linear_qkv_rope(st, rows, (n_q_heads + 2 * n_kv_heads) * head_dim, K, a, wqkv, ro);
}

extern "C" int32_t mc_op_linear_splits(int32_t dtype, int32_t M, int32_t N, int32_t K, int32_t tiled) {
  if (M < 1 || N < 1 || K < 1) return 0;
  return linear_auto_splits(dtype, M, N, K, tiled);
}

extern "C" int mc_op_linear_swiglu(void *stream, int32_t dtype, int32_t M, int32_t N, int32_t K,
                                   const void *a, const void *w_gate, const void *w_up, void *out,
                                   int32_t tiled) {
  MC_TRY(check_dtype(dtype));
  if (M < 0 || N < 1 || K < 1) MC_FAIL(MC_ERR_INVALID, "bad sizes");
  if (!a || !w_gate || !w_up || !out) MC_FAIL(MC_ERR_INVALID, "a pointer is NULL");
  MC_TRY(check_tiled(dtype, tiled, K));
  return launch_linear_swiglu((hipStream_t)stream, dtype, M, N, K, a, w_gate, w_up, out, tiled);
}

extern "C" int mc_op_rope_kv_write(void *stream, int32_t dtype, int32_t rows, int32_t n_q_heads,
                                   int32_t n_kv_heads, int32_t head_dim, int32_t page_tokens,
                                   float rope_base, const float *qkv, int32_t n_splits,
                                   const int32_t *row_pos, const int32_t *row_page,
                                   const int32_t *row_off, void *q_out, void *k_pages,
                                   void *v_pages) {
  MC_TRY(check_dtype(dtype));
  if (rows < 0 || n_q_heads < 1 || n_kv_heads < 1 || head_dim < 2 || head_dim % 2 || page_tokens < 1 ||
      n_splits < 1 || !(rope_base > 0.f))
    MC_FAIL(MC_ERR_INVALID, "bad sizes");
  if (!qkv || !row_pos || !row_page || !row_off || !q_out || !k_pages || !v_pages)
    MC_FAIL(MC_ERR_INVALID, "a pointer is NULL");
  return launch_rope_kv((hipStream_t)stream, dtype, rows, n_q_heads, n_kv_heads, head_dim,
                        page_tokens, (double)rope_base, qkv, n_splits, row_pos, row_page, row_off,
                        q_out, k_pages, v_pages);
}

extern "C" size_t mc_op_attention_decode_ws(int32_t n_cands, int32_t n_q_heads, int32_t n_kv_heads,
                                            int32_t head_dim, int32_t prefix_len,
                                            int32_t suffix_len, int32_t page_tokens) {
  if (n_cands < 1 || n_q_heads < 1 || n_kv_heads < 1 || head_dim < 2 || prefix_len < 0 ||
      suffix_len < 0 || page_tokens < 1)
    return 0;
  return decode_attention_ws_bytes(n_cands, n_q_heads, n_kv_heads, head_dim, prefix_len, suffix_len, page_tokens);
}

extern "C" int mc_op_attention_decode(void *stream, int32_t dtype, int32_t n_cands,
                                      int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                      int32_t page_tokens, int32_t prefix_len, int32_t suffix_len,
                                      const void *q, const void *k_prefix, const void *v_prefix,
                                      const void *k_suffix, const void *v_suffix,
                                      const int32_t *page_table, int32_t table_stride,
                                      const int32_t *row_len, int32_t prefix_splits, void *workspace,
                                      size_t workspace_bytes, void *out, int32_t out_tiled) {
  MC_TRY(check_dtype(dtype));
  if (n_cands < 1 || n_q_heads < 1 || n_kv_heads < 1 || n_q_heads % n_kv_heads || head_dim < 2 ||
      head_dim > 256 || page_tokens < 1 || (page_tokens & (page_tokens - 1)) || prefix_len < 0 ||
      suffix_len < 0 || prefix_len + suffix_len < 1 || prefix_splits < 0)
    MC_FAIL(MC_ERR_INVALID, "bad sizes");
  if (!q || !out || !workspace || (prefix_len && (!k_prefix || !v_prefix)) ||
      (suffix_len && (!k_suffix || !v_suffix || !page_table)))
    MC_FAIL(MC_ERR_INVALID, "a pointer is NULL");
  MC_TRY(check_tiled(dtype, out_tiled, n_q_heads * head_dim));
  if (suffix_len && table_stride < (suffix_len + page_tokens - 1) / page_tokens)
    MC_FAIL(MC_ERR_INVALID, "table_stride %d too small for %d suffix tokens", table_stride, suffix_len);
  const size_t need = decode_attention_ws_bytes(n_cands, n_q_heads, n_kv_heads, head_dim, prefix_len, suffix_len, page_tokens);
  if (workspace_bytes < need) MC_FAIL(MC_ERR_INVALID, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
  DecodeAttnArgs a;
  a.q = q; a.k_prefix = k_prefix; a.v_prefix = v_prefix; a.k_suffix = k_suffix; a.v_suffix = v_suffix;
  a.page_table = page_table; a.table_stride = table_stride; a.n_cands = n_cands;
  a.n_q_heads = n_q_heads; a.n_kv_heads = n_kv_heads; a.head_dim = head_dim;
  a.page_tokens = page_tokens; a.prefix_len = prefix_len; a.suffix_len = suffix_len;
  a.row_len = suffix_len ? row_len : nullptr;
  a.prefix_splits = prefix_splits; a.workspace = workspace; a.workspace_bytes = workspace_bytes;
  a.out = out; a.out_tiled = out_tiled;
  return launch_attention_decode((hipStream_t)stream, dtype, a);
}

// ---- decode attention for callers that cannot allocate ---------------------------------------
// The partial states of the split-K kernels live in a file-scope device array instead of a
// caller's workspace.  The array's name is only a host-side stand-in: its device address is looked
// up once per device (every GPU holds its own copy) and that pointer is what host code uses.
static __device__ __align__(256) unsigned char scratch[MC_STATIC_SCRATCH_BYTES];

namespace mc {
constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

// device address of `scratch` on the current device (looked up on the first call per device)
static int static_scratch(void **out) {
  int dev = -1;
  MC_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) MC_FAIL(MC_ERR_UNSUPPORTED, "device ordinal %d outside [0, %d)", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    MC_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) MC_FAIL(MC_ERR_DEVICE, "hipGetSymbolAddress returned a null address");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return MC_OK;
}
}  // namespace mc

extern "C" int mc_op_attention_decode_static(void *stream, int32_t dtype, int32_t n_cands,
                                             int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                             int32_t page_tokens, int32_t prefix_len, int32_t suffix_len,
                                             const void *q, const void *k_prefix, const void *v_prefix,
                                             const void *k_suffix, const void *v_suffix,
                                             const int32_t *page_table, int32_t table_stride,
                                             const int32_t *row_len, int32_t prefix_splits, void *out,
                                             int32_t out_tiled) {
  const size_t need = mc_op_attention_decode_ws(n_cands, n_q_heads, n_kv_heads, head_dim, prefix_len,
                                                suffix_len, page_tokens);
  if (need == 0) MC_FAIL(MC_ERR_INVALID, "bad sizes");
  if (need > (size_t)MC_STATIC_SCRATCH_BYTES)
    MC_FAIL(MC_ERR_UNSUPPORTED, "decode attention needs %zu bytes of scratch, the static buffer holds %zu: use "
            "mc_op_attention_decode with a workspace", need, (size_t)MC_STATIC_SCRATCH_BYTES);
  void *ws = nullptr;
  MC_TRY(static_scratch(&ws));
  return mc_op_attention_decode(stream, dtype, n_cands, n_q_heads, n_kv_heads, head_dim, page_tokens,
                                prefix_len, suffix_len, q, k_prefix, v_prefix, k_suffix, v_suffix, page_table,
                                table_stride, row_len, prefix_splits, ws, (size_t)MC_STATIC_SCRATCH_BYTES, out,
                                out_tiled);
}

extern "C" int mc_op_attention_decode_plan(int32_t n_cands, int32_t n_q_heads, int32_t n_kv_heads,
                                           int32_t head_dim, int32_t page_tokens, int32_t prefix_len,
                                           int32_t suffix_len, int32_t prefix_splits, int32_t *out9) {
  if (!out9 || n_cands < 1 || n_q_heads < 1 || n_kv_heads < 1 || n_q_heads % n_kv_heads || prefix_len < 0 ||
      suffix_len < 0 || prefix_len + suffix_len < 1 || prefix_splits < 0)
    MC_FAIL(MC_ERR_INVALID, "bad sizes");
  DecodeAttnArgs a{};
  a.n_cands = n_cands; a.n_q_heads = n_q_heads; a.n_kv_heads = n_kv_heads; a.head_dim = head_dim;
  a.page_tokens = page_tokens; a.prefix_len = prefix_len; a.suffix_len = suffix_len;
  a.prefix_splits = prefix_splits;
  return decode_attention_plan(a, out9);
}

extern "C" int mc_op_read_probe(void *stream, const void *buf, size_t bytes, void *out_word) {
  if (!buf || !out_word) MC_FAIL(MC_ERR_INVALID, "mc_op_read_probe: NULL pointer");
  return launch_read_probe((hipStream_t)stream, buf, bytes, (uint32_t *)out_word);
}

extern "C" int mc_op_mfma_probe(void *stream, const void *operands, float *out, int32_t n_workgroups,
                                int32_t iters) {
  if (!operands || !out || n_workgroups < 1 || n_workgroups > (1 << 20) || iters < 1 || iters > (1 << 24))
    MC_FAIL(MC_ERR_INVALID, "mc_op_mfma_probe: NULL pointer or sizes out of range");
  return launch_mfma_probe((hipStream_t)stream, operands, out, n_workgroups, iters);
}

extern "C" int mc_op_attention_prefill(void *stream, int32_t n_items, const int32_t *items,
                                       int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                       int32_t page_tokens, int32_t prefix_len, const void *q,
                                       const void *k_prefix, const void *v_prefix,
                                       const void *k_suffix, const void *v_suffix,
                                       const int32_t *page_table, int32_t table_stride, void *out,
                                       int32_t out_tiled) {
  if (n_items < 0 || n_q_heads < 1 || n_kv_heads < 1 || n_q_heads % n_kv_heads || prefix_len < 1)
    MC_FAIL(MC_ERR_INVALID, "bad sizes");
  if (!items || !q || !k_prefix || !v_prefix || !out) MC_FAIL(MC_ERR_INVALID, "a pointer is NULL");
  MC_TRY(check_tiled(MC_BF16, out_tiled, n_q_heads * head_dim));
  if (!prefill_attention_mfma_supported(page_tokens, head_dim, n_q_heads, n_kv_heads))
    MC_FAIL(MC_ERR_UNSUPPORTED, "prefill attention: bf16, 64-token pages, head_dim 64 or 128 only");
  PrefillAttnArgs a;
  a.q = q; a.k_prefix = k_prefix; a.v_prefix = v_prefix; a.k_suffix = k_suffix; a.v_suffix = v_suffix;
  a.items = (const int4 *)items; a.n_items = n_items; a.page_table = page_table;
  a.table_stride = table_stride; a.n_q_heads = n_q_heads; a.n_kv_heads = n_kv_heads;
  a.head_dim = head_dim; a.page_tokens = page_tokens; a.prefix_len = prefix_len; a.out = out;
  a.out_tiled = out_tiled;
  return launch_attention_prefill_mfma((hipStream_t)stream, a);
}

extern "C" size_t mc_op_top_list_bytes(int32_t rows, int32_t N) {
  if (rows < 1 || N < 64 || N % 64) return 0;
  return (size_t)rows * (N / 64) * kTopPerGroup * 8;
}

extern "C" int mc_op_lm_head(void *stream, int32_t M, int32_t N, int32_t K, const void *a, const void *w,
                             float *logits, void *top_lists) {
  if (M < 1 || N < 1 || K < 1) MC_FAIL(MC_ERR_INVALID, "bad sizes");
  if (!a || !w || !logits || !top_lists) MC_FAIL(MC_ERR_INVALID, "a pointer is NULL");
  if (!linear_top_lists_supported(MC_BF16, M, N, K, 1))
    MC_FAIL(MC_ERR_UNSUPPORTED, "LM head with top lists: at most 32 rows, N %% 128 == 0, N >= 65536, K %% 256 == 0");
  return launch_linear((hipStream_t)stream, MC_BF16, M, N, K, a, w, logits, 1, 1, top_lists);
}

extern "C" int mc_op_sample_lists(void *stream, int32_t n_cands, int32_t vocab, const float *logits,
                                  size_t row_stride, const void *top_lists, float temperature,
                                  int32_t top_k, const float *uniforms, int32_t *out_tokens,
                                  int32_t *out_topk) {
  if (n_cands < 1 || vocab < 64 || vocab % 64) MC_FAIL(MC_ERR_INVALID, "bad sizes (vocab must be a multiple of 64)");
  if (!logits || !top_lists || !uniforms || !out_tokens) MC_FAIL(MC_ERR_INVALID, "a pointer is NULL");
  if (!isfinite(temperature)) MC_FAIL(MC_ERR_INVALID, "temperature is not finite");
  const bool greedy = temperature <= 0.f || top_k == 1;
  const int k = greedy ? 1 : ((top_k <= 0 || top_k >= vocab) ? vocab : top_k);
  if (k > MC_MAX_TOP_K) MC_FAIL(MC_ERR_UNSUPPORTED, "top_k %d exceeds the supported %d", k, MC_MAX_TOP_K);
  const int n_groups = vocab / 64;
  return launch_sample((hipStream_t)stream, n_cands, vocab, logits, row_stride, temperature, top_k, uniforms,
                       out_tokens, out_topk, top_lists, row_stride ? (size_t)n_groups * kTopPerGroup : 0, n_groups);
}

extern "C" int mc_op_sample(void *stream, int32_t n_cands, int32_t vocab, const float *logits,
                            size_t row_stride, float temperature, int32_t top_k,
                            const float *uniforms, int32_t *out_tokens, int32_t *out_topk) {
  if (n_cands < 1 || vocab < 1) MC_FAIL(MC_ERR_INVALID, "bad sizes");
  if (!logits || !uniforms || !out_tokens) MC_FAIL(MC_ERR_INVALID, "a pointer is NULL");
  if (!isfinite(temperature)) MC_FAIL(MC_ERR_INVALID, "temperature is not finite");
  const bool greedy = temperature <= 0.f || top_k == 1;
  const int k = greedy ? 1 : ((top_k <= 0 || top_k >= vocab) ? vocab : top_k);
  if (k > MC_MAX_TOP_K) MC_FAIL(MC_ERR_UNSUPPORTED, "top_k %d exceeds the supported %d", k, MC_MAX_TOP_K);
  return launch_sample((hipStream_t)stream, n_cands, vocab, logits, row_stride, temperature, top_k,
                       uniforms, out_tokens, out_topk);
}

extern "C" int mc_op_reward_score(void *stream, int32_t n_cands, int32_t vocab, const float *logits,
                                  const int32_t *reward_ids, const float *reward_values,
                                  int32_t n_reward, float score_temperature, float *out_logprobs,
                                  float *out_scores, int32_t *out_rank) {
  if (n_cands < 1 || vocab < 1 || n_reward < 1 || n_reward > MC_MAX_REWARD) MC_FAIL(MC_ERR_INVALID, "bad sizes");
  if (!logits || !reward_ids || !reward_values || !out_logprobs) MC_FAIL(MC_ERR_INVALID, "a pointer is NULL");
  if (!(score_temperature > 0.f) || !isfinite(score_temperature)) MC_FAIL(MC_ERR_INVALID, "score_temperature must be positive");
  if ((size_t)n_cands * sizeof(float) > 60000) MC_FAIL(MC_ERR_UNSUPPORTED, "too many candidates for one ranking block");
  return launch_reward_score((hipStream_t)stream, n_cands, vocab, logits, reward_ids, reward_values,
                             n_reward, score_temperature, out_logprobs, out_scores, out_rank);
}
