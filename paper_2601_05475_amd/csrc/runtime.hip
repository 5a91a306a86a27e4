// Host runtime behind the C ABI: models, sessions (shared-prefix KV block, suffix page pool,
// page table), the four calls and the inspection hooks.  No device allocation happens here:
// everything is carved out of the caller's arenas.
#include <limits.h>
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <deque>
#include <new>
#include <vector>

#include "common.h"
#include "kernels_mfma.h"

namespace mc {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline size_t esize(int dtype) { return dtype == MC_F32 ? 4 : 2; }

static int check_config(const mc_config *c) {
  if (!c) MC_FAIL(MC_ERR_INVALID, "config is NULL");
  if (c->n_layers < 1 || c->d_model < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 ||
      c->head_dim < 2 || c->d_ffn < 1 || c->vocab < 1)
    MC_FAIL(MC_ERR_INVALID, "config has a non-positive dimension");
  if (c->n_q_heads % c->n_kv_heads) MC_FAIL(MC_ERR_INVALID, "n_q_heads must be a multiple of n_kv_heads");
  if (c->head_dim % 2 || c->head_dim > 256) MC_FAIL(MC_ERR_INVALID, "head_dim must be even and <= 256");
  if (c->dtype != MC_F32 && c->dtype != MC_BF16) MC_FAIL(MC_ERR_INVALID, "unknown dtype %d", c->dtype);
  if (!(c->rms_eps >= 0.f) || !(c->rope_base > 0.f) || !isfinite(c->rope_base))
    MC_FAIL(MC_ERR_INVALID, "rms_eps / rope_base out of range");
  return MC_OK;
}

// Bump allocator over a caller-owned device range.
struct Bump {
  char *base = nullptr;
  size_t cap = 0, used = 0;
  bool measure = false;       // only add sizes up
  void *take(size_t bytes) {
    const size_t at = align_up(used, 256);
    used = at + bytes;
    if (measure) return nullptr;
    return (used <= cap) ? base + at : nullptr;
  }
};

struct LayerW {
  const void *attn_norm, *wqkv, *wo, *ffn_norm, *w_gate, *w_up, *w_down;
};

}  // namespace mc

using namespace mc;

struct mc_model {
  mc_config cfg;
  int device;
  hipStream_t stream;
  const void *embed, *final_norm, *lm_head;
  std::vector<LayerW> layers;
  int n_qkv;                // (Hq + 2 Hkv) * hd
  int tiled;                // matrices (not the embedding) are kept in the tiled MFMA layout
};

namespace mc {

struct ModelLayout {
  size_t embed, final_norm, lm_head, staging;
  struct L { size_t attn_norm, wqkv, wo, ffn_norm, w_gate, w_up, w_down; };
  std::vector<L> layers;
  size_t total, staging_bytes;
  int tiled, staging_rows;
};

// bf16 models whose every matrix fits the tiled MFMA kernels run entirely on them
static int model_is_tiled(const mc_config &c) {
  const int qd = c.n_q_heads * c.head_dim, kd = c.n_kv_heads * c.head_dim;
  return c.dtype == MC_BF16 && kd % 32 == 0 && tiled_shapes_ok(0, qd + 2 * kd, c.d_model) &&
         tiled_shapes_ok(0, c.d_model, qd) && tiled_shapes_ok(0, c.d_ffn, c.d_model) &&
         tiled_shapes_ok(0, c.d_model, c.d_ffn) && tiled_shapes_ok(0, c.vocab, c.d_model);
}

static void model_layout(const mc_config &c, ModelLayout &o) {
  Bump b;
  b.measure = true;
  const size_t e = esize(c.dtype), d = c.d_model, qd = (size_t)c.n_q_heads * c.head_dim,
               kd = (size_t)c.n_kv_heads * c.head_dim;
  auto at = [&](size_t bytes) { b.take(bytes); return b.used - bytes; };
  o.tiled = model_is_tiled(c);
  o.staging_rows = 2048;
  o.staging_bytes = o.tiled ? (size_t)o.staging_rows * std::max({d, qd, (size_t)c.d_ffn}) * e : 0;
  o.staging = at(o.staging_bytes);
  o.embed = at((size_t)c.vocab * d * e);
  o.final_norm = at(d * e);
  o.lm_head = at((size_t)c.vocab * d * e);
  o.layers.resize(c.n_layers);
  for (auto &l : o.layers) {
    l.attn_norm = at(d * e);
    l.wqkv = at((qd + 2 * kd) * d * e);
    l.wo = at(d * qd * e);
    l.ffn_norm = at(d * e);
    l.w_gate = at((size_t)c.d_ffn * d * e);
    l.w_up = at((size_t)c.d_ffn * d * e);
    l.w_down = at(d * (size_t)c.d_ffn * e);
  }
  o.total = align_up(b.used, 256);
}

}  // namespace mc

extern "C" size_t mc_model_bytes(const mc_config *cfg) {
  if (check_config(cfg) != MC_OK) return 0;
  ModelLayout lay;
  model_layout(*cfg, lay);
  return lay.total;
}

static int check_arena(const mc_arena *a, size_t need, const char *what) {
  if (!a || !a->dev_base) MC_FAIL(MC_ERR_INVALID, "%s arena is NULL", what);
  if (((uintptr_t)a->dev_base) & 255) MC_FAIL(MC_ERR_INVALID, "%s arena is not 256-byte aligned", what);
  if (a->dev_bytes < need)
    MC_FAIL(MC_ERR_OOM, "%s arena has %zu bytes, %zu needed", what, a->dev_bytes, need);
  return MC_OK;
}

extern "C" int mc_model_create(const mc_config *cfg, const mc_weights *w, const mc_arena *arena,
                               mc_model **out) {
  MC_TRY(check_config(cfg));
  if (!w || !out) MC_FAIL(MC_ERR_INVALID, "weights / out is NULL");
  if (!w->embed || !w->final_norm || !w->lm_head || !w->attn_norm || !w->wq || !w->wk || !w->wv ||
      !w->wo || !w->ffn_norm || !w->w_gate || !w->w_up || !w->w_down)
    MC_FAIL(MC_ERR_INVALID, "a weight pointer is NULL");
  for (int l = 0; l < cfg->n_layers; ++l)
    if (!w->attn_norm[l] || !w->wq[l] || !w->wk[l] || !w->wv[l] || !w->wo[l] || !w->ffn_norm[l] ||
        !w->w_gate[l] || !w->w_up[l] || !w->w_down[l])
      MC_FAIL(MC_ERR_INVALID, "a weight pointer of layer %d is NULL", l);
  ModelLayout lay;
  model_layout(*cfg, lay);
  MC_TRY(check_arena(arena, lay.total, "model"));
  MC_HIP(hipSetDevice(arena->device));
  hipStream_t st = (hipStream_t)arena->hip_stream;
  char *base = (char *)arena->dev_base;
  const mc_config &c = *cfg;
  const size_t e = esize(c.dtype), d = c.d_model, qd = (size_t)c.n_q_heads * c.head_dim,
               kd = (size_t)c.n_kv_heads * c.head_dim;
  auto put = [&](size_t off, const void *src, size_t bytes) -> hipError_t {
    return hipMemcpyAsync(base + off, src, bytes, hipMemcpyDefault, st);
  };
  // A matrix [rows][K]: plain copy, or (tiled models) repacked through the staging area in
  // row chunks.  row0 places it below earlier rows of a fused matrix (multiple of 32).
  auto put_matrix = [&](size_t off, size_t row0, const void *src, size_t rows, size_t K,
                        int interleave_hd = 0) -> hipError_t {
    if (!lay.tiled) return put(off + row0 * K * e, src, rows * K * e);
    for (size_t r = 0; r < rows; r += lay.staging_rows) {
      const size_t n = std::min(rows - r, (size_t)lay.staging_rows);
      hipError_t err = hipMemcpyAsync(base + lay.staging, (const char *)src + r * K * e, n * K * e,
                                      hipMemcpyDefault, st);
      if (err != hipSuccess) return err;
      if (launch_pack_tiled(st, (int)n, (int)K, base + lay.staging,
                            base + off + (row0 + r) / 32 * (K / 64) * 4096, interleave_hd) != MC_OK)
        return hipErrorLaunchFailure;
      // the staging area is reused by the next chunk: a copy from pageable host memory is not
      // guaranteed to wait for kernels enqueued earlier on the stream
      err = hipStreamSynchronize(st);
      if (err != hipSuccess) return err;
    }
    return hipSuccess;
  };
  MC_HIP(put(lay.embed, w->embed, (size_t)c.vocab * d * e));
  MC_HIP(put(lay.final_norm, w->final_norm, d * e));
  MC_HIP(put_matrix(lay.lm_head, 0, w->lm_head, c.vocab, d));
  mc_model *m = new (std::nothrow) mc_model();
  if (!m) MC_FAIL(MC_ERR_OOM, "host allocation failed");
  m->cfg = c;
  m->device = arena->device;
  m->stream = st;
  m->embed = base + lay.embed;
  m->final_norm = base + lay.final_norm;
  m->lm_head = base + lay.lm_head;
  m->n_qkv = (int)(qd + 2 * kd);
  m->tiled = lay.tiled;
  m->layers.resize(c.n_layers);
  for (int l = 0; l < c.n_layers; ++l) {
    const auto &L = lay.layers[l];
    hipError_t err = put(L.attn_norm, w->attn_norm[l], d * e);
    // fused QKV: rows of wq, then wk, then wv; tiled models keep the rows of every query / key
    // head interleaved (coordinate i at 2i, i + hd/2 at 2i + 1) for the fused rotary epilogue
    if (err == hipSuccess) err = put_matrix(L.wqkv, 0, w->wq[l], qd, d, c.head_dim);
    if (err == hipSuccess) err = put_matrix(L.wqkv, qd, w->wk[l], kd, d, c.head_dim);
    if (err == hipSuccess) err = put_matrix(L.wqkv, qd + kd, w->wv[l], kd, d);
    if (err == hipSuccess) err = put_matrix(L.wo, 0, w->wo[l], d, qd);
    if (err == hipSuccess) err = put(L.ffn_norm, w->ffn_norm[l], d * e);
    if (err == hipSuccess) err = put_matrix(L.w_gate, 0, w->w_gate[l], c.d_ffn, d);
    if (err == hipSuccess) err = put_matrix(L.w_up, 0, w->w_up[l], c.d_ffn, d);
    if (err == hipSuccess) err = put_matrix(L.w_down, 0, w->w_down[l], d, c.d_ffn);
    if (err != hipSuccess) {
      delete m;
      MC_FAIL(MC_ERR_DEVICE, "weight upload of layer %d failed: %s", l, hipGetErrorString(err));
    }
    m->layers[l] = LayerW{base + L.attn_norm, base + L.wqkv, base + L.wo, base + L.ffn_norm,
                          base + L.w_gate, base + L.w_up, base + L.w_down};
  }
  hipError_t err = hipStreamSynchronize(st);   // source buffers may be released after return
  if (err != hipSuccess) {
    delete m;
    MC_FAIL(MC_ERR_DEVICE, "weight upload failed: %s", hipGetErrorString(err));
  }
  *out = m;
  return MC_OK;
}

extern "C" void mc_model_destroy(mc_model *m) { delete m; }

// =====================================================================================
// Session
// =====================================================================================
namespace mc {

enum { LOGITS_NONE = 0, LOGITS_PREFIX = 1, LOGITS_CANDS = 2, LOGITS_SCORE = 3 };
constexpr int kMaxSplits = 16;
constexpr int kRingSlots = 32;
constexpr int kProfCap = 8192;

struct SessionLayout {
  size_t kpool, vpool, kscr, vscr, x, h, part, q, attn_out, act, logits, prefix_logits, xlast,
      hlast, attn_ws, alive, rope_tab, row_tok, row_pos, row_page, row_off, row_tab, last_idx, page_table,
      page_new, cand_len, row_len, score_table, items, samp_tok, samp_u, topk, top_lists, top_lists_prefix, rw_ids, rw_vals,
      rw_lp, rw_scores, rw_rank;
  size_t total;
  // derived sizes
  int rows_cap, n_prefix_pages, n_pool_pages, pages_per_cand, n_score_pages;
  size_t attn_ws_bytes, page_bytes, part_floats;
};

static int check_params(const mc_session_params *p) {
  if (!p) MC_FAIL(MC_ERR_INVALID, "session params are NULL");
  if (p->max_prefix < 1 || p->max_cands < 1 || p->max_suffix < 1)
    MC_FAIL(MC_ERR_INVALID, "max_prefix / max_cands / max_suffix must be >= 1");
  const int pg = p->page_tokens;
  if (pg < 4 || pg > 128 || (pg & (pg - 1))) MC_FAIL(MC_ERR_INVALID, "page_tokens must be a power of two in 4..128");
  if (p->chunk_rows < 0) MC_FAIL(MC_ERR_INVALID, "chunk_rows < 0");
  if (p->pool_pages < 0) MC_FAIL(MC_ERR_INVALID, "pool_pages < 0");
  return MC_OK;
}

static int effective_chunk_rows(const mc_session_params &p) {
  int c = p.chunk_rows > 0 ? p.chunk_rows : 4096;
  return std::max(c, p.max_suffix);     // a scoring chunk holds at least one whole candidate
}

static void session_layout(const mc_config &c, const mc_session_params &p, SessionLayout &o) {
  Bump b;
  b.measure = true;
  auto at = [&](size_t bytes) { b.take(bytes); return b.used - bytes; };
  const size_t e = esize(c.dtype), d = c.d_model, qd = (size_t)c.n_q_heads * c.head_dim,
               nqkv = qd + 2 * (size_t)c.n_kv_heads * c.head_dim;
  const int pg = p.page_tokens;
  const int chunk = effective_chunk_rows(p);
  o.rows_cap = std::max(chunk, p.max_cands);
  o.n_prefix_pages = (p.max_prefix + pg - 1) / pg;
  o.pages_per_cand = (p.max_suffix + pg - 1) / pg;
  o.n_pool_pages = p.max_cands * o.pages_per_cand;
  if (p.pool_pages > 0) o.n_pool_pages = std::min(o.n_pool_pages, p.pool_pages);
  o.n_score_pages = chunk / pg + std::min(p.max_cands, chunk) + 1;
  o.page_bytes = page_elems(c.n_kv_heads, c.head_dim, pg) * e;
  const size_t R = o.rows_cap;
  o.kpool = at((size_t)c.n_layers * (o.n_prefix_pages + o.n_pool_pages) * o.page_bytes);
  o.vpool = at((size_t)c.n_layers * (o.n_prefix_pages + o.n_pool_pages) * o.page_bytes);
  o.kscr = at((size_t)o.n_score_pages * o.page_bytes);
  o.vscr = at((size_t)o.n_score_pages * o.page_bytes);
  // activation buffers that may be kept tiled hold whole 32-row tiles
  const size_t Rp = align_up(R, 32), Cp = align_up((size_t)p.max_cands, 32);
  o.x = at(R * d * 4);
  o.h = at(Rp * d * e);
  o.part_floats = std::max(R, (size_t)p.max_cands * kMaxSplits) * std::max(nqkv, d);
  o.part = at(o.part_floats * 4);
  o.q = at(R * qd * e);
  o.attn_out = at(Rp * qd * e);
  o.act = at(Rp * (size_t)c.d_ffn * e);
  o.logits = at((size_t)p.max_cands * c.vocab * 4);
  o.prefix_logits = at((size_t)c.vocab * 4);
  o.xlast = at((size_t)p.max_cands * d * 4);
  o.hlast = at(Cp * d * e);
  o.attn_ws_bytes = decode_attention_ws_bytes(p.max_cands, c.n_q_heads, c.n_kv_heads, c.head_dim,
                                              p.max_prefix, p.max_suffix, pg);
  o.attn_ws = at(o.attn_ws_bytes);
  o.alive = at((size_t)p.max_cands * 4);
  o.rope_tab = at((size_t)(p.max_prefix + p.max_suffix) * (c.head_dim / 2) * sizeof(double2));
  o.row_tok = at(R * 4);
  o.row_pos = at(R * 4);
  o.row_page = at(R * 4);
  o.row_off = at(R * 4);
  o.row_tab = at(R * 4);
  o.last_idx = at((size_t)p.max_cands * 4);
  o.page_table = at((size_t)p.max_cands * o.pages_per_cand * 4);
  o.page_new = at((size_t)p.max_cands * o.pages_per_cand * 8);     // table indices, then page ids
  o.cand_len = at((size_t)p.max_cands * 4);
  o.row_len = at((size_t)p.max_cands * 4);
  o.score_table = at((size_t)p.max_cands * o.pages_per_cand * 4);
  o.items = at((R / 32 + p.max_cands + 2) * 16);
  o.samp_tok = at((size_t)p.max_cands * 4);
  o.samp_u = at((size_t)p.max_cands * 4);
  o.topk = at((size_t)p.max_cands * MC_MAX_TOP_K * 4);
  // per-group top lists the LM head leaves beside the logits (candidates' rows, prefix row)
  const size_t list_row = (size_t)(c.vocab / 64 + 1) * kTopPerGroup * 8;
  o.top_lists = at((size_t)p.max_cands * list_row);
  o.top_lists_prefix = at(list_row);
  o.rw_ids = at(MC_MAX_REWARD * 4);
  o.rw_vals = at(MC_MAX_REWARD * 4);
  o.rw_lp = at((size_t)p.max_cands * MC_MAX_REWARD * 4);
  o.rw_scores = at((size_t)p.max_cands * 4);
  o.rw_rank = at((size_t)p.max_cands * 4);
  o.total = align_up(b.used, 256);
}

}  // namespace mc

extern "C" size_t mc_session_bytes(const mc_config *cfg, const mc_session_params *p) {
  if (check_config(cfg) != MC_OK || check_params(p) != MC_OK) return 0;
  SessionLayout lay;
  session_layout(*cfg, *p, lay);
  return lay.total;
}

struct mc_session {
  const mc_model *m;
  mc_session_params p;
  SessionLayout lay;
  char *base;
  hipStream_t stream;
  int chunk_rows;
  // state
  int prefix_len = 0, n_cands = 0, suffix_len = 0, logits_state = LOGITS_NONE, logits_rows = 0;
  bool sampled_on_device = false;
  // the LM head left per-group top lists beside the pending logits (candidates' rows / prefix row)
  bool lists_cands = false, lists_prefix = false;
  // candidates still decoding, ascending ids (all of 0..n_cands-1 until some are dropped); row r
  // of every per-candidate buffer belongs to candidate alive[r]
  std::vector<int32_t> alive;
  bool dropped_any = false;
  // candidates that sit out (mc_pause_candidates): they keep their pages and suffix tokens
  std::vector<int32_t> paused;
  // suffix tokens held by every started candidate (by id).  suffix_len is the longest among the
  // candidates still decoding; ragged: they are not all that long (set by mc_prefill_suffix_ragged,
  // cleared when the survivors of a drop are level again)
  std::vector<int32_t> cand_len;
  bool ragged = false;
  int prefix_splits = 0;
  // The pool's free pages are a queue: at a page boundary the candidates still decoding take
  // pages from its head in ascending candidate order; a dropped candidate's pages go to its tail.
  std::vector<int32_t> free_list;           // initial order of the pool
  std::deque<int32_t> free_q;               // pages free now
  std::vector<int32_t> host_table;          // [max_cands][pages_per_cand], pool-relative ids, -1 = none
  // pinned staging ring for small host->device parameter blocks
  char *ring = nullptr;
  size_t slot_bytes = 0;
  int ring_next = 0;
  hipEvent_t ring_ev[kRingSlots];
  bool ring_used[kRingSlots];
  // kernel-class timing
  int prof_class = MC_K_NONE, prof_stride = 1, prof_seen = 0;
  std::vector<hipEvent_t> prof_ev;          // pairs
  int prof_n = 0;

  template <typename T> T *ptr(size_t off) const { return (T *)(base + off); }
  size_t layer_pool_bytes() const { return (size_t)(lay.n_prefix_pages + lay.n_pool_pages) * lay.page_bytes; }
  char *k_layer(int l) const { return base + lay.kpool + (size_t)l * layer_pool_bytes(); }
  char *v_layer(int l) const { return base + lay.vpool + (size_t)l * layer_pool_bytes(); }
};

namespace mc {

// Times the launches made while it lives, if its class is the one being profiled and this
// occurrence is sampled.  on_kernel: the launcher inside the scope attaches the two events to its
// own kernels (the few-row linear layers and decode attention do), so they carry the kernels'
// begin and end times; otherwise the events are recorded on the stream before and after the
// launches, which adds a few microseconds of event handling to what they enclose.
struct ProfScope {
  mc_session *s;
  bool active = false, on_kernel = false;
  ProfScope(mc_session *s_, int cls, bool on_kernel_ = false) : s(s_), on_kernel(on_kernel_) {
    if (s->prof_class != cls || cls == MC_K_NONE) return;
    if ((s->prof_seen++ % s->prof_stride) != 0 || s->prof_n >= kProfCap) return;
    if ((size_t)(2 * s->prof_n + 2) > s->prof_ev.size()) return;
    if (on_kernel) {
      offer_launch_events(s->prof_ev[2 * s->prof_n], s->prof_ev[2 * s->prof_n + 1]);
      active = true;
    } else {
      active = hipEventRecord(s->prof_ev[2 * s->prof_n], s->stream) == hipSuccess;
    }
  }
  ~ProfScope() {
    if (!active) return;
    if (on_kernel) {
      const LaunchEvents left = take_launch_events();     // not taken: the launch failed before it got there
      if (left.start || left.stop) return;
    } else {
      (void)hipEventRecord(s->prof_ev[2 * s->prof_n + 1], s->stream);
    }
    s->prof_n++;
  }
};

// Stage `bytes` of host data into the pinned ring and enqueue its copy to `dst`.
static int upload(mc_session *s, void *dst, const void *src, size_t bytes) {
  if (bytes == 0) return MC_OK;
  if (bytes > s->slot_bytes) MC_FAIL(MC_ERR_INVALID, "internal: staging block of %zu bytes too large", bytes);
  const int slot = s->ring_next;
  s->ring_next = (slot + 1) % kRingSlots;
  if (s->ring_used[slot]) MC_HIP(hipEventSynchronize(s->ring_ev[slot]));
  char *stage = s->ring + (size_t)slot * s->slot_bytes;
  memcpy(stage, src, bytes);
  MC_HIP(hipMemcpyAsync(dst, stage, bytes, hipMemcpyHostToDevice, s->stream));
  MC_HIP(hipEventRecord(s->ring_ev[slot], s->stream));
  s->ring_used[slot] = true;
  return MC_OK;
}

static int download(mc_session *s, void *dst_host, const void *src_dev, size_t bytes) {
  if (bytes) MC_HIP(hipMemcpyAsync(dst_host, src_dev, bytes, hipMemcpyDeviceToHost, s->stream));
  return MC_OK;
}

// tok_src != nullptr: the tokens drawn on the device become the rows' tokens here as well
__global__ void decode_rows_kernel(int B, int pos, int page_slot, int off, int table_stride,
                                   const int32_t *__restrict__ table, const int32_t *__restrict__ alive,
                                   int32_t *row_pos, int32_t *row_page, int32_t *row_off, int32_t *row_tab,
                                   const int32_t *__restrict__ tok_src, int32_t *row_tok) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  if (tok_src) row_tok[b] = tok_src[b];
  const int cand = alive ? alive[b] : b;
  row_pos[b] = pos;
  row_page[b] = table[(size_t)cand * table_stride + page_slot];
  row_off[b] = off;
  row_tab[b] = cand;
}

// dst[r] = src[idx[r]] for r < n (idx ascending, so in place is safe when done by one thread each
// after all reads: the kernel reads everything first)
__global__ void compact_i32_kernel(int n, const int32_t *__restrict__ idx, int32_t *data) {
  __shared__ int32_t tmp[1024];
  const int r = threadIdx.x;
  if (r < n) tmp[r] = data[idx[r]];
  __syncthreads();
  if (r < n) data[r] = tmp[r];
}

__global__ void copy_row_kernel(int n, const float *__restrict__ src, float *__restrict__ dst) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}

enum { PASS_PREFIX = 0, PASS_DECODE = 1, PASS_SCORE = 2, PASS_SUFFIX = 3 };

// Run all layers on `rows` rows whose metadata (token, position, KV slot, table row) is on the
// device already.  prefix_visible: number of prefix keys that exist (for PASS_PREFIX: the end of
// this chunk).  Leaves the last down-projection's partial sums in `part` (n returned in *tail).
static int run_layers(mc_session *s, int rows, int pass, int prefix_visible, int n_items, int *tail_splits) {
  const mc_model *m = s->m;
  const mc_config &c = m->cfg;
  const SessionLayout &L = s->lay;
  hipStream_t st = s->stream;
  const int dt = c.dtype, d = c.d_model, qd = c.n_q_heads * c.head_dim;
  float *x = s->ptr<float>(L.x);
  float *part = s->ptr<float>(L.part);
  void *h = s->ptr<void>(L.h), *q = s->ptr<void>(L.q), *ao = s->ptr<void>(L.attn_out),
       *act = s->ptr<void>(L.act);
  const int32_t *row_pos = s->ptr<int32_t>(L.row_pos), *row_page = s->ptr<int32_t>(L.row_page),
                *row_off = s->ptr<int32_t>(L.row_off), *row_tab = s->ptr<int32_t>(L.row_tab);
  {
    ProfScope ps(s, MC_K_EMBED);
    MC_TRY(launch_embed(st, dt, rows, d, s->ptr<int32_t>(L.row_tok), m->embed, x));
  }
  const int tl = m->tiled;
  auto splits_for = [&](int N, int K) {
    int sp = linear_auto_splits(dt, rows, N, K, tl);
    sp = std::min(sp, kMaxSplits);
    // fewer splits if the partial sums would not fit; on the tiled few-row path a split count
    // has to divide K / 256
    auto fits = [&](int n) {
      return (size_t)n * rows * N <= L.part_floats && !(tl && rows <= 64 && (K / 64) % (4 * n));
    };
    while (sp > 1 && !fits(sp)) --sp;
    return sp;
  };
  int pending = 0;   // partial sums waiting in `part` to be added to x
  const size_t prefix_bytes = (size_t)L.n_prefix_pages * L.page_bytes;
  for (int l = 0; l < c.n_layers; ++l) {
    const LayerW &W = m->layers[l];
    {
      ProfScope ps(s, MC_K_ADD_RMSNORM);
      MC_TRY(launch_add_rmsnorm(st, dt, rows, d, x, part, pending, W.attn_norm, c.rms_eps, h, tl));
    }
    // tiled path, few rows or a large product: the QKV layer finishes its outputs itself (one K split)
    const bool fuse_qkv = tl && c.head_dim % 4 == 0 && linear_qkv_rope_fused(rows, m->n_qkv, d);
    const int s1 = fuse_qkv ? 1 : splits_for(m->n_qkv, d);
    char *kl = s->k_layer(l), *vl = s->v_layer(l);
    void *kdst, *vdst;
    if (pass == PASS_PREFIX) { kdst = kl; vdst = vl; }
    else if (pass == PASS_DECODE || pass == PASS_SUFFIX) { kdst = kl + prefix_bytes; vdst = vl + prefix_bytes; }
    else { kdst = s->ptr<void>(L.kscr); vdst = s->ptr<void>(L.vscr); }
    const double2 *rope_tab = s->ptr<double2>(L.rope_tab);
    if (fuse_qkv) {
      // the QKV layer rotates and stores queries, keys and values itself
      RopeOut ro;
      ro.row_pos = row_pos; ro.row_page = row_page; ro.row_off = row_off;
      ro.q_out = q; ro.k_pages = kdst; ro.v_pages = vdst; ro.table = rope_tab;
      ro.Hq = c.n_q_heads; ro.Hkv = c.n_kv_heads; ro.hd = c.head_dim; ro.pg = s->p.page_tokens;
      ProfScope ps(s, MC_K_LINEAR_QKV);
      MC_TRY(launch_linear_qkv_rope(st, rows, m->n_qkv, d, h, W.wqkv, ro));
    } else {
      {
        ProfScope ps(s, MC_K_LINEAR_QKV);
        MC_TRY(launch_linear(st, dt, rows, m->n_qkv, d, h, W.wqkv, part, s1, tl));
      }
      ProfScope ps(s, MC_K_ROPE_KV);
      MC_TRY(launch_rope_kv(st, dt, rows, c.n_q_heads, c.n_kv_heads, c.head_dim, s->p.page_tokens,
                            (double)c.rope_base, part, s1, row_pos, row_page, row_off, q, kdst, vdst,
                            rope_tab, tl));
    }
    if (pass == PASS_DECODE) {
      DecodeAttnArgs a;
      a.q = q; a.k_prefix = kl; a.v_prefix = vl; a.k_suffix = kdst; a.v_suffix = vdst;
      a.page_table = s->ptr<int32_t>(L.page_table); a.table_stride = L.pages_per_cand;
      a.n_cands = rows; a.n_q_heads = c.n_q_heads; a.n_kv_heads = c.n_kv_heads;
      a.head_dim = c.head_dim; a.page_tokens = s->p.page_tokens;
      a.prefix_len = s->prefix_len; a.suffix_len = s->suffix_len + 1;
      a.row_len = s->ragged ? s->ptr<int32_t>(L.row_len) : nullptr;
      a.prefix_splits = s->prefix_splits;
      a.row_cand = s->dropped_any ? row_tab : nullptr;
      a.workspace = s->ptr<void>(L.attn_ws); a.workspace_bytes = L.attn_ws_bytes; a.out = ao;
      a.out_tiled = tl;
      ProfScope ps(s, MC_K_ATTN_DECODE, dt == MC_BF16 && decode_attention_mfma_supported(a));
      MC_TRY(launch_attention_decode(st, dt, a));
    } else {
      if (tl && prefill_attention_mfma_supported(s->p.page_tokens, c.head_dim, c.n_q_heads, c.n_kv_heads)) {
        PrefillAttnArgs pa;
        pa.q = q; pa.k_prefix = kl; pa.v_prefix = vl; pa.k_suffix = kdst; pa.v_suffix = vdst;
        pa.items = s->ptr<int4>(L.items); pa.n_items = n_items;
        pa.page_table = (pass == PASS_SCORE) ? s->ptr<int32_t>(L.score_table)
                        : (pass == PASS_SUFFIX) ? s->ptr<int32_t>(L.page_table) : nullptr;
        pa.table_stride = L.pages_per_cand;
        pa.n_q_heads = c.n_q_heads; pa.n_kv_heads = c.n_kv_heads; pa.head_dim = c.head_dim;
        pa.page_tokens = s->p.page_tokens; pa.prefix_len = prefix_visible; pa.out = ao;
        pa.out_tiled = tl;
        ProfScope ps(s, MC_K_ATTN_PREFILL);
        MC_TRY(launch_attention_prefill_mfma(st, pa));
      } else {
      AttnArgs a;
      a.q = q; a.k_prefix = kl; a.v_prefix = vl; a.k_suffix = kdst; a.v_suffix = vdst;
      a.row_pos = row_pos; a.row_tab = row_tab;
      a.page_table = (pass == PASS_SCORE) ? s->ptr<int32_t>(L.score_table)
                     : (pass == PASS_SUFFIX) ? s->ptr<int32_t>(L.page_table) : nullptr;
      a.table_stride = L.pages_per_cand;
      a.rows = rows; a.n_q_heads = c.n_q_heads; a.n_kv_heads = c.n_kv_heads;
      a.head_dim = c.head_dim; a.page_tokens = s->p.page_tokens; a.prefix_len = prefix_visible;
      a.out = ao; a.out_tiled = tl;
      ProfScope ps(s, MC_K_ATTN_PREFILL);
      MC_TRY(launch_attention_generic(st, dt, a));
      }
    }
    // a large product on the tiled path adds to the residual stream in its own epilogue
    const bool acc_o = tl && linear_accumulate_fused(rows, d, qd);
    const int s2 = acc_o ? 0 : splits_for(d, qd);
    {
      ProfScope ps(s, MC_K_LINEAR_O);
      if (acc_o) MC_TRY(launch_linear_accumulate(st, rows, d, qd, ao, W.wo, x));
      else MC_TRY(launch_linear(st, dt, rows, d, qd, ao, W.wo, part, s2, tl));
    }
    {
      ProfScope ps(s, MC_K_ADD_RMSNORM);
      MC_TRY(launch_add_rmsnorm(st, dt, rows, d, x, part, s2, W.ffn_norm, c.rms_eps, h, tl));
    }
    {
      ProfScope ps(s, MC_K_LINEAR_GATE_UP, tl && rows <= 64);
      MC_TRY(launch_linear_swiglu(st, dt, rows, c.d_ffn, d, h, W.w_gate, W.w_up, act, tl));
    }
    const bool acc_d = tl && linear_accumulate_fused(rows, d, c.d_ffn);
    const int s3 = acc_d ? 0 : splits_for(d, c.d_ffn);
    {
      ProfScope ps(s, MC_K_LINEAR_DOWN);
      if (acc_d) MC_TRY(launch_linear_accumulate(st, rows, d, c.d_ffn, act, W.w_down, x));
      else MC_TRY(launch_linear(st, dt, rows, d, c.d_ffn, act, W.w_down, part, s3, tl));
    }
    pending = s3;
  }
  *tail_splits = pending;
  return MC_OK;
}

// Final norm + LM head on n_rows rows gathered from x (indices on device in last_idx, or the
// rows 0..n_rows-1 when idx_on_device is false); logits go to `dst`.
// top_out: per-group top lists of the n_rows logits rows for the sampler, or nullptr; *lists_written
// tells whether the layer's form could leave them.
static int lm_head(mc_session *s, int rows_in_x, int tail_splits, int n_rows, bool gather, float *dst,
                   void *top_out = nullptr, bool *lists_written = nullptr) {
  const mc_model *m = s->m;
  const mc_config &c = m->cfg;
  const SessionLayout &L = s->lay;
  hipStream_t st = s->stream;
  float *x = s->ptr<float>(L.x);
  const void *hin;
  if (gather) {
    // fold the pending partial sums into x (normalised output unused), then gather rows
    {
      ProfScope ps(s, MC_K_ADD_RMSNORM);
      MC_TRY(launch_add_rmsnorm(st, c.dtype, rows_in_x, c.d_model, x, s->ptr<float>(L.part),
                                tail_splits, m->final_norm, c.rms_eps, s->ptr<void>(L.h), m->tiled));
    }
    MC_TRY(launch_gather_rows(st, n_rows, c.d_model, x, s->ptr<int32_t>(L.last_idx),
                              s->ptr<float>(L.xlast)));
    MC_TRY(launch_add_rmsnorm(st, c.dtype, n_rows, c.d_model, s->ptr<float>(L.xlast), nullptr, 0,
                              m->final_norm, c.rms_eps, s->ptr<void>(L.hlast), m->tiled));
    hin = s->ptr<void>(L.hlast);
  } else {
    ProfScope ps(s, MC_K_ADD_RMSNORM);
    MC_TRY(launch_add_rmsnorm(st, c.dtype, rows_in_x, c.d_model, x, s->ptr<float>(L.part),
                              tail_splits, m->final_norm, c.rms_eps, s->ptr<void>(L.h), m->tiled));
    hin = s->ptr<void>(L.h);
  }
  const bool lists = top_out && linear_top_lists_supported(c.dtype, n_rows, c.vocab, c.d_model, m->tiled);
  if (lists_written) *lists_written = lists;
  ProfScope ps(s, MC_K_LINEAR_LM_HEAD);
  MC_TRY(launch_linear(st, c.dtype, n_rows, c.vocab, c.d_model, hin, m->lm_head, dst, 1, m->tiled, lists ? top_out : nullptr));
  return MC_OK;
}

static int check_tokens(const mc_config &c, const int32_t *t, size_t n) {
  for (size_t i = 0; i < n; ++i)
    if (t[i] < 0 || t[i] >= c.vocab) MC_FAIL(MC_ERR_INVALID, "token id %d at index %zu outside [0, %d)", t[i], i, c.vocab);
  return MC_OK;
}

}  // namespace mc

extern "C" int mc_session_create(const mc_model *m, const mc_arena *arena,
                                 const mc_session_params *p, mc_session **out) {
  if (!m || !out) MC_FAIL(MC_ERR_INVALID, "model / out is NULL");
  MC_TRY(check_params(p));
  SessionLayout lay;
  session_layout(m->cfg, *p, lay);
  MC_TRY(check_arena(arena, lay.total, "session"));
  if (arena->device != m->device) MC_FAIL(MC_ERR_INVALID, "session arena is on another device than the model");
  MC_HIP(hipSetDevice(arena->device));
  mc_session *s = new (std::nothrow) mc_session();
  if (!s) MC_FAIL(MC_ERR_OOM, "host allocation failed");
  s->m = m;
  s->p = *p;
  s->lay = lay;
  s->base = (char *)arena->dev_base;
  s->stream = (hipStream_t)arena->hip_stream;
  s->chunk_rows = effective_chunk_rows(*p);
  s->free_list.resize(lay.n_pool_pages);
  for (int i = 0; i < lay.n_pool_pages; ++i) s->free_list[i] = i;
  s->free_q.assign(s->free_list.begin(), s->free_list.end());
  s->host_table.assign((size_t)p->max_cands * lay.pages_per_cand, -1);
  s->slot_bytes = align_up((size_t)lay.rows_cap * 4 * 5 + 256, 256);
  for (int i = 0; i < kRingSlots; ++i) { s->ring_used[i] = false; s->ring_ev[i] = nullptr; }
  hipError_t err = hipHostMalloc((void **)&s->ring, s->slot_bytes * kRingSlots, hipHostMallocDefault);
  for (int i = 0; err == hipSuccess && i < kRingSlots; ++i)
    err = hipEventCreateWithFlags(&s->ring_ev[i], hipEventDisableTiming);
  // KV memory starts at zero so that unused tail slots of a page hold finite values
  if (err == hipSuccess)
    err = hipMemsetAsync(s->base + lay.kpool, 0, lay.vscr + (size_t)lay.n_score_pages * lay.page_bytes - lay.kpool, s->stream);
  if (err == hipSuccess)
    err = hipMemsetAsync(s->base + lay.page_table, 0, (size_t)p->max_cands * lay.pages_per_cand * 4, s->stream);
  // rotary angles of every position this session can hold
  if (err == hipSuccess &&
      launch_rope_table(s->stream, p->max_prefix + p->max_suffix, m->cfg.head_dim, (double)m->cfg.rope_base,
                        s->ptr<double2>(lay.rope_tab)) != MC_OK)
    err = hipErrorLaunchFailure;
  if (err == hipSuccess) err = hipStreamSynchronize(s->stream);
  if (err != hipSuccess) {
    mc_session_destroy(s);
    MC_FAIL(MC_ERR_DEVICE, "session set-up failed: %s", hipGetErrorString(err));
  }
  *out = s;
  return MC_OK;
}

extern "C" void mc_session_destroy(mc_session *s) {
  if (!s) return;
  (void)hipStreamSynchronize(s->stream);
  for (int i = 0; i < kRingSlots; ++i)
    if (s->ring_ev[i]) (void)hipEventDestroy(s->ring_ev[i]);
  for (hipEvent_t e : s->prof_ev) (void)hipEventDestroy(e);
  if (s->ring) (void)hipHostFree(s->ring);
  delete s;
}

extern "C" int mc_session_sync(mc_session *s) {
  if (!s) MC_FAIL(MC_ERR_INVALID, "session is NULL");
  MC_HIP(hipStreamSynchronize(s->stream));
  return MC_OK;
}

extern "C" int mc_session_reset_candidates(mc_session *s) {
  if (!s) MC_FAIL(MC_ERR_INVALID, "session is NULL");
  s->n_cands = 0;
  s->suffix_len = 0;
  s->sampled_on_device = false;
  s->free_q.assign(s->free_list.begin(), s->free_list.end());
  s->alive.clear();
  s->paused.clear();
  s->cand_len.clear();
  s->ragged = false;
  s->dropped_any = false;
  std::fill(s->host_table.begin(), s->host_table.end(), -1);
  if (s->prefix_len > 0) {
    s->logits_state = LOGITS_PREFIX;
    s->logits_rows = 1;
  } else {
    s->logits_state = LOGITS_NONE;
    s->logits_rows = 0;
  }
  return MC_OK;
}

// Run n_tokens tokens at positions start .. start + n_tokens - 1 of the shared sequence (the
// positions below start are in the prefix pages already), write their keys and values into the
// prefix pages and leave the logits of the last one in prefix_logits.
static int prefill_range(mc_session *s, const int32_t *tokens, int n_tokens, int start) {
  const SessionLayout &L = s->lay;
  const int pg = s->p.page_tokens;
  std::vector<int32_t> meta, items;
  int tail = 0, rows = 0;
  for (int p0 = 0; p0 < n_tokens; p0 += s->chunk_rows) {
    rows = std::min(s->chunk_rows, n_tokens - p0);
    meta.resize((size_t)rows * 4);
    for (int r = 0; r < rows; ++r) {
      const int pos = start + p0 + r;
      meta[r] = tokens[p0 + r];
      meta[rows + r] = pos;
      meta[2 * rows + r] = pos / pg;
      meta[3 * rows + r] = pos % pg;
    }
    // the four blocks land in row_tok, row_pos, row_page, row_off
    MC_TRY(upload(s, s->ptr<void>(L.row_tok), meta.data(), (size_t)rows * 4));
    MC_TRY(upload(s, s->ptr<void>(L.row_pos), meta.data() + rows, (size_t)rows * 4));
    MC_TRY(upload(s, s->ptr<void>(L.row_page), meta.data() + 2 * rows, (size_t)rows * 4));
    MC_TRY(upload(s, s->ptr<void>(L.row_off), meta.data() + 3 * rows, (size_t)rows * 4));
    // attention work items: 64 consecutive positions each
    items.clear();
    for (int r = 0; r < rows; r += 64) {
      items.push_back(r); items.push_back(std::min(64, rows - r)); items.push_back(start + p0 + r); items.push_back(-1);
    }
    MC_TRY(upload(s, s->ptr<void>(L.items), items.data(), items.size() * 4));
    MC_TRY(run_layers(s, rows, PASS_PREFIX, start + p0 + rows, (int)items.size() / 4, &tail));
  }
  // logits of the last position only
  const int32_t last = rows - 1;
  MC_TRY(upload(s, s->ptr<void>(L.last_idx), &last, 4));
  s->lists_prefix = false;
  bool lists = false;
  MC_TRY(lm_head(s, rows, tail, 1, true, s->ptr<float>(L.prefix_logits), s->ptr<void>(L.top_lists_prefix), &lists));
  s->lists_prefix = lists;
  return MC_OK;
}

extern "C" int mc_prefill_shared(mc_session *s, const int32_t *tokens, int32_t n_tokens) {
  if (!s || !tokens) MC_FAIL(MC_ERR_INVALID, "session / tokens is NULL");
  if (n_tokens < 1 || n_tokens > s->p.max_prefix)
    MC_FAIL(MC_ERR_INVALID, "n_tokens %d outside [1, %d]", n_tokens, s->p.max_prefix);
  MC_TRY(check_tokens(s->m->cfg, tokens, n_tokens));
  MC_HIP(hipSetDevice(s->m->device));
  // the old prefix and candidates are gone from here on
  s->prefix_len = 0;
  mc_session_reset_candidates(s);
  MC_TRY(prefill_range(s, tokens, n_tokens, 0));
  s->prefix_len = n_tokens;
  s->logits_state = LOGITS_PREFIX;
  s->logits_rows = 1;
  return MC_OK;
}

extern "C" int mc_extend_shared(mc_session *s, const int32_t *tokens, int32_t n_tokens) {
  if (!s || !tokens) MC_FAIL(MC_ERR_INVALID, "session / tokens is NULL");
  if (s->prefix_len <= 0) MC_FAIL(MC_ERR_STATE, "mc_extend_shared before mc_prefill_shared");
  if (n_tokens < 1 || n_tokens > s->p.max_prefix - s->prefix_len)
    MC_FAIL(MC_ERR_INVALID, "n_tokens %d outside [1, %d] (prefix holds %d of %d)", n_tokens,
            s->p.max_prefix - s->prefix_len, s->prefix_len, s->p.max_prefix);
  MC_TRY(check_tokens(s->m->cfg, tokens, n_tokens));
  MC_HIP(hipSetDevice(s->m->device));
  const int start = s->prefix_len;
  // candidates were conditioned on the shorter prefix: they are gone; a failure below leaves
  // the old prefix intact (pages past it may have been written, which nothing reads)
  mc_session_reset_candidates(s);
  s->logits_state = LOGITS_NONE;
  s->logits_rows = 0;
  MC_TRY(prefill_range(s, tokens, n_tokens, start));
  s->prefix_len = start + n_tokens;
  s->logits_state = LOGITS_PREFIX;
  s->logits_rows = 1;
  return MC_OK;
}

namespace mc {
// Copy the keys and values of suffix tokens 0 .. t-1 of one candidate (pages table_row[.] of the
// pool) to prefix positions P .. P + t - 1, element by element: the two sides may sit at
// different offsets inside their pages.  One block per (token, layer).
template <typename T>
__global__ __launch_bounds__(256) void kv_promote_kernel(
    char *kbase, char *vbase, size_t layer_bytes, int n_prefix_pages, const int32_t *__restrict__ table_row,
    int Hkv, int hd, int pg, int P) {
  const int j = blockIdx.x, l = blockIdx.y;
  const size_t pelems = (size_t)Hkv * hd * pg;
  T *k = (T *)(kbase + (size_t)l * layer_bytes), *v = (T *)(vbase + (size_t)l * layer_bytes);
  const size_t src = (size_t)(n_prefix_pages + table_row[j / pg]) * pelems;
  const size_t dst = (size_t)((P + j) / pg) * pelems;
  const int so = j % pg, dof = (P + j) % pg;
  for (int e = threadIdx.x; e < Hkv * hd; e += 256) {
    const int kvh = e / hd, d = e % hd;
    const size_t head = (size_t)kvh * pg * hd;
    k[dst + head + k_elem_offset(dof, d, pg, hd)] = k[src + head + k_elem_offset(so, d, pg, hd)];
    v[dst + head + v_elem_offset(dof, d, pg, hd)] = v[src + head + v_elem_offset(so, d, pg, hd)];
  }
}
}  // namespace mc

extern "C" int mc_promote_candidate(mc_session *s, int32_t cand) {
  if (!s) MC_FAIL(MC_ERR_INVALID, "session is NULL");
  if (s->n_cands < 1 || s->suffix_len < 1) MC_FAIL(MC_ERR_STATE, "mc_promote_candidate: no candidate has decoded a token");
  if (cand < 0 || cand >= s->n_cands) MC_FAIL(MC_ERR_INVALID, "candidate %d outside [0, %d)", cand, s->n_cands);
  const int ri = (int)(std::find(s->alive.begin(), s->alive.end(), cand) - s->alive.begin());
  if (ri >= (int)s->alive.size()) MC_FAIL(MC_ERR_INVALID, "candidate %d was dropped", cand);
  const int t = s->cand_len[cand], P = s->prefix_len;
  if (t < 1) MC_FAIL(MC_ERR_STATE, "mc_promote_candidate: candidate %d holds no token", cand);
  if (t > s->p.max_prefix - P)
    MC_FAIL(MC_ERR_OOM, "prefix of %d + suffix of %d tokens exceeds max_prefix %d", P, t, s->p.max_prefix);
  MC_HIP(hipSetDevice(s->m->device));
  const mc_config &c = s->m->cfg;
  const SessionLayout &L = s->lay;
  const int32_t *row = s->ptr<int32_t>(L.page_table) + (size_t)cand * L.pages_per_cand;
  dim3 grid(t, c.n_layers);
  if (c.dtype == MC_F32)
    kv_promote_kernel<float><<<grid, 256, 0, s->stream>>>(s->k_layer(0), s->v_layer(0), s->layer_pool_bytes(),
                                                          L.n_prefix_pages, row, c.n_kv_heads, c.head_dim, s->p.page_tokens, P);
  else
    kv_promote_kernel<bf16_t><<<grid, 256, 0, s->stream>>>(s->k_layer(0), s->v_layer(0), s->layer_pool_bytes(),
                                                           L.n_prefix_pages, row, c.n_kv_heads, c.head_dim, s->p.page_tokens, P);
  MC_HIP(hipGetLastError());
  // the candidate's last logits become the logits of the last prefix position
  const bool have_logits = s->logits_state == LOGITS_CANDS && s->logits_rows == (int)s->alive.size();
  s->lists_prefix = false;                      // the prefix row changes: its top lists are not copied along
  if (have_logits)
    MC_HIP(hipMemcpyAsync(s->ptr<void>(L.prefix_logits), s->ptr<float>(L.logits) + (size_t)ri * c.vocab,
                          (size_t)c.vocab * 4, hipMemcpyDeviceToDevice, s->stream));
  s->prefix_len = P + t;
  mc_session_reset_candidates(s);
  if (!have_logits) {
    s->logits_state = LOGITS_NONE;
    s->logits_rows = 0;
  }
  return MC_OK;
}

// The number of candidates is fixed by the first call that names it; from then on calls name the
// number still decoding.
static int check_cand_count(mc_session *s, int n_cands) {
  if (n_cands < 1 || n_cands > s->p.max_cands)
    MC_FAIL(MC_ERR_INVALID, "n_cands %d outside [1, %d]", n_cands, s->p.max_cands);
  if (s->n_cands && n_cands != (int)s->alive.size())
    MC_FAIL(MC_ERR_INVALID, "n_cands %d, but %d candidates are decoding (%d were started)", n_cands,
            (int)s->alive.size(), s->n_cands);
  return MC_OK;
}
static void fix_cands(mc_session *s, int n_cands) {
  if (s->n_cands) return;
  s->n_cands = n_cands;
  s->alive.resize(n_cands);
  for (int b = 0; b < n_cands; ++b) s->alive[b] = b;
  s->cand_len.assign(n_cands, 0);
  s->ragged = false;
}
static void refresh_lengths(mc_session *s) {
  int lo = INT32_MAX, hi = 0;
  for (int b : s->alive) { lo = std::min(lo, s->cand_len[b]); hi = std::max(hi, s->cand_len[b]); }
  s->suffix_len = hi;
  s->ragged = lo != hi;
}
static void unfix_cands(mc_session *s, int saved_total) {
  if (saved_total == 0) { s->n_cands = 0; s->alive.clear(); s->cand_len.clear(); }
}

__global__ void scatter_i32_kernel(int n, const int32_t *__restrict__ idx, const int32_t *__restrict__ val,
                                   int32_t *dst) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[idx[i]] = val[i];
}

// host -> device for blocks that may exceed one staging slot
static int upload_long(mc_session *s, void *dst, const void *src, size_t bytes) {
  for (size_t at = 0; at < bytes; at += s->slot_bytes)
    MC_TRY(upload(s, (char *)dst + at, (const char *)src + at, std::min(s->slot_bytes, bytes - at)));
  return MC_OK;
}

// Pages for the table entries idx[.] (candidate * pages_per_cand + slot, in the order the
// candidates take them), read off the head of the queue without removing them and written into
// the device page table.  The queue and the host table change only in commit_pages, once the
// step that needed the pages has been enqueued, so a refused or failed step leaves nothing behind.
static int stage_pages(mc_session *s, const std::vector<int32_t> &idx, std::vector<int32_t> &fresh) {
  const SessionLayout &L = s->lay;
  fresh.clear();
  const size_t n = idx.size();
  if (n == 0) return MC_OK;
  if (n > s->free_q.size())
    MC_FAIL(MC_ERR_OOM, "page pool exhausted: %zu page(s) needed, %zu of %d pages are free", n, s->free_q.size(),
            L.n_pool_pages);
  if (n > (size_t)s->p.max_cands * L.pages_per_cand) MC_FAIL(MC_ERR_INVALID, "internal: page list too long");
  fresh.assign(s->free_q.begin(), s->free_q.begin() + n);
  int32_t *d_idx = s->ptr<int32_t>(L.page_new), *d_val = d_idx + (size_t)s->p.max_cands * L.pages_per_cand;
  MC_TRY(upload_long(s, d_idx, idx.data(), n * 4));
  MC_TRY(upload_long(s, d_val, fresh.data(), n * 4));
  scatter_i32_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s->stream>>>((int)n, d_idx, d_val, s->ptr<int32_t>(L.page_table));
  MC_HIP(hipGetLastError());
  return MC_OK;
}
static void commit_pages(mc_session *s, const std::vector<int32_t> &idx, const std::vector<int32_t> &fresh) {
  for (size_t i = 0; i < fresh.size(); ++i) {
    s->host_table[idx[i]] = fresh[i];
    s->free_q.pop_front();
  }
}

// rows of a decode step whose candidates differ in length: everything per row comes from the
// candidate's own length (cand_len, by candidate id)
__global__ void decode_rows_ragged_kernel(int B, int prefix_len, int pg, int table_stride,
                                          const int32_t *__restrict__ table, const int32_t *__restrict__ alive,
                                          const int32_t *__restrict__ cand_len, int32_t *row_pos,
                                          int32_t *row_page, int32_t *row_off, int32_t *row_tab, int32_t *row_len,
                                          const int32_t *__restrict__ tok_src, int32_t *row_tok) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  if (tok_src) row_tok[b] = tok_src[b];
  const int cand = alive ? alive[b] : b;
  const int t = cand_len[cand];
  row_pos[b] = prefix_len + t;
  row_page[b] = table[(size_t)cand * table_stride + t / pg];
  row_off[b] = t % pg;
  row_tab[b] = cand;
  row_len[b] = t + 1;
}

extern "C" int mc_decode_step(mc_session *s, const int32_t *tokens, int32_t n_cands) {
  if (!s) MC_FAIL(MC_ERR_INVALID, "session is NULL");
  if (s->prefix_len <= 0) MC_FAIL(MC_ERR_STATE, "mc_decode_step before mc_prefill_shared");
  MC_TRY(check_cand_count(s, n_cands));
  if (s->suffix_len >= s->p.max_suffix)
    MC_FAIL(MC_ERR_OOM, "suffix is full (%d tokens): a candidate has reached max_suffix", s->suffix_len);
  const mc_config &c = s->m->cfg;
  if (tokens) MC_TRY(check_tokens(c, tokens, n_cands));
  else if (!s->sampled_on_device) MC_FAIL(MC_ERR_STATE, "tokens is NULL but no mc_sample result is pending on the device");
  MC_HIP(hipSetDevice(s->m->device));
  const SessionLayout &L = s->lay;
  const int pg = s->p.page_tokens, t = s->suffix_len;
  const int saved_n = s->n_cands;
  fix_cands(s, n_cands);
  // candidates at a page boundary take a page each, in ascending order
  std::vector<int32_t> idx, fresh;
  for (int b : s->alive)
    if (s->cand_len[b] % pg == 0) idx.push_back(b * L.pages_per_cand + s->cand_len[b] / pg);
  if (int rc0 = stage_pages(s, idx, fresh)) { unfix_cands(s, saved_n); return rc0; }
  // from here on every failure leaves through `fail`, which forgets candidates that this call started
  auto fail = [&](int code) { unfix_cands(s, saved_n); return code; };
  if (tokens) {
    if (int rc1 = upload(s, s->ptr<void>(L.row_tok), tokens, (size_t)n_cands * 4)) return fail(rc1);
  }
  const int32_t *tok_src = tokens ? nullptr : s->ptr<int32_t>(L.samp_tok);      // copied by the row kernel below
  if (s->ragged) {
    if (int rc1 = upload(s, s->ptr<void>(L.cand_len), s->cand_len.data(), (size_t)s->n_cands * 4)) return fail(rc1);
    decode_rows_ragged_kernel<<<(n_cands + 63) / 64, 64, 0, s->stream>>>(
        n_cands, s->prefix_len, pg, L.pages_per_cand, s->ptr<int32_t>(L.page_table),
        s->dropped_any ? s->ptr<int32_t>(L.alive) : nullptr, s->ptr<int32_t>(L.cand_len), s->ptr<int32_t>(L.row_pos),
        s->ptr<int32_t>(L.row_page), s->ptr<int32_t>(L.row_off), s->ptr<int32_t>(L.row_tab), s->ptr<int32_t>(L.row_len),
        tok_src, s->ptr<int32_t>(L.row_tok));
  } else {
    decode_rows_kernel<<<(n_cands + 63) / 64, 64, 0, s->stream>>>(
        n_cands, s->prefix_len + t, t / pg, t % pg, L.pages_per_cand, s->ptr<int32_t>(L.page_table),
        s->dropped_any ? s->ptr<int32_t>(L.alive) : nullptr, s->ptr<int32_t>(L.row_pos), s->ptr<int32_t>(L.row_page), s->ptr<int32_t>(L.row_off),
        s->ptr<int32_t>(L.row_tab), tok_src, s->ptr<int32_t>(L.row_tok));
  }
  if (hipGetLastError() != hipSuccess) {
    set_error("launch of the decode-row kernel failed");
    return fail(MC_ERR_DEVICE);
  }
  int tail = 0;
  int rc = run_layers(s, n_cands, PASS_DECODE, s->prefix_len, 0, &tail);
  bool lists = false;
  s->lists_cands = false;
  if (rc == MC_OK) rc = lm_head(s, n_cands, tail, n_cands, false, s->ptr<float>(L.logits), s->ptr<void>(L.top_lists), &lists);
  if (rc != MC_OK) return fail(rc);
  s->lists_cands = lists;
  commit_pages(s, idx, fresh);
  for (int b : s->alive) s->cand_len[b]++;
  s->suffix_len = t + 1;
  s->logits_state = LOGITS_CANDS;
  s->logits_rows = n_cands;
  s->sampled_on_device = false;
  return MC_OK;
}

extern "C" int mc_sample(mc_session *s, int32_t n_cands, float temperature, int32_t top_k,
                         const float *uniforms, int32_t *out_tokens, int32_t *out_topk_ids) {
  if (!s || !uniforms) MC_FAIL(MC_ERR_INVALID, "session / uniforms is NULL");
  if (s->logits_state != LOGITS_PREFIX && s->logits_state != LOGITS_CANDS)
    MC_FAIL(MC_ERR_STATE, "mc_sample without pending logits (call mc_prefill_shared or mc_decode_step first)");
  MC_TRY(check_cand_count(s, n_cands));
  if (!isfinite(temperature)) MC_FAIL(MC_ERR_INVALID, "temperature is not finite");
  for (int b = 0; b < n_cands; ++b)
    if (!(uniforms[b] >= 0.f && uniforms[b] < 1.f)) MC_FAIL(MC_ERR_INVALID, "uniforms[%d] = %g outside [0, 1)", b, uniforms[b]);
  const mc_config &c = s->m->cfg;
  const bool greedy = temperature <= 0.f || top_k == 1;
  const int k = greedy ? 1 : ((top_k <= 0 || top_k >= c.vocab) ? c.vocab : top_k);
  if (k > MC_MAX_TOP_K) MC_FAIL(MC_ERR_UNSUPPORTED, "top_k %d exceeds the supported %d", k, MC_MAX_TOP_K);
  MC_HIP(hipSetDevice(s->m->device));
  const SessionLayout &L = s->lay;
  MC_TRY(upload(s, s->ptr<void>(L.samp_u), uniforms, (size_t)n_cands * 4));
  const bool shared_row = s->logits_state == LOGITS_PREFIX;
  const float *lg = shared_row ? s->ptr<float>(L.prefix_logits) : s->ptr<float>(L.logits);
  const int n_groups = c.vocab / 64;
  const void *lists = shared_row ? (s->lists_prefix ? s->ptr<void>(L.top_lists_prefix) : nullptr)
                                 : (s->lists_cands ? s->ptr<void>(L.top_lists) : nullptr);
  {
    ProfScope ps(s, MC_K_SAMPLE);
    MC_TRY(launch_sample(s->stream, n_cands, c.vocab, lg, shared_row ? 0 : (size_t)c.vocab,
                         temperature, top_k, s->ptr<float>(L.samp_u), s->ptr<int32_t>(L.samp_tok),
                         out_topk_ids ? s->ptr<int32_t>(L.topk) : nullptr, lists,
                         shared_row ? 0 : (size_t)n_groups * kTopPerGroup, n_groups));
  }
  s->sampled_on_device = true;
  fix_cands(s, n_cands);
  if (out_tokens || out_topk_ids) {
    if (out_tokens) MC_TRY(download(s, out_tokens, s->ptr<void>(L.samp_tok), (size_t)n_cands * 4));
    if (out_topk_ids) MC_TRY(download(s, out_topk_ids, s->ptr<void>(L.topk), (size_t)n_cands * k * 4));
    MC_HIP(hipStreamSynchronize(s->stream));
  }
  return MC_OK;
}

extern "C" int mc_score_candidates(mc_session *s, const int32_t *suffix_tokens,
                                   const int32_t *suffix_lens, int32_t n_cands, int32_t max_len,
                                   const int32_t *reward_ids, const float *reward_values,
                                   int32_t n_reward, float score_temperature, float *out_logprobs,
                                   float *out_scores, int32_t *out_rank) {
  if (!s || !suffix_tokens || !suffix_lens || !reward_ids || !reward_values)
    MC_FAIL(MC_ERR_INVALID, "a required pointer is NULL");
  if (s->prefix_len <= 0) MC_FAIL(MC_ERR_STATE, "mc_score_candidates before mc_prefill_shared");
  if (n_cands < 1 || n_cands > s->p.max_cands)
    MC_FAIL(MC_ERR_INVALID, "n_cands %d outside [1, %d]", n_cands, s->p.max_cands);
  if (max_len < 1 || max_len > s->p.max_suffix)
    MC_FAIL(MC_ERR_INVALID, "max_len %d outside [1, %d]", max_len, s->p.max_suffix);
  if (n_reward < 1 || n_reward > MC_MAX_REWARD)
    MC_FAIL(MC_ERR_INVALID, "n_reward %d outside [1, %d]", n_reward, MC_MAX_REWARD);
  if (!(score_temperature > 0.f) || !isfinite(score_temperature))
    MC_FAIL(MC_ERR_INVALID, "score_temperature must be positive and finite");
  const mc_config &c = s->m->cfg;
  for (int r = 0; r < n_reward; ++r) {
    if (reward_ids[r] < 0 || reward_ids[r] >= c.vocab) MC_FAIL(MC_ERR_INVALID, "reward id %d outside the vocabulary", reward_ids[r]);
    if (!isfinite(reward_values[r])) MC_FAIL(MC_ERR_INVALID, "reward value %d is not finite", r);
    for (int q = 0; q < r; ++q)
      if (reward_ids[q] == reward_ids[r]) MC_FAIL(MC_ERR_INVALID, "reward id %d is repeated", reward_ids[r]);
  }
  for (int b = 0; b < n_cands; ++b) {
    if (suffix_lens[b] < 1 || suffix_lens[b] > max_len)
      MC_FAIL(MC_ERR_INVALID, "suffix_lens[%d] = %d outside [1, %d]", b, suffix_lens[b], max_len);
    MC_TRY(check_tokens(c, suffix_tokens + (size_t)b * max_len, suffix_lens[b]));
  }
  MC_HIP(hipSetDevice(s->m->device));
  const SessionLayout &L = s->lay;
  const int pg = s->p.page_tokens;
  s->lists_cands = false;                       // the candidates' logits rows are overwritten below
  MC_TRY(upload(s, s->ptr<void>(L.rw_ids), reward_ids, (size_t)n_reward * 4));
  MC_TRY(upload(s, s->ptr<void>(L.rw_vals), reward_values, (size_t)n_reward * 4));
  std::vector<int32_t> tok, pos, page, off, tab, last, table, items;
  int b0 = 0;
  while (b0 < n_cands) {
    // a chunk holds whole candidates, at most chunk_rows rows
    int b1 = b0, rows = 0;
    while (b1 < n_cands && rows + suffix_lens[b1] <= s->chunk_rows) rows += suffix_lens[b1++];
    const int nc = b1 - b0;
    tok.resize(rows); pos.resize(rows); page.resize(rows); off.resize(rows); tab.resize(rows);
    last.resize(nc);
    table.assign((size_t)nc * L.pages_per_cand, 0);
    int r = 0, next_page = 0;
    items.clear();
    for (int b = b0; b < b1; ++b) {
      const int len = suffix_lens[b];
      for (int j = 0; j < len; j += 64) {
        items.push_back(r + j); items.push_back(std::min(64, len - j));
        items.push_back(s->prefix_len + j); items.push_back(b - b0);
      }
      for (int j = 0; j < len; ++j, ++r) {
        if (j % pg == 0) table[(size_t)(b - b0) * L.pages_per_cand + j / pg] = next_page++;
        tok[r] = suffix_tokens[(size_t)b * max_len + j];
        pos[r] = s->prefix_len + j;
        page[r] = table[(size_t)(b - b0) * L.pages_per_cand + j / pg];
        off[r] = j % pg;
        tab[r] = b - b0;
      }
      last[b - b0] = r - 1;
    }
    if (next_page > L.n_score_pages) MC_FAIL(MC_ERR_OOM, "internal: scoring scratch pages exhausted");
    MC_TRY(upload(s, s->ptr<void>(L.row_tok), tok.data(), (size_t)rows * 4));
    MC_TRY(upload(s, s->ptr<void>(L.row_pos), pos.data(), (size_t)rows * 4));
    MC_TRY(upload(s, s->ptr<void>(L.row_page), page.data(), (size_t)rows * 4));
    MC_TRY(upload(s, s->ptr<void>(L.row_off), off.data(), (size_t)rows * 4));
    MC_TRY(upload(s, s->ptr<void>(L.row_tab), tab.data(), (size_t)rows * 4));
    MC_TRY(upload(s, s->ptr<void>(L.last_idx), last.data(), (size_t)nc * 4));
    MC_TRY(upload_long(s, s->ptr<void>(L.score_table), table.data(), table.size() * 4));   // through the pinned ring: no host stall
    int tail = 0;
    MC_TRY(upload(s, s->ptr<void>(L.items), items.data(), items.size() * 4));
    MC_TRY(run_layers(s, rows, PASS_SCORE, s->prefix_len, (int)items.size() / 4, &tail));
    MC_TRY(lm_head(s, rows, tail, nc, true, s->ptr<float>(L.logits) + (size_t)b0 * c.vocab));
    b0 = b1;
  }
  {
    ProfScope ps(s, MC_K_REWARD);
    MC_TRY(launch_reward_score(s->stream, n_cands, c.vocab, s->ptr<float>(L.logits),
                               s->ptr<int32_t>(L.rw_ids), s->ptr<float>(L.rw_vals), n_reward,
                               score_temperature, s->ptr<float>(L.rw_lp), s->ptr<float>(L.rw_scores),
                               s->ptr<int32_t>(L.rw_rank)));
  }
  if (out_logprobs) MC_TRY(download(s, out_logprobs, s->ptr<void>(L.rw_lp), (size_t)n_cands * n_reward * 4));
  if (out_scores) MC_TRY(download(s, out_scores, s->ptr<void>(L.rw_scores), (size_t)n_cands * 4));
  if (out_rank) MC_TRY(download(s, out_rank, s->ptr<void>(L.rw_rank), (size_t)n_cands * 4));
  MC_HIP(hipStreamSynchronize(s->stream));
  // scoring overwrote the candidates' logits buffer: sampling must be preceded by a new step
  s->logits_state = LOGITS_SCORE;
  s->logits_rows = n_cands;
  return MC_OK;
}

// Take the n candidates cands[.] out of the set that decodes.  release: their pages go back to
// the pool (a drop); otherwise they keep pages and tokens and wait in `paused`.
static int take_out(mc_session *s, const int32_t *cands, int32_t n, bool release, const char *who) {
  if (!s || !cands) MC_FAIL(MC_ERR_INVALID, "session / cands is NULL");
  if (s->n_cands < 1) MC_FAIL(MC_ERR_STATE, "%s: no candidates", who);
  const int old_n = (int)s->alive.size();
  if (n < 1 || n >= old_n) MC_FAIL(MC_ERR_INVALID, "n %d outside [1, %d): at least one candidate must go on decoding", n, old_n);
  std::vector<char> gone(s->n_cands, 0);
  for (int i = 0; i < n; ++i) {
    const int b = cands[i];
    if (b < 0 || b >= s->n_cands || gone[b] || std::find(s->alive.begin(), s->alive.end(), b) == s->alive.end())
      MC_FAIL(MC_ERR_INVALID, "cands[%d] = %d is not a candidate that is still decoding (or is repeated)", i, b);
    gone[b] = 1;
  }
  MC_HIP(hipSetDevice(s->m->device));
  const mc_config &c = s->m->cfg;
  const SessionLayout &L = s->lay;
  std::vector<int32_t> keep_rows, new_alive;
  for (int r = 0; r < old_n; ++r)
    if (!gone[s->alive[r]]) { keep_rows.push_back(r); new_alive.push_back(s->alive[r]); }
  const int new_n = (int)new_alive.size();
  s->lists_cands = false;                       // rows move: the sampler reads whole rows until the next step
  // pending per-candidate results move up to the rows of the survivors (ascending, so a row is
  // never overwritten before it has been copied)
  if (s->logits_state == LOGITS_CANDS && s->logits_rows == old_n)
    for (int r = 0; r < new_n; ++r)
      if (keep_rows[r] != r)
        MC_HIP(hipMemcpyAsync(s->ptr<float>(L.logits) + (size_t)r * c.vocab, s->ptr<float>(L.logits) + (size_t)keep_rows[r] * c.vocab,
                              (size_t)c.vocab * 4, hipMemcpyDeviceToDevice, s->stream));
  if (s->sampled_on_device) {
    if (old_n > 1024) MC_FAIL(MC_ERR_UNSUPPORTED, "more than 1024 candidates");
    MC_TRY(upload(s, s->ptr<void>(L.last_idx), keep_rows.data(), (size_t)new_n * 4));
    compact_i32_kernel<<<1, 1024, 0, s->stream>>>(new_n, s->ptr<int32_t>(L.last_idx), s->ptr<int32_t>(L.samp_tok));
    MC_HIP(hipGetLastError());
  }
  MC_TRY(upload(s, s->ptr<void>(L.alive), new_alive.data(), (size_t)new_n * 4));
  for (int b = 0; b < s->n_cands; ++b) {
    if (!gone[b]) continue;
    if (!release) { s->paused.push_back(b); continue; }
    for (int p = 0; p < L.pages_per_cand; ++p) {
      int32_t &id = s->host_table[(size_t)b * L.pages_per_cand + p];
      if (id >= 0) s->free_q.push_back(id);
      id = -1;
    }
  }
  s->alive = new_alive;
  s->dropped_any = true;
  refresh_lengths(s);
  if (s->logits_state == LOGITS_CANDS) s->logits_rows = new_n;
  return MC_OK;
}

extern "C" int mc_drop_candidates(mc_session *s, const int32_t *cands, int32_t n) {
  return take_out(s, cands, n, true, "mc_drop_candidates");
}

extern "C" int mc_pause_candidates(mc_session *s, const int32_t *cands, int32_t n) {
  return take_out(s, cands, n, false, "mc_pause_candidates");
}

extern "C" int mc_resume_candidates(mc_session *s, const int32_t *cands, int32_t n) {
  if (!s || !cands) MC_FAIL(MC_ERR_INVALID, "session / cands is NULL");
  if (n < 1 || n > (int)s->paused.size()) MC_FAIL(MC_ERR_INVALID, "n %d outside [1, %d paused candidates]", n, (int)s->paused.size());
  std::vector<int32_t> back(cands, cands + n);
  std::sort(back.begin(), back.end());
  for (int i = 0; i < n; ++i)
    if ((i > 0 && back[i] == back[i - 1]) || std::find(s->paused.begin(), s->paused.end(), back[i]) == s->paused.end())
      MC_FAIL(MC_ERR_INVALID, "candidate %d is not paused (or is repeated)", back[i]);
  MC_HIP(hipSetDevice(s->m->device));
  std::vector<int32_t> new_alive(s->alive);
  new_alive.insert(new_alive.end(), back.begin(), back.end());
  std::sort(new_alive.begin(), new_alive.end());
  MC_TRY(upload(s, s->ptr<void>(s->lay.alive), new_alive.data(), new_alive.size() * 4));
  for (int b : back) s->paused.erase(std::find(s->paused.begin(), s->paused.end(), b));
  s->alive = new_alive;
  s->dropped_any = true;
  refresh_lengths(s);
  // the rows of the per-candidate buffers are renumbered and the resumed candidates have none:
  // nothing is pending any more
  s->lists_cands = false;
  s->sampled_on_device = false;
  if (s->logits_state == LOGITS_CANDS || s->logits_state == LOGITS_SCORE) {
    s->logits_state = LOGITS_NONE;
    s->logits_rows = 0;
  }
  return MC_OK;
}

// lens == nullptr: every candidate gets max_len tokens.  Row r of suffix_tokens ([n_cands][max_len])
// belongs to the r-th candidate still decoding.
static int prefill_suffix_impl(mc_session *s, const int32_t *suffix_tokens, const int32_t *lens, int32_t n_cands,
                               int32_t max_len, const char *who) {
  if (!s || !suffix_tokens) MC_FAIL(MC_ERR_INVALID, "session / suffix_tokens is NULL");
  if (s->prefix_len <= 0) MC_FAIL(MC_ERR_STATE, "%s before mc_prefill_shared", who);
  MC_TRY(check_cand_count(s, n_cands));
  if (max_len < 1) MC_FAIL(MC_ERR_INVALID, "len %d < 1", max_len);
  const mc_config &c = s->m->cfg;
  const SessionLayout &L = s->lay;
  const int pg = s->p.page_tokens;
  auto len_of = [&](int r) { return lens ? lens[r] : max_len; };
  for (int r = 0; r < n_cands; ++r) {
    if (len_of(r) < 1 || len_of(r) > max_len) MC_FAIL(MC_ERR_INVALID, "lens[%d] = %d outside [1, %d]", r, len_of(r), max_len);
    if (len_of(r) > s->chunk_rows) MC_FAIL(MC_ERR_INVALID, "lens[%d] = %d exceeds the chunk of %d rows", r, len_of(r), s->chunk_rows);
    MC_TRY(check_tokens(c, suffix_tokens + (size_t)r * max_len, len_of(r)));
  }
  const int saved_n = s->n_cands;
  fix_cands(s, n_cands);
  for (int r = 0; r < n_cands; ++r)
    if (len_of(r) > s->p.max_suffix - s->cand_len[s->alive[r]]) {
      const int have = s->cand_len[s->alive[r]];
      unfix_cands(s, saved_n);
      MC_FAIL(MC_ERR_OOM, "suffix of %d + %d tokens exceeds max_suffix %d", have, len_of(r), s->p.max_suffix);
    }
  MC_HIP(hipSetDevice(s->m->device));
  // New pages in the order a lock-step decode of these tokens would take them: token by token,
  // candidates ascending, a candidate stepping aside once its tokens are used up.
  std::vector<int32_t> idx, fresh;
  {
    std::vector<int32_t> next(n_cands);           // first slot candidate r does not hold yet
    for (int r = 0; r < n_cands; ++r) next[r] = (s->cand_len[s->alive[r]] + pg - 1) / pg;
    for (;;) {
      // the earliest token index at which some candidate opens its next slot
      int j = INT32_MAX;
      for (int r = 0; r < n_cands; ++r) {
        const int at = next[r] * pg - s->cand_len[s->alive[r]];
        if (at < len_of(r)) j = std::min(j, at);
      }
      if (j == INT32_MAX) break;
      for (int r = 0; r < n_cands; ++r)
        if (next[r] * pg - s->cand_len[s->alive[r]] == j && j < len_of(r))
          idx.push_back(s->alive[r] * L.pages_per_cand + next[r]++);
    }
  }
  if (int rc0 = stage_pages(s, idx, fresh)) { unfix_cands(s, saved_n); return rc0; }
  s->lists_cands = false;                       // this pass writes logits rows without top lists
  std::vector<int32_t> now(s->host_table);       // the table with the staged pages in place
  for (size_t i = 0; i < idx.size(); ++i) now[idx[i]] = fresh[i];
  std::vector<int32_t> tok, pos, page, off, tab, last, items;
  for (int b0 = 0; b0 < n_cands;) {
    int b1 = b0, rows = 0;                         // whole candidates per chunk
    while (b1 < n_cands && rows + len_of(b1) <= s->chunk_rows) rows += len_of(b1++);
    const int nc = b1 - b0;
    tok.resize(rows); pos.resize(rows); page.resize(rows); off.resize(rows); tab.resize(rows);
    last.resize(nc);
    items.clear();
    int r = 0;
    for (int b = b0; b < b1; ++b) {               // b: row among the candidates still decoding
      const int cand = s->alive[b], t = s->cand_len[cand], len = len_of(b);
      for (int j = 0; j < len; j += 64) {
        items.push_back(r + j); items.push_back(std::min(64, len - j));
        items.push_back(s->prefix_len + t + j); items.push_back(cand);
      }
      for (int j = 0; j < len; ++j, ++r) {
        tok[r] = suffix_tokens[(size_t)b * max_len + j];
        pos[r] = s->prefix_len + t + j;
        page[r] = now[(size_t)cand * L.pages_per_cand + (t + j) / pg];
        off[r] = (t + j) % pg;
        tab[r] = cand;
      }
      last[b - b0] = r - 1;
    }
    int rc = upload(s, s->ptr<void>(L.row_tok), tok.data(), (size_t)rows * 4);
    if (rc == MC_OK) rc = upload(s, s->ptr<void>(L.row_pos), pos.data(), (size_t)rows * 4);
    if (rc == MC_OK) rc = upload(s, s->ptr<void>(L.row_page), page.data(), (size_t)rows * 4);
    if (rc == MC_OK) rc = upload(s, s->ptr<void>(L.row_off), off.data(), (size_t)rows * 4);
    if (rc == MC_OK) rc = upload(s, s->ptr<void>(L.row_tab), tab.data(), (size_t)rows * 4);
    if (rc == MC_OK) rc = upload(s, s->ptr<void>(L.last_idx), last.data(), (size_t)nc * 4);
    if (rc == MC_OK) rc = upload(s, s->ptr<void>(L.items), items.data(), items.size() * 4);
    int tail = 0;
    if (rc == MC_OK) rc = run_layers(s, rows, PASS_SUFFIX, s->prefix_len, (int)items.size() / 4, &tail);
    if (rc == MC_OK) rc = lm_head(s, rows, tail, nc, true, s->ptr<float>(L.logits) + (size_t)b0 * c.vocab);
    if (rc != MC_OK) { unfix_cands(s, saved_n); return rc; }
    b0 = b1;
  }
  commit_pages(s, idx, fresh);
  for (int r = 0; r < n_cands; ++r) s->cand_len[s->alive[r]] += len_of(r);
  refresh_lengths(s);
  s->logits_state = LOGITS_CANDS;
  s->logits_rows = n_cands;
  s->sampled_on_device = false;
  return MC_OK;
}

extern "C" int mc_prefill_suffix(mc_session *s, const int32_t *suffix_tokens, int32_t n_cands, int32_t len) {
  return prefill_suffix_impl(s, suffix_tokens, nullptr, n_cands, len, "mc_prefill_suffix");
}

extern "C" int mc_prefill_suffix_ragged(mc_session *s, const int32_t *suffix_tokens, const int32_t *lens,
                                        int32_t n_cands, int32_t max_len) {
  if (!lens) MC_FAIL(MC_ERR_INVALID, "lens is NULL");
  return prefill_suffix_impl(s, suffix_tokens, lens, n_cands, max_len, "mc_prefill_suffix_ragged");
}

// ---- inspection hooks -----------------------------------------------------------------
extern "C" int mc_debug_copy_logits(mc_session *s, float *out, int32_t n_rows) {
  if (!s || !out) MC_FAIL(MC_ERR_INVALID, "session / out is NULL");
  if (s->logits_state == LOGITS_NONE) MC_FAIL(MC_ERR_STATE, "no logits pending");
  if (n_rows != s->logits_rows) MC_FAIL(MC_ERR_INVALID, "n_rows %d, but %d rows are pending", n_rows, s->logits_rows);
  const SessionLayout &L = s->lay;
  const float *src = s->logits_state == LOGITS_PREFIX ? s->ptr<float>(L.prefix_logits) : s->ptr<float>(L.logits);
  MC_TRY(download(s, out, src, (size_t)n_rows * s->m->cfg.vocab * 4));
  MC_HIP(hipStreamSynchronize(s->stream));
  return MC_OK;
}

extern "C" int mc_debug_page_table(mc_session *s, int32_t *out, int32_t *n_pages, int32_t max_pages) {
  if (!s || !out || !n_pages) MC_FAIL(MC_ERR_INVALID, "a pointer is NULL");
  int longest = s->suffix_len;
  for (int b : s->paused) longest = std::max(longest, s->cand_len[b]);
  const int most = (longest + s->p.page_tokens - 1) / s->p.page_tokens;
  if (max_pages < most) MC_FAIL(MC_ERR_INVALID, "max_pages %d < %d pages held", max_pages, most);
  for (int b = 0; b < s->p.max_cands; ++b) {
    const bool holds = std::find(s->alive.begin(), s->alive.end(), b) != s->alive.end() ||
                       std::find(s->paused.begin(), s->paused.end(), b) != s->paused.end();
    const int held = holds ? (s->cand_len[b] + s->p.page_tokens - 1) / s->p.page_tokens : 0;
    n_pages[b] = held;
    for (int p = 0; p < max_pages; ++p)
      out[(size_t)b * max_pages + p] = (holds && p < held) ? s->host_table[(size_t)b * s->lay.pages_per_cand + p] : -1;
  }
  return MC_OK;
}

extern "C" int32_t mc_debug_pool_pages(const mc_session *s) { return s ? s->lay.n_pool_pages : 0; }

extern "C" int mc_debug_set_free_list(mc_session *s, const int32_t *perm, int32_t n) {
  if (!s || !perm) MC_FAIL(MC_ERR_INVALID, "session / perm is NULL");
  if (s->n_cands != 0) MC_FAIL(MC_ERR_STATE, "free list can only change while no candidate holds a page");
  if (n != s->lay.n_pool_pages) MC_FAIL(MC_ERR_INVALID, "n %d != pool size %d", n, s->lay.n_pool_pages);
  std::vector<char> seen(n, 0);
  for (int i = 0; i < n; ++i) {
    if (perm[i] < 0 || perm[i] >= n || seen[perm[i]]) MC_FAIL(MC_ERR_INVALID, "perm is not a permutation");
    seen[perm[i]] = 1;
  }
  s->free_list.assign(perm, perm + n);
  s->free_q.assign(s->free_list.begin(), s->free_list.end());
  return MC_OK;
}

extern "C" int mc_debug_set_prefix_splits(mc_session *s, int32_t n_splits) {
  if (!s) MC_FAIL(MC_ERR_INVALID, "session is NULL");
  if (n_splits < 0 || n_splits > 1024) MC_FAIL(MC_ERR_INVALID, "n_splits %d outside [0, 1024]", n_splits);
  s->prefix_splits = n_splits;
  return MC_OK;
}

extern "C" const char *mc_last_error(void) { return g_err; }

// ---- timing ----------------------------------------------------------------------------
extern "C" int mc_profile_begin(mc_session *s, int32_t kernel_class, int32_t stride) {
  if (!s) MC_FAIL(MC_ERR_INVALID, "session is NULL");
  if (kernel_class < 0 || kernel_class >= MC_K_COUNT) MC_FAIL(MC_ERR_INVALID, "unknown kernel class %d", kernel_class);
  if (stride < 1) MC_FAIL(MC_ERR_INVALID, "stride must be >= 1");
  MC_HIP(hipSetDevice(s->m->device));
  if (kernel_class != MC_K_NONE && s->prof_ev.empty()) {
    s->prof_ev.resize(2 * kProfCap);
    for (auto &e : s->prof_ev) MC_HIP(hipEventCreate(&e));
  }
  s->prof_class = kernel_class;
  s->prof_stride = stride;
  s->prof_seen = 0;
  s->prof_n = 0;
  return MC_OK;
}

extern "C" int mc_profile_end(mc_session *s, int32_t *n_timed, double *total_ms) {
  if (!s || !n_timed || !total_ms) MC_FAIL(MC_ERR_INVALID, "a pointer is NULL");
  MC_HIP(hipStreamSynchronize(s->stream));
  double tot = 0.0;
  for (int i = 0; i < s->prof_n; ++i) {
    float ms = 0.f;
    MC_HIP(hipEventElapsedTime(&ms, s->prof_ev[2 * i], s->prof_ev[2 * i + 1]));
    tot += ms;
  }
  *n_timed = s->prof_n;
  *total_ms = tot;
  s->prof_class = MC_K_NONE;
  return MC_OK;
}
