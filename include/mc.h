/*
 * mc.h - C ABI of the MI355X shared-prefix candidate decoding / scoring library.
 *
 * The computation is the LLM step inside the MaxCode search loop: a frozen
 * autoregressive policy proposes several candidates from ONE search state (Sec. 3,
 * "The Markov Decision Process": stochastic token sampling yields M distinct
 * candidates for the same state; Sec. 3.2, CUDA-LLM reformulation: k candidates per
 * state), and a generative value model reranks candidate states by the expected
 * value of a categorical reward-to-go (Sec. 3.3, "Generative Value Function Guided
 * Search").  All candidates share the prompt (problem, trajectory, critiques, best
 * result so far), so its keys/values are computed once and read once per step.
 *
 * Conventions
 *  - Every function returns an mc_status (0 = ok, negative = error) unless noted.
 *    mc_last_error() gives a message for the last failure on the calling thread.
 *  - "host" pointers are ordinary CPU memory, read or written during the call only.
 *    "device" pointers are HIP device memory on the session's / call's device.
 *  - The library never calls hipMalloc for device memory: models and sessions live
 *    inside arenas supplied by the caller (mc_arena), sized by mc_model_bytes /
 *    mc_session_bytes.  The caller keeps ownership and frees them after destroy.
 *  - All work is enqueued on the arena's HIP stream.  Calls with host outputs return
 *    after the outputs are valid; calls without host outputs are asynchronous.
 *  - On error no output is valid and the session keeps its pre-call state
 *    (MC_ERR_DEVICE excepted).  Handles are not thread-safe.
 *  - Matrices are row-major [out_features][in_features]; element type is the
 *    model's dtype (MC_F32: float, MC_BF16: 16-bit bfloat16 bit patterns).
 */
#ifndef MC_H_
#define MC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mc_model mc_model;     /* immutable weights + shape, on device      */
typedef struct mc_session mc_session; /* shared prefix KV + candidates' KV pages   */

typedef enum { MC_F32 = 0, MC_BF16 = 1 } mc_dtype;

typedef enum {
  MC_OK = 0,
  MC_ERR_INVALID = -1,     /* bad argument (null, out of range, non-finite)       */
  MC_ERR_STATE = -2,       /* call out of order (decode before prefill, ...)      */
  MC_ERR_OOM = -3,         /* arena or page pool too small                        */
  MC_ERR_DEVICE = -4,      /* a HIP call failed                                   */
  MC_ERR_UNSUPPORTED = -5  /* shape or option the kernels do not cover            */
} mc_status;

/* Decoder shape: pre-norm blocks of grouped-query attention with rotary position
 * embedding (pairs (i, i + head_dim/2), angle pos * rope_base^(-2i/head_dim)) and a
 * SwiGLU feed-forward, RMSNorm (x * g / sqrt(mean(x^2) + rms_eps)), no biases,
 * untied LM head.  Query head a reads KV head a / (n_q_heads / n_kv_heads). */
typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rms_eps, rope_base;
  int32_t dtype; /* mc_dtype of weights, activations and KV */
} mc_config;

/* Weight pointers (host or device memory; copied during mc_model_create and free
 * to release afterwards).  Per-layer members are arrays of n_layers pointers. */
typedef struct {
  const void *embed;              /* [vocab][d_model]                              */
  const void *const *attn_norm;   /* [d_model]                                     */
  const void *const *wq;          /* [n_q_heads*head_dim][d_model]                 */
  const void *const *wk;          /* [n_kv_heads*head_dim][d_model]                */
  const void *const *wv;          /* [n_kv_heads*head_dim][d_model]                */
  const void *const *wo;          /* [d_model][n_q_heads*head_dim]                 */
  const void *const *ffn_norm;    /* [d_model]                                     */
  const void *const *w_gate;      /* [d_ffn][d_model]                              */
  const void *const *w_up;        /* [d_ffn][d_model]                              */
  const void *const *w_down;      /* [d_model][d_ffn]                              */
  const void *final_norm;         /* [d_model]                                     */
  const void *lm_head;            /* [vocab][d_model]                              */
} mc_weights;

/* Device memory owned by the caller (e.g. a torch tensor) plus the stream to use. */
typedef struct {
  void *dev_base;     /* device pointer, 256-byte aligned                         */
  size_t dev_bytes;
  void *hip_stream;   /* hipStream_t; NULL = the default stream                   */
  int32_t device;     /* HIP device ordinal                                       */
} mc_arena;

typedef struct {
  int32_t max_prefix;   /* longest shared prefix, tokens                          */
  int32_t max_cands;    /* most candidates B                                      */
  int32_t max_suffix;   /* longest per-candidate suffix (decode steps / scoring)  */
  int32_t page_tokens;  /* KV page size in tokens: power of two, 4..128           */
  int32_t chunk_rows;   /* rows processed at once by prefill/scoring (0 = default)*/
  int32_t pool_pages;   /* KV pages shared by the candidates' suffixes; 0 = max_cands *
                           ceil(max_suffix / page_tokens), enough for every candidate to
                           reach max_suffix.  A smaller pool serves searches that start
                           many candidates and keep few (mc_drop_candidates returns pages
                           to the pool); a step that needs more pages than are free fails
                           with MC_ERR_OOM and changes nothing                          */
} mc_session_params;

/* ---- lifecycle ------------------------------------------------------------------ */
size_t mc_model_bytes(const mc_config *cfg);                   /* 0 if cfg is invalid */
int mc_model_create(const mc_config *cfg, const mc_weights *w, const mc_arena *arena,
                    mc_model **out);
void mc_model_destroy(mc_model *m);

size_t mc_session_bytes(const mc_config *cfg, const mc_session_params *p);
int mc_session_create(const mc_model *m, const mc_arena *arena, const mc_session_params *p,
                      mc_session **out);
void mc_session_destroy(mc_session *s);
/* Drop all candidates (their pages return to the free list in its initial order) and
 * keep the prefix; the next mc_sample draws again from the prefix's last position. */
int mc_session_reset_candidates(mc_session *s);
/* Wait for everything enqueued by this session. */
int mc_session_sync(mc_session *s);

/* ---- the four calls -------------------------------------------------------------- */

/* 1. One context -> shared KV (policy paragraph of Sec. 3: all candidates of a step
 *    are conditioned on the same state).  tokens: host, n_tokens in [1, max_prefix].
 *    Replaces any earlier prefix and drops all candidates.  Leaves the logits of the
 *    last prefix position on the device for mc_sample.  Asynchronous. */
int mc_prefill_shared(mc_session *s, const int32_t *tokens, int32_t n_tokens);

/* 1b. Grow the shared context in place (Sec. 3: the state of step i+1 is the state of step i
 *    plus the chosen candidate, its feedback and the critique, so the prompt of the next depth
 *    extends the prompt of this one).  mc_extend_shared appends n_tokens host tokens at positions
 *    prefix_len .. of the shared sequence: only the new tokens are run, attending to the
 *    prefix KV already there, and the logits of the last new position are left for mc_sample.
 *    n_tokens in [1, max_prefix - prefix_len].  mc_promote_candidate appends the tokens candidate
 *    cand has decoded so far (its suffix KV, copied on the device; nothing is recomputed) and
 *    makes that candidate's pending logits the prefix logits.  Both drop all candidates.
 *    Errors: MC_ERR_STATE without a prefix / without a decoded token, MC_ERR_OOM or
 *    MC_ERR_INVALID when max_prefix would be exceeded.  Asynchronous. */
int mc_extend_shared(mc_session *s, const int32_t *tokens, int32_t n_tokens);
int mc_promote_candidate(mc_session *s, int32_t cand);

/* 1c. Several new tokens per candidate in one pass (the critic of Sec. 3.3 reads, per candidate,
 *    the candidate and its execution feedback after the shared trajectory, then writes its
 *    critique token by token).  suffix_tokens: host [n_cands][len]; every candidate gets len
 *    tokens after the suffix tokens it already holds, attending causally to the
 *    shared prefix and to its own suffix; their K/V go to the candidate's pages and stay, the
 *    logits of each candidate's last new token are left for mc_sample / mc_decode_step to go on
 *    from.  One common len for all candidates here.  Errors: MC_ERR_STATE without a
 *    prefix, MC_ERR_OOM beyond max_suffix, MC_ERR_INVALID for a changed n_cands.  Asynchronous. */
int mc_prefill_suffix(mc_session *s, const int32_t *suffix_tokens, int32_t n_cands, int32_t len);
/*    The same with a length of its own for every candidate (the candidates and their feedback
 *    differ in length): row r of suffix_tokens (host [n_cands][max_len]) holds lens[r] tokens,
 *    1 <= lens[r] <= max_len, for the r-th candidate still decoding.  From then on the
 *    candidates sit at different suffix positions: mc_decode_step appends each one's token at its
 *    own position (own rotary angle, own page slot, attention over its own keys), a candidate
 *    takes a new page when its own length reaches a page boundary (candidates in ascending order
 *    at every token index, as a lock-step decode of the same tokens would), mc_promote_candidate
 *    moves that candidate's own length, and MC_ERR_OOM is returned once any candidate would
 *    exceed max_suffix (drop it to go on with the others). */
int mc_prefill_suffix_ragged(mc_session *s, const int32_t *suffix_tokens, const int32_t *lens,
                             int32_t n_cands, int32_t max_len);

/* 1d. Candidates end at different lengths, and a value-guided search keeps only the promising
 *    ones (Sec. 3.3).  mc_drop_candidates removes the n candidates cands[.] (ids as numbered when
 *    the candidates were started, each still decoding, at least one other must stay): they take
 *    no further part in mc_decode_step / mc_sample / mc_prefill_suffix, whose work (rows, KV
 *    traffic) shrinks accordingly, and their pages go back to the pool: the free pages are a
 *    queue, a page boundary hands its head to the candidates still decoding in ascending id
 *    order, and the pages of dropped candidates join its tail (ascending candidate id, each
 *    one's pages in the order it took them), so later boundaries reuse them.  From then on those calls
 *    are given the number of candidates still decoding, and every per-candidate array (tokens,
 *    uniforms, sampled ids, logits rows) lists the survivors in ascending id order; results that
 *    were pending for the survivors (logits, sampled tokens) stay valid.
 *    mc_session_reset_candidates starts over with all candidates. */
int mc_drop_candidates(mc_session *s, const int32_t *cands, int32_t n);

/* 1e. A candidate that sits out some steps and goes on later (it waits for its execution feedback
 *    while the others keep decoding, Sec. 3.3).  mc_pause_candidates takes the n candidates cands[.]
 *    (each still decoding, at least one other must go on) out of the set that decodes, exactly as
 *    mc_drop_candidates does (rows, KV traffic and per-candidate arrays shrink to the others, whose
 *    pending results stay valid), but they keep their pages and suffix tokens.
 *    mc_resume_candidates puts n paused candidates back, in ascending id order among the others,
 *    each at its own suffix length (the candidates may then differ in length as after
 *    mc_prefill_suffix_ragged).  Resuming renumbers the rows of the per-candidate arrays, so nothing
 *    is pending afterwards: the next call is mc_decode_step with host tokens for every candidate
 *    now decoding (or mc_prefill_suffix / mc_prefill_suffix_ragged).  mc_session_reset_candidates
 *    forgets paused candidates too.  A paused candidate cannot be dropped or promoted; resume it first. */
int mc_pause_candidates(mc_session *s, const int32_t *cands, int32_t n);
int mc_resume_candidates(mc_session *s, const int32_t *cands, int32_t n);

/* 2. One new token per candidate: appends its K/V to the candidate's current page
 *    and leaves logits [n_cands][vocab] on the device.  tokens: host [n_cands], or
 *    NULL to consume the tokens drawn by the latest mc_sample without leaving the
 *    device.  n_cands is fixed by the first call after a prefill/reset.
 *    Asynchronous. */
int mc_decode_step(mc_session *s, const int32_t *tokens, int32_t n_cands);

/* 3. Draw the next token of every candidate from the logits left by call 1 (one row,
 *    shared by all candidates) or call 2 (one row each).  With z = logit / T, keep
 *    the top_k entries under the order (z descending, id ascending), softmax over
 *    them (sums taken left to right in that order, fp32) and pick the first entry
 *    whose cumulative probability exceeds uniforms[b]; the last entry if none does.
 *    temperature <= 0 or top_k == 1: argmax (lowest id on ties).  top_k <= 0 or
 *    >= vocab: whole vocabulary (supported up to MC_MAX_TOP_K entries).
 *    uniforms: host [n_cands], each in [0, 1).  out_tokens: host [n_cands] or NULL
 *    (NULL keeps the call asynchronous).  out_topk_ids: host [n_cands][k] sorted by
 *    that order, or NULL. */
int mc_sample(mc_session *s, int32_t n_cands, float temperature, int32_t top_k,
              const float *uniforms, int32_t *out_tokens, int32_t *out_topk_ids);

/* 4. Rerank candidates by the generative reward-to-go score (Sec. 3.3): run each
 *    candidate's suffix against the shared prefix, take the log-probabilities of the
 *    reward tokens (log-softmax over the whole vocabulary) at its last position,
 *    score = sum_r reward_values[r] * softmax_r(logprob_r / score_temperature), and
 *    rank by (score descending, candidate index ascending).  Does not touch the
 *    candidates' decode state.  suffix_tokens: host [n_cands][max_len] (entries past
 *    suffix_lens[b] ignored); suffix_lens[b] in [1, max_len]; reward_ids distinct.
 *    Outputs: host out_logprobs [n_cands][n_reward], out_scores [n_cands],
 *    out_rank [n_cands] (best first); any may be NULL. */
int mc_score_candidates(mc_session *s, const int32_t *suffix_tokens,
                        const int32_t *suffix_lens, int32_t n_cands, int32_t max_len,
                        const int32_t *reward_ids, const float *reward_values,
                        int32_t n_reward, float score_temperature, float *out_logprobs,
                        float *out_scores, int32_t *out_rank);

#define MC_MAX_TOP_K 4096
#define MC_MAX_REWARD 64

/* ---- host-side bookkeeping of the search loop (no device work) -------------------- */

/* Categorical reward f_r (Sec. 3.3, "Categorical Reward Formulation"): 0 if the candidate is
 * incorrect or its speedup is <= 100 %, else 1..4 by the thresholds (s1, s2, s3) in percent
 * (intervals closed on the right).  thresholds: host, 3 values, 100 <= s1 <= s2 <= s3.
 * Returns the bin, or a negative mc_status. */
int32_t mc_reward_bin(double speedup_percent, int32_t correct, const double *thresholds);

/* Best discounted reward so far (Sec. 3.2): u_out[i] = max_{j <= i} gamma^depths[j] * rewards[j].
 * All arrays host, n >= 1, gamma in (0, 1]. */
int mc_best_so_far(const double *rewards, const int32_t *depths, int32_t n, double gamma, double *u_out);

/* Training targets of the value model along one trajectory (Sec. 3.3): with rewards[t] =
 * f_r(e_{t+1}), t = 0..n-1,  u_out[t] = max_{k <= t} gamma^k rewards[k]  and
 * v_out[t] = max(u_out[t] / gamma, max_{k >= t} gamma^(k-t) rewards[k]). */
int mc_value_targets(const double *rewards, int32_t n, double gamma, double *u_out, double *v_out);

/* Beam step of the CUDA-LLM search (Sec. 3.2): the index of the largest speedup ratio if any is
 * > 1 (lowest index on ties), else MC_SELECT_NONE (no candidate is correct and faster). */
#define MC_SELECT_NONE (-100)
int32_t mc_select_candidate(const double *speedups, int32_t n);

/* Evaluation statistics (Sec. 4, "Evaluation Metrics").  mc_median_of_max: speedups holds the
 * generations of problem 0, then of problem 1, ... (counts[p] >= 1 each); *out = the median over
 * problems of the per-problem maximum (mean of the two middle values for an even count).
 * mc_average_rank: max_speedup is [n_methods][n_problems]; avg_rank[m] = mean over problems of
 * 1 + the number of methods strictly better on that problem. */
int mc_median_of_max(const double *speedups, const int32_t *counts, int32_t n_problems, double *out);
int mc_average_rank(const double *max_speedup, int32_t n_methods, int32_t n_problems, double *avg_rank);

/* ---- inspection hooks (tests and tools; not on the fast path) -------------------- */
/* Copy the pending logits to host as fp32: n_rows rows of vocab floats (1 row after
 * a prefill, n_cands after a decode step, n_cands after scoring). */
int mc_debug_copy_logits(mc_session *s, float *out, int32_t n_rows);
/* Page ids of every candidate's allocated suffix pages.  out: host
 * [max_cands][max_pages] (unused entries -1), n_pages: host [max_cands]. */
int mc_debug_page_table(mc_session *s, int32_t *out, int32_t *n_pages, int32_t max_pages);
/* Replace the order in which an untouched pool hands out its pages (a permutation of
 * 0..n-1, n = pool size; mc_session_reset_candidates returns to this order); only
 * allowed while no candidate holds a page.  mc_debug_pool_pages gives n. */
int mc_debug_set_free_list(mc_session *s, const int32_t *perm, int32_t n);
int32_t mc_debug_pool_pages(const mc_session *s);
/* Override the number of key-axis splits used for the shared prefix (0 = automatic). */
int mc_debug_set_prefix_splits(mc_session *s, int32_t n_splits);
const char *mc_last_error(void);

/* ---- timing of one kernel class inside a session --------------------------------- */
typedef enum {
  MC_K_NONE = 0, MC_K_EMBED, MC_K_ADD_RMSNORM, MC_K_LINEAR_QKV, MC_K_ROPE_KV,
  MC_K_ATTN_DECODE, MC_K_ATTN_MERGE, MC_K_ATTN_PREFILL, MC_K_LINEAR_O,
  MC_K_LINEAR_GATE_UP, MC_K_LINEAR_DOWN, MC_K_LINEAR_LM_HEAD, MC_K_SAMPLE,
  MC_K_REWARD, MC_K_COUNT
} mc_kernel_class;
/* Time every `stride`-th launch of one kernel class with HIP events on the session stream
 * (kernel_class = MC_K_NONE switches it off; at most 8192 launches recorded).  For the few-row
 * gate/up layer and for decode attention (+ merge) the events are attached to the kernel launches
 * themselves and carry the kernels' own begin and end times; for the other classes they are
 * recorded on the stream before and after the launch, which adds a few microseconds. */
int mc_profile_begin(mc_session *s, int32_t kernel_class, int32_t stride);
/* Synchronise, then report how many launches were timed and their total duration. */
int mc_profile_end(mc_session *s, int32_t *n_timed, double *total_ms);

/* ---- single operations on device buffers (kernel-level tests and measurement) ---- */
/* All pointers below are DEVICE pointers unless marked host; `stream` is a hipStream_t
 * (NULL = default).  `dtype` selects float or bf16 for buffers marked (T). */

/* Tiled operand layout of the bf16 MFMA linear kernels.  A [rows][K] matrix (K % 64 == 0) is
 * stored as 4 KB blocks, rows padded to a multiple of 32: block (row / 32, k / 64) sits at byte
 * ((row / 32) * (K / 64) + k / 64) * 4096, and inside it the 16-byte chunk c = (k % 32) / 8 of
 * lane l = row % 32 + 32 * ((k % 64) / 32), at byte (c * 64 + l) * 16, holds the 8 elements
 * k - k % 8 .. +7 of that row.  mc_op_tiled_bytes gives the buffer size (0 if K is unsuitable);
 * mc_op_pack_tiled converts a row-major bf16 matrix (padding rows are zero-filled). */
size_t mc_op_tiled_bytes(int32_t rows, int32_t K);
int mc_op_pack_tiled(void *stream, int32_t rows, int32_t K, const void *src, void *dst);

/* Residual update + RMSNorm: x[r][:] += sum_s partials[s][r][:] (n_partials may be 0),
 * then h[r][:] = (T)(x * gain / sqrt(mean(x^2) + eps)).  x: fp32 [rows][d], in/out.
 * h_tiled = 1 stores h in the tiled layout (bf16, d % 64 == 0). */
int mc_op_add_rmsnorm(void *stream, int32_t dtype, int32_t rows, int32_t d, float *x,
                      const float *partials, int32_t n_partials, const void *gain /*(T)[d]*/,
                      float eps, void *h_out /*(T)[rows][d]*/, int32_t h_tiled);

/* out[s][m][n] = sum over the s-th K range of a[m][k] * w[n][k]; n_splits partial sums
 * (fp32, row-major) that add up to a * w^T.  a: (T)[M][K], w: (T)[N][K], out: fp32
 * [n_splits][M][N].  tiled = 1: a and w are in the tiled layout (bf16, N % 128 == 0,
 * K % 256 == 0; M <= 64 streams the weights once and n_splits must divide K / 256; larger M
 * runs the MFMA GEMM with n_splits = 1).  mc_op_linear_splits: the split count the session
 * would choose. */
int mc_op_linear(void *stream, int32_t dtype, int32_t M, int32_t N, int32_t K, const void *a,
                 const void *w, float *out, int32_t n_splits, int32_t tiled);
int32_t mc_op_linear_splits(int32_t dtype, int32_t M, int32_t N, int32_t K, int32_t tiled);

/* bf16 tiled operands, many rows: x[m][n] += sum_k a[m][k] w[n][k] in the epilogue of the
 * 256-row-tile matrix-core GEMM (the residual update of the O and down projections in prefill and
 * scoring).  x: fp32 [M][N] row-major, device, updated in
 * place; every element is read and written by exactly one lane, so the result does not depend on
 * scheduling.  MC_ERR_UNSUPPORTED unless N % 128 == 0, K % 256 == 0 and M > 64 (fewer rows keep
 * mc_op_linear + mc_op_add_rmsnorm). */
int mc_op_linear_accumulate(void *stream, int32_t M, int32_t N, int32_t K, const void *a,
                            const void *w, float *x);

/* bf16 tiled operands: the QKV projection fused with mc_op_rope_kv_write.  a: tiled [rows][K];
 * wqkv: tiled [(Hq + 2 Hkv) * hd][K] whose query and key heads have their rows interleaved
 * (row 2i of a head holds coordinate i, row 2i + 1 coordinate i + hd/2; value heads in natural
 * order).  table: device scratch of n_pos * hd/2 * 16 bytes, filled here with cos / sin (double)
 * of pos * base^(-2i/hd); every row_pos[r] must be < n_pos.  Outputs as mc_op_rope_kv_write
 * (bf16).  Covers rows <= 64 (weight-streaming kernel) and more rows (256-row-tile GEMM) when
 * N % 128 == 0 and K % 256 == 0; else MC_ERR_UNSUPPORTED. */
int mc_op_linear_qkv_rope(void *stream, int32_t rows, int32_t n_q_heads, int32_t n_kv_heads,
                          int32_t head_dim, int32_t page_tokens, int32_t K, float rope_base,
                          int32_t n_pos, const void *a, const void *wqkv, const int32_t *row_pos,
                          const int32_t *row_page, const int32_t *row_off, void *table,
                          void *q_out, void *k_pages, void *v_pages);

/* out[m][n] = (T)( silu(a . w_gate[n]) * (a . w_up[n]) ).  out: (T)[M][N]; with tiled = 1 the
 * inputs and the output are tiled. */
int mc_op_linear_swiglu(void *stream, int32_t dtype, int32_t M, int32_t N, int32_t K,
                        const void *a, const void *w_gate, const void *w_up, void *out,
                        int32_t tiled);

/* Sum the n_splits partial QKV rows, rotate q and k of row r by position row_pos[r],
 * store q as (T)[rows][Hq][hd] and write k, v of row r into KV page row_page[r] at
 * offset row_off[r].  qkv: fp32 [n_splits][rows][(Hq+2Hkv)*hd].
 *
 * KV page layout (all attention entry points read what this one writes).  A K page and a V
 * page each hold Hkv regions of page_tokens * hd elements, one per KV head.  If page_tokens
 * or hd is not a multiple of 32 a region is plain: K as [key][hd], V transposed as [hd][key].
 * Otherwise it is a sequence of 32-key blocks of 32 * hd elements, each block a run of
 * 1 KB fragments in the order one 32x32x16 MFMA reads its A operand; fragment f keeps, for
 * lane l = 0..63, eight elements at (f * 64 + l) * 8:
 *   K fragment c:          key l % 32, coordinates 16c + 8 (l / 32) + 0..7;
 *   V fragment 2 dt + sl:  coordinate 32 dt + l % 32, keys 16 sl + 4 (l / 32) + {0,1,2,3,8,9,10,11}. */
int mc_op_rope_kv_write(void *stream, int32_t dtype, int32_t rows, int32_t n_q_heads,
                        int32_t n_kv_heads, int32_t head_dim, int32_t page_tokens,
                        float rope_base, const float *qkv, int32_t n_splits,
                        const int32_t *row_pos, const int32_t *row_page,
                        const int32_t *row_off, void *q_out, void *k_pages, void *v_pages);

/* Decode attention for n_cands candidates: candidate b attends to the prefix_len keys of the
 * shared prefix (pages 0.. of k_prefix/v_prefix, in order) and to its own suffix keys (pages
 * page_table[b][0..] of k_suffix/v_suffix): suffix_len of them, or, with row_len (device,
 * [n_cands]) given, row_len[b] of them, 1 <= row_len[b] <= suffix_len (other values are
 * clamped into that range) for candidates of different lengths.
 * q, out: (T)[n_cands][Hq][hd].  workspace: fp32 scratch of mc_op_attention_decode_ws
 * bytes.  prefix_splits: key-axis splits of the prefix (0 = automatic).  out_tiled = 1 stores
 * out as a tiled [n_cands][Hq*hd] matrix. */
size_t mc_op_attention_decode_ws(int32_t n_cands, int32_t n_q_heads, int32_t n_kv_heads,
                                 int32_t head_dim, int32_t prefix_len, int32_t suffix_len,
                                 int32_t page_tokens);
int mc_op_attention_decode(void *stream, int32_t dtype, int32_t n_cands, int32_t n_q_heads,
                           int32_t n_kv_heads, int32_t head_dim, int32_t page_tokens,
                           int32_t prefix_len, int32_t suffix_len, const void *q,
                           const void *k_prefix, const void *v_prefix, const void *k_suffix,
                           const void *v_suffix, const int32_t *page_table,
                           int32_t table_stride, const int32_t *row_len, int32_t prefix_splits,
                           void *workspace, size_t workspace_bytes, void *out, int32_t out_tiled);

/* mc_op_attention_decode for callers that cannot allocate device memory or bring a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same
 * kernels and arguments, with the partial states kept in a buffer of MC_STATIC_SCRATCH_BYTES that
 * the library holds in every GPU's memory from load to process exit.  The call allocates nothing.
 * MC_ERR_UNSUPPORTED when mc_op_attention_decode_ws(...) for these sizes exceeds that buffer (the
 * 1B and 8B decode shapes fit, a 16k-token prefix with 64 candidates does not).  All calls on one
 * GPU share the buffer: calls that overlap on one GPU (two streams, two threads) race; calls on
 * one stream are ordered and safe.  Nothing in the buffer has to survive between calls. */
#define MC_STATIC_SCRATCH_BYTES (32u << 20)
int mc_op_attention_decode_static(void *stream, int32_t dtype, int32_t n_cands, int32_t n_q_heads,
                                  int32_t n_kv_heads, int32_t head_dim, int32_t page_tokens,
                                  int32_t prefix_len, int32_t suffix_len, const void *q,
                                  const void *k_prefix, const void *v_prefix, const void *k_suffix,
                                  const void *v_suffix, const int32_t *page_table,
                                  int32_t table_stride, const int32_t *row_len, int32_t prefix_splits,
                                  void *out, int32_t out_tiled);

/* Host-only: the work-item plan mc_op_attention_decode would launch for these sizes on the bf16
 * MFMA path (MC_ERR_UNSUPPORTED for shapes that path does not cover).  out9 (host, nine values):
 * prefix items incl. padding ids, suffix items, prefix key splits, 32-key blocks per prefix split,
 * suffix key splits, blocks per suffix split, partial states per (candidate, head), id distance
 * between the items of one prefix split, blocks of 32 query rows per prefix item (1 or 4). */
int mc_op_attention_decode_plan(int32_t n_cands, int32_t n_q_heads, int32_t n_kv_heads,
                                int32_t head_dim, int32_t page_tokens, int32_t prefix_len,
                                int32_t suffix_len, int32_t prefix_splits, int32_t *out9);

/* Causal attention for many query rows (prefix prefill, candidate scoring); bf16, 64-token
 * pages, head_dim 64 or 128.  items: device int32 [n_items][4] = (first row, rows <= 64,
 * position of the first row, page-table row or -1): up to 64 consecutive positions of one sequence.
 * A row at position p attends to keys 0..p: positions < prefix_len from the prefix pages (in
 * order), later ones from pages page_table[row][.] of the suffix pool.  q: [rows][Hq][hd];
 * out: [rows][Hq*hd], row-major or tiled (out_tiled = 1). */
int mc_op_attention_prefill(void *stream, int32_t n_items, const int32_t *items,
                            int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                            int32_t page_tokens, int32_t prefix_len, const void *q,
                            const void *k_prefix, const void *v_prefix, const void *k_suffix,
                            const void *v_suffix, const int32_t *page_table,
                            int32_t table_stride, void *out, int32_t out_tiled);

/* HBM read-rate probe (a measurement aid): reads `bytes` of device memory once (a multiple of
 * 64 MiB; larger than the 256 MB memory-side cache for an HBM figure) with 16-byte streaming
 * loads and nothing else; out_word: device, 4 bytes, may be written. */
int mc_op_read_probe(void *stream, const void *buf, size_t bytes, void *out_word);

/* Matrix-core rate probe (a measurement aid, not part of the path): n_workgroups * 256 threads
 * each read 96 bytes of bf16 operands (device, n_workgroups * 256 * 96 bytes) once and then issue
 * iters * 8 MFMAs (32x32x16, bf16) on them, no other memory traffic; out: device, one float per
 * thread.  Flops = n_workgroups * 4 waves * iters * 8 * 32768.  The rate depends on the operand
 * values through the power-dependent clock. */
int mc_op_mfma_probe(void *stream, const void *operands, float *out, int32_t n_workgroups,
                     int32_t iters);

/* Sampling from fp32 logits [rows][vocab] (row_stride 0 = every candidate reads row 0).
 * uniforms: device [n_cands].  out_tokens: device [n_cands]; out_topk: device
 * [n_cands][k] or NULL.  Same rule as mc_sample. */
int mc_op_sample(void *stream, int32_t n_cands, int32_t vocab, const float *logits,
                 size_t row_stride, float temperature, int32_t top_k, const float *uniforms,
                 int32_t *out_tokens, int32_t *out_topk);

/* The LM head's share of sampling (bf16 tiled operands; at most 32 rows, N % 128 == 0, N >= 65536,
 * K % 256 == 0, else MC_ERR_UNSUPPORTED): logits[m][n] = sum_k a[m][k] w[n][k] (fp32 [M][N]) and,
 * beside them, for every row and every group of 64 consecutive ids the four largest (logit, id)
 * pairs under (logit descending, id ascending): top_lists[(m * N / 64 + g) * 4 + t] = {float bits,
 * int32 id}, mc_op_top_list_bytes(M, N) bytes.  mc_op_sample_lists is mc_op_sample reading those
 * lists (1 / 16 of a row) instead of the rows wherever that yields the rule's result: for
 * top_k <= 64 it selects from the lists and checks that no group's fourth entry reaches the k-th
 * selected value after the division by the temperature (an unlisted id of that group could then
 * belong to the top k or tie with its last member); a row that fails the check is selected from
 * the whole row, so ids and top-k lists are the rule's in every case.  row_stride 0 = every
 * candidate reads row 0 of both. */
size_t mc_op_top_list_bytes(int32_t rows, int32_t N);
int mc_op_lm_head(void *stream, int32_t M, int32_t N, int32_t K, const void *a, const void *w,
                  float *logits, void *top_lists);
int mc_op_sample_lists(void *stream, int32_t n_cands, int32_t vocab, const float *logits,
                       size_t row_stride, const void *top_lists, float temperature, int32_t top_k,
                       const float *uniforms, int32_t *out_tokens, int32_t *out_topk);

/* Reward log-probs, expected-value scores and ranking from fp32 logits [n_cands][vocab].
 * reward_ids, reward_values: device [n_reward].  Outputs: device. */
int mc_op_reward_score(void *stream, int32_t n_cands, int32_t vocab, const float *logits,
                       const int32_t *reward_ids, const float *reward_values,
                       int32_t n_reward, float score_temperature, float *out_logprobs,
                       float *out_scores, int32_t *out_rank);

#ifdef __cplusplus
}
#endif
#endif /* MC_H_ */
