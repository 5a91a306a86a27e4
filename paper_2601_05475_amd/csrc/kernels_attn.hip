// Decode attention for B candidates that share one prefix (bf16, gfx950 MFMA).
//
// Candidate b's query heads attend to the shared prefix (read ONCE for all candidates) and to
// b's own suffix pages.  One launch runs a list of work items, one workgroup (4 waves) each:
//   prefix item (kv head, key split s, row block rb): a range of prefix pages against up to 128
//     query rows (row = b * G + g, G = query heads per KV head); wave w owns rows 32w..32w+31.
//   suffix item (candidate b, kv head): all of b's suffix pages against its G query rows; the
//     four waves take the four 32-key blocks of each staged page pair and merge in LDS.
// Every item leaves an un-normalised partial (max m, sum l, weighted values o) per query head;
// a second small kernel merges the partials of each (candidate, head) and writes bf16.
//
// Tiles: two 64-key pages per iteration are staged through LDS (K as [key][hd], V as stored,
// [hd][key]); loads for the next pair are in flight while the current pair is consumed.
// Scores are computed transposed, S^T = K Q^T, so that a lane owns ONE query column: the softmax
// reductions are 16 in-lane steps plus one cross-half shuffle, the running rescale of O^T is a
// per-lane scalar, and the probability registers are, as they stand, the B operand of
// O^T += V^T P^T once V's key order follows the accumulator layout (see kmap below).
#include "kernels_mfma.h"

#include <stdlib.h>

#include <algorithm>

namespace mc {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
// native 16- and 8-byte vectors: register arrays of these are promoted out of scratch
typedef __attribute__((ext_vector_type(4))) uint32_t v4u;
typedef __attribute__((ext_vector_type(2))) uint32_t v2u;
__device__ inline v4u make_v4u(uint32_t a, uint32_t b, uint32_t c, uint32_t d) { return v4u{a, b, c, d}; }

__device__ inline f32x16 mfma32a(v4u a, v4u b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// two floats -> packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32)
__device__ inline uint32_t pack2_bf16(float a, float b) {
  typedef __attribute__((ext_vector_type(2))) float f32x2;
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, b}, bf16x2));
}

constexpr int PG = 64;                       // keys per page (the only page size of this kernel)

template <int HD> struct AttnTile {
  static constexpr int KLD = HD + 8;         // K row stride (elements): 16-byte aligned, conflict-free b128 reads
  static constexpr int VLD = PG + 8;         // V row stride (elements): 16-byte aligned, conflict-free b64 reads
  static constexpr int K_ELEMS = PG * KLD;
  static constexpr int V_ELEMS = HD * VLD;
  static constexpr int PAGE_ELEMS = K_ELEMS + V_ELEMS;
  static constexpr int LDS_BYTES = 2 * PAGE_ELEMS * 2;
  static constexpr int CHUNKS = PG * HD / 8;            // 16-byte chunks of one K (or V) page
  static constexpr int CPT = CHUNKS / 256;              // chunks per thread per page per tensor
};

constexpr int kStages = 1;                   // register stages of the page pipeline
constexpr int kMaxSuffixSplits = 8;
constexpr int kMaxPids = 512;                // suffix page ids kept in LDS (longer suffixes read them from memory)

struct AttnItems {
  int n_prefix_items, n_suffix_items;
  int splits, row_blocks, pages_per_split;   // prefix
  int suffix_splits, suffix_pps;             // suffix: key splits per (candidate, kv head), pages per split
  int n_prefix_pages, rows;                  // rows = B * G
  int pid_offset;                            // byte offset of the page-id array in LDS
};

template <int HD>
__global__ __launch_bounds__(256, 2)
void decode_attention_kernel(DecodeAttnArgs a, AttnItems it,
                                                               float *__restrict__ part_o,
                                                               float *__restrict__ part_ml) {
  using TL = AttnTile<HD>;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  bf16_t *lds = (bf16_t *)lds_raw;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, col = lane & 31, h = lane >> 5;
  const int Hq = a.n_q_heads, Hkv = a.n_kv_heads, G = Hq / Hkv, B = a.n_cands;
  const bool is_prefix = (int)blockIdx.x < it.n_prefix_items;

  // ---- decode the work item
  int kvh, part, first_page, n_pages, n_keys;       // n_keys: valid keys counted from first_page * 64
  const bf16_t *kpool, *vpool;
  const int32_t *table = nullptr;
  int b_of_col, g_of_col;
  bool col_valid;
  if (is_prefix) {
    int id = blockIdx.x;
    const int rb = id % it.row_blocks; id /= it.row_blocks;
    const int s = id % it.splits; kvh = id / it.splits;
    part = s;
    first_page = s * it.pages_per_split;
    n_pages = min(it.pages_per_split, it.n_prefix_pages - first_page);
    n_keys = min(a.prefix_len - first_page * PG, n_pages * PG);
    kpool = (const bf16_t *)a.k_prefix; vpool = (const bf16_t *)a.v_prefix;
    const int rho = rb * 128 + wave * 32 + col;
    col_valid = rho < it.rows;
    b_of_col = col_valid ? rho / G : 0;
    g_of_col = col_valid ? rho % G : 0;
  } else {
    int id = blockIdx.x - it.n_prefix_items;
    const int ss = id % it.suffix_splits; id /= it.suffix_splits;
    kvh = id % Hkv;
    const int b = id / Hkv;
    part = ((a.prefix_len > 0) ? it.splits : 0) + ss;
    first_page = ss * it.suffix_pps;
    n_pages = min(it.suffix_pps, (a.suffix_len + PG - 1) / PG - first_page);
    n_keys = min(a.suffix_len - first_page * PG, n_pages * PG);
    kpool = (const bf16_t *)a.k_suffix; vpool = (const bf16_t *)a.v_suffix;
    table = a.page_table + (size_t)b * a.table_stride;
    col_valid = col < G;
    b_of_col = b;
    g_of_col = col_valid ? col : 0;
  }
  const int head = kvh * G + g_of_col;

  // ---- query fragments: B operand of S^T = K Q^T, lane (col, h) holds Q[row][16c + 8h .. +7]
  v4u qf[HD / 16];
  {
    const bf16_t *qrow = (const bf16_t *)a.q + ((size_t)b_of_col * Hq + head) * HD + 8 * h;
#pragma unroll
    for (int c = 0; c < HD / 16; ++c) qf[c] = *(const v4u *)(qrow + 16 * c);
  }
  const float scale2 = 1.4426950408889634f / sqrtf((float)HD);   // 1/sqrt(hd) * log2(e)

  f32x16 o[HD / 32];
#pragma unroll
  for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
  float m = -INFINITY, l = 0.f;

  // ---- staging: thread t carries chunks t + 256 i of the K and of the V page in flight
  const size_t page_stride = (size_t)Hkv * PG * HD;           // elements per page (all kv heads)
  const size_t head_off = (size_t)kvh * PG * HD;
  // kStages register stages: that many pages are in flight while one is consumed.  Two stages
  // keep the kernel within 256 registers, so two workgroups share a CU and overlap each other's
  // load, softmax and MFMA phases.
  v4u sk[kStages][TL::CPT], sv[kStages][TL::CPT];
  // A suffix item's page ids are copied to LDS once: fetching one from global memory inside the
  // loop would put a full memory round trip in front of every prefetch.
  int *pids = (int *)(lds_raw + it.pid_offset);
  const bool pids_in_lds = table != nullptr && n_pages <= kMaxPids;
  if (pids_in_lds) {
    for (int i = tid; i < n_pages; i += 256) pids[i] = table[first_page + i];
    __syncthreads();
  }
  auto page_id = [&](int pi) __attribute__((always_inline)) -> int {
    return table ? (pids_in_lds ? pids[pi - first_page] : table[pi]) : pi;
  };
  // Every call issues the same number of loads, whether or not page pi exists: past the end all
  // lanes re-read one 16-byte piece of the item's first page (the data is never used).  With no
  // branch around the loads the compiler's load counters stay exact, so a commit waits for its own
  // stage only and the two younger stages stay in flight.
  auto issue = [&](int stage, int pi) __attribute__((always_inline)) {
    const bool real = pi < n_pages;
    const size_t base = (size_t)page_id(first_page + (real ? pi : 0)) * page_stride + head_off;
    const size_t lane_off = real ? (size_t)tid * 8 : 0, step = real ? 256 * 8 : 0;
#pragma unroll
    for (int i = 0; i < TL::CPT; ++i) {
      sk[stage][i] = *(const v4u *)(kpool + base + lane_off + step * i);
      sv[stage][i] = *(const v4u *)(vpool + base + lane_off + step * i);
    }
  };
  auto commit = [&](int stage, int buf) __attribute__((always_inline)) {
    bf16_t *kt = lds + buf * TL::PAGE_ELEMS, *vt = kt + TL::K_ELEMS;
#pragma unroll
    for (int i = 0; i < TL::CPT; ++i) {
      const int ci = tid + 256 * i;
      *(v4u *)(kt + (ci / (HD / 8)) * TL::KLD + (ci % (HD / 8)) * 8) = sk[stage][i];
      *(v4u *)(vt + (ci / (PG / 8)) * TL::VLD + (ci % (PG / 8)) * 8) = sv[stage][i];
    }
  };

  // one 32-key block: half `blk` of the page held in LDS buffer `buf`
  auto process = [&](int buf, int blk, int n_valid) __attribute__((always_inline)) {
    const bf16_t *kt = lds + buf * TL::PAGE_ELEMS, *vt = kt + TL::K_ELEMS;
    const int kb = blk * 32;
    f32x16 s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int c = 0; c < HD / 16; ++c) {
      const v4u kf = *(const v4u *)(kt + (kb + col) * TL::KLD + 16 * c + 8 * h);
      s = mfma32a(kf, qf[c], s);
    }
    // s[r] = raw score of key kmap(r) = 8 (r / 4) + 4 h + r % 4 against this lane's query column.
    // The running maximum m lives in the base-2 domain: m = max(score * scale * log2(e)).
    if (n_valid < 32) {
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (8 * (r >> 2) + 4 * h + (r & 3) >= n_valid) s[r] = -INFINITY;
    }
    float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
#pragma unroll
    for (int r = 4; r < 16; r += 4) mx = fmaxf(mx, fmaxf(fmaxf(s[r], s[r + 1]), fmaxf(s[r + 2], s[r + 3])));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    // Lazy reference: m only has to stay within kTau of the true running maximum (then every
    // 2^(score - m) <= 2^kTau, harmless in fp32 and bf16); sums and weighted values are all taken
    // against the same m, so the normalised result does not depend on it.  The costly rescale of
    // the 16 * HD/32 accumulators then happens in the first block(s) only.
    constexpr float kTau = 8.0f;
    const float mx2 = mx * scale2;                // finite: a processed block has a valid key
    if (__any(mx2 > m + kTau)) {
      const float m_new = fmaxf(m, mx2);
      const float corr = __builtin_amdgcn_exp2f(m - m_new);   // m = -inf at the start: 0
      l *= corr;
      m = m_new;
#pragma unroll
      for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] *= corr;
    }
    float rs = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      s[r] = __builtin_amdgcn_exp2f(fmaf(s[r], scale2, -m));
      rs += s[r];
    }
    rs += __shfl_xor(rs, 32, 64);
    l += rs;
    // probabilities as the B operand: slab sl holds keys kmap(8 sl .. 8 sl + 7)
    v4u pb[2];
    pb[0] = make_v4u(pack2_bf16(s[0], s[1]), pack2_bf16(s[2], s[3]), pack2_bf16(s[4], s[5]), pack2_bf16(s[6], s[7]));
    pb[1] = make_v4u(pack2_bf16(s[8], s[9]), pack2_bf16(s[10], s[11]), pack2_bf16(s[12], s[13]), pack2_bf16(s[14], s[15]));
#pragma unroll
    for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
      for (int sl = 0; sl < 2; ++sl) {
        const bf16_t *vrow = vt + (dt * 32 + col) * TL::VLD + kb + 16 * sl + 4 * h;
        const v2u lo = *(const v2u *)vrow, hi = *(const v2u *)(vrow + 8);
        o[dt] = mfma32a(make_v4u(lo.x, lo.y, hi.x, hi.y), pb[sl], o[dt]);
      }
  };

  // Page i is consumed from LDS buffer i % 2 while page i + 1 is in flight to registers.  One
  // barrier per page: commit(i + 1) overwrites the buffer read during page i - 1, and every wave
  // has left that page before it reaches the barrier of page i.
  auto consume = [&](int i) __attribute__((always_inline)) {
    const int buf = i & 1;
    const int key0 = i * PG;         // first key of this page, relative to the item's first page
    if (is_prefix) {
#pragma unroll 1
      for (int blk = 0; blk < 2; ++blk) {
        const int nv = min(32, n_keys - (key0 + 32 * blk));
        if (nv > 0) process(buf, blk, nv);
      }
    } else if (wave < 2) {           // a suffix page has two blocks: waves 2, 3 only help to stage
      const int nv = min(32, n_keys - (key0 + 32 * wave));
      if (nv > 0) process(buf, wave, nv);
    }
  };
  // Page pi is consumed from LDS buffer pi % 2.  One barrier per page is enough: commit(pi)
  // overwrites the buffer read during page pi - 2, and every wave has left that page before it
  // arrives at the barrier of page pi - 1.  Stages past the last page run as no-ops on dummy
  // data (n_pages >= 1 for every item).
#pragma unroll
  for (int st = 0; st < kStages; ++st) issue(st, st);
  for (int i = 0; i < n_pages; i += kStages) {
#pragma unroll
    for (int st = 0; st < kStages; ++st) {
      const int pi = i + st;
      commit(st, pi & 1);
      __syncthreads();
      issue(st, pi + kStages);
      if (pi < n_pages) consume(pi);
    }
  }

  // ---- epilogue
  if (is_prefix) {
    if (col_valid) {
      const size_t row = ((size_t)part * B + b_of_col) * Hq + head;
      if (h == 0) {
        part_ml[row * 2] = m;
        part_ml[row * 2 + 1] = l;
      }
#pragma unroll
      for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4)
          *(float4 *)(part_o + row * HD + dt * 32 + 8 * r4 + 4 * h) =
              make_float4(o[dt][4 * r4], o[dt][4 * r4 + 1], o[dt][4 * r4 + 2], o[dt][4 * r4 + 3]);
    }
  } else {
    // the four waves hold four partial states of the same G columns: merge them in LDS
    __syncthreads();
    float *sm = (float *)lds_raw;                       // [4][32] m, then [4][32] l
    float *so = sm + 256;                               // [4][G][HD]
    if (h == 0) {
      sm[wave * 32 + col] = m;
      sm[128 + wave * 32 + col] = l;
    }
    __syncthreads();
    float mm = sm[col];
#pragma unroll
    for (int w = 1; w < 4; ++w) mm = fmaxf(mm, sm[w * 32 + col]);
    // a wave that saw no key has m = -inf and contributes nothing
    const float f = (m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m - mm);
    if (col_valid) {
#pragma unroll
      for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          so[((size_t)wave * G + col) * HD + dt * 32 + 8 * (r >> 2) + 4 * h + (r & 3)] = o[dt][r] * f;
    }
    __syncthreads();
    for (int e = tid; e < G * HD; e += 256) {
      const int g = e / HD, d = e % HD;
      const float v = so[e] + so[G * HD + e] + so[2 * G * HD + e] + so[3 * G * HD + e];
      const size_t row = ((size_t)part * B + b_of_col) * Hq + kvh * G + g;
      part_o[row * HD + d] = v;
      if (d == 0) {
        float mg = sm[g], lg = 0.f;
#pragma unroll
        for (int w = 1; w < 4; ++w) mg = fmaxf(mg, sm[w * 32 + g]);
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const float mw = sm[w * 32 + g];
          lg += (mw == -INFINITY) ? 0.f : sm[128 + w * 32 + g] * __builtin_amdgcn_exp2f(mw - mg);
        }
        part_ml[row * 2] = mg;
        part_ml[row * 2 + 1] = lg;
      }
    }
  }
}

// out[b][head] = sum_p 2^{m_p - M} o_p / sum_p 2^{m_p - M} l_p   (m in the base-2 domain)
template <int HD>
__global__ __launch_bounds__(HD) void decode_attention_merge_kernel(
    int n_parts, int B, int Hq, const float *__restrict__ part_o, const float *__restrict__ part_ml,
    bf16_t *__restrict__ out, int out_tiled) {
  // The (m, l) pairs are fetched by one thread each, in parallel, and turned into weights in
  // LDS; the value sums then run over independent loads, eight parts in flight at a time.
  constexpr int kMaxParts = 1024;
  __shared__ float sw[kMaxParts], sl[kMaxParts];
  const int bh = blockIdx.x, d = threadIdx.x;
  const size_t stride = (size_t)B * Hq;
  for (int p = d; p < n_parts; p += HD) {
    const float2 ml = *(const float2 *)(part_ml + (p * stride + bh) * 2);
    sw[p] = ml.x;
    sl[p] = ml.y;
  }
  __syncthreads();
  float M = -INFINITY;
  for (int p = 0; p < n_parts; ++p) M = fmaxf(M, sw[p]);
  __syncthreads();
  for (int p = d; p < n_parts; p += HD) sw[p] = __builtin_amdgcn_exp2f(sw[p] - M);
  __syncthreads();
  float den = 0.f;
  for (int p = 0; p < n_parts; ++p) den += sw[p] * sl[p];
  float num = 0.f;
  const float *po = part_o + (size_t)bh * HD + d;
  int p = 0;
  for (; p + 8 <= n_parts; p += 8) {
    float v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = po[(p + j) * stride * HD];
#pragma unroll
    for (int j = 0; j < 8; ++j) num += sw[p + j] * v[j];
  }
  for (; p < n_parts; ++p) num += sw[p] * po[p * stride * HD];
  const int b = bh / Hq, head = bh % Hq;
  const size_t at = out_tiled ? tiled_offset(b, head * HD + d, Hq * HD) : (size_t)bh * HD + d;
  out[at] = f32_to_bf16(num / den);
}

static AttnItems plan_items(const DecodeAttnArgs &a) {
  AttnItems it;
  const int G = a.n_q_heads / a.n_kv_heads;
  it.rows = a.n_cands * G;
  it.row_blocks = (it.rows + 127) / 128;
  it.n_prefix_pages = (a.prefix_len + PG - 1) / PG;
  int splits = 0;
  if (it.n_prefix_pages > 0) {
    const int pairs = (it.n_prefix_pages + 1) / 2;
    splits = a.prefix_splits;
    if (splits <= 0) {
      // enough items to cover the chip, but at least four page pairs (512 keys) per item so that
      // the partial sums written per item stay small next to the keys/values read
      const int per_head = std::max(1, 256 / std::max(1, a.n_kv_heads * it.row_blocks));
      splits = std::min(per_head, std::max(1, pairs / 4));
    }
    splits = std::max(1, std::min(splits, pairs));
    it.pages_per_split = ((pairs + splits - 1) / splits) * 2;
    splits = (it.n_prefix_pages + it.pages_per_split - 1) / it.pages_per_split;   // drop empty splits
  } else {
    it.pages_per_split = 0;
  }
  it.splits = splits;
  it.n_prefix_items = a.n_kv_heads * splits * it.row_blocks;
  // suffix: split a candidate's pages when that fills idle workgroup slots (two per CU); the
  // partial state of a suffix item is small (G rows), so splitting costs little
  const int s_pages = (a.suffix_len + PG - 1) / PG;
  int ssplits = 1;
  if (s_pages > 0) {
    const char *env = getenv("MC_ATTN_SUFFIX_SPLITS");         // measurement override
    if (env && atoi(env) > 0) ssplits = atoi(env);
    else {
      const int base_items = a.n_cands * a.n_kv_heads;
      while (ssplits < kMaxSuffixSplits && base_items * ssplits * 2 + it.n_prefix_items <= 640 &&
             (s_pages + ssplits * 2 - 1) / (ssplits * 2) >= 2)
        ssplits *= 2;
    }
    ssplits = std::max(1, std::min(std::min(ssplits, kMaxSuffixSplits), s_pages));
    it.suffix_pps = (s_pages + ssplits - 1) / ssplits;
    ssplits = (s_pages + it.suffix_pps - 1) / it.suffix_pps;
  } else {
    it.suffix_pps = 0;
  }
  it.suffix_splits = ssplits;
  it.n_suffix_items = (a.suffix_len > 0) ? a.n_cands * a.n_kv_heads * ssplits : 0;
  return it;
}

bool decode_attention_mfma_supported(const DecodeAttnArgs &a) {
  const int G = a.n_q_heads / a.n_kv_heads;
  return a.page_tokens == PG && (a.head_dim == 64 || a.head_dim == 128) && G >= 1 && G <= 32 &&
         a.n_q_heads % a.n_kv_heads == 0;
}

// partials: every (part, candidate, head) holds hd + 2 floats; parts <= prefix pairs + 1
size_t decode_attention_mfma_ws_bytes(int n_cands, int Hq, int Hkv, int hd, int prefix_len,
                                      int suffix_len, int page_tokens) {
  (void)Hkv; (void)suffix_len;
  if (page_tokens != PG) return 0;
  const int pairs = ((prefix_len + PG - 1) / PG + 1) / 2;
  const size_t parts = (size_t)pairs + kMaxSuffixSplits;
  return parts * n_cands * Hq * (size_t)(hd + 2) * sizeof(float) + 512;
}

template <int HD>
static int launch_decode_attention_t(hipStream_t st, const DecodeAttnArgs &a, const AttnItems &it_in) {
  using TL = AttnTile<HD>;
  const int n_parts = (a.prefix_len > 0 ? it_in.splits : 0) + (a.suffix_len > 0 ? it_in.suffix_splits : 0);
  const size_t rows = (size_t)a.n_cands * a.n_q_heads;
  const size_t need = (size_t)n_parts * rows * (HD + 2) * sizeof(float);
  if (a.workspace_bytes < need) MC_FAIL(MC_ERR_INVALID, "attention workspace has %zu bytes, %zu needed", a.workspace_bytes, need);
  if (n_parts > 1024) MC_FAIL(MC_ERR_UNSUPPORTED, "decode attention: %d partial states exceed 1024", n_parts);
  float *part_o = (float *)a.workspace;
  float *part_ml = part_o + (size_t)n_parts * rows * HD;
  const int G = a.n_q_heads / a.n_kv_heads;
  const size_t lds_main = (std::max((size_t)TL::LDS_BYTES, (size_t)(256 + 4 * G * HD) * sizeof(float)) + 15) / 16 * 16;
  const size_t lds = lds_main + kMaxPids * sizeof(int);
  AttnItems it = it_in;
  it.pid_offset = (int)lds_main;
  static bool attr_set = false;          // per template instance
  if (!attr_set) {
    MC_HIP(hipFuncSetAttribute((const void *)decode_attention_kernel<HD>,
                               hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 1024));
    attr_set = true;
  }
  decode_attention_kernel<HD><<<it.n_prefix_items + it.n_suffix_items, 256, lds, st>>>(a, it, part_o, part_ml);
  MC_HIP(hipGetLastError());
  decode_attention_merge_kernel<HD><<<(unsigned)rows, HD, 0, st>>>(
      n_parts, a.n_cands, a.n_q_heads, part_o, part_ml, (bf16_t *)a.out, a.out_tiled);
  MC_HIP(hipGetLastError());
  return MC_OK;
}

int launch_attention_decode_mfma(hipStream_t st, const DecodeAttnArgs &a) {
  if (!decode_attention_mfma_supported(a)) MC_FAIL(MC_ERR_UNSUPPORTED, "decode attention: shape not covered");
  const AttnItems it = plan_items(a);
  if (it.n_prefix_items + it.n_suffix_items == 0) MC_FAIL(MC_ERR_INVALID, "decode attention without keys");
  return a.head_dim == 128 ? launch_decode_attention_t<128>(st, a, it) : launch_decode_attention_t<64>(st, a, it);
}

}  // namespace mc
