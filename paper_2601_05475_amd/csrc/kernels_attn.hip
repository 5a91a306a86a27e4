// Decode attention for B candidates that share one prefix (bf16, gfx950 MFMA).
//
// Candidate b's query heads attend to the shared prefix (read from HBM once for all candidates)
// and to b's own suffix pages.  KV pages are stored in MFMA fragment order, so a wave loads the
// operands of a 32-key block straight from global memory into registers, 1 KB per instruction,
// and no tile is staged through LDS: every wave is an independent stream that always has the
// K or the V fragments of its next block in flight, and eight such waves per CU keep enough
// bytes in flight to cover the memory latency.
// One launch runs a list of work items, one workgroup (4 waves) each.  An item is a range of
// 32-key blocks of one KV head against up to 32 query columns; wave w takes blocks w, w + 4, ...
// of the range and the four partial states are merged in LDS:
//   prefix item (row block rb, kv head, key split s): columns are query rows 32 rb .. 32 rb + 31
//     (row = b * G + g, G = query heads per KV head).  The items of one (kv head, split) differ
//     in rb only and are numbered a multiple of 8 apart: workgroups are dealt round-robin to the
//     8 XCDs, so they share one L2 and the keys come from HBM once.
//     With eight or more row blocks per KV head an item takes four of them instead, one per wave:
//     every wave walks all blocks of the range and nothing is merged across waves.
//   suffix item (candidate b, kv head, key split): columns are b's G query heads.
// Every item leaves an un-normalised partial (max m, sum l, weighted values o) per query head;
// a second small kernel merges the partials of each (candidate, head) and writes bf16.  (An item
// that holds the only partial of its rows normalises and writes them itself.)
//
// Scores are computed transposed, S^T = K Q^T, so that a lane owns ONE query column: the softmax
// reductions are 16 in-lane steps plus one cross-half shuffle, the running rescale of O^T is a
// per-lane scalar, and the probability registers are, as they stand, the B operand of
// O^T += V^T P^T because V's fragments list their keys in the accumulator's order.
#include "kernels_mfma.h"

#include <hip/hip_ext.h>

#include <algorithm>

namespace mc {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
// native 16-byte vectors: register arrays of these are promoted out of scratch
typedef __attribute__((ext_vector_type(4))) uint32_t v4u;
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
constexpr int kMaxSuffixSplits = 8;

struct AttnItems {
  int n_prefix_items, n_suffix_items;
  int splits, row_blocks, blocks_per_split;  // prefix: key splits, blocks of 32 rows, 32-key blocks per split
  int prefix_groups, prefix_stride;          // (kv head, split) pairs; id distance between row blocks (multiple of 8)
  int suffix_splits, suffix_bps;             // suffix: key splits per (candidate, kv head), blocks per split
  int n_prefix_blocks, n_suffix_blocks, rows;   // rows = B * G
  int rb_per_item;                           // prefix: row blocks per item, 1 (waves split the keys) or 4 (one per wave)
};

template <int HD>
__global__ __launch_bounds__(256, 2)
void decode_attention_kernel(DecodeAttnArgs a, AttnItems it, float *__restrict__ part_o,
                             float *__restrict__ part_ml, int n_parts) {
  constexpr int NF = HD / 16;                // 1 KB fragments per 32-key block, K and V alike
  constexpr int BLK = 32 * HD;               // elements of one block
  constexpr int SOLD = HD + 4;               // row stride of the merge buffer (floats)
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, h = lane >> 5;
  // the wave index as a scalar: block ranges, page ids and addresses derived from it stay in
  // scalar registers and the loop branches are uniform
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int swap_addr = (lane ^ 32) << 2;    // ds_bpermute address of the lane with the other 16 keys
  const int Hq = a.n_q_heads, Hkv = a.n_kv_heads, G = Hq / Hkv, B = a.n_cands;
  const bool is_prefix = (int)blockIdx.x < it.n_prefix_items;

  // ---- decode the work item.  Column c of the item is query row (b, head) with
  //      rho = col0 + c, b = rho / G (prefix) or the item's candidate (suffix), g = rho % G.
  int kvh, part, first_blk, blk_end, len, n_cols, col0, b_item;
  const bf16_t *kpool, *vpool;
  const int32_t *table = nullptr;
  // Many query rows per KV head (more than 7 blocks of 32): a prefix item takes four row blocks,
  // one per wave, and every wave walks all key blocks of the item's range.  The four waves ask
  // for the same key and value fragments at about the same time, so the range crosses the L2-to-CU
  // path about once per item instead of once per row block, which is what bounds the kernel
  // there; nothing is merged across waves.  With few row blocks (wave_rows false) the waves
  // split the key blocks of one row block instead, which keeps more items in flight.
  const bool wave_rows = is_prefix && it.rb_per_item == 4;
  if (is_prefix) {
    const int rbg = blockIdx.x / it.prefix_stride, grp = blockIdx.x % it.prefix_stride;
    if (grp >= it.prefix_groups) return;                       // padding id
    const int s = grp % it.splits;
    kvh = grp / it.splits;
    part = s;
    first_blk = s * it.blocks_per_split;
    blk_end = min(first_blk + it.blocks_per_split, it.n_prefix_blocks);
    len = a.prefix_len;
    kpool = (const bf16_t *)a.k_prefix; vpool = (const bf16_t *)a.v_prefix;
    col0 = (wave_rows ? rbg * 4 + wave : rbg) * 32;
    n_cols = max(0, min(32, it.rows - col0));                  // 0: a wave past the last row block idles
    b_item = -1;
  } else {
    int id = blockIdx.x - it.n_prefix_items;
    const int ss = id % it.suffix_splits; id /= it.suffix_splits;
    kvh = id % Hkv;
    b_item = id / Hkv;
    part = ((a.prefix_len > 0) ? it.splits : 0) + ss;
    first_blk = ss * it.suffix_bps;
    // candidates of different lengths: the plan is laid out for the longest, an item past its
    // candidate's last block has nothing to do and writes an empty partial state
    len = a.row_len ? min(max(a.row_len[b_item], 1), a.suffix_len) : a.suffix_len;
    blk_end = min(first_blk + it.suffix_bps, (len + 31) >> 5);
    kpool = (const bf16_t *)a.k_suffix; vpool = (const bf16_t *)a.v_suffix;
    table = a.page_table + (size_t)(a.row_cand ? a.row_cand[b_item] : b_item) * a.table_stride;
    col0 = 0;
    n_cols = G;
  }
  const bool col_valid = col < n_cols;
  const int rho = n_cols > 0 ? col0 + (col_valid ? col : 0) : 0;   // a wave without columns reads row 0 (never stored)
  const int b_of_col = (b_item >= 0) ? b_item : rho / G;
  const int head = kvh * G + rho % G;
  const int bstep = wave_rows ? 1 : 4;                       // distance between this wave's key blocks
  const int blk_begin = first_blk + (wave_rows ? 0 : wave);
  const int n_mine = n_cols > 0 ? (blk_end - blk_begin + bstep - 1) / bstep : 0;   // <= 0: idle wave

  // ---- query fragments: B operand of S^T = K Q^T, lane (col, h) holds Q[row][16c + 8h .. +7].
  // They are parked in LDS (each lane reads back only what it wrote) to leave the registers to
  // the accumulators and the fragments in flight.
  v4u *qs = (v4u *)lds_raw + wave * NF * 64 + lane;
  {
    const bf16_t *qrow = (const bf16_t *)a.q + ((size_t)b_of_col * Hq + head) * HD + 8 * h;
#pragma unroll
    for (int c = 0; c < NF; ++c) qs[c * 64] = *(const v4u *)(qrow + 16 * c);
  }
  const float scale2 = 1.4426950408889634f / sqrtf((float)HD);   // 1/sqrt(hd) * log2(e)

  f32x16 o[HD / 32];
#pragma unroll
  for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
  float m = -INFINITY, l = 0.f;

  const size_t page_stride = (size_t)Hkv * PG * HD;           // elements per page (all kv heads)
  const size_t head_off = (size_t)kvh * PG * HD;
  v4u kf[NF], vf[NF];
  // Page ids of the next 64 blocks of this wave, one per lane; block j of the window reads lane j.
  int my_pid = 0;
  auto load_pids = [&](int w0) __attribute__((always_inline)) {
    int g = blk_begin + (w0 + lane) * bstep;
    if (g >= blk_end) g = first_blk;                            // any valid block of the item
    my_pid = table ? table[g >> 1] : (g >> 1);
  };
  // Byte address of block j of the window (wave-uniform) and this lane's offset in a fragment.
  // Past the end of the window the loads are still issued, all lanes re-reading the same 16-byte
  // pieces of the window's first block (never used): with no branch around the loads the
  // compiler's load counters stay exact, so waiting for the keys of a block leaves its values,
  // issued later, in flight, and the other way round.
  // A lane all of whose keys lie past the end of the sequence (only in the sequence's last block)
  // reads the fragment's first 16 bytes instead of its own: finite values of valid keys, which
  // meet a masked score (keys) or a zero probability (values), and no memory traffic of their own.
  auto block_base = [&](int w0, int j, int wn, uint32_t &voff, int &n_valid) __attribute__((always_inline)) -> size_t {
    const bool real = j < wn;
    const int jj = real ? j : 0;
    const int g = blk_begin + (w0 + jj) * bstep;
    const int page = __builtin_amdgcn_readlane(my_pid, jj);
    voff = real ? lane * 16u : 0u;
    n_valid = len - 32 * g;
    return ((size_t)page * page_stride + head_off + (size_t)(g & 1) * BLK) * sizeof(bf16_t);
  };
  auto issue_k = [&](int w0, int j, int wn) __attribute__((always_inline)) {
    uint32_t voff;
    int n_valid;
    const char *kb = (const char *)kpool + block_base(w0, j, wn, voff, n_valid);
    if (col >= n_valid) voff = 0u;                               // lane (col, h) holds key col
#pragma unroll
    for (int c = 0; c < NF; ++c) kf[c] = *(const v4u *)(kb + voff + 1024 * c);
  };
  auto issue_v = [&](int w0, int j, int wn) __attribute__((always_inline)) {
    uint32_t voff;
    int n_valid;
    const char *vb = (const char *)vpool + block_base(w0, j, wn, voff, n_valid);
#pragma unroll
    for (int c = 0; c < NF; ++c)                                 // fragment c: keys 16 (c & 1) + 4 h + {0..3, 8..11}
      vf[c] = *(const v4u *)(vb + ((16 * (c & 1) + 4 * h >= n_valid) ? 0u : voff) + 1024 * c);
  };

  // Windows of 64 blocks (the page ids one wave register holds).  Inside a window: scores of
  // block j from kf, then kf is refilled for block j + 1 while the softmax and the value MFMAs of
  // block j run, then vf is refilled.
  for (int w0 = 0; w0 < n_mine; w0 += 64) {
    const int wn = min(64, n_mine - w0);
    load_pids(w0);
    issue_k(w0, 0, wn);
    issue_v(w0, 0, wn);
    for (int j = 0; j < wn; ++j) {
      const int n_valid = min(32, len - 32 * (blk_begin + (w0 + j) * bstep));
      // an offset the compiler cannot see through (always 0): the query reads stay inside the
      // loop instead of being hoisted back into 4 * NF registers
      int q_at = 0;
      asm volatile("" : "+v"(q_at));
      f32x16 s;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
      for (int c = 0; c < NF; ++c) s = mfma32a(kf[c], qs[c * 64 + q_at], s);
      issue_k(w0, j + 1, wn);
      // s[r] = raw score of key kmap(r) = 8 (r / 4) + 4 h + r % 4 against this lane's query column.
      // The running maximum m lives in the base-2 domain: m = max(score * scale * log2(e)).
      if (n_valid < 32) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (8 * (r >> 2) + 4 * h + (r & 3) >= n_valid) s[r] = -INFINITY;
      }
      // Lazy reference: sums and weighted values are all taken against the same m, so the
      // normalised result does not depend on it; m only has to keep the numbers in range.  The
      // probabilities are therefore computed against m as it stands, and only if a lane's sum
      // leaves the range (a score far above m, or the first block, where m = -inf gives inf or
      // NaN) the block's maximum is taken, m moved there and the 16 * HD/32 accumulators
      // rescaled.  The common case spends no instruction on maxima.
      f32x16 p;
      float rs = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        p[r] = __builtin_amdgcn_exp2f(fmaf(s[r], scale2, -m));
        rs += p[r];
      }
      if (__any(!(rs <= kSoftmaxSumLimit))) {
        float mx = max16f(s);
        mx = fmaxf(mx, swap_halves(mx, swap_addr));
        const float m_new = fmaxf(m, mx * scale2);              // finite: a processed block has a valid key
        const float corr = __builtin_amdgcn_exp2f(m - m_new);   // m = -inf at the start: 0
        l *= corr;
        m = m_new;
#pragma unroll
        for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[dt][r] *= corr;
        rs = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          p[r] = __builtin_amdgcn_exp2f(fmaf(s[r], scale2, -m));
          rs += p[r];
        }
      }
      rs += swap_halves(rs, swap_addr);
      l += rs;
      // probabilities as the B operand: slab sl holds keys kmap(8 sl .. 8 sl + 7)
      v4u pb[2];
      pb[0] = make_v4u(pack2_bf16(p[0], p[1]), pack2_bf16(p[2], p[3]), pack2_bf16(p[4], p[5]), pack2_bf16(p[6], p[7]));
      pb[1] = make_v4u(pack2_bf16(p[8], p[9]), pack2_bf16(p[10], p[11]), pack2_bf16(p[12], p[13]), pack2_bf16(p[14], p[15]));
#pragma unroll
      for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
        for (int sl = 0; sl < 2; ++sl) o[dt] = mfma32a(vf[dt * 2 + sl], pb[sl], o[dt]);
      issue_v(w0, j + 1, wn);
    }
  }

  // ---- epilogue: the four waves hold four partial states of the same columns; merge in LDS
  __syncthreads();                                      // the query fragments are no longer read
  float *sm = (float *)lds_raw;                         // [4][32] m, [4][32] l, [32] merged m, [32] merged l
  float *so = sm + 320;                                 // [4][n_cols][SOLD]
  if (wave_rows) {
    // every wave holds the finished partial state of its own 32 columns: through LDS only to
    // turn lane-per-column registers into row-contiguous stores
    if (h == 0) {
      sm[wave * 32 + col] = m;
      sm[128 + wave * 32 + col] = l;
    }
    if (col_valid) {
      float *dst = so + (size_t)(wave * 32 + col) * SOLD + 4 * h;
#pragma unroll
      for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4)
          *(float4 *)(dst + dt * 32 + 8 * r4) = make_float4(o[dt][4 * r4], o[dt][4 * r4 + 1],
                                                            o[dt][4 * r4 + 2], o[dt][4 * r4 + 3]);
    }
    __syncthreads();
    const int row0 = (int)(blockIdx.x / it.prefix_stride) * 128;      // first query row of the item
#pragma unroll 4
    for (int i = 0; i < HD / 8; ++i) {                  // 128 columns x HD / 4 quads, 256 per round
      const int e = tid + 256 * i;
      const int cg = e / (HD / 4), d = (e % (HD / 4)) * 4;
      const int rc = row0 + cg;
      if (rc >= it.rows) continue;
      const float4 v = *(const float4 *)(so + (size_t)cg * SOLD + d);
      const int bc = rc / G, hq = kvh * G + rc % G;
      if (n_parts == 1) {
        const float lg = sm[128 + cg];
        const size_t at = a.out_tiled ? tiled_offset(bc, hq * HD + d, Hq * HD) : ((size_t)bc * Hq + hq) * HD + d;
        uint2 pk;
        pk.x = pack2_bf16(v.x / lg, v.y / lg);
        pk.y = pack2_bf16(v.z / lg, v.w / lg);
        *(uint2 *)((bf16_t *)a.out + at) = pk;
        continue;
      }
      const size_t row = ((size_t)part * B + bc) * Hq + hq;
      *(float4 *)(part_o + row * HD + d) = v;
      if (d == 0) *(float2 *)(part_ml + row * 2) = make_float2(sm[cg], sm[128 + cg]);
    }
    return;
  }
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
  if (wave == 0 && h == 0) {                            // the column's merged maximum and sum, once
    float lg = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float mw = sm[w * 32 + col];
      lg += (mw == -INFINITY) ? 0.f : sm[128 + w * 32 + col] * __builtin_amdgcn_exp2f(mw - mm);
    }
    sm[256 + col] = mm;
    sm[288 + col] = lg;
  }
  if (col_valid) {
    float *dst = so + (size_t)(wave * n_cols + col) * SOLD + 4 * h;
#pragma unroll
    for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4)
        *(float4 *)(dst + dt * 32 + 8 * r4) = make_float4(o[dt][4 * r4] * f, o[dt][4 * r4 + 1] * f,
                                                          o[dt][4 * r4 + 2] * f, o[dt][4 * r4 + 3] * f);
  }
  __syncthreads();
  const int wstride = n_cols * SOLD;
  // 32 columns x HD / 4 quads at most: a fixed number of rounds, so that the LDS reads of all of
  // them are in flight together
#pragma unroll
  for (int i = 0; i < HD / 32; ++i) {
    const int e = tid + 256 * i;
    if (e >= n_cols * (HD / 4)) continue;
    const int c = e / (HD / 4), d = (e % (HD / 4)) * 4;
    const float *p0 = so + c * SOLD + d;
    float4 v = *(const float4 *)p0;
#pragma unroll
    for (int w = 1; w < 4; ++w) {
      const float4 u = *(const float4 *)(p0 + w * wstride);
      v.x += u.x; v.y += u.y; v.z += u.z; v.w += u.w;
    }
    const int rc = col0 + c;
    const int bc = (b_item >= 0) ? b_item : rc / G;
    const int hq = kvh * G + rc % G;
    if (n_parts == 1) {
      // the only partial state of its (candidate, head): normalise and store the output here
      const float lg = sm[288 + c];
      const size_t at = a.out_tiled ? tiled_offset(bc, hq * HD + d, Hq * HD) : ((size_t)bc * Hq + hq) * HD + d;
      uint2 pk;
      pk.x = pack2_bf16(v.x / lg, v.y / lg);
      pk.y = pack2_bf16(v.z / lg, v.w / lg);
      *(uint2 *)((bf16_t *)a.out + at) = pk;
      continue;
    }
    const size_t row = ((size_t)part * B + bc) * Hq + hq;
    *(float4 *)(part_o + row * HD + d) = v;
    if (d == 0) *(float2 *)(part_ml + row * 2) = make_float2(sm[256 + c], sm[288 + c]);
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
  if (n_parts <= 16) {
    // few parts (the decode shapes up to a 4k prefix): every thread fetches all (m, l) pairs and
    // its own coordinate of every part in one batch of independent loads, one memory round trip
    // instead of three; same sums in the same order as below
    float2 ml[16];
    float v[16];
#pragma unroll
    for (int p = 0; p < 16; ++p) {
      ml[p] = make_float2(-INFINITY, 0.f);
      v[p] = 0.f;
      if (p < n_parts) {                           // uniform: the loads of the parts that exist go out back to back
        ml[p] = *(const float2 *)(part_ml + (p * stride + bh) * 2);
        v[p] = part_o[(p * stride + bh) * HD + d];
      }
    }
    float M = -INFINITY;
#pragma unroll
    for (int p = 0; p < 16; ++p)
      if (p < n_parts) M = fmaxf(M, ml[p].x);
    float den = 0.f, num = 0.f;
#pragma unroll
    for (int p = 0; p < 16; ++p)
      if (p < n_parts) {
        const float wgt = __builtin_amdgcn_exp2f(ml[p].x - M);
        den += wgt * ml[p].y;
        num += wgt * v[p];
      }
    const int b = bh / Hq, head = bh % Hq;
    const size_t at = out_tiled ? tiled_offset(b, head * HD + d, Hq * HD) : (size_t)bh * HD + d;
    out[at] = f32_to_bf16(num / den);
    return;
  }
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
  it.row_blocks = (it.rows + 31) / 32;
  it.n_prefix_blocks = (a.prefix_len + 31) / 32;
  it.n_suffix_blocks = (a.suffix_len + 31) / 32;
  // Blocks per wave: every wave (2048 run at once, 8 per CU) gets about an equal share of all
    // (block, 32 columns) pairs, and at least four blocks, because each item pays a fixed cost
    // (query fetch, merge, partial sums written and read again) that more, shorter items multiply.
  const long wave_blocks = (long)it.n_prefix_blocks * a.n_kv_heads * it.row_blocks +
                           (long)it.n_suffix_blocks * a.n_kv_heads * a.n_cands;
  const int per_wave = (int)std::max(4L, (wave_blocks + 2047) / 2048);
  int splits = 0;
  it.blocks_per_split = 0;
  if (it.n_prefix_blocks > 0) {
    const int max_splits = (it.n_prefix_blocks + 3) / 4;        // at least 128 keys per split
    splits = a.prefix_splits;
    if (splits <= 0) splits = (it.n_prefix_blocks + 4 * per_wave - 1) / (4 * per_wave);
    splits = std::max(1, std::min(splits, max_splits));
    it.blocks_per_split = (it.n_prefix_blocks + splits - 1) / splits;
    splits = (it.n_prefix_blocks + it.blocks_per_split - 1) / it.blocks_per_split;   // drop empty splits
  }
  // many row blocks: four per item (one per wave), and key splits for about 384 items
  it.rb_per_item = it.row_blocks >= 8 ? 4 : 1;
  const int rb_groups = (it.row_blocks + it.rb_per_item - 1) / it.rb_per_item;
  if (it.rb_per_item == 4 && it.n_prefix_blocks > 0) {
    const int max_splits = (it.n_prefix_blocks + 3) / 4;
    splits = a.prefix_splits > 0 ? a.prefix_splits : (384 + a.n_kv_heads * rb_groups - 1) / (a.n_kv_heads * rb_groups);
    // 16 partial states per row are what the merge kernel fetches in one batch: leave one to the suffix
    if (a.prefix_splits <= 0 && a.suffix_len > 0 && splits == 16) splits = 15;
    splits = std::max(1, std::min(splits, max_splits));
    it.blocks_per_split = (it.n_prefix_blocks + splits - 1) / splits;
    splits = (it.n_prefix_blocks + it.blocks_per_split - 1) / it.blocks_per_split;
  }
  it.splits = splits;
  it.prefix_groups = a.n_kv_heads * splits;
  it.prefix_stride = (it.prefix_groups + 7) / 8 * 8;
  it.n_prefix_items = (splits > 0) ? it.prefix_stride * rb_groups : 0;
  // suffix: the same share per wave
  int ssplits = 1;
  it.suffix_bps = 0;
  if (it.n_suffix_blocks > 0) {
    ssplits = (it.n_suffix_blocks + 4 * per_wave - 1) / (4 * per_wave);
    ssplits = std::max(1, std::min(std::min(ssplits, kMaxSuffixSplits), it.n_suffix_blocks));
    it.suffix_bps = (it.n_suffix_blocks + ssplits - 1) / ssplits;
    ssplits = (it.n_suffix_blocks + it.suffix_bps - 1) / it.suffix_bps;
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

// partials: every (part, candidate, head) holds hd + 2 floats; parts <= prefix blocks / 4 + suffix splits
size_t decode_attention_mfma_ws_bytes(int n_cands, int Hq, int Hkv, int hd, int prefix_len,
                                      int suffix_len, int page_tokens) {
  (void)Hkv; (void)suffix_len;
  if (page_tokens != PG) return 0;
  const size_t parts = (size_t)(((prefix_len + 31) / 32 + 3) / 4) + kMaxSuffixSplits;
  return parts * n_cands * Hq * (size_t)(hd + 2) * sizeof(float) + 512;
}

template <int HD>
static int launch_decode_attention_t(hipStream_t st, const DecodeAttnArgs &a, const AttnItems &it_in) {
  const int n_parts = (a.prefix_len > 0 ? it_in.splits : 0) + (a.suffix_len > 0 ? it_in.suffix_splits : 0);
  const size_t rows = (size_t)a.n_cands * a.n_q_heads;
  const size_t need = (size_t)n_parts * rows * (HD + 2) * sizeof(float);
  if (a.workspace_bytes < need) MC_FAIL(MC_ERR_INVALID, "attention workspace has %zu bytes, %zu needed", a.workspace_bytes, need);
  if (n_parts > 1024) MC_FAIL(MC_ERR_UNSUPPORTED, "decode attention: %d partial states exceed 1024", n_parts);
  float *part_o = (float *)a.workspace;
  float *part_ml = part_o + (size_t)n_parts * rows * HD;
  const int G = a.n_q_heads / a.n_kv_heads;
  // query fragments of four waves, later reused by the suffix items' merge
  const int max_cols = (a.prefix_len > 0) ? std::min(32, a.n_cands * G) : G;
  const size_t lds = std::max((size_t)4 * (HD / 16) * 1024, (size_t)(320 + 4 * max_cols * (HD + 4)) * sizeof(float));
  const AttnItems &it = it_in;
  MC_TRY(raise_dynamic_lds_limit((const void *)decode_attention_kernel<HD>, 160 * 1024 - 1024));
  // events offered by a profiling scope: begin of the first kernel, end of the last
  const LaunchEvents ev = take_launch_events();
  hipEvent_t stop1 = n_parts == 1 ? ev.stop : nullptr;
  if (ev.start || stop1)
    hipExtLaunchKernelGGL(decode_attention_kernel<HD>, dim3(it.n_prefix_items + it.n_suffix_items), dim3(256),
                          (uint32_t)lds, st, ev.start, stop1, 0, a, it, part_o, part_ml, n_parts);
  else
    decode_attention_kernel<HD><<<it.n_prefix_items + it.n_suffix_items, 256, lds, st>>>(a, it, part_o, part_ml, n_parts);
  MC_HIP(hipGetLastError());
  if (n_parts == 1) return MC_OK;          // every item finished its own outputs
  if (ev.stop)
    hipExtLaunchKernelGGL(decode_attention_merge_kernel<HD>, dim3((unsigned)rows), dim3(HD), 0, st, nullptr, ev.stop, 0,
                          n_parts, a.n_cands, a.n_q_heads, (const float *)part_o, (const float *)part_ml,
                          (bf16_t *)a.out, a.out_tiled);
  else
    decode_attention_merge_kernel<HD><<<(unsigned)rows, HD, 0, st>>>(
        n_parts, a.n_cands, a.n_q_heads, part_o, part_ml, (bf16_t *)a.out, a.out_tiled);
  MC_HIP(hipGetLastError());
  return MC_OK;
}

// The launch plan as numbers, for host-side checks: {prefix items (with padding ids), suffix
// items, prefix splits, blocks per prefix split, suffix splits, blocks per suffix split, partial
// states per (candidate, head), prefix id stride, row blocks per prefix item}.
int decode_attention_plan(const DecodeAttnArgs &a, int32_t out[9]) {
  if (!decode_attention_mfma_supported(a)) MC_FAIL(MC_ERR_UNSUPPORTED, "decode attention: shape not covered");
  const AttnItems it = plan_items(a);
  out[0] = it.n_prefix_items; out[1] = it.n_suffix_items; out[2] = it.splits; out[3] = it.blocks_per_split;
  out[4] = it.suffix_splits; out[5] = it.suffix_bps;
  out[6] = (a.prefix_len > 0 ? it.splits : 0) + (a.suffix_len > 0 ? it.suffix_splits : 0);
  out[7] = it.prefix_stride;
  out[8] = it.rb_per_item;
  return MC_OK;
}

int launch_attention_decode_mfma(hipStream_t st, const DecodeAttnArgs &a) {
  if (!decode_attention_mfma_supported(a)) MC_FAIL(MC_ERR_UNSUPPORTED, "decode attention: shape not covered");
  const AttnItems it = plan_items(a);
  if (it.n_prefix_items + it.n_suffix_items == 0) MC_FAIL(MC_ERR_INVALID, "decode attention without keys");
  return a.head_dim == 128 ? launch_decode_attention_t<128>(st, a, it) : launch_decode_attention_t<64>(st, a, it);
}

}  // namespace mc
