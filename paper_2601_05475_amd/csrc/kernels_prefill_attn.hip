// Causal attention for many query rows (prefix prefill and candidate scoring), bf16, gfx950 MFMA.
//
// A work item is up to 64 consecutive positions of one sequence, one KV head and up to four of
// its query heads.  The workgroup has 8 waves: wave w owns head 4 * hg + w % 4 of the group and
// positions 32 (w / 4) .. + 31 of the item, which are its MFMA columns.  Two waves per SIMD let
// one wave's softmax run under the other's MFMAs, and the LDS only reaches its full read rate
// with eight waves per CU.
// Keys are streamed page by page (64 keys) through LDS and shared by the four waves: first the
// shared-prefix pages that are visible to the block, then (scoring) the sequence's own suffix
// pages.  Pages are stored in MFMA fragment order, so a page is copied to LDS as it is (by
// loads that write LDS directly, two pages ahead, three buffers) and an operand is one
// conflict-free 16-byte read per lane.  Each item sees all keys of its rows, so
// it normalises and writes bf16 itself.  Operand mapping and the softmax scheme are those of
// the decode kernel (transposed scores, lazy base-2 reference maximum); the addition is the
// causal mask, applied only to blocks that reach past the first position of the item.
#include "kernels_mfma.h"

#include <algorithm>

namespace mc {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t v4u;
typedef __attribute__((ext_vector_type(2))) uint32_t v2u;

__device__ inline f32x16 mfma32p(v4u a, v4u b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
__device__ inline uint32_t pack2p_bf16(float a, float b) {
  typedef __attribute__((ext_vector_type(2))) float f32x2;
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, b}, bf16x2));
}

constexpr int PPG = 64;                       // keys per page

template <int HD> struct PTile {
  static constexpr int K_ELEMS = PPG * HD, V_ELEMS = PPG * HD, PAGE_ELEMS = K_ELEMS + V_ELEMS;
  static constexpr int NF = HD / 16;          // 1 KB fragments per 32-key block (K and V alike)
  static constexpr int LDS_BYTES = 3 * PAGE_ELEMS * 2;      // three page buffers
  static constexpr int CPT = PPG * HD / 8 / 512;
};

constexpr int kPrefillMaxPids = 1024;

template <int HD>
__global__ __launch_bounds__(512)
void prefill_attention_kernel(PrefillAttnArgs a) {
  using TL = PTile<HD>;
  extern __shared__ __attribute__((aligned(16))) unsigned char plds_raw[];
  bf16_t *lds = (bf16_t *)plds_raw;
  int *pids = (int *)(plds_raw + TL::LDS_BYTES);
  const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hw = wave & 3, half = wave >> 2;    // head within the group, half of the item's rows
  const int swap_addr = (lane ^ 32) << 2;       // ds_bpermute address of the lane with the other 16 keys
  const int Hq = a.n_q_heads, Hkv = a.n_kv_heads, G = Hq / Hkv, HG = (G + 3) / 4;

  int id = blockIdx.x;
  const int hg = id % HG; id /= HG;
  const int kvh = id % Hkv; id /= Hkv;
  const int4 item = a.items[id];               // row_start, n_rows (<= 64), pos_start, table row
  const int n_rows = item.y, tab = item.w;
  const int row_start = item.x + 32 * half;     // this wave's rows and their first position
  const int pos_start = item.z + 32 * half;
  const int my_rows = min(32, n_rows - 32 * half);
  const int g = 4 * hg + hw;
  const bool wave_active = g < G && my_rows > 0;   // uniform per wave
  const int head = kvh * G + (g < G ? g : 0);
  const bool col_valid = col < my_rows;
  const int my_pos = pos_start + (col_valid ? col : 0);
  const int my_last = pos_start + my_rows - 1;     // last position of this wave's rows

  // visible keys: prefix [0, nA), then own suffix [0, nB) at absolute positions prefix_len + j
  const int last_pos = item.z + n_rows - 1;        // of the whole item: pages every wave helps to stage
  const int nA = min(a.prefix_len, last_pos + 1);
  const int nB = (tab >= 0 && last_pos >= a.prefix_len) ? last_pos - a.prefix_len + 1 : 0;
  const int nPA = (nA + PPG - 1) / PPG, nPB = (nB + PPG - 1) / PPG, n_pages = nPA + nPB;
  const int32_t *table = (nPB > 0) ? a.page_table + (size_t)tab * a.table_stride : nullptr;
  const bool pids_in_lds = nPB <= kPrefillMaxPids;
  if (nPB > 0 && pids_in_lds) {
    for (int i = tid; i < nPB; i += 512) pids[i] = table[i];
    __syncthreads();
  }

  v4u qf[HD / 16];
  {
    // a wave without rows reads the item's first row (its result is never stored)
    const int qr = wave_active ? row_start + (col_valid ? col : 0) : item.x;
    const bf16_t *qrow = (const bf16_t *)a.q + ((size_t)qr * Hq + head) * HD + 8 * h;
#pragma unroll
    for (int c = 0; c < HD / 16; ++c) qf[c] = *(const v4u *)(qrow + 16 * c);
  }
  const float scale2 = 1.4426950408889634f / sqrtf((float)HD);
  f32x16 o[HD / 32];
#pragma unroll
  for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
  float m = -INFINITY, l = 0.f;

  const size_t page_stride = (size_t)Hkv * PPG * HD, head_off = (size_t)kvh * PPG * HD;
  const bf16_t *kA = (const bf16_t *)a.k_prefix, *vA = (const bf16_t *)a.v_prefix;
  const bf16_t *kB = (const bf16_t *)a.k_suffix, *vB = (const bf16_t *)a.v_suffix;
  // Pages go from global memory straight into LDS (lane i of a wave-wide 16-byte load lands at
  // the wave's base + 16 i: the page is copied as it is), two pages ahead of the one in use, into
  // three buffers.  The same number of loads is issued whether or not the page exists (a page
  // past the end re-reads 16 bytes of page 0 into a buffer nobody reads), so the wait before the
  // barrier can count: all but the newest page's loads have landed.
  auto issue = [&](int pi, int buf) __attribute__((always_inline)) {
    const bool real = pi < n_pages;
    const int p = real ? pi : 0;
    const bool in_a = p < nPA;
    const int page = in_a ? p : (pids_in_lds ? pids[p - nPA] : table[p - nPA]);
    const bf16_t *kp = (in_a ? kA : kB) + (size_t)page * page_stride + head_off;
    const bf16_t *vp = (in_a ? vA : vB) + (size_t)page * page_stride + head_off;
    const size_t lane_off = real ? (size_t)tid * 8 : 0, step = real ? 512 * 8 : 0;
    bf16_t *kt = lds + buf * TL::PAGE_ELEMS + wave * 512, *vt = kt + TL::K_ELEMS;
#pragma unroll
    for (int i = 0; i < TL::CPT; ++i) {
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(kp + lane_off + step * i),
                                       (__attribute__((address_space(3))) void *)(kt + 4096 * i), 16, 0, 0);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(vp + lane_off + step * i),
                                       (__attribute__((address_space(3))) void *)(vt + 4096 * i), 16, 0, 0);
    }
  };
  // one 32-key block whose key 0 sits at absolute position abs0; n_valid keys exist
  auto process = [&](int buf, int blk, int n_valid, int abs0) __attribute__((always_inline)) {
    const bf16_t *kt = lds + buf * TL::PAGE_ELEMS, *vt = kt + TL::K_ELEMS;
    const bf16_t *kblk = kt + (blk * TL::NF * 64 + lane) * 8, *vblk = vt + (blk * TL::NF * 64 + lane) * 8;
    f32x16 s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int c = 0; c < HD / 16; ++c) {
      const v4u kf = *(const v4u *)(kblk + c * 512);
      s = mfma32p(kf, qf[c], s);
    }
    // key of register r: 8 (r / 4) + 4 h + r % 4; it is masked if it does not exist or lies
    // after this lane's query position
    if (n_valid < 32 || abs0 + 31 > pos_start) {
      const int lim = min(n_valid, my_pos - abs0 + 1);      // keys [0, lim) are visible
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (8 * (r >> 2) + 4 * h + (r & 3) >= lim) s[r] = -INFINITY;
    }
    // Probabilities against the reference m as it stands (see the decode kernel: any reference
    // gives the same normalised result, it only has to keep the numbers in range).  Only if a
    // lane's sum leaves the range - a score far above the reference, or no reference yet (m =
    // -inf yields inf or NaN) - the block's maximum is taken, the reference moved and the
    // accumulators rescaled; the common case spends no instruction on maxima.
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
      const float m_new = fmaxf(m, mx * scale2);    // stays -inf for a column that has seen no key
      const float corr = (m_new == -INFINITY) ? 1.0f : __builtin_amdgcn_exp2f(m - m_new);
      l *= corr;
      m = m_new;
#pragma unroll
      for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] *= corr;
      // a column with no visible key so far: 0 as reference, all its p are 0
      const float mref = (m == -INFINITY) ? 0.f : m;
      rs = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        p[r] = __builtin_amdgcn_exp2f(fmaf(s[r], scale2, -mref));
        rs += p[r];
      }
    }
    rs += swap_halves(rs, swap_addr);
    l += rs;
    v4u pb[2];
    pb[0] = v4u{pack2p_bf16(p[0], p[1]), pack2p_bf16(p[2], p[3]), pack2p_bf16(p[4], p[5]), pack2p_bf16(p[6], p[7])};
    pb[1] = v4u{pack2p_bf16(p[8], p[9]), pack2p_bf16(p[10], p[11]), pack2p_bf16(p[12], p[13]), pack2p_bf16(p[14], p[15])};
#pragma unroll
    for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
      for (int sl = 0; sl < 2; ++sl) {
        const v4u vf = *(const v4u *)(vblk + (dt * 2 + sl) * 512);
        o[dt] = mfma32p(vf, pb[sl], o[dt]);
      }
  };
  auto consume = [&](int pi, int buf) __attribute__((always_inline)) {
    if (!wave_active) return;
    const bool in_a = pi < nPA;
    const int abs_page = in_a ? pi * PPG : a.prefix_len + (pi - nPA) * PPG;
    const int keys_here = in_a ? min(PPG, nA - pi * PPG) : min(PPG, nB - (pi - nPA) * PPG);
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
      const int nv = min(32, keys_here - 32 * blk);
      if (nv > 0 && abs_page + 32 * blk <= my_last) process(buf, blk, nv, abs_page + 32 * blk);   // else all masked
    }
  };

  issue(0, 0);
  issue(1, 1);
  int buf = 0;
  for (int pi = 0; pi < n_pages; ++pi) {
    // page pi has landed once at most the loads of page pi + 1 are outstanding
    if (TL::CPT == 2) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
    __syncthreads();                             // ... for every wave; and page pi - 1 is no longer read
    issue(pi + 2, buf >= 1 ? buf - 1 : 2);       // into page pi - 1's buffer, (buf + 2) % 3
    consume(pi, buf);
    buf = buf == 2 ? 0 : buf + 1;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // no load into LDS outlives the workgroup

  if (wave_active && col_valid) {
    const float inv = 1.0f / l;                  // l > 0: every row sees at least its own key
    bf16_t *out = (bf16_t *)a.out;
    const int row = row_start + col;
#pragma unroll
    for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int d = dt * 32 + 8 * r4 + 4 * h;
        const size_t at = a.out_tiled ? tiled_offset(row, head * HD + d, Hq * HD)
                                      : ((size_t)row * Hq + head) * HD + d;
        v2u pk = {pack2p_bf16(o[dt][4 * r4] * inv, o[dt][4 * r4 + 1] * inv),
                  pack2p_bf16(o[dt][4 * r4 + 2] * inv, o[dt][4 * r4 + 3] * inv)};
        *(v2u *)(out + at) = pk;
      }
  }
}

bool prefill_attention_mfma_supported(int page_tokens, int head_dim, int Hq, int Hkv) {
  return page_tokens == PPG && (head_dim == 64 || head_dim == 128) && Hq % Hkv == 0;
}

template <int HD>
static int launch_prefill_t(hipStream_t st, const PrefillAttnArgs &a) {
  using TL = PTile<HD>;
  const int G = a.n_q_heads / a.n_kv_heads, HG = (G + 3) / 4;
  const size_t lds = TL::LDS_BYTES + kPrefillMaxPids * sizeof(int);
  MC_TRY(raise_dynamic_lds_limit((const void *)prefill_attention_kernel<HD>, 160 * 1024 - 1024));
  const unsigned grid = (unsigned)a.n_items * a.n_kv_heads * HG;
  prefill_attention_kernel<HD><<<grid, 512, lds, st>>>(a);
  MC_HIP(hipGetLastError());
  return MC_OK;
}

int launch_attention_prefill_mfma(hipStream_t st, const PrefillAttnArgs &a) {
  if (a.n_items <= 0) return MC_OK;
  if (!prefill_attention_mfma_supported(a.page_tokens, a.head_dim, a.n_q_heads, a.n_kv_heads))
    MC_FAIL(MC_ERR_UNSUPPORTED, "prefill attention: shape not covered");
  return a.head_dim == 128 ? launch_prefill_t<128>(st, a) : launch_prefill_t<64>(st, a);
}

}  // namespace mc
