// bf16 MFMA kernels for gfx950 (wave64, v_mfma_f32_32x32x16_bf16).
//
// Operand layout of the 32x32x16 instruction, D[32][32] += A[32][16] * B[16][32], as used here:
//   A: lane l holds row (l % 32), contraction slots 8*(l / 32) .. +7   (8 bf16 = 16 bytes)
//   B: lane l holds column (l % 32), the same contraction slots
//   D: lane l holds column (l % 32); register r holds row 8*(r / 4) + 4*(l / 32) + (r % 4)
// Only the pairing of A and B slots matters for a dot product, so kernels are free to map a slot
// to any element of the contracted axis as long as both operands use the same map.
//
// Tiled operand layout ("tiled" below).  A [rows][K] bf16 matrix, rows % 32 == 0 and K % 64 == 0,
// is stored as 4 KB blocks, block (row tile rt, unit u) at ((rt * K/64 + u) * 4096) bytes, and
// inside a block chunk c (0..3) of lane l (0..63) at (c * 64 + l) * 16 bytes holds
//   M[32 rt + l % 32][64 u + 32 (l / 32) + 8 c + 0..7].
// One wave-wide 16-byte load of chunk c therefore reads 1 KB of contiguous memory and lands
// directly in the A (or B) operand registers of four consecutive MFMA steps.
#include "kernels_mfma.h"

#include <hip/hip_ext.h>

#include <algorithm>

namespace mc {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
// 16-byte register quantity as a native vector: arrays of it are promoted to registers (arrays
// of the runtime's struct-based uint4 that are updated under a condition end up in scratch)
typedef __attribute__((ext_vector_type(4))) uint32_t v4u;
__device__ inline v4u make_v4u(uint32_t a, uint32_t b, uint32_t c, uint32_t d) { return v4u{a, b, c, d}; }

__device__ inline f32x16 mfma32(v4u a, v4u b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

__device__ inline float silu_f(float g) { return g / (1.0f + expf(-g)); }

__device__ inline uint2 pack4_bf16(float a, float b, float c, float d) {
  uint2 r;
  r.x = (uint32_t)f32_to_bf16(a) | ((uint32_t)f32_to_bf16(b) << 16);
  r.y = (uint32_t)f32_to_bf16(c) | ((uint32_t)f32_to_bf16(d) << 16);
  return r;
}

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
// streaming 16-byte load: the data is used once, keep it out of the way of reusable lines
__device__ inline v4u load_stream(const bf16_t *p) {
  const u32x4 v = __builtin_nontemporal_load((const u32x4 *)p);
  return make_v4u(v[0], v[1], v[2], v[3]);
}

// ---- row-major -> tiled repack (one thread per 16-byte chunk of the destination) -----------
__global__ void pack_tiled_kernel(int rows, int rows_pad, int K, const bf16_t *__restrict__ src,
                                  bf16_t *__restrict__ dst, int interleave_hd) {
  const size_t chunk = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t total = (size_t)rows_pad * K / 8;
  if (chunk >= total) return;
  const int lane = chunk & 63, c = (chunk >> 6) & 3;
  const size_t blk = chunk >> 8;
  const int U = K >> 6;
  const int rt = (int)(blk / U), u = (int)(blk % U);
  const int row = 32 * rt + (lane & 31), k = 64 * u + 32 * (lane >> 5) + 8 * c;
  int srow = row;
  if (interleave_hd > 0) {                      // destination row 2i <- i, 2i + 1 <- i + hd / 2
    const int jp = row % interleave_hd;
    srow = row - jp + (jp >> 1) + ((jp & 1) ? interleave_hd / 2 : 0);
  }
  v4u v = make_v4u(0, 0, 0, 0);
  if (row < rows) v = *(const v4u *)(src + (size_t)srow * K + k);
  *(v4u *)(dst + chunk * 8) = v;
}

int launch_pack_tiled(hipStream_t st, int rows, int K, const void *src, void *dst, int interleave_hd) {
  if (rows <= 0) return MC_OK;
  if (K % 64) MC_FAIL(MC_ERR_UNSUPPORTED, "tiled layout needs K %% 64 == 0 (K = %d)", K);
  if (interleave_hd < 0 || (interleave_hd > 0 && (interleave_hd % 2 || rows % interleave_hd)))
    MC_FAIL(MC_ERR_INVALID, "row interleave of %d does not fit %d rows", interleave_hd, rows);
  const int rows_pad = (rows + 31) / 32 * 32;
  const size_t chunks = (size_t)rows_pad * K / 8;
  pack_tiled_kernel<<<(unsigned)((chunks + 255) / 256), 256, 0, st>>>(rows, rows_pad, K, (const bf16_t *)src, (bf16_t *)dst, interleave_hd);
  MC_HIP(hipGetLastError());
  return MC_OK;
}

// ---- streaming-read probe: what a kernel that only reads (16-byte non-temporal loads, eight in
// flight per thread, one contiguous range per workgroup) gets out of HBM
__global__ __launch_bounds__(256) void read_probe_kernel(const u32x4 *__restrict__ p, size_t per_wg,
                                                         uint32_t *__restrict__ out) {
  const u32x4 *q = p + (size_t)blockIdx.x * per_wg + threadIdx.x;
  u32x4 acc = {0, 0, 0, 0};
  for (size_t i = 0; i < per_wg; i += 256 * 8) {
    u32x4 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = __builtin_nontemporal_load(q + i + j * 256);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc ^= v[j];
  }
  if (acc[0] == 0x12345678u && acc[1] == 0x9abcdef0u) out[0] = acc[2];      // keeps the loads alive
}

int launch_read_probe(hipStream_t st, const void *buf, size_t bytes, uint32_t *out) {
  const int n_wg = 2048;
  const size_t per_wg = bytes / 16 / n_wg;
  if (per_wg == 0 || per_wg % 2048) MC_FAIL(MC_ERR_INVALID, "read probe: bytes must be a positive multiple of %d", 2048 * 2048 * 16);
  read_probe_kernel<<<n_wg, 256, 0, st>>>((const u32x4 *)buf, per_wg, out);
  MC_HIP(hipGetLastError());
  return MC_OK;
}

// =====================================================================================
// Few-row linear layer on tiled operands: weights streamed once from HBM straight into MFMA
// operands.  A workgroup owns one 32-row weight tile; its 4 waves take 4 slices of the K range
// and meet in LDS.  Loads run two units (2 x 4 KB per operand) ahead of the MFMAs.
// MB = number of 32-row tiles of the activations (M <= 32 MB).
// =====================================================================================
// ROPE (the fused QKV layer, one K split): instead of storing the sums, rotate the query / key
// coordinates by the row's position and write queries (bf16, row-major), keys and values (into
// their page slots).  The weight rows of every query / key head are interleaved so that the two
// members of a rotary pair are neighbours in a thread's four consecutive outputs.
// PAIR (plain sums, one K split, an even number of weight tiles; used where the tiles outnumber
// the CUs many times: the LM head): every WAVE takes its own pair of weight tiles (w2 = the second
// one) over the whole K range, so an activation fragment serves two weight tiles, the four waves
// of a workgroup fetch the same activation units at about the same time (L1), and there is
// nothing to reduce across waves: each wave stores its own 64 output columns.
// Sorted list of the kTopPerGroup best (value, id) pairs under the order (value descending, id
// ascending), kept in registers.  insert() takes `first` = "the new pair ranks before entry s".
struct Top4 {
  float v[kTopPerGroup];
  int id[kTopPerGroup];
  __device__ inline void clear() {
#pragma unroll
    for (int s = 0; s < kTopPerGroup; ++s) { v[s] = -INFINITY; id[s] = 0x7FFFFFFF; }
  }
  template <typename Before>
  __device__ inline void insert(float x, int xi, Before before) {
    bool c[kTopPerGroup];
#pragma unroll
    for (int s = 0; s < kTopPerGroup; ++s) c[s] = before(x, xi, v[s], id[s]);      // c[s] implies c[s + 1]
#pragma unroll
    for (int s = kTopPerGroup - 1; s > 0; --s) {
      v[s] = c[s - 1] ? v[s - 1] : (c[s] ? x : v[s]);
      id[s] = c[s - 1] ? id[s - 1] : (c[s] ? xi : id[s]);
    }
    v[0] = c[0] ? x : v[0];
    id[0] = c[0] ? xi : id[0];
  }
};

enum { SKINNY_PLAIN = 0, SKINNY_SWIGLU = 1, SKINNY_PAIR = 2 };
template <int MB, int MODE, bool ROPE>
__global__ __launch_bounds__(256) void skinny_linear_kernel(
    int M, int N, int K, int units_per_wave, const bf16_t *__restrict__ a,
    const bf16_t *__restrict__ w, const bf16_t *__restrict__ w2, float *__restrict__ out,
    bf16_t *__restrict__ out_t, RopeOut ro, uint2 *__restrict__ top_out) {
  constexpr bool SWIGLU = MODE == SKINNY_SWIGLU, PAIR = MODE == SKINNY_PAIR;
  constexpr int NW = MODE != SKINNY_PLAIN ? 2 : 1;
  __shared__ float4 red[4][NW][MB][4][64];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, nl = lane & 31, h = lane >> 5;
  // PAIR: the grid is rounded up to a multiple of 8 and every XCD (workgroups are dealt to them
  // round-robin) takes a contiguous range of tile pairs, so that the pieces its workgroups write
  // into a row of the output sit next to each other in one L2
  int rt = blockIdx.x;
  if (PAIR) {
    const int per_xcd = gridDim.x >> 3;
    rt = 4 * ((int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3)) + wave;   // this wave's tile pair
    if (rt >= N / 64) return;                                 // no barrier on this path
  }
  const int split = blockIdx.y;
  const int U = K >> 6;
  const int u0 = PAIR ? 0 : (split * 4 + wave) * units_per_wave;
  const int wt = PAIR ? 2 * rt : rt;                          // weight tile of w (and of w2)
  const bf16_t *wp = w + ((size_t)wt * U + u0) * 2048 + lane * 8;
  const bf16_t *up = NW == 2 ? w2 + ((size_t)wt * U + u0) * 2048 + lane * 8 : nullptr;
  const bf16_t *ap = a + (size_t)u0 * 2048 + lane * 8;      // activation tile mb adds mb * U * 2048
  f32x16 acc[NW][MB];
#pragma unroll
  for (int i = 0; i < NW; ++i)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][mb][r] = 0.f;

  v4u wf[2][4], uf[2][4], af[2][MB][4];
  auto issue = [&](int slot, int u) __attribute__((always_inline)) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      wf[slot][c] = load_stream(wp + (size_t)u * 2048 + c * 512);
      if (NW == 2) uf[slot][c] = load_stream(up + (size_t)u * 2048 + c * 512);
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
        af[slot][mb][c] = *(const v4u *)(ap + ((size_t)mb * U + u) * 2048 + c * 512);
    }
  };
  auto compute = [&](int slot) __attribute__((always_inline)) {
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        acc[0][mb] = mfma32(wf[slot][c], af[slot][mb][c], acc[0][mb]);
        if (NW == 2) acc[NW - 1][mb] = mfma32(uf[slot][c], af[slot][mb][c], acc[NW - 1][mb]);
      }
  };
  issue(0, 0);
  int u = 0;
  for (; u + 2 <= units_per_wave; u += 2) {
    issue(1, u + 1);
    compute(0);
    if (u + 2 < units_per_wave) issue(0, u + 2);
    compute(1);
  }
  if (u < units_per_wave) compute(0);

  if (PAIR) {
    // the wave's own sums: lane (nl, h) holds row nl of the tile and, per register quad r4,
    // columns 8 r4 + 4 h .. + 3
#pragma unroll
    for (int i = 0; i < NW; ++i)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        const int m = mb * 32 + nl;
        if (m >= M) continue;
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4)
          *(float4 *)(out + (size_t)m * N + 32 * (wt + i) + 8 * r4 + 4 * h) =
              make_float4(acc[i][mb][4 * r4], acc[i][mb][4 * r4 + 1], acc[i][mb][4 * r4 + 2], acc[i][mb][4 * r4 + 3]);
      }
    if (!top_out) return;
    // The LM head's share of sampling: the kTopPerGroup largest of this wave's 64 outputs of every
    // row, under (value descending, id ascending), so that the sampler reads 2004 short lists
    // instead of 128256 logits per row.  A lane walks its 32 outputs in ascending id (a later equal
    // value never displaces an earlier one), then the two half-waves merge their lists.
    const int swap_addr = (lane ^ 32) << 2;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      Top4 t;
      t.clear();
#pragma unroll
      for (int i = 0; i < NW; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          t.insert(acc[i][mb][r] + 0.0f, 32 * (wt + i) + 8 * (r >> 2) + 4 * h + (r & 3),
                   [](float x, int, float y, int) { return x > y; });
      float pv[kTopPerGroup];
      int pi[kTopPerGroup];
#pragma unroll
      for (int s = 0; s < kTopPerGroup; ++s) {
        pv[s] = swap_halves(t.v[s], swap_addr);
        pi[s] = __builtin_amdgcn_ds_bpermute(swap_addr, t.id[s]);
      }
#pragma unroll
      for (int s = 0; s < kTopPerGroup; ++s)
        t.insert(pv[s], pi[s], [](float x, int xi, float y, int yi) { return x > y || (x == y && xi < yi); });
      const int m = mb * 32 + nl;
      if (h == 0 && m < M) {
        uint2 *dst = top_out + ((size_t)m * (N / 64) + rt) * kTopPerGroup;
#pragma unroll
        for (int s = 0; s < kTopPerGroup; s += 2)
          *(uint4 *)(dst + s) = make_uint4(__float_as_uint(t.v[s]), (uint32_t)t.id[s], __float_as_uint(t.v[s + 1]), (uint32_t)t.id[s + 1]);
      }
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < NW; ++i)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4)
        red[wave][i][mb][r4][lane] = make_float4(acc[i][mb][4 * r4], acc[i][mb][4 * r4 + 1],
                                                 acc[i][mb][4 * r4 + 2], acc[i][mb][4 * r4 + 3]);
  __syncthreads();
  // thread (r4 = wave, lane) adds the four waves' quads in a fixed order and stores 4 outputs
  const int r4 = wave;
  const int n = 32 * wt + 8 * r4 + 4 * h;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    const int m = mb * 32 + nl;
    float4 s[NW];
#pragma unroll
    for (int i = 0; i < NW; ++i) {
      s[i] = red[0][i][mb][r4][lane];
#pragma unroll
      for (int sw = 1; sw < 4; ++sw) {
        const float4 t = red[sw][i][mb][r4][lane];
        s[i].x += t.x; s[i].y += t.y; s[i].z += t.z; s[i].w += t.w;
      }
    }
    if (m < M) {
      if (SWIGLU) {
        // the product feeds the next linear layer: store it tiled, as a [*][N] activation
        *(uint2 *)(out_t + tiled_offset(m, n, N)) =
            pack4_bf16(silu_f(s[0].x) * s[NW - 1].x, silu_f(s[0].y) * s[NW - 1].y,
                       silu_f(s[0].z) * s[NW - 1].z, silu_f(s[0].w) * s[NW - 1].w);
      } else if (ROPE) {
        rope_store_quad(ro, m, n, s[0], rope_load_quad(ro, m, n));
      } else {
        *(float4 *)(out + ((size_t)split * M + m) * N + n) = s[0];
      }
    }
  }
}

// =====================================================================================
// The one-split fused layers (gate/up + SwiGLU, QKV + rotary) in row-range form, for up to 32
// activation rows.  With one workgroup per 32-row weight tile the 8B gate/up layer has 448
// workgroups for 256 compute units: 192 units hold two and 64 hold one, and since a unit pulls
// no more than its share of the HBM rate the layer takes as long as the units with two (measured:
// the others idle from 22 us on, the layer ends at 40 us); the QKV layer has 192 workgroups and
// leaves 64 units empty.  Here every one of gridDim.x workgroups takes the same number of weight
// rows, R = N / gridDim.x (a multiple of 8: an output quad group of the MFMA layout), over the
// whole K range, wherever they fall in the 32-row tiles.  The MFMA does not care which weight rows
// sit in its operand (result row i depends on operand row i only), so a workgroup treats its
// range as NB blocks of 32 consecutive rows: lane (row nl, half h) of block b fetches row
// r0 + 32 b + nl from whatever tile holds it; lanes past the range read its last row (a valid
// address, no bytes fetched for a neighbour's rows) and their results are never stored.  The
// four waves split K and meet in LDS as in the form above.
// =====================================================================================
template <int NB, int MODE, bool ROPE>
__global__ __launch_bounds__(256) void skinny_rows_kernel(
    int M, int N, int K, int rows_per_wg, const bf16_t *__restrict__ a, const bf16_t *__restrict__ w,
    const bf16_t *__restrict__ w2, bf16_t *__restrict__ out_t, RopeOut ro) {
  constexpr bool SWIGLU = MODE == SKINNY_SWIGLU;
  constexpr int NW = SWIGLU ? 2 : 1;
  extern __shared__ float4 red_rows[];                        // [4 waves][NB][NW][4 quads][64 lanes]
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, nl = lane & 31, h = lane >> 5;
  const int r0 = blockIdx.x * rows_per_wg, r1 = r0 + rows_per_wg;
  const int U = K >> 6, units_per_wave = U >> 2, u0 = wave * units_per_wave;
  const bf16_t *wp[NB], *up[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b) {
    const int row = min(r0 + 32 * b + nl, r1 - 1);
    const size_t off = ((size_t)(row >> 5) * U + u0) * 2048 + (size_t)(32 * h + (row & 31)) * 8;
    wp[b] = w + off;
    up[b] = NW == 2 ? w2 + off : nullptr;
  }
  const bf16_t *ap = a + (size_t)u0 * 2048 + lane * 8;
  f32x16 acc[NB][NW];
#pragma unroll
  for (int b = 0; b < NB; ++b)
#pragma unroll
    for (int i = 0; i < NW; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[b][i][r] = 0.f;

  v4u wf[2][NB][4], uf[2][NB][4], af[2][4];
  auto issue = [&](int slot, int u) __attribute__((always_inline)) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        wf[slot][b][c] = load_stream(wp[b] + (size_t)u * 2048 + c * 512);
        if (NW == 2) uf[slot][b][c] = load_stream(up[b] + (size_t)u * 2048 + c * 512);
      }
      af[slot][c] = *(const v4u *)(ap + (size_t)u * 2048 + c * 512);
    }
  };
  auto compute = [&](int slot) __attribute__((always_inline)) {
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        acc[b][0] = mfma32(wf[slot][b][c], af[slot][c], acc[b][0]);
        if (NW == 2) acc[b][NW - 1] = mfma32(uf[slot][b][c], af[slot][c], acc[b][NW - 1]);
      }
  };
  issue(0, 0);
  int u = 0;
  for (; u + 2 <= units_per_wave; u += 2) {
    issue(1, u + 1);
    compute(0);
    if (u + 2 < units_per_wave) issue(0, u + 2);
    compute(1);
  }
  if (u < units_per_wave) compute(0);

#pragma unroll
  for (int b = 0; b < NB; ++b)
#pragma unroll
    for (int i = 0; i < NW; ++i)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4)
        red_rows[((((wave * NB + b) * NW + i) * 4 + r4) << 6) + lane] =
            make_float4(acc[b][i][4 * r4], acc[b][i][4 * r4 + 1], acc[b][i][4 * r4 + 2], acc[b][i][4 * r4 + 3]);
  __syncthreads();
  // thread (r4 = wave, lane) adds the four waves' quads of every block in a fixed order and
  // stores the 4 outputs of activation row m = nl if their weight rows lie in the range
  const int r4 = wave, m = nl;
#pragma unroll
  for (int b = 0; b < NB; ++b) {
    const int n = r0 + 32 * b + 8 * r4 + 4 * h;
    if (n >= r1 || m >= M) continue;
    float4 s[NW];
#pragma unroll
    for (int i = 0; i < NW; ++i) {
      s[i] = red_rows[((((0 * NB + b) * NW + i) * 4 + r4) << 6) + lane];
#pragma unroll
      for (int sw = 1; sw < 4; ++sw) {
        const float4 t = red_rows[((((sw * NB + b) * NW + i) * 4 + r4) << 6) + lane];
        s[i].x += t.x; s[i].y += t.y; s[i].z += t.z; s[i].w += t.w;
      }
    }
    if (SWIGLU) {
      *(uint2 *)(out_t + tiled_offset(m, n, N)) =
          pack4_bf16(silu_f(s[0].x) * s[NW - 1].x, silu_f(s[0].y) * s[NW - 1].y,
                     silu_f(s[0].z) * s[NW - 1].z, silu_f(s[0].w) * s[NW - 1].w);
    } else if (ROPE) {
      rope_store_quad(ro, m, n, s[0], rope_load_quad(ro, m, n));
    }
  }
}

// =====================================================================================
// The same layer for 33..64 rows (two 32-row activation tiles).  In the form above every wave
// fetches its own activation units, and with two tiles per weight tile that is as many bytes
// from L2 as the weights bring from HBM (twice as many in the plain form), all of them addressed
// to the same few hundred kilobytes: the layer then runs at 3-5 TB/s.  Here the four waves of a
// workgroup take four different weight tiles over one common K range and share the activation
// units through LDS (staged four units at a time, two buffers, one barrier per four units), so
// the activations cross the L2-to-CU path once per workgroup instead of once per wave, and each
// wave ends with complete sums for its tile: nothing to reduce across waves.  Weights stream
// straight into MFMA operand registers, four units per wave in flight (a unit's registers are
// refilled as soon as its MFMAs have been issued).  K splits are separate workgroups
// (gridDim.y), each writing its own fp32 partial.
// =====================================================================================
template <bool SWIGLU>
__global__ __launch_bounds__(256) void skinny_shared_kernel(
    int M, int N, int K, int units_per_split, const bf16_t *__restrict__ a,
    const bf16_t *__restrict__ w, const bf16_t *__restrict__ w2, float *__restrict__ out,
    bf16_t *__restrict__ out_t) {
  constexpr int MB = 2, NW = SWIGLU ? 2 : 1, CH = 4;
  __shared__ v4u act[2][CH][MB][256];                         // 64 KB
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, nl = lane & 31, h = lane >> 5;
  const int tiles = N >> 5, U = K >> 6;
  // every XCD (workgroups are dealt to them round-robin) takes a contiguous range of tile groups
  const int per_xcd = gridDim.x >> 3;
  const int wt_raw = 4 * ((int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3)) + wave;
  const bool live = wt_raw < tiles;                           // a wave past the last tile only helps staging
  const int wt = live ? wt_raw : tiles - 1;
  const int split = blockIdx.y, u0 = split * units_per_split, n_chunks = units_per_split / CH;
  const bf16_t *wp = w + ((size_t)wt * U + u0) * 2048 + lane * 8;
  const bf16_t *up = SWIGLU ? w2 + ((size_t)wt * U + u0) * 2048 + lane * 8 : nullptr;
  const bf16_t *ap = a + (size_t)u0 * 2048 + tid * 8;         // tile mb, unit u: + (mb * U + u) * 2048
  f32x16 acc[NW][MB];
#pragma unroll
  for (int i = 0; i < NW; ++i)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][mb][r] = 0.f;

  v4u stg[CH][MB], wf[CH][4], uf[CH][4];
  auto load_act = [&](int chunk) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < CH; ++j)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
        stg[j][mb] = *(const v4u *)(ap + ((size_t)mb * U + chunk * CH + j) * 2048);
  };
  auto store_act = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < CH; ++j)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) act[buf][j][mb][tid] = stg[j][mb];
  };
  auto issue_w = [&](int j, int u) __attribute__((always_inline)) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      wf[j][c] = load_stream(wp + (size_t)u * 2048 + c * 512);
      if (SWIGLU) uf[j][c] = load_stream(up + (size_t)u * 2048 + c * 512);
    }
  };
  load_act(0);
#pragma unroll
  for (int j = 0; j < CH; ++j) issue_w(j, j);
  store_act(0);
  if (n_chunks > 1) load_act(1);
  __syncthreads();
  for (int i = 0; i < n_chunks; ++i) {
    const int buf = i & 1;
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      v4u af[MB][4];
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int c = 0; c < 4; ++c) af[mb][c] = act[buf][j][mb][c * 64 + lane];
#pragma unroll
      for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
          acc[0][mb] = mfma32(wf[j][c], af[mb][c], acc[0][mb]);
          if (SWIGLU) acc[NW - 1][mb] = mfma32(uf[j][c], af[mb][c], acc[NW - 1][mb]);
        }
      if (i + 1 < n_chunks) issue_w(j, (i + 1) * CH + j);
    }
    // the other buffer was last read during chunk i - 1, which every wave left before the barrier
    // that ended it
    if (i + 1 < n_chunks) {
      store_act(buf ^ 1);
      if (i + 2 < n_chunks) load_act(i + 2);
    }
    __syncthreads();
  }
  if (!live) return;
  // the wave's own sums: lane (nl, h) holds row nl of each activation tile and, per register
  // quad r4, columns 8 r4 + 4 h .. + 3 of the weight tile
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    const int m = mb * 32 + nl;
    if (m >= M) continue;
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      const int n = 32 * wt + 8 * r4 + 4 * h;
      const f32x16 &g = acc[0][mb];
      if (SWIGLU) {
        const f32x16 &v = acc[NW - 1][mb];
        *(uint2 *)(out_t + tiled_offset(m, n, N)) =
            pack4_bf16(silu_f(g[4 * r4]) * v[4 * r4], silu_f(g[4 * r4 + 1]) * v[4 * r4 + 1],
                       silu_f(g[4 * r4 + 2]) * v[4 * r4 + 2], silu_f(g[4 * r4 + 3]) * v[4 * r4 + 3]);
      } else {
        *(float4 *)(out + ((size_t)split * M + m) * N + n) =
            make_float4(g[4 * r4], g[4 * r4 + 1], g[4 * r4 + 2], g[4 * r4 + 3]);
      }
    }
  }
}

bool skinny_linear_supported(int M, int N, int K) {
  return M >= 1 && M <= 64 && N % 32 == 0 && K % 256 == 0;
}

// Two activation tiles: the shared-activation form, if its workgroups (four weight tiles each)
// can fill the chip; fewer of them leave CUs idle and the one-tile-per-workgroup form is faster
// (measured at 112 workgroups: 57 against 45 us).
static bool skinny_shared_form(int M, int N, int n_splits, bool rope) {
  return M > 32 && !rope && (N / 32 + 3) / 4 * n_splits >= 160;
}

int skinny_linear_splits(int M, int N, int K) {
  const int tiles = N / 32, units = K / 64;
  if (M > 32) {
    // any divisor of units / 4 will do there
    const int groups = (tiles + 3) / 4;
    int best = 1;
    for (int s = 1; s <= 16; ++s) {
      if (units % (4 * s)) continue;
      best = s;
      if (groups * s >= 192) break;
    }
    if (skinny_shared_form(M, N, best, false)) return best;
  }
  int best = 1;
  for (int s = 1; s <= 16; s *= 2) {
    if (units % (4 * s)) break;
    best = s;
    if (tiles * s >= 192) break;      // measured: more splits only add partial sums to write and re-read
  }
  return best;
}

// many more tiles than CUs, plain sums: every wave takes a pair of weight tiles (SKINNY_PAIR)
static bool skinny_pair_form(int N, int n_splits, bool rope, bool swiglu) {
  return !rope && !swiglu && n_splits == 1 && (N / 32) % 2 == 0 && N / 32 >= 2048;
}

// Rows per workgroup of the row-range form, or 0 where it does not apply: one of the two fused
// one-split layers, up to 32 activation rows, a row count that splits into equal multiples of 8
// over the chip's 256 compute units, and a tile count that does not already do so.
static int skinny_rows_per_wg(int M, int N, int n_splits, bool rope, bool swiglu) {
  constexpr int kComputeUnits = 256;
  if (M > 32 || n_splits != 1 || rope == swiglu) return 0;
  if (N % (8 * kComputeUnits) || (N / 32) % kComputeUnits == 0) return 0;
  const int R = N / kComputeUnits;
  return R <= 64 ? R : 0;                                     // at most two 32-row blocks
}

bool skinny_top_lists_supported(int M, int N, int K) {
  return skinny_linear_supported(M, N, K) && N % 64 == 0 && skinny_pair_form(N, 1, false, false) &&
         !skinny_shared_form(M, N, 1, false);
}

int launch_linear_skinny(hipStream_t st, int M, int N, int K, const void *a, const void *w,
                         const void *w2, float *out, void *out_t, int n_splits, const RopeOut *rope,
                         void *top_out) {
  const int units = K / 64;
  if (!skinny_linear_supported(M, N, K) || n_splits < 1 || units % (4 * n_splits))
    MC_FAIL(MC_ERR_UNSUPPORTED, "few-row linear: M=%d N=%d K=%d splits=%d not covered", M, N, K, n_splits);
  if (w2 && n_splits != 1) MC_FAIL(MC_ERR_INVALID, "the SwiGLU form cannot be split over K");
  if (w2 && N % 64) MC_FAIL(MC_ERR_UNSUPPORTED, "tiled SwiGLU output needs N %% 64 == 0");
  if (rope && (w2 || n_splits != 1 || rope->hd % 4 || N != (rope->Hq + 2 * rope->Hkv) * rope->hd))
    MC_FAIL(MC_ERR_INVALID, "fused QKV output: one K split, N = (Hq + 2 Hkv) hd, hd %% 4 == 0");
  const RopeOut none{};
  if (top_out && !(n_splits == 1 && !rope && !w2 && skinny_top_lists_supported(M, N, K)))
    MC_FAIL(MC_ERR_UNSUPPORTED, "per-group top lists: M=%d N=%d K=%d not covered", M, N, K);
  if (const int R = skinny_rows_per_wg(M, N, n_splits, rope != nullptr, w2 != nullptr)) {
    const LaunchEvents ev3 = take_launch_events();
    auto go3 = [&](auto kernel, int n_blocks, int n_w, const RopeOut &ro) -> int {
      const int lds = 4 * n_blocks * n_w * 4 * 64 * (int)sizeof(float4);
      MC_TRY(raise_dynamic_lds_limit((const void *)kernel, lds));
      if (ev3.start || ev3.stop)
        hipExtLaunchKernelGGL(kernel, dim3(N / R), dim3(256), lds, st, ev3.start, ev3.stop, 0, M, N, K, R,
                              (const bf16_t *)a, (const bf16_t *)w, (const bf16_t *)w2, (bf16_t *)out_t, ro);
      else
        kernel<<<dim3(N / R), 256, lds, st>>>(M, N, K, R, (const bf16_t *)a, (const bf16_t *)w,
                                              (const bf16_t *)w2, (bf16_t *)out_t, ro);
      return MC_OK;
    };
    if (w2 && R > 32) MC_TRY(go3(skinny_rows_kernel<2, SKINNY_SWIGLU, false>, 2, 2, none));
    else if (w2) MC_TRY(go3(skinny_rows_kernel<1, SKINNY_SWIGLU, false>, 1, 2, none));
    else if (R > 32) MC_TRY(go3(skinny_rows_kernel<2, SKINNY_PLAIN, true>, 2, 1, *rope));
    else MC_TRY(go3(skinny_rows_kernel<1, SKINNY_PLAIN, true>, 1, 1, *rope));
    MC_HIP(hipGetLastError());
    return MC_OK;
  }
  if (skinny_shared_form(M, N, n_splits, rope != nullptr)) {
    const int groups = (N / 32 + 3) / 4;
    const dim3 grid2((groups + 7) / 8 * 8, n_splits);
    const LaunchEvents ev2 = take_launch_events();
    auto go2 = [&](auto kernel) {
      if (ev2.start || ev2.stop)
        hipExtLaunchKernelGGL(kernel, grid2, dim3(256), 0, st, ev2.start, ev2.stop, 0, M, N, K, units / n_splits,
                              (const bf16_t *)a, (const bf16_t *)w, (const bf16_t *)w2, out, (bf16_t *)out_t);
      else
        kernel<<<grid2, 256, 0, st>>>(M, N, K, units / n_splits, (const bf16_t *)a, (const bf16_t *)w,
                                      (const bf16_t *)w2, out, (bf16_t *)out_t);
    };
    if (w2) go2(skinny_shared_kernel<true>);
    else go2(skinny_shared_kernel<false>);
    MC_HIP(hipGetLastError());
    return MC_OK;
  }
  int upw = units / (4 * n_splits);
  const bf16_t *A = (const bf16_t *)a, *W = (const bf16_t *)w, *W2 = (const bf16_t *)w2;
  bf16_t *OT = (bf16_t *)out_t;
  const bool pair = skinny_pair_form(N, n_splits, rope != nullptr, w2 != nullptr);
  dim3 grid(pair ? ((N / 64 + 3) / 4 + 7) / 8 * 8 : N / 32, n_splits);
  if (pair) {
    W2 = W + (size_t)units * 2048;                             // the tile after w's
    upw = units;                                               // every wave walks the whole K range
  }
  // events offered by a profiling scope ride on the launch itself
  const LaunchEvents ev = take_launch_events();
  auto go = [&](auto kernel, const RopeOut &ro) {
    if (ev.start || ev.stop)
      hipExtLaunchKernelGGL(kernel, grid, dim3(256), 0, st, ev.start, ev.stop, 0, M, N, K, upw, A, W, W2, out, OT, ro, (uint2 *)top_out);
    else
      kernel<<<grid, 256, 0, st>>>(M, N, K, upw, A, W, W2, out, OT, ro, (uint2 *)top_out);
  };
  if (M <= 32) {
    if (rope) go(skinny_linear_kernel<1, SKINNY_PLAIN, true>, *rope);
    else if (pair) go(skinny_linear_kernel<1, SKINNY_PAIR, false>, none);
    else if (w2) go(skinny_linear_kernel<1, SKINNY_SWIGLU, false>, none);
    else go(skinny_linear_kernel<1, SKINNY_PLAIN, false>, none);
  } else {
    if (rope) go(skinny_linear_kernel<2, SKINNY_PLAIN, true>, *rope);
    else if (pair) go(skinny_linear_kernel<2, SKINNY_PAIR, false>, none);
    else if (w2) go(skinny_linear_kernel<2, SKINNY_SWIGLU, false>, none);
    else go(skinny_linear_kernel<2, SKINNY_PLAIN, false>, none);
  }
  MC_HIP(hipGetLastError());
  return MC_OK;
}

}  // namespace mc
