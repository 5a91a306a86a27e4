// Plain-ALU kernels: embedding, residual + RMSNorm, RoPE + KV page write, a generic
// tiled linear layer, a generic attention kernel, sampling, reward scoring.
// They serve every dtype and shape; the bf16 MFMA kernels in kernels_mfma.hip take over
// the large contractions when the shape allows.
#include "common.h"

namespace mc {

// ------------------------------------------------------------------ block reductions
__device__ inline float wave_sum(float v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ inline float wave_max(float v) {
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ inline double wave_sum_d(double v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// sum over a block of up to 1024 threads; every thread gets the result; fixed order
template <typename F>
__device__ inline F block_sum(F v, F *scratch /* >= 16 */) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  __syncthreads();
  if (lane == 0) scratch[wave] = v;
  __syncthreads();
  F t = 0;
  for (int w = 0; w < nw; ++w) t += scratch[w];
  return t;
}
__device__ inline float block_max(float v, float *scratch) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  v = wave_max(v);
  __syncthreads();
  if (lane == 0) scratch[wave] = v;
  __syncthreads();
  float t = scratch[0];
  for (int w = 1; w < nw; ++w) t = fmaxf(t, scratch[w]);
  return t;
}

// ------------------------------------------------------------------ embedding gather
template <typename T>
__global__ void embed_kernel(int d, const int32_t *__restrict__ tok, const T *__restrict__ table,
                             float *__restrict__ x) {
  const int r = blockIdx.x;
  const T *src = table + (size_t)tok[r] * d;
  float *dst = x + (size_t)r * d;
  if (sizeof(T) == 2 && d % 8 == 0) {
    // bf16 rows in 16-byte pieces (rows start on a multiple of 16 bytes: d % 8 == 0)
    for (int i = 8 * threadIdx.x; i < d; i += 8 * blockDim.x) {
      const uint4 e = *(const uint4 *)((const bf16_t *)src + i);
      *(float4 *)(dst + i) = make_float4(bf16_to_f32((bf16_t)(e.x & 0xFFFF)), bf16_to_f32((bf16_t)(e.x >> 16)),
                                         bf16_to_f32((bf16_t)(e.y & 0xFFFF)), bf16_to_f32((bf16_t)(e.y >> 16)));
      *(float4 *)(dst + i + 4) = make_float4(bf16_to_f32((bf16_t)(e.z & 0xFFFF)), bf16_to_f32((bf16_t)(e.z >> 16)),
                                             bf16_to_f32((bf16_t)(e.w & 0xFFFF)), bf16_to_f32((bf16_t)(e.w >> 16)));
    }
    return;
  }
  for (int i = threadIdx.x; i < d; i += blockDim.x) dst[i] = Cvt<T>::to_f32(src[i]);
}

int launch_embed(hipStream_t st, int dtype, int rows, int d, const int32_t *tokens,
                 const void *table, float *x) {
  if (rows <= 0) return MC_OK;
  if (dtype == MC_F32)
    embed_kernel<float><<<rows, 256, 0, st>>>(d, tokens, (const float *)table, x);
  else
    embed_kernel<bf16_t><<<rows, 256, 0, st>>>(d, tokens, (const bf16_t *)table, x);
  MC_HIP(hipGetLastError());
  return MC_OK;
}

// ------------------------------------------------------------------ residual + RMSNorm
// x[r] += sum_s partials[s][r];  h[r] = x[r] * gain / sqrt(mean(x[r]^2) + eps)
template <typename T>
__global__ __launch_bounds__(256) void add_rmsnorm_kernel(
    int d, float *__restrict__ x, const float *__restrict__ partials, int n_partials,
    size_t pstride, const T *__restrict__ gain, float eps, T *__restrict__ h, int h_tiled) {
  __shared__ float scratch[16];
  const int r = blockIdx.x;
  const size_t row = (size_t)blockIdx.x * d;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) {
    float v = x[row + i];
    for (int s = 0; s < n_partials; ++s) v += partials[s * pstride + row + i];
    if (n_partials) x[row + i] = v;
    ss += v * v;
  }
  ss = block_sum<float>(ss, scratch);
  const float inv = 1.0f / sqrtf(ss / (float)d + eps);
  for (int i = threadIdx.x; i < d; i += 256) {
    const size_t at = h_tiled ? tiled_offset(r, i, d) : row + i;
    h[at] = Cvt<T>::from_f32(x[row + i] * inv * Cvt<T>::to_f32(gain[i]));
  }
}

// The same, four elements per thread and the row kept in registers between the two phases
// (d % 4 == 0, d <= 4 * VEC * blockDim).  bf16 output goes out as 8-byte stores; in the tiled
// layout four consecutive k stay inside one 16-byte chunk.
// rows_per_xcd > 0 (many rows): workgroups are dealt round-robin to the 8 XCDs, so block b works
// on row (b % 8) * rows_per_xcd + b / 8 and every XCD gets a contiguous range of rows.  In the
// tiled layout the 16-byte pieces of 8 consecutive rows share a 128-byte line; written from one
// L2 they leave as whole lines instead of eight partial ones.
template <typename T, int VEC>
__global__ __launch_bounds__(1024) void add_rmsnorm_vec_kernel(
    int rows, int rows_per_xcd, int d, float *__restrict__ x, const float *__restrict__ partials, int n_partials,
    size_t pstride, const T *__restrict__ gain, float eps, T *__restrict__ h, int h_tiled) {
  __shared__ float scratch[16];
  const int nt = blockDim.x;
  const int r = rows_per_xcd > 0 ? (int)(blockIdx.x & 7) * rows_per_xcd + (int)(blockIdx.x >> 3) : (int)blockIdx.x;
  if (r >= rows) return;
  const size_t row = (size_t)r * d;
  float4 v[VEC];
  float ss = 0.f;
#pragma unroll
  for (int j = 0; j < VEC; ++j) {
    const int i = 4 * (threadIdx.x + j * nt);
    v[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < d) {
      v[j] = *(const float4 *)(x + row + i);
      for (int s = 0; s < n_partials; ++s) {
        const float4 p = *(const float4 *)(partials + s * pstride + row + i);
        v[j].x += p.x; v[j].y += p.y; v[j].z += p.z; v[j].w += p.w;
      }
      if (n_partials) *(float4 *)(x + row + i) = v[j];
      ss += v[j].x * v[j].x + v[j].y * v[j].y + v[j].z * v[j].z + v[j].w * v[j].w;
    }
  }
  ss = block_sum<float>(ss, scratch);
  const float inv = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
  for (int j = 0; j < VEC; ++j) {
    const int i = 4 * (threadIdx.x + j * nt);
    if (i < d) {
      const size_t at = h_tiled ? tiled_offset(r, i, d) : row + i;
      const float o0 = v[j].x * inv * Cvt<T>::to_f32(gain[i]), o1 = v[j].y * inv * Cvt<T>::to_f32(gain[i + 1]),
                  o2 = v[j].z * inv * Cvt<T>::to_f32(gain[i + 2]), o3 = v[j].w * inv * Cvt<T>::to_f32(gain[i + 3]);
      if (sizeof(T) == 2) {
        uint2 pk;
        pk.x = (uint32_t)f32_to_bf16(o0) | ((uint32_t)f32_to_bf16(o1) << 16);
        pk.y = (uint32_t)f32_to_bf16(o2) | ((uint32_t)f32_to_bf16(o3) << 16);
        *(uint2 *)(h + at) = pk;
      } else {
        *(float4 *)(h + at) = make_float4(o0, o1, o2, o3);
      }
    }
  }
}

template <typename T>
static void launch_add_rmsnorm_t(hipStream_t st, int rows, int d, float *x, const float *partials,
                                 int n_partials, size_t ps, const T *gain, float eps, T *h, int h_tiled) {
  if (d % 4 == 0 && d <= 16384) {
    // enough threads for one float4 each where possible; at least one wave
    const int quads = d / 4;
    // many rows: 512 threads with two loads each in flight were measured faster than 1024 x 1
    const int nt_max = (rows >= 2048 && quads <= 4 * 512) ? 512 : 1024;
    int nt = 64;
    while (nt < nt_max && nt < quads) nt *= 2;
    const int vec = (quads + nt - 1) / nt;
    // many rows into the tiled layout: a contiguous range of rows per XCD
    const int rpx = (h_tiled && rows >= 256) ? ((rows + 7) / 8 + 7) / 8 * 8 : 0;
    const int grid = rpx > 0 ? 8 * rpx : rows;
    if (vec <= 1) add_rmsnorm_vec_kernel<T, 1><<<grid, nt, 0, st>>>(rows, rpx, d, x, partials, n_partials, ps, gain, eps, h, h_tiled);
    else if (vec <= 2) add_rmsnorm_vec_kernel<T, 2><<<grid, nt, 0, st>>>(rows, rpx, d, x, partials, n_partials, ps, gain, eps, h, h_tiled);
    else add_rmsnorm_vec_kernel<T, 4><<<grid, nt, 0, st>>>(rows, rpx, d, x, partials, n_partials, ps, gain, eps, h, h_tiled);
  } else {
    add_rmsnorm_kernel<T><<<rows, 256, 0, st>>>(d, x, partials, n_partials, ps, gain, eps, h, h_tiled);
  }
}

int launch_add_rmsnorm(hipStream_t st, int dtype, int rows, int d, float *x, const float *partials,
                       int n_partials, const void *gain, float eps, void *h_out, int h_tiled) {
  if (rows <= 0) return MC_OK;
  const size_t ps = (size_t)rows * d;
  if (dtype == MC_F32)
    launch_add_rmsnorm_t<float>(st, rows, d, x, partials, n_partials, ps, (const float *)gain, eps, (float *)h_out, h_tiled);
  else
    launch_add_rmsnorm_t<bf16_t>(st, rows, d, x, partials, n_partials, ps, (const bf16_t *)gain, eps, (bf16_t *)h_out, h_tiled);
  MC_HIP(hipGetLastError());
  return MC_OK;
}

__global__ void gather_rows_kernel(int d, const float *__restrict__ x,
                                   const int32_t *__restrict__ idx, float *__restrict__ out) {
  const float *src = x + (size_t)idx[blockIdx.x] * d;
  float *dst = out + (size_t)blockIdx.x * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) dst[i] = src[i];
}

int launch_gather_rows(hipStream_t st, int rows, int d, const float *x, const int32_t *idx,
                       float *out) {
  if (rows <= 0) return MC_OK;
  gather_rows_kernel<<<rows, 256, 0, st>>>(d, x, idx, out);
  MC_HIP(hipGetLastError());
  return MC_OK;
}

// ------------------------------------------------------------------ generic linear layer
// out[s][m][n] = sum_{k in split s} a[m][k] * w[n][k]; 64x64 tile, 16-deep slabs, 4x4 per thread.
// SWIGLU: two weight matrices, out[m][n] = silu(a.wg[n]) * (a.wu[n]) in the model dtype.
template <typename T, bool SWIGLU>
__global__ __launch_bounds__(256) void linear_generic_kernel(
    int M, int N, int K, int k_per_split, const T *__restrict__ a, const T *__restrict__ w,
    const T *__restrict__ w2, float *__restrict__ out, T *__restrict__ out_t) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float As[BK][BM + 4];
  __shared__ float Ws[BK][BN + 4];
  __shared__ float Us[SWIGLU ? BK : 1][BN + 4];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN, split = blockIdx.z;
  const int k_begin = split * k_per_split;
  const int k_end = min(K, k_begin + k_per_split);
  float acc[4][4] = {}, acc2[4][4] = {};
  const int lr = tid >> 2, lk = (tid & 3) * 4;   // each thread stages 4 consecutive k of one row
  for (int k0 = k_begin; k0 < k_end; k0 += BK) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int k = k0 + lk + j;
      const bool kin = k < k_end;
      As[lk + j][lr] = (kin && m0 + lr < M) ? Cvt<T>::to_f32(a[(size_t)(m0 + lr) * K + k]) : 0.f;
      Ws[lk + j][lr] = (kin && n0 + lr < N) ? Cvt<T>::to_f32(w[(size_t)(n0 + lr) * K + k]) : 0.f;
      if (SWIGLU)
        Us[lk + j][lr] = (kin && n0 + lr < N) ? Cvt<T>::to_f32(w2[(size_t)(n0 + lr) * K + k]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float av[4], wv[4], uv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        av[i] = As[kk][ty * 4 + i];
        wv[i] = Ws[kk][tx * 4 + i];
        if (SWIGLU) uv[i] = Us[kk][tx * 4 + i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          acc[i][j] += av[i] * wv[j];
          if (SWIGLU) acc2[i][j] += av[i] * uv[j];
        }
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      if (SWIGLU) {
        const float g = acc[i][j];
        out_t[(size_t)m * N + n] = Cvt<T>::from_f32(g / (1.0f + expf(-g)) * acc2[i][j]);
      } else {
        out[((size_t)split * M + m) * N + n] = acc[i][j];
      }
    }
  }
}

int launch_linear_generic(hipStream_t st, int dtype, int M, int N, int K, const void *a,
                          const void *w, float *out, int n_splits) {
  if (M <= 0 || N <= 0) return MC_OK;
  int kps = (K + n_splits - 1) / n_splits;
  kps = (kps + 15) / 16 * 16;
  dim3 grid((N + 63) / 64, (M + 63) / 64, n_splits);
  if (dtype == MC_F32)
    linear_generic_kernel<float, false><<<grid, 256, 0, st>>>(
        M, N, K, kps, (const float *)a, (const float *)w, nullptr, out, nullptr);
  else
    linear_generic_kernel<bf16_t, false><<<grid, 256, 0, st>>>(
        M, N, K, kps, (const bf16_t *)a, (const bf16_t *)w, nullptr, out, nullptr);
  MC_HIP(hipGetLastError());
  return MC_OK;
}

int launch_linear_swiglu_generic(hipStream_t st, int dtype, int M, int N, int K, const void *a,
                                 const void *wg, const void *wu, void *out) {
  if (M <= 0 || N <= 0) return MC_OK;
  dim3 grid((N + 63) / 64, (M + 63) / 64, 1);
  if (dtype == MC_F32)
    linear_generic_kernel<float, true><<<grid, 256, 0, st>>>(
        M, N, K, (K + 15) / 16 * 16, (const float *)a, (const float *)wg, (const float *)wu,
        nullptr, (float *)out);
  else
    linear_generic_kernel<bf16_t, true><<<grid, 256, 0, st>>>(
        M, N, K, (K + 15) / 16 * 16, (const bf16_t *)a, (const bf16_t *)wg, (const bf16_t *)wu,
        nullptr, (bf16_t *)out);
  MC_HIP(hipGetLastError());
  return MC_OK;
}

// ------------------------------------------------------------------ RoPE + KV page write
__global__ void rope_table_kernel(int n_pos, int half, int hd, double rope_base, double2 *__restrict__ table) {
  const size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= (size_t)n_pos * half) return;
  const int pos = (int)(e / half), i = (int)(e % half);
  double sn, cs;
  sincos((double)pos * pow(rope_base, -2.0 * (double)i / (double)hd), &sn, &cs);
  table[e] = make_double2(cs, sn);
}

int launch_rope_table(hipStream_t st, int n_pos, int hd, double rope_base, double2 *table) {
  const size_t n = (size_t)n_pos * (hd / 2);
  if (n == 0) return MC_OK;
  rope_table_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(n_pos, hd / 2, hd, rope_base, table);
  MC_HIP(hipGetLastError());
  return MC_OK;
}

// One block per (row, head).  Heads 0..Hq-1 are queries, then Hkv key heads, then Hkv value
// heads.  The angle pos * base^(-2i/hd) and its sine/cosine are taken in double (from the table
// of the same expressions when one is given).  qk_interleaved: coordinate i of a query / key head
// sits at 2i and coordinate i + hd/2 at 2i + 1 of the input row (see launch_pack_tiled).
template <typename T>
__global__ __launch_bounds__(64) void rope_kv_kernel(
    int rows, int Hq, int Hkv, int hd, int pg, double rope_base,
    const float *__restrict__ qkv, int n_splits, const int32_t *__restrict__ row_pos,
    const int32_t *__restrict__ row_page, const int32_t *__restrict__ row_off,
    T *__restrict__ q_out, T *__restrict__ k_pages, T *__restrict__ v_pages,
    const double2 *__restrict__ table, int qk_interleaved) {
  const int r = blockIdx.x, h = blockIdx.y;
  const int nqkv = (Hq + 2 * Hkv) * hd, half = hd >> 1;
  const size_t sstride = (size_t)rows * nqkv;
  const float *src = qkv + (size_t)r * nqkv + (size_t)h * hd;
  const size_t pelems = (size_t)Hkv * hd * pg;
  if (h < Hq + Hkv) {
    const double pos = (double)row_pos[r];
    // queries go out row-major; a key goes to its slot of the page, in the page's layout
    T *dst = (h < Hq) ? q_out + ((size_t)r * Hq + h) * hd
                      : k_pages + (size_t)row_page[r] * pelems + (size_t)(h - Hq) * pg * hd;
    const int key = row_off[r];
    for (int i = threadIdx.x; i < half; i += 64) {
      float lo = 0.f, hi = 0.f;
      const int at_l = qk_interleaved ? 2 * i : i, at_h = qk_interleaved ? 2 * i + 1 : i + half;
      for (int s = 0; s < n_splits; ++s) {
        lo += src[s * sstride + at_l];
        hi += src[s * sstride + at_h];
      }
      double sn, cs;
      if (table) {
        const double2 t = table[(size_t)row_pos[r] * half + i];
        cs = t.x; sn = t.y;
      } else {
        sincos(pos * pow(rope_base, -2.0 * (double)i / (double)hd), &sn, &cs);
      }
      const size_t at_lo = (h < Hq) ? (size_t)i : k_elem_offset(key, i, pg, hd);
      const size_t at_hi = (h < Hq) ? (size_t)(i + half) : k_elem_offset(key, i + half, pg, hd);
      dst[at_lo] = Cvt<T>::from_f32((float)((double)lo * cs - (double)hi * sn));
      dst[at_hi] = Cvt<T>::from_f32((float)((double)hi * cs + (double)lo * sn));
    }
  } else {
    const int kvh = h - Hq - Hkv;
    T *dst = v_pages + (size_t)row_page[r] * pelems + (size_t)kvh * hd * pg;
    const int key = row_off[r];
    for (int i = threadIdx.x; i < hd; i += 64) {
      float v = 0.f;
      for (int s = 0; s < n_splits; ++s) v += src[s * sstride + i];
      dst[v_elem_offset(key, i, pg, hd)] = Cvt<T>::from_f32(v);
    }
  }
}

int launch_rope_kv(hipStream_t st, int dtype, int rows, int Hq, int Hkv, int hd, int page_tokens,
                   double rope_base, const float *qkv, int n_splits, const int32_t *row_pos,
                   const int32_t *row_page, const int32_t *row_off, void *q_out, void *k_pages,
                   void *v_pages, const double2 *table, int qk_interleaved) {
  if (rows <= 0) return MC_OK;
  dim3 grid(rows, Hq + 2 * Hkv);
  if (dtype == MC_F32)
    rope_kv_kernel<float><<<grid, 64, 0, st>>>(rows, Hq, Hkv, hd, page_tokens, rope_base, qkv,
                                               n_splits, row_pos, row_page, row_off,
                                               (float *)q_out, (float *)k_pages, (float *)v_pages,
                                               table, qk_interleaved);
  else
    rope_kv_kernel<bf16_t><<<grid, 64, 0, st>>>(rows, Hq, Hkv, hd, page_tokens, rope_base, qkv,
                                                n_splits, row_pos, row_page, row_off,
                                                (bf16_t *)q_out, (bf16_t *)k_pages,
                                                (bf16_t *)v_pages, table, qk_interleaved);
  MC_HIP(hipGetLastError());
  return MC_OK;
}

// ------------------------------------------------------------------ generic attention
// One wave per (query row, query head).  Keys 0..pos of the row's sequence are walked 64 at a
// time with a running (max, sum, weighted value) state.  Lane j scores key j of the block; then
// lane d accumulates coordinates d, d+64, ... of the value sum.
template <typename T>
__global__ __launch_bounds__(64) void attention_generic_kernel(AttnArgs a) {
  constexpr int MAXD = 4;   // head_dim <= 256
  __shared__ float qs[256];
  __shared__ float ps[64];
  __shared__ long long kbase[64];   // element offset of the key's page+head base, -1 if masked
  __shared__ int koff[64];
  const int r = blockIdx.x, qh = blockIdx.y, lane = threadIdx.x;
  const int hd = a.head_dim, pg = a.page_tokens, Hkv = a.n_kv_heads;
  const int kvh = qh / (a.n_q_heads / Hkv);
  const int pos = a.row_pos[r];
  const int n_keys = pos + 1;
  const int n_pre = min(n_keys, a.prefix_len);
  const size_t pelems = (size_t)Hkv * hd * pg;
  const T *q = (const T *)a.q + ((size_t)r * a.n_q_heads + qh) * hd;
  for (int i = lane; i < hd; i += 64) qs[i] = Cvt<T>::to_f32(q[i]);
  const int32_t *tab = a.page_table ? a.page_table + (size_t)a.row_tab[r] * a.table_stride : nullptr;
  const float scale = 1.0f / sqrtf((float)hd);
  float m = -INFINITY, l = 0.f, o[MAXD] = {0.f, 0.f, 0.f, 0.f};
  __syncthreads();
  for (int j0 = 0; j0 < n_keys; j0 += 64) {
    const int j = j0 + lane;
    float s = -INFINITY;
    long long base = -1;
    int off = 0;
    bool in_prefix = true;
    if (j < n_keys) {
      int page;
      if (j < n_pre) {
        page = j / pg;
        off = j % pg;
      } else {
        const int jj = j - a.prefix_len;
        page = tab[jj / pg];
        off = jj % pg;
        in_prefix = false;
      }
      base = (long long)((size_t)page * pelems + (size_t)kvh * hd * pg);
      const T *kp = (const T *)(in_prefix ? a.k_prefix : a.k_suffix) + base;
      float dot = 0.f;
      if (kv_fragment_layout(pg, hd)) {
        for (int i = 0; i < hd; i += 8) {
          const T *k8 = kp + k_elem_offset(off, i, pg, hd);      // 8 consecutive d are contiguous
#pragma unroll
          for (int j = 0; j < 8; ++j) dot += qs[i + j] * Cvt<T>::to_f32(k8[j]);
        }
      } else {
        kp += (size_t)off * hd;
        for (int i = 0; i < hd; ++i) dot += qs[i] * Cvt<T>::to_f32(kp[i]);
      }
      s = dot * scale;
    }
    // bit 62 marks "suffix pool" so that the value pass picks the right pool
    kbase[lane] = (base < 0) ? -1 : (in_prefix ? base : (base | (1ll << 62)));
    koff[lane] = off;
    const float m_new = fmaxf(m, wave_max(s));
    const float p = (j < n_keys) ? expf(s - m_new) : 0.f;
    const float corr = expf(m - m_new);      // m = -inf on the first block: exp(-inf) = 0
    l = l * corr + wave_sum(p);
    ps[lane] = p;
    m = m_new;
    __syncthreads();
    const int nblk = min(64, n_keys - j0);
#pragma unroll
    for (int c = 0; c < MAXD; ++c) {
      const int d = lane + 64 * c;
      if (d < hd) {
        float acc = o[c] * corr;
        for (int t = 0; t < nblk; ++t) {
          const long long kb = kbase[t];
          const T *vp = (const T *)((kb >> 62) & 1 ? a.v_suffix : a.v_prefix) +
                        (kb & ~(1ll << 62)) + v_elem_offset(koff[t], d, pg, hd);
          acc += ps[t] * Cvt<T>::to_f32(*vp);
        }
        o[c] = acc;
      }
    }
    __syncthreads();
  }
  T *out = (T *)a.out;
#pragma unroll
  for (int c = 0; c < MAXD; ++c) {
    const int d = lane + 64 * c;
    if (d < hd) {
      const size_t at = a.out_tiled ? tiled_offset(r, qh * hd + d, a.n_q_heads * hd)
                                    : ((size_t)r * a.n_q_heads + qh) * hd + d;
      out[at] = Cvt<T>::from_f32(o[c] / l);
    }
  }
}

int launch_attention_generic(hipStream_t st, int dtype, const AttnArgs &a) {
  if (a.rows <= 0) return MC_OK;
  if (a.head_dim > 256) MC_FAIL(MC_ERR_UNSUPPORTED, "head_dim %d > 256", a.head_dim);
  dim3 grid(a.rows, a.n_q_heads);
  if (dtype == MC_F32)
    attention_generic_kernel<float><<<grid, 64, 0, st>>>(a);
  else
    attention_generic_kernel<bf16_t><<<grid, 64, 0, st>>>(a);
  MC_HIP(hipGetLastError());
  return MC_OK;
}

// ------------------------------------------------------------------ sampling
// Order-preserving map of a float to an unsigned integer (larger float -> larger integer).
__device__ inline uint32_t float_order_bits(float f) {
  const uint32_t b = __float_as_uint(f + 0.0f);       // -0 -> +0
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ inline float float_from_order_bits(uint32_t o) {
  return __uint_as_float((o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o);
}
// 64-bit key whose descending order is (z descending, id ascending)
__device__ inline unsigned long long sample_key(float z, int id) {
  return ((unsigned long long)float_order_bits(z) << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)id);
}

__device__ inline unsigned long long block_max_u64(unsigned long long v, unsigned long long *scratch) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  for (int o = 32; o > 0; o >>= 1) {
    unsigned long long t = __shfl_xor(v, o, 64);
    v = t > v ? t : v;
  }
  __syncthreads();
  if (lane == 0) scratch[wave] = v;
  __syncthreads();
  unsigned long long t = scratch[0];
  for (int w = 1; w < nw; ++w) t = scratch[w] > t ? scratch[w] : t;
  return t;
}

__device__ inline unsigned int block_reduce_u32(unsigned int v, bool take_max, unsigned int *scratch) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  for (int o = 32; o > 0; o >>= 1) {
    const unsigned int t = __shfl_xor(v, o, 64);
    v = take_max ? max(v, t) : min(v, t);
  }
  __syncthreads();
  if (lane == 0) scratch[wave] = v;
  __syncthreads();
  unsigned int t = scratch[0];
  for (int w = 1; w < nw; ++w) t = take_max ? max(t, scratch[w]) : min(t, scratch[w]);
  return t;
}

// Slot in a shared list for every lane with `want` set: one atomic per wave, not per lane.
__device__ inline unsigned int wave_claim(bool want, unsigned int *counter) {
  const unsigned long long m = __ballot(want);
  if (m == 0) return 0;
  const int leader = __ffsll((long long)m) - 1;
  unsigned int base = 0;
  if ((int)(threadIdx.x & 63) == leader) base = atomicAdd(counter, (unsigned int)__popcll(m));
  base = __shfl(base, leader, 64);
  return base + (unsigned int)__popcll(m & ((1ull << (threadIdx.x & 63)) - 1ull));
}

// Walk one row with all 1024 threads: f(valid, logit, index) is called the same number of times
// by every thread (so f may use wave-wide operations).  Loads go out in batches of eight 16-byte
// vectors per thread; a loop of single dependent-looking loads would pay the memory latency
// once per element.
template <typename F>
__device__ inline void scan_row(const float *row, int V, F f) {
  constexpr int NB = 8;
  const int tid = threadIdx.x;
  const int V4 = (((uintptr_t)row & 15) == 0) ? V / 4 : 0;
  const float4 *row4 = (const float4 *)row;
  for (int g0 = 0; g0 < V4; g0 += NB * 1024) {
    float4 z[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const int g = g0 + j * 1024 + tid;
      z[j] = (g < V4) ? row4[g] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const int g = g0 + j * 1024 + tid;
      const bool ok = g < V4;
      f(ok, z[j].x, 4 * g);
      f(ok, z[j].y, 4 * g + 1);
      f(ok, z[j].z, 4 * g + 2);
      f(ok, z[j].w, 4 * g + 3);
    }
  }
  for (int v0 = 4 * V4; v0 < V; v0 += 1024) {
    const int v = v0 + tid;
    const bool ok = v < V;
    f(ok, ok ? row[v] : 0.f, v);
  }
}

// The same walk over a list of (value bits, id) pairs: the per-group top lists the LM head leaves
// beside the logits (n even).
template <typename F>
__device__ inline void scan_pairs(const uint2 *list, int n, F f) {
  constexpr int NB = 4;
  const int tid = threadIdx.x;
  const int n2 = n / 2;
  const uint4 *l4 = (const uint4 *)list;
  for (int g0 = 0; g0 < n2; g0 += NB * 1024) {
    uint4 e[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const int g = g0 + j * 1024 + tid;
      e[j] = (g < n2) ? l4[g] : make_uint4(0u, 0u, 0u, 0u);
    }
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const bool ok = g0 + j * 1024 + tid < n2;
      f(ok, __uint_as_float(e[j].x), (int)e[j].y);
      f(ok, __uint_as_float(e[j].z), (int)e[j].w);
    }
  }
}

// LDS of the sampling kernel
struct SampleShared {
  unsigned long long sel[MC_MAX_TOP_K];
  float ev[MC_MAX_TOP_K];
  unsigned int hist[2048];
  unsigned long long scratch64[16];
  unsigned int scratch32[16];
  unsigned int s_bin, s_above, s_cnt, s_cnt2;
};

// Threshold selection of the k largest keys of the elements `scan` walks (k <= 1024, at least
// 4096 elements, every thread sees some and no two threads see the same): pass 1 takes every
// thread's largest value; the threads form n_g >= k groups (n_g the next power of two), and the
// smallest of the n_g group maxima, L, is a lower bound of the k-th largest value (n_g >= k
// distinct elements are >= L); M is the overall maximum.  Pass 2 looks only at elements >= L (a
// fraction of a percent of a row for k = 50): they are kept in an LDS list and counted in a
// histogram over (M - value) in order-preserving integer units, 2047 bins.  The bin B in which the
// count reaches k bounds the top k from below, the list is cut down to bins <= B (k plus a few).
// Returns the number of keys left in sh.sel (>= k, the top k among them), or 0 if the list or the
// cut overflowed (many equal values).  Division by T > 0, correctly rounded, never reverses an
// order, so maxima are taken on the values themselves and only candidates are divided.
template <typename Scan>
__device__ inline int threshold_select(Scan scan, float temperature, int k, SampleShared &sh) {
  const int tid = threadIdx.x;
  unsigned int mine = 0;
  scan([&](bool ok, float z, int) {
    if (ok) mine = max(mine, float_order_bits(z));
  });
  const unsigned int M = float_order_bits(
      __fdiv_rn(float_from_order_bits(block_reduce_u32(mine, true, sh.scratch32)), temperature));
  int n_g = 1;
  while (n_g < k) n_g <<= 1;
  sh.hist[tid] = mine;
  __syncthreads();
  unsigned int gmax = 0xFFFFFFFFu;
  if (tid < n_g) {
    const int per = 1024 / n_g;
    gmax = 0;
    for (int i = 0; i < per; ++i) gmax = max(gmax, sh.hist[tid * per + i]);
  }
  const float z_l = float_from_order_bits(block_reduce_u32(gmax, false, sh.scratch32));
  const unsigned int L = float_order_bits(__fdiv_rn(z_l, temperature));
  // a value below z_low cannot reach L after the division (its quotient is smaller by dozens of
  // ulps): a cheap test that spares the division for nearly every element
  const float z_low = z_l - fabsf(z_l) * 3.8147e-06f - 1e-30f;
  const unsigned int range = M - L;
  int shift = 0;
  while ((range >> shift) > 2046u) ++shift;
  for (int i = tid; i < 2048; i += 1024) sh.hist[i] = 0;
  if (tid == 0) { sh.s_cnt = 0; sh.s_cnt2 = 0; }
  __syncthreads();
  scan([&](bool ok, float z, int v) {
    const bool maybe = ok && z >= z_low;
    if (__ballot(maybe) == 0) return;             // wave-uniform: most batches hold no candidate
    const unsigned int ob = maybe ? float_order_bits(__fdiv_rn(z, temperature)) : 0u;
    const bool keep = maybe && ob >= L;
    const unsigned int slot = wave_claim(keep, &sh.s_cnt);
    if (keep) {
      atomicAdd(&sh.hist[(M - ob) >> shift], 1u);
      if (slot < MC_MAX_TOP_K) sh.sel[slot] = ((unsigned long long)ob << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)v);
    }
  });
  __syncthreads();
  const unsigned int n_cand = sh.s_cnt;
  if (tid < 64) {
    // lane L owns bins [32L, 32L + 32): find the bin in which the running count reaches k
    unsigned int own = 0;
    for (int i = 0; i < 32; ++i) own += sh.hist[32 * tid + i];
    unsigned int incl = own;
    for (int o = 1; o < 64; o <<= 1) {
      const unsigned int t = __shfl_up(incl, o, 64);
      if (tid >= o) incl += t;
    }
    const unsigned int excl = incl - own;
    if (excl < (unsigned int)k && incl >= (unsigned int)k) {   // exactly one lane (count >= n_g >= k)
      unsigned int run = excl;
      for (int i = 0; i < 32; ++i) {
        run += sh.hist[32 * tid + i];
        if (run >= (unsigned int)k) {
          sh.s_bin = (unsigned int)(32 * tid + i);
          sh.s_above = run;                          // elements in bins <= s_bin
          break;
        }
      }
    }
  }
  __syncthreads();
  const unsigned int B = sh.s_bin, G = sh.s_above;
  int n_sel = 0;
  if (n_cand <= MC_MAX_TOP_K && G <= MC_MAX_TOP_K) {
    // cut the list down to bins <= B: read everything, then write the survivors back
    unsigned long long mykeys[MC_MAX_TOP_K / 1024];
#pragma unroll
    for (int j = 0; j < MC_MAX_TOP_K / 1024; ++j) {
      const unsigned int i = tid + 1024 * j;
      mykeys[j] = (i < n_cand) ? sh.sel[i] : 0ull;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < MC_MAX_TOP_K / 1024; ++j) {
      const unsigned int i = tid + 1024 * j;
      const bool keep = i < n_cand && ((M - (unsigned int)(mykeys[j] >> 32)) >> shift) <= B;
      const unsigned int slot = wave_claim(keep, &sh.s_cnt2);
      if (keep) sh.sel[slot] = mykeys[j];
    }
    __syncthreads();
    n_sel = (int)sh.s_cnt2;                           // == G
  }
  __syncthreads();
  return n_sel;
}

// Radix selection of the k largest keys of a row: up to six passes on the 64-bit key (11/11/10-bit
// digits), exact for any input and any k.  Leaves exactly k keys in sh.sel.
__device__ inline int radix_select(const float *row, int V, float temperature, int k, SampleShared &sh) {
  const int tid = threadIdx.x;
  unsigned long long prefix = 0, pmask = 0;
  unsigned int need = (unsigned int)k;
  const int shifts[6] = {53, 42, 32, 21, 10, 0};
  const int nbits[6] = {11, 11, 10, 11, 11, 10};
  for (int pass = 0; pass < 6; ++pass) {
    const int shift = shifts[pass];
    const unsigned int bmask = (1u << nbits[pass]) - 1u;
    for (int i = tid; i < 2048; i += 1024) sh.hist[i] = 0;
    __syncthreads();
    for (int v = tid; v < V; v += 1024) {
      const unsigned long long key = sample_key(__fdiv_rn(row[v], temperature), v);
      if ((key & pmask) == prefix) atomicAdd(&sh.hist[(unsigned int)(key >> shift) & bmask], 1u);
    }
    __syncthreads();
    if (tid < 64) {
      // lane L owns bins [2048-32(L+1), 2048-32L): walk from the top bin down
      const int hi = 2048 - 32 * tid;
      unsigned int mine = 0;
      for (int i = 1; i <= 32; ++i) mine += sh.hist[hi - i];
      unsigned int incl = mine;                   // inclusive scan over lanes 0..L
      for (int o = 1; o < 64; o <<= 1) {
        const unsigned int t = __shfl_up(incl, o, 64);
        if (tid >= o) incl += t;
      }
      const unsigned int excl = incl - mine;
      if (excl < need && incl >= need) {          // exactly one lane
        unsigned int above = excl;
        for (int i = 1; i <= 32; ++i) {
          const unsigned int c = sh.hist[hi - i];
          if (above + c >= need) {
            sh.s_bin = (unsigned int)(hi - i);
            sh.s_above = above;
            sh.s_cnt = c;
            break;
          }
          above += c;
        }
      }
    }
    __syncthreads();
    prefix |= (unsigned long long)sh.s_bin << shift;
    pmask |= (unsigned long long)bmask << shift;
    need -= sh.s_above;
    const bool done = (sh.s_cnt == need);            // the whole bin belongs to the top k
    __syncthreads();
    if (done) break;
  }
  // every key >= prefix (low bits zero) is selected: exactly k of them
  if (tid == 0) sh.s_cnt = 0;
  __syncthreads();
  for (int v = tid; v < V; v += 1024) {
    const unsigned long long key = sample_key(__fdiv_rn(row[v], temperature), v);
    if (key >= prefix) {
      const unsigned int slot = atomicAdd(&sh.s_cnt, 1u);
      if (slot < MC_MAX_TOP_K) sh.sel[slot] = key;
    }
  }
  return k;
}

// Bitonic sort of sh.sel[0 .. n_sel), descending: the first k entries are the top k in order.
__device__ inline void sort_selected(int n_sel, SampleShared &sh) {
  const int tid = threadIdx.x;
  int kp = 1;
  while (kp < n_sel) kp <<= 1;
  __syncthreads();
  for (int i = n_sel + tid; i < kp; i += 1024) sh.sel[i] = 0ull;
  __syncthreads();
  for (int size = 2; size <= kp; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      for (int i = tid; i < kp; i += 1024) {
        const int j = i ^ stride;
        if (j > i) {
          const unsigned long long x = sh.sel[i], y = sh.sel[j];
          const bool desc = ((i & size) == 0);
          if ((x < y) == desc) { sh.sel[i] = y; sh.sel[j] = x; }
        }
      }
      __syncthreads();
    }
  }
}

// One block of 1024 threads per candidate: exact top-k of z / T under the order (value
// descending, id ascending), a bitonic sort of the survivors in LDS, then the softmax and the
// cumulative walk done left to right by one thread, as the rule demands.
//
// Where the LM head left per-group top lists beside the logits (top != nullptr: for every group
// of 64 consecutive ids its kTopListLen largest (value, id) pairs in order) and k <= kTopListMaxK,
// the selection runs on those lists, 1 / 16 of a row.  The result is the row's top k provided
// no group's last listed entry reaches the k-th selected value after the division (then an
// unlisted element of that group could belong to the top k, or tie with its last member): that
// is checked, and such a row is selected from the whole row instead, so the ids are the rule's
// in every case.  Selection from a row: threshold selection (two passes, k <= 1024, V >= 4096),
// else radix selection.
constexpr int kTopListLen = 4, kTopListMaxK = 64;
__global__ __launch_bounds__(1024) void sample_kernel(
    int V, const float *__restrict__ logits, size_t row_stride, const uint2 *__restrict__ top,
    size_t top_stride, int n_groups, float temperature, int top_k,
    const float *__restrict__ uniforms, int32_t *__restrict__ out_tokens,
    int32_t *__restrict__ out_topk) {
  __shared__ SampleShared sh;
  const int b = blockIdx.x, tid = threadIdx.x;
  const float *row = logits + (size_t)b * row_stride;
  const uint2 *list = top ? top + (size_t)b * top_stride : nullptr;

  if (temperature <= 0.f || top_k == 1) {
    unsigned long long best = 0;
    if (list) {                                    // the arg max is the best of the groups' first entries
      for (int g = tid; g < n_groups; g += 1024) {
        const uint2 e = list[(size_t)g * kTopListLen];
        const unsigned long long key = sample_key(__uint_as_float(e.x), (int)e.y);
        best = key > best ? key : best;
      }
    } else {
      for (int v = tid; v < V; v += 1024) {
        const unsigned long long key = sample_key(row[v], v);
        best = key > best ? key : best;
      }
    }
    best = block_max_u64(best, sh.scratch64);
    if (tid == 0) {
      const int tok = (int)(0xFFFFFFFFu - (uint32_t)(best & 0xFFFFFFFFull));
      out_tokens[b] = tok;
      if (out_topk) out_topk[b] = tok;
    }
    return;
  }
  const int k = (top_k <= 0 || top_k >= V) ? V : top_k;
  int n_sel = 0;                                   // keys in sel[] (>= k; the top k are among them)

  if (list && k <= kTopListMaxK && n_groups * kTopListLen >= 4096) {
    n_sel = threshold_select([&](auto f) { scan_pairs(list, n_groups * kTopListLen, f); }, temperature, k, sh);
    if (n_sel) {
      sort_selected(n_sel, sh);
      // conclusive only if every group's last listed entry stays below the k-th selected value
      const unsigned int z_k = (unsigned int)(sh.sel[k - 1] >> 32);
      unsigned int open = 0;
      for (int g = tid; g < n_groups; g += 1024) {
        const uint2 e = list[(size_t)g * kTopListLen + kTopListLen - 1];
        open |= float_order_bits(__fdiv_rn(__uint_as_float(e.x), temperature)) >= z_k ? 1u : 0u;
      }
      if (block_reduce_u32(open, true, sh.scratch32)) n_sel = 0;
      __syncthreads();
    }
  }
  if (n_sel == 0) {
    if (k <= 1024 && V >= 4096)
      n_sel = threshold_select([&](auto f) { scan_row(row, V, f); }, temperature, k, sh);
    if (n_sel == 0) n_sel = radix_select(row, V, temperature, k, sh);
    sort_selected(n_sel, sh);
  }
  const float z0 = float_from_order_bits((uint32_t)(sh.sel[0] >> 32));
  for (int i = tid; i < k; i += 1024)
    sh.ev[i] = expf(float_from_order_bits((uint32_t)(sh.sel[i] >> 32)) - z0);
  if (out_topk)
    for (int i = tid; i < k; i += 1024)
      out_topk[(size_t)b * k + i] = (int)(0xFFFFFFFFu - (uint32_t)(sh.sel[i] & 0xFFFFFFFFull));
  __syncthreads();
  if (tid == 0) {
    float total = 0.f;
    for (int i = 0; i < k; ++i) total += sh.ev[i];
    const float u = uniforms[b];
    float run = 0.f;
    int pick = k - 1;
    for (int i = 0; i < k; ++i) {
      run += sh.ev[i];
      if (__fdiv_rn(run, total) > u) { pick = i; break; }
    }
    out_tokens[b] = (int)(0xFFFFFFFFu - (uint32_t)(sh.sel[pick] & 0xFFFFFFFFull));
  }
}

int launch_sample(hipStream_t st, int n_cands, int vocab, const float *logits, size_t row_stride,
                  float temperature, int top_k, const float *uniforms, int32_t *out_tokens,
                  int32_t *out_topk, const void *top_lists, size_t top_stride, int n_groups) {
  if (n_cands <= 0) return MC_OK;
  sample_kernel<<<n_cands, 1024, 0, st>>>(vocab, logits, row_stride, (const uint2 *)top_lists, top_stride, n_groups,
                                          temperature, top_k, uniforms, out_tokens, out_topk);
  MC_HIP(hipGetLastError());
  return MC_OK;
}

// ------------------------------------------------------------------ reward scoring
// log-softmax over the whole vocabulary read at the reward tokens (sums kept in double)
__global__ __launch_bounds__(1024) void reward_logprob_kernel(
    int V, const float *__restrict__ logits, const int32_t *__restrict__ ids, int R,
    float *__restrict__ out_lp) {
  __shared__ float scr_f[16];
  __shared__ double scr_d[16];
  const float *row = logits + (size_t)blockIdx.x * V;
  float m = -INFINITY;
  for (int v = threadIdx.x; v < V; v += 1024) m = fmaxf(m, row[v]);
  m = block_max(m, scr_f);
  double s = 0.0;
  for (int v = threadIdx.x; v < V; v += 1024) s += exp((double)row[v] - (double)m);
  s = block_sum<double>(s, scr_d);
  const double lse = (double)m + log(s);
  for (int r = threadIdx.x; r < R; r += 1024)
    out_lp[(size_t)blockIdx.x * R + r] = (float)((double)row[ids[r]] - lse);
}

// score_b = sum_r w_r softmax_r(lp_r / Ts); rank by (score descending, index ascending)
__global__ __launch_bounds__(1024) void score_rank_kernel(
    int B, int R, const float *__restrict__ lp, const float *__restrict__ w, float ts,
    float *__restrict__ scores, int32_t *__restrict__ rank) {
  extern __shared__ float sc[];
  for (int b = threadIdx.x; b < B; b += 1024) {
    const float *p = lp + (size_t)b * R;
    double mx = -1e300;
    for (int r = 0; r < R; ++r) mx = fmax(mx, (double)p[r] / (double)ts);
    double den = 0.0, num = 0.0;
    for (int r = 0; r < R; ++r) {
      const double e = exp((double)p[r] / (double)ts - mx);
      den += e;
      num += e * (double)w[r];
    }
    const float v = (float)(num / den);
    sc[b] = v;
    if (scores) scores[b] = v;
  }
  __syncthreads();
  if (rank)
    for (int b = threadIdx.x; b < B; b += 1024) {
      const float mine = sc[b];
      int ahead = 0;
      for (int c = 0; c < B; ++c) ahead += (sc[c] > mine) || (sc[c] == mine && c < b);
      rank[ahead] = b;
    }
}

int launch_reward_score(hipStream_t st, int n_cands, int vocab, const float *logits,
                        const int32_t *reward_ids, const float *reward_values, int n_reward,
                        float score_temperature, float *out_logprobs, float *out_scores,
                        int32_t *out_rank) {
  if (n_cands <= 0) return MC_OK;
  reward_logprob_kernel<<<n_cands, 1024, 0, st>>>(vocab, logits, reward_ids, n_reward,
                                                  out_logprobs);
  MC_HIP(hipGetLastError());
  score_rank_kernel<<<1, 1024, (size_t)n_cands * sizeof(float), st>>>(
      n_cands, n_reward, out_logprobs, reward_values, score_temperature, out_scores, out_rank);
  MC_HIP(hipGetLastError());
  return MC_OK;
}

}  // namespace mc
