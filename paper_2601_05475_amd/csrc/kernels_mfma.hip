// bf16 MFMA kernels for gfx950 (wave64, v_mfma_f32_32x32x16_bf16).
//
// Operand layout of the 32x32x16 instruction, D[32][32] += A[32][16] * B[16][32], as used here:
//   A: lane l holds row (l % 32), contraction slots 8*(l / 32) .. +7   (8 bf16 = 16 bytes)
//   B: lane l holds column (l % 32), the same contraction slots
//   D: lane l holds column (l % 32); register r holds row 8*(r / 4) + 4*(l / 32) + (r % 4)
// Only the pairing of A and B slots matters for a dot product, so kernels are free to map a slot
// to any element of the contracted axis as long as both operands use the same map.
#include "kernels_mfma.h"

#include <algorithm>

namespace mc {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ inline f32x16 mfma32(uint4 a, uint4 b, f32x16 c) {
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

// =====================================================================================
// Few-row linear layer: weights streamed once, straight from HBM into MFMA operands.
// A workgroup owns 32 weight rows; its 4 waves take 4 different slices of the K range and
// meet in LDS.  Lane (row n, half h) reads 64 contiguous bytes of its weight row per step,
// the activation operand uses the same slot map.  MB = number of 32-row blocks of `a`.
// =====================================================================================
template <int MB, bool SWIGLU>
__global__ __launch_bounds__(256) void skinny_linear_kernel(
    int M, int N, int K, int units_per_wave, const bf16_t *__restrict__ a,
    const bf16_t *__restrict__ w, const bf16_t *__restrict__ w2, float *__restrict__ out,
    bf16_t *__restrict__ out_t) {
  constexpr int NW = SWIGLU ? 2 : 1;
  __shared__ float4 red[4][NW][MB][4][64];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, nl = lane & 31, h = lane >> 5;
  const int n0 = blockIdx.x * 32, split = blockIdx.y;
  const size_t k_begin = ((size_t)(split * 4 + wave) * units_per_wave) * 64 + 32 * h;
  const bf16_t *wrow = w + (size_t)(n0 + nl) * K + k_begin;
  const bf16_t *urow = SWIGLU ? w2 + (size_t)(n0 + nl) * K + k_begin : nullptr;
  const bf16_t *arow[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) arow[mb] = a + (size_t)min(mb * 32 + nl, M - 1) * K + k_begin;
  f32x16 acc[NW][MB];
#pragma unroll
  for (int i = 0; i < NW; ++i)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][mb][r] = 0.f;

#pragma unroll 2
  for (int u = 0; u < units_per_wave; ++u) {
    uint4 wf[4], uf[4], af[MB][4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      wf[c] = *(const uint4 *)(wrow + u * 64 + 8 * c);
      if (SWIGLU) uf[c] = *(const uint4 *)(urow + u * 64 + 8 * c);
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int c = 0; c < 4; ++c) af[mb][c] = *(const uint4 *)(arow[mb] + u * 64 + 8 * c);
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        acc[0][mb] = mfma32(wf[c], af[mb][c], acc[0][mb]);
        if (SWIGLU) acc[1][mb] = mfma32(uf[c], af[mb][c], acc[1][mb]);
      }
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
  const int n = n0 + 8 * r4 + 4 * h;
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
        *(uint2 *)(out_t + (size_t)m * N + n) =
            pack4_bf16(silu_f(s[0].x) * s[NW - 1].x, silu_f(s[0].y) * s[NW - 1].y,
                       silu_f(s[0].z) * s[NW - 1].z, silu_f(s[0].w) * s[NW - 1].w);
      } else {
        *(float4 *)(out + ((size_t)split * M + m) * N + n) = s[0];
      }
    }
  }
}

bool skinny_linear_supported(int M, int N, int K) {
  return M >= 1 && M <= 64 && N % 32 == 0 && K % 256 == 0;
}

int skinny_linear_splits(int M, int N, int K) {
  (void)M;
  const int tiles = N / 32, units = K / 64;
  int best = 1;
  for (int s = 1; s <= 16; s *= 2) {
    if (units % (4 * s)) break;
    best = s;
    if (tiles * s >= 512) break;
  }
  return best;
}

int launch_linear_skinny(hipStream_t st, int M, int N, int K, const void *a, const void *w,
                         const void *w2, float *out, void *out_t, int n_splits) {
  const int units = K / 64;
  if (!skinny_linear_supported(M, N, K) || n_splits < 1 || units % (4 * n_splits))
    MC_FAIL(MC_ERR_UNSUPPORTED, "few-row linear: M=%d N=%d K=%d splits=%d not covered", M, N, K, n_splits);
  if (w2 && n_splits != 1) MC_FAIL(MC_ERR_INVALID, "the SwiGLU form cannot be split over K");
  const int upw = units / (4 * n_splits);
  dim3 grid(N / 32, n_splits);
  const bf16_t *A = (const bf16_t *)a, *W = (const bf16_t *)w, *W2 = (const bf16_t *)w2;
  bf16_t *OT = (bf16_t *)out_t;
  if (M <= 32) {
    if (w2) skinny_linear_kernel<1, true><<<grid, 256, 0, st>>>(M, N, K, upw, A, W, W2, out, OT);
    else skinny_linear_kernel<1, false><<<grid, 256, 0, st>>>(M, N, K, upw, A, W, W2, out, OT);
  } else {
    if (w2) skinny_linear_kernel<2, true><<<grid, 256, 0, st>>>(M, N, K, upw, A, W, W2, out, OT);
    else skinny_linear_kernel<2, false><<<grid, 256, 0, st>>>(M, N, K, upw, A, W, W2, out, OT);
  }
  MC_HIP(hipGetLastError());
  return MC_OK;
}

// =====================================================================================
// Many-row GEMM: out[m][n] = sum_k a[m][k] w[n][k].  128 x 128 tile per workgroup, 64-deep
// slabs staged through LDS, 2 x 2 waves each owning 64 x 64 (2 x 2 MFMA tiles).  Weight rows
// feed the A operand so that a lane ends up with runs of 4 consecutive n for 16-byte stores.
// =====================================================================================
constexpr int GB = 128, GK = 64, GLD = GK + 8;   // LDS row stride in elements (144 bytes)

template <bool SWIGLU>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(
    int M, int N, int K, const bf16_t *__restrict__ a, const bf16_t *__restrict__ w,
    const bf16_t *__restrict__ w2, float *__restrict__ out, bf16_t *__restrict__ out_t) {
  constexpr int NW = SWIGLU ? 2 : 1;
  __shared__ __attribute__((aligned(16))) bf16_t As[GB * GLD];
  __shared__ __attribute__((aligned(16))) bf16_t Ws[NW][GB * GLD];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, j = lane & 31, h = lane >> 5;
  const int wn = wave & 1, wm = wave >> 1;
  const int n0 = blockIdx.x * GB, m0 = blockIdx.y * GB;
  // staging: thread t moves 16-byte chunk (t % 8) of rows t / 8 + 32 i
  const int srow = tid >> 3, schunk = (tid & 7) * 8;
  const bf16_t *ag[4], *wg[4], *ug[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    ag[i] = a + (size_t)min(m0 + srow + 32 * i, M - 1) * K + schunk;
    wg[i] = w + (size_t)(n0 + srow + 32 * i) * K + schunk;
    ug[i] = SWIGLU ? w2 + (size_t)(n0 + srow + 32 * i) * K + schunk : nullptr;
  }
  f32x16 acc[NW][2][2];
#pragma unroll
  for (int i = 0; i < NW; ++i)
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int y = 0; y < 2; ++y)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][x][y][r] = 0.f;
  uint4 pa[4], pw[4], pu[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    pa[i] = *(const uint4 *)(ag[i]);
    pw[i] = *(const uint4 *)(wg[i]);
    if (SWIGLU) pu[i] = *(const uint4 *)(ug[i]);
  }
  for (int k0 = 0; k0 < K; k0 += GK) {
    __syncthreads();           // everyone is done reading the previous slab
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      *(uint4 *)(As + (srow + 32 * i) * GLD + schunk) = pa[i];
      *(uint4 *)(Ws[0] + (srow + 32 * i) * GLD + schunk) = pw[i];
      if (SWIGLU) *(uint4 *)(Ws[NW - 1] + (srow + 32 * i) * GLD + schunk) = pu[i];
    }
    __syncthreads();
    if (k0 + GK < K) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        pa[i] = *(const uint4 *)(ag[i] + k0 + GK);
        pw[i] = *(const uint4 *)(wg[i] + k0 + GK);
        if (SWIGLU) pu[i] = *(const uint4 *)(ug[i] + k0 + GK);
      }
    }
#pragma unroll
    for (int ks = 0; ks < GK / 16; ++ks) {
      uint4 fa[2], fw[NW][2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        fa[t] = *(const uint4 *)(As + (64 * wm + 32 * t + j) * GLD + 16 * ks + 8 * h);
        fw[0][t] = *(const uint4 *)(Ws[0] + (64 * wn + 32 * t + j) * GLD + 16 * ks + 8 * h);
        if (SWIGLU) fw[NW - 1][t] = *(const uint4 *)(Ws[NW - 1] + (64 * wn + 32 * t + j) * GLD + 16 * ks + 8 * h);
      }
#pragma unroll
      for (int i = 0; i < NW; ++i)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
          for (int mt = 0; mt < 2; ++mt) acc[i][nt][mt] = mfma32(fw[i][nt], fa[mt], acc[i][nt][mt]);
    }
  }
#pragma unroll
  for (int mt = 0; mt < 2; ++mt) {
    const int m = m0 + 64 * wm + 32 * mt + j;
    if (m >= M) continue;
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int n = n0 + 64 * wn + 32 * nt + 8 * r4 + 4 * h;
        const f32x16 &g = acc[0][nt][mt];
        if (SWIGLU) {
          const f32x16 &u = acc[NW - 1][nt][mt];
          *(uint2 *)(out_t + (size_t)m * N + n) =
              pack4_bf16(silu_f(g[4 * r4]) * u[4 * r4], silu_f(g[4 * r4 + 1]) * u[4 * r4 + 1],
                         silu_f(g[4 * r4 + 2]) * u[4 * r4 + 2], silu_f(g[4 * r4 + 3]) * u[4 * r4 + 3]);
        } else {
          *(float4 *)(out + (size_t)m * N + n) =
              make_float4(g[4 * r4], g[4 * r4 + 1], g[4 * r4 + 2], g[4 * r4 + 3]);
        }
      }
  }
}

bool gemm_supported(int M, int N, int K) { return M > 64 && N % GB == 0 && K % GK == 0; }

int launch_gemm_mfma(hipStream_t st, int M, int N, int K, const void *a, const void *w,
                     const void *w2, float *out, void *out_t) {
  if (!gemm_supported(M, N, K)) MC_FAIL(MC_ERR_UNSUPPORTED, "GEMM: M=%d N=%d K=%d not covered", M, N, K);
  dim3 grid(N / GB, (M + GB - 1) / GB);
  if (w2)
    gemm_mfma_kernel<true><<<grid, 256, 0, st>>>(M, N, K, (const bf16_t *)a, (const bf16_t *)w,
                                                 (const bf16_t *)w2, out, (bf16_t *)out_t);
  else
    gemm_mfma_kernel<false><<<grid, 256, 0, st>>>(M, N, K, (const bf16_t *)a, (const bf16_t *)w,
                                                  nullptr, out, (bf16_t *)out_t);
  MC_HIP(hipGetLastError());
  return MC_OK;
}

bool decode_attention_mfma_supported(const DecodeAttnArgs &) { return false; }
size_t decode_attention_mfma_ws_bytes(int, int, int, int, int, int, int) { return 0; }
int launch_attention_decode_mfma(hipStream_t, const DecodeAttnArgs &) { MC_FAIL(MC_ERR_UNSUPPORTED, "not built"); }

}  // namespace mc
