// Many-row bf16 GEMM on tiled operands (gfx950, v_mfma_f32_32x32x16_bf16):
//   out[m][n] = sum_k a[m][k] w[n][k]                 (fp32, row-major), or
//   out_t[m][n] = silu(a . wg[n]) * (a . wu[n])        (bf16, tiled; the SwiGLU form).
//
// A workgroup of 8 waves (4 x 2) owns 256 rows of a and 256 rows of w (128 of wg and of wu in
// the SwiGLU form); a wave keeps 8 accumulator tiles of 32 x 32 (64 rows of a x 128 rows of w).
// Eight waves per CU, two per SIMD, is what the LDS needs to deliver its full read rate (one
// wave per SIMD reaches about half), and the second wave fills the matrix core while the first
// waits for operands.  Per 16-deep chunk a wave reads 6 fragments and issues 8 MFMAs.
// One 64-deep unit of both operands (16 blocks of 4 KB, already in MFMA operand order, so they
// are copied to LDS as they are and read back conflict-free) is staged per step in one of two
// alternating buffers: the global loads of unit u + 1 are issued before the MFMAs of unit u,
// land in registers meanwhile and are written to the other buffer before the single barrier
// that ends the unit.
//
// Workgroup numbering follows the hardware's round-robin deal of workgroups to the 8 XCDs: the
// ids that land on one XCD walk a compact 8 x 4 patch of output tiles, so that XCD's L2 serves
// each operand tile to several workgroups and HBM sees it about once per patch row/column.
#include "kernels_mfma.h"

#include <algorithm>

namespace mc {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t v4u;

__device__ inline f32x16 mfma32g(v4u a, v4u b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
__device__ inline float silu_g(float g) { return g / (1.0f + expf(-g)); }
__device__ inline uint32_t pack2g_bf16(float a, float b) {
  typedef __attribute__((ext_vector_type(2))) float f32x2;
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, b}, bf16x2));
}

constexpr int kPatchRows = 8;     // output-tile patch walked by one XCD: 8 row tiles x 4 column tiles

// tile (tm, tn) of workgroup `id`; false if the id is padding
__device__ inline bool gemm_tile_of(int id, int tiles_m, int tiles_n, int &tm, int &tn) {
  const int total = tiles_m * tiles_n;
  const int per_xcd = (total + 7) >> 3;
  const int L = (id & 7) * per_xcd + (id >> 3);
  if ((id >> 3) >= per_xcd || L >= total) return false;
  const int band = L / (kPatchRows * tiles_n);              // band of kPatchRows row tiles
  const int rows_here = min(kPatchRows, tiles_m - band * kPatchRows);
  const int in_band = L - band * kPatchRows * tiles_n;
  tn = in_band / rows_here;
  tm = band * kPatchRows + in_band % rows_here;
  return true;
}

// What a workgroup does with its 256 x 256 sums: store them (fp32), the SwiGLU product of two
// weight matrices (bf16, tiled), the fused QKV epilogue (rope_store_quad), or out += sums.
enum { GEMM_STORE = 0, GEMM_SWIGLU = 1, GEMM_ROPE = 2, GEMM_ACCUM = 3 };
// row stride (floats) of a wave's 32 x 128 parking area in the GEMM_ROPE epilogue: 128 + 4, so
// that the 16-byte writes of eight lanes (eight rows) fall into different banks
constexpr int kParkStride = 132;

template <int MODE>
__global__ __launch_bounds__(512)
void gemm256_kernel(int M, int N, int K, int tiles_m, int tiles_n, const bf16_t *__restrict__ a,
                    const bf16_t *__restrict__ w, const bf16_t *__restrict__ w2,
                    float *__restrict__ out, bf16_t *__restrict__ out_t, RopeOut ro) {
  constexpr bool SWIGLU = MODE == GEMM_SWIGLU;
  constexpr int NW = SWIGLU ? 2 : 1;       // weight matrices
  constexpr int TM = 2;                    // 32-row tiles of a per wave
  constexpr int TN = SWIGLU ? 2 : 4;       // 32-row tiles of each weight matrix per wave
  constexpr int WT = NW * TN;              // weight tiles of one wave (4)
  constexpr int AB = 8;                    // blocks of a per unit (workgroup): 256 rows
  constexpr int WB = 2 * TN;               // blocks of each weight matrix per unit (workgroup)
  constexpr int NB = AB + NW * WB;         // 16 blocks of 256 chunks
  extern __shared__ __attribute__((aligned(16))) unsigned char gemm_lds[];
  v4u *lds = (v4u *)gemm_lds;              // [2][NB][256]
  const int tid = threadIdx.x, lane = tid & 63, j = lane & 31, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wn = wave & 1, wm = wave >> 1;
  int tm, tn;
  if (!gemm_tile_of(blockIdx.x, tiles_m, tiles_n, tm, tn)) return;
  const int U = K >> 6;
  const int mt0 = tm * AB, nt0 = tn * WB;  // first 32-row tile of a / of each weight matrix
  const int m_tiles = (M + 31) >> 5;

  // staging: thread t carries chunk t % 256 of blocks 2i + t / 256, i = 0..7; the block base is
  // wave-uniform (scalar registers), the rest a 32-bit byte offset
  const int half = wave >> 2;
  const char *src[NB / 2];
#pragma unroll
  for (int i = 0; i < NB / 2; ++i) {
    const int b = 2 * i + half;            // block of the unit: a first, then w, then w2
    const bf16_t *p;
    if (b < AB) p = a + (size_t)min(mt0 + b, m_tiles - 1) * U * 2048;
    else if (b < AB + WB) p = w + (size_t)(nt0 + b - AB) * U * 2048;
    else p = w2 + (size_t)(nt0 + b - AB - WB) * U * 2048;
    src[i] = (const char *)p;
  }
  const uint32_t s_off = (tid & 255) * 16u;
  const int s_lds = half * 256 + (tid & 255);       // + (buf * NB + 2 i) * 256

  f32x16 acc[WT][TM];
#pragma unroll
  for (int x = 0; x < WT; ++x)
#pragma unroll
    for (int y = 0; y < TM; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;

  // Loads past the last unit re-read the last unit (in bounds, never used), so that every
  // iteration issues the same loads and the compiler's load counters stay exact.
  v4u st[NB / 2];
  auto load_unit = [&](int u) __attribute__((always_inline)) {
    const uint32_t at = s_off + (uint32_t)min(u, U - 1) * 4096u;
#pragma unroll
    for (int i = 0; i < NB / 2; ++i) st[i] = *(const v4u *)(src[i] + at);
  };
  auto store_unit = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < NB / 2; ++i) lds[(buf * NB + 2 * i) * 256 + s_lds] = st[i];
  };

  // fragments of chunk c of the unit in LDS buffer `buf`
  auto read_frags = [&](v4u (&fa)[TM], v4u (&fw)[WT], int buf, int c) __attribute__((always_inline)) {
    const v4u *ca = lds + (buf * NB + TM * wm) * 256 + lane + c * 64;
    const v4u *cw = lds + (buf * NB + AB + TN * wn) * 256 + lane + c * 64;
#pragma unroll
    for (int t = 0; t < TM; ++t) fa[t] = ca[t * 256];
#pragma unroll
    for (int x = 0; x < TN; ++x) {
      fw[x] = cw[x * 256];
      if (SWIGLU) fw[TN + x] = cw[(WB + x) * 256];
    }
  };
  auto multiply = [&](const v4u (&fa)[TM], const v4u (&fw)[WT]) __attribute__((always_inline)) {
#pragma unroll
    for (int x = 0; x < WT; ++x)
#pragma unroll
      for (int y = 0; y < TM; ++y) acc[x][y] = mfma32g(fw[x], fa[y], acc[x][y]);
  };

  load_unit(0);
  store_unit(0);
  __syncthreads();
  // Per unit: the global loads of unit u + 1 go out first.  The fragments of chunk c + 1 are read
  // from LDS while the MFMAs of chunk c run (two register sets), and the LDS writes of unit u + 1
  // are spread between the MFMAs of the last chunk, so that only the barrier itself and the
  // first fragment reads after it are not covered by matrix work.  The scheduling directives pin
  // this interleaving; without them the compiler sinks loads next to their uses.
  for (int u = 0; u < U; ++u) {
    const int buf = u & 1;
    v4u fa[2][TM], fw[2][WT];
    load_unit(u + 1);
    read_frags(fa[0], fw[0], buf, 0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int c = 0; c < 3; ++c) {
      read_frags(fa[(c + 1) & 1], fw[(c + 1) & 1], buf, c + 1);
      multiply(fa[c & 1], fw[c & 1]);
#pragma unroll
      for (int i = 0; i < TM + WT; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);    // one LDS read
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);    // one MFMA
      }
      __builtin_amdgcn_sched_group_barrier(0x008, TM * WT - TM - WT, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    // the other buffer was last read during unit u - 1, which every wave left before the
    // barrier that ended it
    store_unit(buf ^ 1);
    multiply(fa[1], fw[1]);
#pragma unroll
    for (int i = 0; i < NB / 2; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      // one MFMA
      __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);      // one LDS write
    }
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
  }

  // weight rows are the A operand: a lane holds column m = j of the tile and, per register quad,
  // four consecutive n
  if (MODE == GEMM_ROPE) {
    // The rotation epilogue is long; it runs as a rolled loop over quads that the wave first
    // parks in its own slice of LDS (free after the last barrier above).  The loop hands
    // consecutive lanes consecutive quads of one row, so table reads and query stores coalesce.
    float *park = (float *)gemm_lds + wave * (32 * kParkStride);
    const int n_wave = 32 * (nt0 + TN * wn);
#pragma unroll
    for (int y = 0; y < TM; ++y) {
      const int m0 = 32 * (mt0 + TM * wm + y);
#pragma unroll
      for (int x = 0; x < TN; ++x)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const f32x16 &g = acc[x][y];
          *(float4 *)(park + j * kParkStride + 32 * x + 8 * r4 + 4 * h) =
              make_float4(g[4 * r4], g[4 * r4 + 1], g[4 * r4 + 2], g[4 * r4 + 3]);
        }
      constexpr int kBatch = 4;        // quads per lane whose loads go out together
#pragma unroll 1
      for (int it0 = 0; it0 < 32 * TN * 8 / 64; it0 += kBatch) {
        float4 s[kBatch];
        RopeQuad rq[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
          const int e = (it0 + u) * 64 + lane, row = e / (TN * 8), quad = e % (TN * 8);
          s[u] = *(const float4 *)(park + row * kParkStride + 4 * quad);
          rq[u] = rope_load_quad(ro, min(m0 + row, M - 1), n_wave + 4 * quad);
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
          const int e = (it0 + u) * 64 + lane, row = e / (TN * 8), quad = e % (TN * 8);
          if (m0 + row < M) rope_store_quad(ro, m0 + row, n_wave + 4 * quad, s[u], rq[u]);
        }
      }
    }
    return;
  }
#pragma unroll
  for (int y = 0; y < TM; ++y) {
    const int m = 32 * (mt0 + TM * wm + y) + j;
    if (m >= M) continue;
#pragma unroll
    for (int x = 0; x < TN; ++x)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int n = 32 * (nt0 + TN * wn + x) + 8 * r4 + 4 * h;
        const f32x16 &g = acc[x][y];
        if (SWIGLU) {
          const f32x16 &uu = acc[TN + x][y];
          uint2 pk;
          pk.x = pack2g_bf16(silu_g(g[4 * r4]) * uu[4 * r4], silu_g(g[4 * r4 + 1]) * uu[4 * r4 + 1]);
          pk.y = pack2g_bf16(silu_g(g[4 * r4 + 2]) * uu[4 * r4 + 2], silu_g(g[4 * r4 + 3]) * uu[4 * r4 + 3]);
          *(uint2 *)(out_t + tiled_offset(m, n, N)) = pk;
        } else if (MODE == GEMM_ACCUM) {
          float4 *p = (float4 *)(out + (size_t)m * N + n);
          const float4 old = *p;
          *p = make_float4(old.x + g[4 * r4], old.y + g[4 * r4 + 1], old.z + g[4 * r4 + 2], old.w + g[4 * r4 + 3]);
        } else {
          *(float4 *)(out + (size_t)m * N + n) =
              make_float4(g[4 * r4], g[4 * r4 + 1], g[4 * r4 + 2], g[4 * r4 + 3]);
        }
      }
  }
}

// Matrix-core rate with nothing else going on: every wave keeps 8 accumulator tiles and issues
// MFMAs on operands it loaded once.  What this reaches with realistic operand values is the
// practical ceiling of any GEMM on the part (the clock follows the power drawn, which depends on
// the data: all-zero operands run markedly faster).
__global__ __launch_bounds__(256) void mfma_probe_kernel(const v4u *__restrict__ operands,
                                                         float *__restrict__ out, int iters) {
  const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
  v4u a[2], b[4];
#pragma unroll
  for (int i = 0; i < 2; ++i) a[i] = operands[t * 6 + i];
#pragma unroll
  for (int i = 0; i < 4; ++i) b[i] = operands[t * 6 + 2 + i];
  f32x16 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
      for (int y = 0; y < 2; ++y) acc[x * 2 + y] = mfma32g(b[x], a[y], acc[x * 2 + y]);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  out[t] = s;
}

int launch_mfma_probe(hipStream_t st, const void *operands, float *out, int n_workgroups, int iters) {
  mfma_probe_kernel<<<n_workgroups, 256, 0, st>>>((const v4u *)operands, out, iters);
  MC_HIP(hipGetLastError());
  return MC_OK;
}

bool gemm256_supported(int M, int N, int K, bool swiglu) {
  return M >= 1 && K >= 64 && K % 64 == 0 && N % (swiglu ? 128 : 256) == 0;
}

int launch_gemm256(hipStream_t st, int M, int N, int K, const void *a, const void *w,
                   const void *w2, float *out, void *out_t, const RopeOut *rope, int accumulate) {
  const bool swiglu = w2 != nullptr;
  if (!gemm256_supported(M, N, K, swiglu)) MC_FAIL(MC_ERR_UNSUPPORTED, "GEMM: M=%d N=%d K=%d not covered", M, N, K);
  if ((swiglu && (rope || accumulate)) || (rope && accumulate))
    MC_FAIL(MC_ERR_INVALID, "GEMM: one output form at a time");
  if (rope && (rope->hd % 4 || N != (rope->Hq + 2 * rope->Hkv) * rope->hd))
    MC_FAIL(MC_ERR_INVALID, "fused QKV output: N = (Hq + 2 Hkv) hd, hd %% 4 == 0");
  const int mode = swiglu ? GEMM_SWIGLU : rope ? GEMM_ROPE : accumulate ? GEMM_ACCUM : GEMM_STORE;
  const int tiles_m = (M + 255) / 256, tiles_n = N / (swiglu ? 128 : 256);
  const int per_xcd = (tiles_m * tiles_n + 7) / 8;
  // two buffers of 16 blocks; the parking areas of the rotation epilogue need a little more
  const size_t lds = std::max<size_t>(2 * 16 * 4096, mode == GEMM_ROPE ? 8 * 32 * kParkStride * sizeof(float) : 0);
  const void *kernels[4] = {(const void *)gemm256_kernel<GEMM_STORE>, (const void *)gemm256_kernel<GEMM_SWIGLU>,
                            (const void *)gemm256_kernel<GEMM_ROPE>, (const void *)gemm256_kernel<GEMM_ACCUM>};
  static bool attr_set[4] = {false, false, false, false};
  if (!attr_set[mode]) {
    MC_HIP(hipFuncSetAttribute(kernels[mode], hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr_set[mode] = true;
  }
  const RopeOut none{};
  const bf16_t *A = (const bf16_t *)a, *W = (const bf16_t *)w, *W2 = (const bf16_t *)w2;
  bf16_t *OT = (bf16_t *)out_t;
  const dim3 grid(8 * per_xcd);
  switch (mode) {
    case GEMM_SWIGLU: gemm256_kernel<GEMM_SWIGLU><<<grid, 512, lds, st>>>(M, N, K, tiles_m, tiles_n, A, W, W2, out, OT, none); break;
    case GEMM_ROPE: gemm256_kernel<GEMM_ROPE><<<grid, 512, lds, st>>>(M, N, K, tiles_m, tiles_n, A, W, W2, out, OT, *rope); break;
    case GEMM_ACCUM: gemm256_kernel<GEMM_ACCUM><<<grid, 512, lds, st>>>(M, N, K, tiles_m, tiles_n, A, W, W2, out, OT, none); break;
    default: gemm256_kernel<GEMM_STORE><<<grid, 512, lds, st>>>(M, N, K, tiles_m, tiles_n, A, W, W2, out, OT, none); break;
  }
  MC_HIP(hipGetLastError());
  return MC_OK;
}

}  // namespace mc
