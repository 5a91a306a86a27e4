// Many-row bf16 GEMM on tiled operands (gfx950, v_mfma_f32_32x32x16_bf16):
//   out[m][n] = sum_k a[m][k] w[n][k]                 (fp32, row-major), or
//   out_t[m][n] = silu(a . wg[n]) * (a . wu[n])        (bf16, tiled; the SwiGLU form).
//
// A workgroup of 4 waves owns 256 rows of a and 128 rows of w (64 of wg and of wu in the SwiGLU
// form); a wave keeps 8 accumulator tiles of 32 x 32 (its own 64 rows of a x all 128 rows of w).
// Two workgroups share a CU (two waves per SIMD, 215 registers each): they run out of step, so
// the barrier, prologue and epilogue of one are covered by the matrix work of the other.
// The two operands reach the matrix cores by different roads, which splits the traffic between
// LDS and the vector memory path instead of loading one of them with everything:
//   * w is shared by the four waves: one 64-deep unit (4 blocks of 4 KB, already in MFMA operand
//     order, so they are copied to LDS as they are and read back conflict-free) is staged per
//     step in one of three LDS stages.  The global loads of unit u + 2 go out at the top of
//     unit u, land in registers meanwhile and are written to LDS during its last chunk; the one
//     barrier per unit then makes stage u + 2 visible a whole unit before it is read, so the first
//     fragments of unit u + 1 are read before the barrier that ends unit u and no wave starts a
//     unit waiting for LDS.
//   * a rows belong to one wave only, and the tiled layout holds them in operand order: a wave
//     loads its fragments straight from memory into the registers the MFMAs read (1 KB per wave
//     and fragment, fully coalesced), one unit ahead, refilling each fragment's registers as soon
//     as the chunk that used them has been issued.
// Per 16-deep chunk a wave reads 4 fragments from LDS, loads 2 from memory and issues 8 MFMAs.
// With both operands in LDS (the earlier form: 256 x 256 per 8-wave workgroup) the matrix pipes
// were busy 61 % and the LDS 63 %; this form reaches 75 % at a lower clock: the part is then at
// its power limit, and variants that differ in barrier scope or fragment look-ahead all
// land on the same rate.
//
// Workgroup numbering follows the hardware's round-robin deal of workgroups to the 8 XCDs: the
// ids that land on one XCD walk a compact patch of output tiles (8 row tiles deep), so that XCD's
// L2 serves each operand tile to several workgroups and HBM sees it about once per patch
// row/column.
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

constexpr int kPatchRows = 8;     // output-tile patch walked by one XCD: 8 row tiles deep

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

// What a workgroup does with its 256 x 128 sums: store them (fp32), the SwiGLU product of two
// weight matrices (bf16, tiled), the fused QKV epilogue (rope_store_quad), or out += sums.
enum { GEMM_STORE = 0, GEMM_SWIGLU = 1, GEMM_ROPE = 2, GEMM_ACCUM = 3 };
// row stride (floats) of a wave's 32 x 128 parking area in the GEMM_ROPE epilogue: 128 + 4, so
// that the 16-byte writes of eight lanes (eight rows) fall into different banks
constexpr int kParkStride = 132;

template <int MODE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void gemm256_kernel(int M, int N, int K, int tiles_m, int tiles_n, const bf16_t *__restrict__ a,
                    const bf16_t *__restrict__ w, const bf16_t *__restrict__ w2,
                    float *__restrict__ out, bf16_t *__restrict__ out_t, RopeOut ro) {
  constexpr bool SWIGLU = MODE == GEMM_SWIGLU;
  constexpr int NW = SWIGLU ? 2 : 1;       // weight matrices
  constexpr int TM = 2;                    // 32-row tiles of a per wave
  constexpr int TN = SWIGLU ? 2 : 4;       // 32-row tiles of each weight matrix per wave
  constexpr int WT = NW * TN;              // weight tiles of one wave (4)
  constexpr int AB = 8;                    // 32-row tiles of a per workgroup: 256 rows
  constexpr int WB = TN;                   // blocks of each weight matrix per unit (workgroup)
  constexpr int NBW = NW * WB;             // 4 weight blocks of 256 chunks per unit
  constexpr int kStages = 3;
  extern __shared__ __attribute__((aligned(16))) unsigned char gemm_lds[];
  v4u *lds = (v4u *)gemm_lds;              // [kStages][NBW][256]
  const int tid = threadIdx.x, lane = tid & 63, j = lane & 31, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave;
  int tm, tn;
  if (!gemm_tile_of(blockIdx.x, tiles_m, tiles_n, tm, tn)) return;
  const int U = K >> 6;
  const int mt0 = tm * AB, nt0 = tn * WB;  // first 32-row tile of a / of each weight matrix
  const int m_tiles = (M + 31) >> 5;

  // weight staging: thread t carries chunk t of every block of the unit
  const char *src[NBW];
#pragma unroll
  for (int i = 0; i < NBW; ++i) {
    // blocks of the unit: w first, then w2
    const bf16_t *p = i < WB ? w + (size_t)(nt0 + i) * U * 2048 : w2 + (size_t)(nt0 + i - WB) * U * 2048;
    src[i] = (const char *)p;
  }
  const uint32_t s_off = tid * 16u;
  const int s_lds = tid;       // + (stage * NBW + i) * 256
  // the rows of a come straight from memory in operand order: a chunk of a tile is 1 KB, 16 bytes per lane
  const char *asrc[TM];
#pragma unroll
  for (int y = 0; y < TM; ++y)
    asrc[y] = (const char *)(a + (size_t)min(mt0 + TM * wm + y, m_tiles - 1) * U * 2048);
  const uint32_t a_off = lane * 16u;

  f32x16 acc[WT][TM];
#pragma unroll
  for (int x = 0; x < WT; ++x)
#pragma unroll
    for (int y = 0; y < TM; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;

  // Loads past the last unit re-read the last unit (in bounds, never used), so that every
  // iteration issues the same loads and the compiler's load counters stay exact.
  v4u st[NBW];
  auto load_w = [&](int u) __attribute__((always_inline)) {
    const uint32_t at = s_off + (uint32_t)min(u, U - 1) * 4096u;
#pragma unroll
    for (int i = 0; i < NBW; ++i) st[i] = *(const v4u *)(src[i] + at);
  };
  auto store_w = [&](int stage) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < NBW; ++i) lds[(stage * NBW + i) * 256 + s_lds] = st[i];
  };
  v4u fa[4][TM];
  auto load_a = [&](int u, int c) __attribute__((always_inline)) {
    const uint32_t at = a_off + (uint32_t)min(u, U - 1) * 4096u + (uint32_t)c * 1024u;
#pragma unroll
    for (int y = 0; y < TM; ++y) fa[c][y] = *(const v4u *)(asrc[y] + at);
  };
  auto read_w = [&](v4u (&fw)[WT], int stage, int c) __attribute__((always_inline)) {
    const v4u *cw = lds + stage * NBW * 256 + lane + c * 64;
#pragma unroll
    for (int x = 0; x < TN; ++x) {
      fw[x] = cw[x * 256];
      if (SWIGLU) fw[TN + x] = cw[(WB + x) * 256];
    }
  };
  auto multiply = [&](const v4u (&fa_)[TM], const v4u (&fw)[WT]) __attribute__((always_inline)) {
#pragma unroll
    for (int y = 0; y < TM; ++y)
#pragma unroll
      for (int x = 0; x < WT; ++x) acc[x][y] = mfma32g(fw[x], fa_[y], acc[x][y]);
  };

  v4u fw[2][WT];
  load_w(0);
#pragma unroll
  for (int c = 0; c < 4; ++c) load_a(0, c);
  store_w(0);
  load_w(1);
  store_w(1);
  __syncthreads();
  read_w(fw[0], 0, 0);
  int cur = 0, nxt = 1, wr = 2;
  for (int u = 0; u < U; ++u) {
    load_w(u + 2);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int c = 0; c < 3; ++c) {
      read_w(fw[(c + 1) & 1], cur, c + 1);
      multiply(fa[c], fw[c & 1]);
      load_a(u + 1, c);
#pragma unroll
      for (int i = 0; i < WT; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);    // one LDS read
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);    // one MFMA
      }
      __builtin_amdgcn_sched_group_barrier(0x008, TM * WT - WT, 0);
      __builtin_amdgcn_sched_group_barrier(0x020, TM, 0);     // the loads of a for the next unit
      __builtin_amdgcn_sched_barrier(0);
    }
    // stage wr was last read during unit u - 1, which every wave left before the barrier that
    // ended it; stage nxt was written during unit u - 1 and is complete since that barrier
    store_w(wr);
    read_w(fw[0], nxt, 0);
    multiply(fa[3], fw[1]);
    load_a(u + 1, 3);
#pragma unroll
    for (int i = 0; i < NBW; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      // one MFMA
      __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);      // one LDS write
    }
#pragma unroll
    for (int i = 0; i < WT; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      // one MFMA
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);      // one LDS read
    }
    __builtin_amdgcn_sched_group_barrier(0x020, TM, 0);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    const int t = cur; cur = nxt; nxt = wr; wr = t;
  }

  // weight rows are the A operand: a lane holds column m = j of the tile and, per register quad,
  // four consecutive n
  if (MODE == GEMM_ROPE) {
    // The rotation epilogue is long; it runs as a rolled loop over quads that the wave first
    // parks in its own slice of LDS (free after the last barrier above).  The loop hands
    // consecutive lanes consecutive quads of one row, so table reads and query stores coalesce.
    float *park = (float *)gemm_lds + wave * (32 * kParkStride);
    const int n_wave = 32 * nt0;
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
        const int n = 32 * (nt0 + x) + 8 * r4 + 4 * h;
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
  (void)swiglu;
  return M >= 1 && K >= 64 && K % 64 == 0 && N % 128 == 0;
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
  const int tiles_m = (M + 255) / 256, tiles_n = N / (swiglu ? 64 : 128);
  const int per_xcd = (tiles_m * tiles_n + 7) / 8;
  // three stages of 4 weight blocks; the parking areas of the rotation epilogue need a little more
  const size_t lds = std::max<size_t>(3 * 4 * 4096, mode == GEMM_ROPE ? 4 * 32 * kParkStride * sizeof(float) : 0);
  const void *kernels[4] = {(const void *)gemm256_kernel<GEMM_STORE>, (const void *)gemm256_kernel<GEMM_SWIGLU>,
                            (const void *)gemm256_kernel<GEMM_ROPE>, (const void *)gemm256_kernel<GEMM_ACCUM>};
  // the largest request of this mode (the rotation epilogue's parking areas included)
  MC_TRY(raise_dynamic_lds_limit(kernels[mode], (int)lds));
  const RopeOut none{};
  const bf16_t *A = (const bf16_t *)a, *W = (const bf16_t *)w, *W2 = (const bf16_t *)w2;
  bf16_t *OT = (bf16_t *)out_t;
  const dim3 grid(8 * per_xcd);
  switch (mode) {
    case GEMM_SWIGLU: gemm256_kernel<GEMM_SWIGLU><<<grid, 256, lds, st>>>(M, N, K, tiles_m, tiles_n, A, W, W2, out, OT, none); break;
    case GEMM_ROPE: gemm256_kernel<GEMM_ROPE><<<grid, 256, lds, st>>>(M, N, K, tiles_m, tiles_n, A, W, W2, out, OT, *rope); break;
    case GEMM_ACCUM: gemm256_kernel<GEMM_ACCUM><<<grid, 256, lds, st>>>(M, N, K, tiles_m, tiles_n, A, W, W2, out, OT, none); break;
    default: gemm256_kernel<GEMM_STORE><<<grid, 256, lds, st>>>(M, N, K, tiles_m, tiles_n, A, W, W2, out, OT, none); break;
  }
  MC_HIP(hipGetLastError());
  return MC_OK;
}

}  // namespace mc
