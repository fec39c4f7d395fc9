// GEMM with bf16 operands and fp32 accumulation on the matrix cores (v_mfma_f32_32x32x16_bf16),
// for the wide edge layers of the bilinear block (paper Sec. 3.4; Table 4 widths).  Matrices
// stay fp32 in HBM; operands are rounded to bf16 (round-to-nearest-even) on their way into LDS,
// the fused epilogue and all outputs are fp32.
//
// LDS tiles are As[m][k], Bs[n][k] with k contiguous (rows padded to 80 bytes), so the 8
// consecutive k that one lane feeds to an MFMA are a single 16-byte read.  A 256-thread
// workgroup owns a 128 x BN tile, each wavefront 32x32 blocks of it; K advances 32 per slab,
// global loads for the next slab are issued before the current one is multiplied.
#include <stdarg.h>

#include <type_traits>

#include "gemm_common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int BKH = 32;        // k per slab
constexpr int LDK = BKH + 8;   // bf16 per LDS row: 80 bytes, 16-byte reads of 8 lanes cover all banks
constexpr int K8 = BKH / 8;    // 16-byte groups per row

__device__ __forceinline__ bf16x8 to_bf16x8(const float* v, uint32_t bits) {
  bf16x8 r;
#pragma unroll
  for (int c = 0; c < 8; ++c) r[c] = (__bf16)(((bits >> c) & 1u) ? v[c] : 0.f);
  return r;
}

// source rows = tile rows, contraction index contiguous; item = (row, group of 8 k)
template <int X, bool VEC>
struct bl_kcontig {
  static constexpr int ITEMS = X * K8;
  static constexpr int NV = (ITEMS + THREADS - 1) / THREADS;
  float r[NV][8];
  uint32_t mask;
  __device__ __forceinline__ void fetch(const float* __restrict__ src, int64_t ld, int64_t row0, int64_t n_rows,
                                        int64_t k0, int64_t k_end) {
    mask = 0;
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      const int row = idx / K8, kq = (idx % K8) * 8;
      const bool in_tile = (ITEMS % THREADS == 0) || idx < ITEMS;
      const int64_t gr = row0 + row, gk = k0 + kq;
      const bool row_ok = in_tile && gr < n_rows;
      const float* p = src + (gr < n_rows ? gr : n_rows - 1) * ld;
      if (VEC) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int64_t k = gk + 4 * h;
          const f32x4 v = ld4(p + (k < k_end ? k : k_end - 4));
#pragma unroll
          for (int c = 0; c < 4; ++c) r[it][4 * h + c] = v[c];
          mask |= ((row_ok && k < k_end) ? 0xFu : 0u) << (8 * it + 4 * h);
        }
      } else {
#pragma unroll
        for (int c = 0; c < 8; ++c) {
          const int64_t k = gk + c;
          r[it][c] = p[k < k_end ? k : k_end - 1];
          mask |= ((row_ok && k < k_end) ? 1u : 0u) << (8 * it + c);
        }
      }
    }
  }
  __device__ __forceinline__ void store(__bf16* __restrict__ S) const {
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      if (ITEMS % THREADS != 0 && idx >= ITEMS) continue;
      const int row = idx / K8, kq = (idx % K8) * 8;
      *reinterpret_cast<bf16x8*>(&S[row * LDK + kq]) = to_bf16x8(r[it], (mask >> (8 * it)) & 0xFFu);
    }
  }
};

// source has the tile's m/n index contiguous and the contraction index strided; item = (x, group of 8 k);
// consecutive lanes take consecutive x, so every one of the 8 loads is coalesced
template <int X, bool VEC>
struct bl_xcontig {
  static constexpr int ITEMS = X * K8;
  static constexpr int NV = (ITEMS + THREADS - 1) / THREADS;
  float r[NV][8];
  uint32_t mask;
  __device__ __forceinline__ void fetch(const float* __restrict__ src, int64_t ld, int64_t x0, int64_t n_x,
                                        int64_t k0, int64_t k_end) {
    mask = 0;
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      const int x = idx % X, kq = (idx / X) * 8;
      const bool in_tile = (ITEMS % THREADS == 0) || idx < ITEMS;
      const int64_t gx = x0 + x;
      const bool x_ok = in_tile && gx < n_x;
      const float* p = src + (gx < n_x ? gx : n_x - 1);
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const int64_t k = k0 + kq + c;
        r[it][c] = p[(k < k_end ? k : k_end - 1) * ld];
        mask |= ((x_ok && k < k_end) ? 1u : 0u) << (8 * it + c);
      }
    }
  }
  __device__ __forceinline__ void store(__bf16* __restrict__ S) const {
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      if (ITEMS % THREADS != 0 && idx >= ITEMS) continue;
      const int x = idx % X, kq = (idx / X) * 8;
      *reinterpret_cast<bf16x8*>(&S[x * LDK + kq]) = to_bf16x8(r[it], (mask >> (8 * it)) & 0xFFu);
    }
  }
};

template <int BM, int BN, int WAVES_M, int WAVES_N, int MODE, bool VEC>
__global__ void __launch_bounds__(THREADS)
gemm_bf16_kernel(const gemm_args g) {
  static_assert(WAVES_M * WAVES_N == 4, "four wavefronts per workgroup");
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int MB = WM / 32, NB = WN / 32;
  using loadA = typename std::conditional<MODE != MODE_TN, bl_kcontig<BM, VEC>, bl_xcontig<BM, VEC>>::type;
  using loadB = typename std::conditional<MODE == MODE_NT, bl_kcontig<BN, VEC>, bl_xcontig<BN, VEC>>::type;
  extern __shared__ __attribute__((aligned(16))) float smem[];
  __bf16* As = reinterpret_cast<__bf16*>(smem);
  __bf16* Bs = As + BM * LDK;

  const int tiles_n = (g.N + BN - 1) / BN;
  const int tiles_m = (int)((g.M + BM - 1) / BM);
  const int tile = xcd_remap(blockIdx.x, tiles_m * tiles_n);
  const int64_t m0 = (int64_t)(tile / tiles_n) * BM;
  const int n0 = (tile % tiles_n) * BN;

  int64_t k_begin = 0, k_end = g.K;
  if (MODE == MODE_TN) {
    k_begin = (int64_t)blockIdx.y * g.k_per_split;
    k_end = k_begin + g.k_per_split < (int64_t)g.K ? k_begin + g.k_per_split : (int64_t)g.K;
  }

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
  const int kh = lane >> 5, l32 = lane & 31;

  f32x16 acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  loadA la;
  loadB lb;
  auto fetch = [&](int64_t k0) {
    la.fetch(g.A, g.lda, m0, g.M, k0, k_end);
    lb.fetch(g.B, g.ldb, n0, g.N, k0, k_end);
  };

  if (k_begin < k_end) {
    fetch(k_begin);
    la.store(As);
    lb.store(Bs);
  }
  __syncthreads();

  for (int64_t k0 = k_begin; k0 < k_end; k0 += BKH) {
    const bool more = k0 + BKH < k_end;
    if (more) fetch(k0 + BKH);
#pragma unroll
    for (int kk = 0; kk < BKH; kk += 16) {
      bf16x8 a[MB], b[NB];
#pragma unroll
      for (int i = 0; i < MB; ++i) a[i] = *reinterpret_cast<const bf16x8*>(&As[(wm0 + i * 32 + l32) * LDK + kk + kh * 8]);
#pragma unroll
      for (int j = 0; j < NB; ++j) b[j] = *reinterpret_cast<const bf16x8*>(&Bs[(wn0 + j * 32 + l32) * LDK + kk + kh * 8]);
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
    if (more) {
      la.store(As);
      lb.store(Bs);
    }
    __syncthreads();
  }

  // epilogue: same register layout as the fp32 32x32 MFMA; transposed through a per-wavefront
  // LDS slice so that loads and stores are 16-byte accesses
  float* stage = smem + wave * (32 * EPI_LD);
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j) {
#pragma unroll
      for (int v = 0; v < 16; ++v) stage[((v >> 2) * 8 + kh * 4 + (v & 3)) * EPI_LD + l32] = acc[i][j][v];
      wave_lds_sync();
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int r = it * 8 + (lane >> 3), c4 = (lane & 7) * 4;
        const f32x4 v4 = *reinterpret_cast<const f32x4*>(&stage[r * EPI_LD + c4]);
        const int64_t row = m0 + wm0 + i * 32 + r;
        const int col = n0 + wn0 + j * 32 + c4;
        if (row >= g.M || col >= g.N) continue;
        if (MODE == MODE_TN) {
          float* dst = g.part + ((int64_t)blockIdx.y * g.M + row) * g.N + col;
          if (g.vecC) *reinterpret_cast<f32x4*>(dst) = v4;
          else
            for (int c = 0; c < 4; ++c)
              if (col + c < g.N) dst[c] = v4[c];
        } else {
          if (g.vecC) epilogue_store4(g.epi, row, col, g.N, v4);
          else
            for (int c = 0; c < 4; ++c)
              if (col + c < g.N) epilogue_store(g.epi, row, col + c, g.N, v4[c]);
        }
      }
      wave_lds_sync();
    }
}

template <int BM, int BN, int WMS, int WNS, int MODE, bool VEC>
int launch_v(gp_ctx* ctx, gemm_args& g, int splits) {
  const int64_t tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
  if (tiles > INT32_MAX) return gp_fail(ctx, GP_BAD_ARG, "gemm: too many tiles");
  dim3 grid((unsigned)tiles, (unsigned)splits, 1);
  static char name[48];
  if (!name[0]) snprintf(name, sizeof(name), "gemm_bf16_%s_%dx%d", MODE == MODE_NN ? "nn" : MODE == MODE_NT ? "nt" : "tn", BM, BN);
  const double mnk = (double)g.M * g.N * g.K;
  gp_prof_scope prof(ctx, name, 2.0 * mnk,
                     4.0 * ((double)g.M * g.K + (double)g.K * g.N + (double)g.M * g.N * (MODE == MODE_TN ? splits : 1)));
  constexpr size_t lds_main = sizeof(__bf16) * (size_t)(BM + BN) * LDK;
  constexpr size_t lds_epi = sizeof(float) * 4 * 32 * EPI_LD;
  constexpr size_t lds = lds_main > lds_epi ? lds_main : lds_epi;
  gemm_bf16_kernel<BM, BN, WMS, WNS, MODE, VEC><<<grid, THREADS, lds, ctx->stream>>>(g);
  GP_LAUNCH_CHECK(ctx, "gemm_bf16_kernel");
  return GP_OK;
}

template <int MODE>
int dispatch(gp_ctx* ctx, gemm_args& g, int splits) {
#define GP_BF16_LAUNCH(BN, WMS, WNS)                                                      \
  do {                                                                                    \
    if (g.vecA && g.vecB) return launch_v<128, BN, WMS, WNS, MODE, true>(ctx, g, splits); \
    return launch_v<128, BN, WMS, WNS, MODE, false>(ctx, g, splits);                      \
  } while (0)
  if (g.N > 64) GP_BF16_LAUNCH(128, 2, 2);
  if (g.N > 32) GP_BF16_LAUNCH(64, 2, 2);
  GP_BF16_LAUNCH(32, 4, 1);
#undef GP_BF16_LAUNCH
}

}  // namespace

// Called by gp_gemm_nn / gp_gemm_nt / gp_gemm_tn when the context asks for bf16 operands; `g` has
// been filled exactly as for the fp32 kernels (same tile geometry, same split-K plan).
int gp_gemm_bf16_launch(gp_ctx* ctx, int mode, void* args, int splits) {
  gemm_args& g = *static_cast<gemm_args*>(args);
  if (mode == MODE_NN) return dispatch<MODE_NN>(ctx, g, splits);
  if (mode == MODE_NT) return dispatch<MODE_NT>(ctx, g, splits);
  return dispatch<MODE_TN>(ctx, g, splits);
}
