// fp32 GEMM on the matrix cores (v_mfma_f32_32x32x2_f32) with fused epilogues, plus the small
// reductions and elementwise kernels the edge MLPs need (EdgeUpdate of paper Sec. 2.1 / 3.3).
//
// Tiling: a 256-thread workgroup (4 wavefronts of 64) owns a BM x BN tile of C; the K loop
// advances BK = 32 at a time through LDS tiles As[k][m], Bs[k][n] (k-major, so the 32 lanes that
// feed one MFMA operand read consecutive LDS words).  Each wavefront owns
// (BM/WAVES_M) x (BN/WAVES_N) of the tile as 32x32 MFMA blocks.  The next K-slab is fetched
// into registers while the current one is multiplied and written to LDS between two barriers.
// With 32 k per slab a row of a k-contiguous operand contributes a whole 128-byte line to each
// load instruction, which the memory pipeline delivers faster than two half lines (BK = 16
// measured 5 % slower; two LDS buffers with one barrier per slab can be compiled in and measured
// slower still, because they halve the number of resident workgroups).
#include <stdarg.h>

#include <type_traits>

#include "gemm_common.h"

namespace {

#ifndef GP_GEMM_BK
#define GP_GEMM_BK 32
#endif
#ifndef GP_GEMM_NBUF
#define GP_GEMM_NBUF 1
#endif
constexpr int BK = GP_GEMM_BK;
constexpr int NBUF = GP_GEMM_NBUF;   // LDS buffers per operand (2: one barrier per slab)
// Operand loaders.  A fetch only ISSUES global loads (addresses are clamped into the matrix, so
// no branch surrounds a load and nothing waits on the data); the out-of-range elements are
// zeroed later, in store(), from a bit mask.  That keeps the loads of the next K-slab in flight
// while the current slab is multiplied.  VEC: 16-byte loads are legal (extent % 4 == 0, aligned).

// Source has the contraction index contiguous: tile of X rows by BK k's, stored transposed.
template <int X, bool VEC>
struct loader_kcontig {
  static constexpr int KV = BK / 4;               // 16-byte vectors per row
  static constexpr int TOTAL = X * KV;
  static constexpr int NV = (TOTAL + THREADS - 1) / THREADS;
  static constexpr int LD = X + 1;                // odd stride: transposed stores hit distinct banks
  f32x4 r[NV];
  uint32_t mask;
  __device__ __forceinline__ void fetch(const float* __restrict__ src, int64_t ld, int64_t row0,
                                        int64_t n_rows, int64_t k0, int64_t k_end) {
    mask = 0;
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      const int row = idx / KV, kq = (idx % KV) * 4;
      const bool in_tile = (TOTAL % THREADS == 0) || idx < TOTAL;
      const int64_t gr = row0 + row, gk = k0 + kq;
      const bool row_ok = in_tile && gr < n_rows;
      const float* p = src + (gr < n_rows ? gr : n_rows - 1) * ld;
      if (VEC) {
        const bool ok = row_ok && gk < k_end;
        r[it] = ld4(p + (gk < k_end ? gk : k_end - 4));
        mask |= (ok ? 0xFu : 0u) << (4 * it);
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int64_t kc = gk + c;
          r[it][c] = p[kc < k_end ? kc : k_end - 1];
          mask |= ((row_ok && kc < k_end) ? 1u : 0u) << (4 * it + c);
        }
      }
    }
  }
  __device__ __forceinline__ void store(float* __restrict__ S) const {
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      const int row = idx / KV, kq = (idx % KV) * 4;
      if (TOTAL % THREADS != 0 && idx >= TOTAL) continue;
#pragma unroll
      for (int c = 0; c < 4; ++c) S[(kq + c) * LD + row] = ((mask >> (4 * it + c)) & 1u) ? r[it][c] : 0.f;
    }
  }
};

// Source has the tile's m/n index contiguous: BK rows by X columns, stored as is.
template <int X, bool VEC>
struct loader_xcontig {
  static constexpr int TOTAL = X * BK / 4;
  static constexpr int NV = (TOTAL + THREADS - 1) / THREADS;
  static constexpr int LD = X + 4;
  f32x4 r[NV];
  uint32_t mask;
  __device__ __forceinline__ void fetch(const float* __restrict__ src, int64_t ld, int64_t x0,
                                        int64_t n_x, int64_t k0, int64_t k_end) {
    mask = 0;
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      const int k = idx / (X / 4), xq = (idx % (X / 4)) * 4;
      const bool in_tile = (TOTAL % THREADS == 0) || idx < TOTAL;
      const int64_t gk = k0 + k, gx = x0 + xq;
      const bool k_ok = in_tile && gk < k_end;
      const float* p = src + (gk < k_end ? gk : k_end - 1) * ld;
      if (VEC) {
        const bool ok = k_ok && gx < n_x;
        r[it] = ld4(p + (gx < n_x ? gx : n_x - 4));
        mask |= (ok ? 0xFu : 0u) << (4 * it);
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int64_t xc = gx + c;
          r[it][c] = p[xc < n_x ? xc : n_x - 1];
          mask |= ((k_ok && xc < n_x) ? 1u : 0u) << (4 * it + c);
        }
      }
    }
  }
  __device__ __forceinline__ void store(float* __restrict__ S) const {
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      const int k = idx / (X / 4), xq = (idx % (X / 4)) * 4;
      if (TOTAL % THREADS != 0 && idx >= TOTAL) continue;
      f32x4 v;
#pragma unroll
      for (int c = 0; c < 4; ++c) v[c] = ((mask >> (4 * it + c)) & 1u) ? r[it][c] : 0.f;
      *reinterpret_cast<f32x4*>(&S[k * LD + xq]) = v;
    }
  }
};

template <int BM, int BN, int WAVES_M, int WAVES_N, int MODE, bool VEC>
__global__ void __launch_bounds__(THREADS)
gemm_f32_kernel(const gemm_args g) {
  static_assert(WAVES_M * WAVES_N == 4, "four wavefronts per workgroup");
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int MB = WM / 32, NB = WN / 32;
  using loadA = typename std::conditional<MODE != MODE_TN, loader_kcontig<BM, VEC>, loader_xcontig<BM, VEC>>::type;
  using loadB = typename std::conditional<MODE == MODE_NT, loader_kcontig<BN, VEC>, loader_xcontig<BN, VEC>>::type;
  constexpr int LDA = loadA::LD, LDB = loadB::LD;
  extern __shared__ __attribute__((aligned(16))) float smem[];
  auto As = [&](int buf) -> float* { return smem + buf * (BK * LDA); };
  auto Bs = [&](int buf) -> float* { return smem + NBUF * BK * LDA + buf * (BK * LDB); };

  const int tiles_n = (g.N + BN - 1) / BN;
  const int tiles_m = (int)((g.M + BM - 1) / BM);
  const int tile = xcd_remap(blockIdx.x, tiles_m * tiles_n);
  const int tile_m = tile / tiles_n;
  const int64_t m0 = (int64_t)tile_m * BM;
  const int n0 = (tile % tiles_n) * BN;

  int64_t k_begin = 0, k_end = g.K;
  if (MODE == MODE_TN) {
    k_begin = (int64_t)blockIdx.y * g.k_per_split;
    k_end = k_begin + g.k_per_split < (int64_t)g.K ? k_begin + g.k_per_split : (int64_t)g.K;
  }

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;

  f32x16 acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  float colsum = 0.f;   // TN: column threadIdx.x of the B tile, over the slabs this workgroup owns

  loadA la;
  loadB lb;
  auto fetch = [&](int64_t k0) {
    la.fetch(g.A, g.lda, m0, g.M, k0, k_end);
    lb.fetch(g.B, g.ldb, n0, g.N, k0, k_end);
  };

  if (k_begin < k_end) {
    fetch(k_begin);
    la.store(As(0));
    lb.store(Bs(0));
  }
  __syncthreads();

  const int kh = lane >> 5, l32 = lane & 31;
  int cur = 0, slab = 0;
  for (int64_t k0 = k_begin; k0 < k_end; k0 += BK, ++slab) {
    const bool more = k0 + BK < k_end;
    if (more) fetch(k0 + BK);
    const float* __restrict__ Ac = As(cur);
    const float* __restrict__ Bc = Bs(cur);
    // LDS operands for step kk+2 are requested before the MFMAs of step kk are issued
    float a[2][MB], b[2][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i) a[0][i] = Ac[kh * LDA + wm0 + i * 32 + l32];
#pragma unroll
    for (int j = 0; j < NB; ++j) b[0][j] = Bc[kh * LDB + wn0 + j * 32 + l32];
#pragma unroll
    for (int kk = 0; kk < BK; kk += 2) {
      const int cb = (kk >> 1) & 1;
      if (kk + 2 < BK) {
#pragma unroll
        for (int i = 0; i < MB; ++i) a[cb ^ 1][i] = Ac[(kk + 2 + kh) * LDA + wm0 + i * 32 + l32];
#pragma unroll
        for (int j = 0; j < NB; ++j) b[cb ^ 1][j] = Bc[(kk + 2 + kh) * LDB + wn0 + j * 32 + l32];
      }
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cb][i], b[cb][j], acc[i][j], 0, 0, 0);
    }
    if (MODE == MODE_TN && g.colsum_part && (slab % tiles_m) == tile_m && threadIdx.x < BN) {
#pragma unroll
      for (int kk = 0; kk < BK; ++kk) colsum += Bc[kk * LDB + threadIdx.x];
    }
    if (more) {
      if (NBUF == 1) __syncthreads();
      la.store(As(cur ^ (NBUF - 1)));
      lb.store(Bs(cur ^ (NBUF - 1)));
    }
    __syncthreads();
    cur ^= (NBUF - 1);
  }

  __syncthreads();   // all wavefronts are done with the operand tiles; LDS is reused below
  tile_epilogue_f32<MB, NB, MODE>(g, acc, smem, m0, n0, wm0, wn0, blockIdx.y);
  if (MODE == MODE_TN && g.colsum_part && threadIdx.x < BN && n0 + (int)threadIdx.x < g.N)
    g.colsum_part[((int64_t)blockIdx.y * tiles_m + tile_m) * g.N + n0 + threadIdx.x] = colsum;
}

// out[i] = sum_z part[z*n + i] for i < n;  out2[i] = sum_z part2[z*n2 + i] for i < n2.
// 16 column groups x 16 split lanes per workgroup: every lane issues its (few) 16-byte loads
// back to back, the 16 lanes of a column group are combined in a fixed order through LDS, so
// the result is reproducible.  The second (narrow) array is handled the same way, one float
// per column group.
constexpr int RED_COLS = 16, RED_LANES = 16;
__global__ void __launch_bounds__(RED_COLS* RED_LANES)
reduce_parts_kernel(const float* __restrict__ part, int splits, int64_t n, int vec, float* __restrict__ out,
                    int blocks1, const float* __restrict__ part2, int splits2, int64_t n2,
                    float* __restrict__ out2) {
  __shared__ f32x4 red[RED_LANES][RED_COLS];
  const int cg = threadIdx.x % RED_COLS, sl = threadIdx.x / RED_COLS;
  f32x4 s = {0.f, 0.f, 0.f, 0.f};
  if ((int)blockIdx.x < blocks1) {
    const int64_t i = ((int64_t)blockIdx.x * RED_COLS + cg) * 4;
    if (i < n) {
      if (vec) {
#pragma unroll 8
        for (int z = sl; z < splits; z += RED_LANES) s += ld4(part + (int64_t)z * n + i);
      } else {
        for (int z = sl; z < splits; z += RED_LANES)
          for (int c = 0; c < 4; ++c)
            if (i + c < n) s[c] += part[(int64_t)z * n + i + c];
      }
    }
    red[sl][cg] = s;
    __syncthreads();
    if (sl == 0 && i < n) {
      f32x4 t = red[0][cg];
      for (int k = 1; k < RED_LANES; ++k) t += red[k][cg];
      if (vec) st4(out + i, t);
      else
        for (int c = 0; c < 4; ++c)
          if (i + c < n) out[i + c] = t[c];
    }
  } else {
    const int64_t i = (int64_t)(blockIdx.x - blocks1) * RED_COLS + cg;
    if (i < n2) {
#pragma unroll 8
      for (int z = sl; z < splits2; z += RED_LANES) s[0] += part2[(int64_t)z * n2 + i];
    }
    red[sl][cg] = s;
    __syncthreads();
    if (sl == 0 && i < n2) {
      float t = red[0][cg][0];
      for (int k = 1; k < RED_LANES; ++k) t += red[k][cg][0];
      out2[i] = t;
    }
  }
}

int launch_reduce(gp_ctx* ctx, const float* part, int splits, int64_t n, float* out, const float* part2, int splits2,
                  int64_t n2, float* out2) {
  const int per_block = RED_COLS * 4;
  const int blocks1 = (int)((n + per_block - 1) / per_block);
  const int blocks2 = (int)((n2 + RED_COLS - 1) / RED_COLS);
  const int vec = (n % 4 == 0) && (((uintptr_t)part | (uintptr_t)out) & 15) == 0;
  gp_prof_scope prof(ctx, "reduce_parts", 0.0, 4.0 * ((double)(splits + 1) * n + (double)(splits2 + 1) * n2));
  reduce_parts_kernel<<<blocks1 + blocks2, RED_COLS * RED_LANES, 0, ctx->stream>>>(part, splits, n, vec, out, blocks1,
                                                                                  part2, splits2, n2, out2);
  GP_LAUNCH_CHECK(ctx, "reduce_parts_kernel");
  return GP_OK;
}

// part[b*N + c] = sum over the b-th slab of rows of X[r, c]
__global__ void colsum_part_kernel(const float* __restrict__ X, int64_t rows, int N, int64_t rows_per_block,
                                   float* __restrict__ part) {
  const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
  const int64_t r1 = r0 + rows_per_block < rows ? r0 + rows_per_block : rows;
  for (int c = threadIdx.x; c < N; c += blockDim.x) {
    float s = 0.f;
    for (int64_t r = r0; r < r1; ++r) s += X[r * N + c];
    part[(int64_t)blockIdx.x * N + c] = s;
  }
}

__global__ void ew_dsilu_mul_kernel(const float* __restrict__ g, const float* __restrict__ z,
                                    float* __restrict__ out, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = g[i] * dsilu_f(z[i]);
}

__global__ void ew_gate_bwd_kernel(const float* __restrict__ dxg, const float* __restrict__ z,
                                   const float* __restrict__ gate, float* __restrict__ dz,
                                   float* __restrict__ dgate, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float d = dxg[i], zz = z[i];
  dz[i] = d * gate[i] * dsilu_f(zz);
  dgate[i] = d * silu_f(zz);
}

__global__ void ew_add3_kernel(const float* __restrict__ a, const float* __restrict__ b,
                               const float* __restrict__ c, float* __restrict__ out, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float v = a[i] + b[i];
  if (c) v += c[i];
  out[i] = v;
}

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }
inline int nblk(int64_t n) { return (int)((n + 255) / 256); }

template <int BM, int BN, int WMS, int WNS, int MODE, bool VEC>
int launch_gemm_v(gp_ctx* ctx, gemm_args& g, int splits) {
  const int64_t tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
  if (tiles > INT32_MAX) return gp_fail(ctx, GP_BAD_ARG, "gemm: too many tiles");
  dim3 grid((unsigned)tiles, (unsigned)splits, 1);
  static char name[48];
  if (!name[0]) snprintf(name, sizeof(name), "gemm_f32_%s_%dx%d", MODE == MODE_NN ? "nn" : MODE == MODE_NT ? "nt" : "tn", BM, BN);
  const double mnk = (double)g.M * g.N * g.K;
  gp_prof_scope prof(ctx, name, 2.0 * mnk,
                     4.0 * ((double)g.M * g.K + (double)g.K * g.N + (double)g.M * g.N * (MODE == MODE_TN ? splits : 1)));
  using loadA = typename std::conditional<MODE != MODE_TN, loader_kcontig<BM, VEC>, loader_xcontig<BM, VEC>>::type;
  using loadB = typename std::conditional<MODE == MODE_NT, loader_kcontig<BN, VEC>, loader_xcontig<BN, VEC>>::type;
  constexpr size_t lds_main = sizeof(float) * NBUF * BK * (loadA::LD + loadB::LD);
  constexpr size_t lds_epi = sizeof(float) * 4 * 32 * EPI_LD;
  constexpr size_t lds = lds_main > lds_epi ? lds_main : lds_epi;
  static bool attr_set = false;
  if (!attr_set) {
    GP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_f32_kernel<BM, BN, WMS, WNS, MODE, VEC>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr_set = true;
  }
  gemm_f32_kernel<BM, BN, WMS, WNS, MODE, VEC><<<grid, THREADS, lds, ctx->stream>>>(g);
  GP_LAUNCH_CHECK(ctx, "gemm_f32_kernel");
  return GP_OK;
}

template <int BM, int BN, int WMS, int WNS, int MODE>
int launch_gemm(gp_ctx* ctx, gemm_args& g, int splits) {
  if (g.vecA && g.vecB) return launch_gemm_v<BM, BN, WMS, WNS, MODE, true>(ctx, g, splits);
  return launch_gemm_v<BM, BN, WMS, WNS, MODE, false>(ctx, g, splits);
}

// tile shape by output width
inline int tile_bn(int N) { return N > 64 ? 128 : N > 32 ? 64 : 32; }
constexpr int TILE_BM = 128;

template <int MODE>
int dispatch_gemm(gp_ctx* ctx, gemm_args& g, int splits) {
  // bf16 operands (fp32 accumulate) when the calling block asks for them; the fused column
  // sums exist only in the fp32 kernel
  if (ctx->gemm_bf16 && !(MODE == MODE_TN && g.colsum_part)) return gp_gemm_bf16_launch(ctx, MODE, &g, splits);
  if (g.a_bf16 || g.b_bf16 || g.epi.bf16)
    return gp_fail(ctx, GP_BAD_ARG, "gemm: bf16 storage is only handled by the bf16-operand kernels");
  if (g.epi.lr_a) return gp_fail(ctx, GP_BAD_ARG, "gemm: a low-rank epilogue factor is only taken by the global->LDS bf16 kernel");
  // the reduction over rows in that form has one tile shape (128 x 128) and wants 16-byte aligned rows
  if (ctx->f32_split && (MODE != MODE_TN || gp_gemm_split_tn_ok(g.M, g.N, g.vecA, g.vecB))) return gp_gemm_split_launch(ctx, MODE, &g, splits);
  if (MODE == MODE_TN) {   // tile widths the split plan (tn_plan / tile_bn) was made for
    if (g.N > 64) return launch_gemm<TILE_BM, 128, 2, 2, MODE>(ctx, g, splits);
    if (g.N > 32) return launch_gemm<TILE_BM, 64, 2, 2, MODE>(ctx, g, splits);
    return launch_gemm<TILE_BM, 32, 4, 1, MODE>(ctx, g, splits);
  }
  // Row-panel GEMMs: narrower tiles than the MFMA rate alone would ask for.  The layers here have K <= a few
  // hundred, so a workgroup is mostly prologue (first loads) and epilogue; more, smaller workgroups per CU let
  // those phases of one workgroup overlap the main loop of another (measured at E = 43 372 and 300 000).
  if (g.N > 64) return launch_gemm<TILE_BM, 64, 2, 2, MODE>(ctx, g, splits);
  return launch_gemm<TILE_BM, 32, 4, 1, MODE>(ctx, g, splits);
}

int check_epi(gp_ctx* ctx, const gp_epilogue& e) {
  GP_REQUIRE(ctx, e.out || e.out2 || e.save_pre, "gemm: epilogue has no output");
  GP_REQUIRE(ctx, e.act != 2 || e.zsrc, "gemm: act=2 needs zsrc");
  GP_REQUIRE(ctx, !e.out2 || e.z2src, "gemm: out2 needs z2src");
  return GP_OK;
}

bool epi_vec_ok(const gp_epilogue& e, int N) {
  return N % 4 == 0 && aligned16(e.bias) && aligned16(e.add_pre) && aligned16(e.save_pre) && aligned16(e.zsrc) &&
         aligned16(e.mul) && aligned16(e.add_post) && aligned16(e.out) && aligned16(e.out2) && aligned16(e.z2src);
}

struct tn_plan_t {
  int splits, tiles_m, tiles_n;
  int64_t per;
};

// Split the reduction so that about three workgroups per CU exist (what the register file holds), each
// reducing >= 256 rows.
// `light`: the three-plane kernel multiplies 2.7 times faster, so what its workgroups wait for is the partial sums they
// write (as many bytes as the operands at 169 splits of 43 372 rows): two workgroups per CU instead of three, a third fewer
// partial sums (configuration 2: 44 -> 41 us per weight gradient, 10 -> 9 us per reduction)
tn_plan_t tn_plan(int64_t rows, int M, int N, bool light = false) {
  tn_plan_t p;
  p.tiles_m = (M + TILE_BM - 1) / TILE_BM;
  p.tiles_n = (N + tile_bn(N) - 1) / tile_bn(N);
  const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
  int64_t s = ((light ? 512 : 768) + tiles - 1) / tiles;
  const int64_t max_s = (rows + 255) / 256;
  if (s > max_s) s = max_s;
  if (s < 1) s = 1;
  int64_t per = (rows + s - 1) / s;
  per = (per + BK - 1) / BK * BK;
  s = (rows + per - 1) / per;
  if (s < 1) s = 1;
  p.splits = (int)s;
  p.per = per;
  return p;
}

}  // namespace

int gp_gemm_nn(gp_ctx* ctx, const float* A, const float* B, int64_t M, int N, int K, const gp_epilogue& epi, int a_bf16,
               int b_bf16) {
  GP_REQUIRE(ctx, A && B && M >= 0 && N > 0 && K > 0, "gemm_nn: bad arguments");
  GP_TRY(check_epi(ctx, epi));
  if (M == 0) return GP_OK;
  gemm_args g{};
  g.A = A; g.B = B; g.M = M; g.N = N; g.K = K; g.lda = K; g.ldb = N;
  g.a_bf16 = a_bf16;
  g.b_bf16 = b_bf16;
  g.vecA = (K % (a_bf16 ? 8 : 4) == 0) && aligned16(A);
  g.vecB = b_bf16 ? (N % 2 == 0 && ((uintptr_t)B & 3) == 0) : (N % 4 == 0) && aligned16(B);
  g.epi = epi;
  g.vecC = epi_vec_ok(epi, N);
  g.epi_kind = gp_epilogue_kind(g.epi, g.vecC);
  g.epi_mask = gp_epilogue_mask(g.epi, g.vecC);
  return dispatch_gemm<MODE_NN>(ctx, g, 1);
}

int gp_gemm_nt(gp_ctx* ctx, const float* A, const float* Bt, int64_t M, int N, int K, const gp_epilogue& epi, int a_bf16,
               int b_bf16) {
  GP_REQUIRE(ctx, A && Bt && M >= 0 && N > 0 && K > 0, "gemm_nt: bad arguments");
  GP_TRY(check_epi(ctx, epi));
  if (M == 0) return GP_OK;
  gemm_args g{};
  g.A = A; g.B = Bt; g.M = M; g.N = N; g.K = K; g.lda = K; g.ldb = K;
  g.a_bf16 = a_bf16;
  g.b_bf16 = b_bf16;
  g.vecA = (K % (a_bf16 ? 8 : 4) == 0) && aligned16(A);
  g.vecB = (K % (b_bf16 ? 8 : 4) == 0) && aligned16(Bt);
  g.epi = epi;
  g.vecC = epi_vec_ok(epi, N);
  g.epi_kind = gp_epilogue_kind(g.epi, g.vecC);
  g.epi_mask = gp_epilogue_mask(g.epi, g.vecC);
  return dispatch_gemm<MODE_NT>(ctx, g, 1);
}

// the conditions of the global->LDS bf16 kernel on the shape (its operands must also be bf16 and 16-byte aligned)
bool gp_gemm_nt_takes_lowrank(const gp_ctx* ctx, int64_t M, int N, int K) {
  return ctx->gemm_bf16 && M >= 8192 && N > 128 && N % 4 == 0 && K % 64 == 0 && K >= 128;
}

// whether gp_gemm_nt2 can run as one launch (the conditions of the global->LDS bf16 kernel)
bool gp_gemm_nt2_fused(const gp_ctx* ctx, const float* A, const float* Bt, const float* A2, const float* B2t, int64_t M, int N,
                       int K, int a_bf16, int b_bf16) {
  return ctx->gemm_bf16 && a_bf16 && b_bf16 && M >= 8192 && N > 128 && K % 64 == 0 && K >= 128 && aligned16(A) && aligned16(Bt) &&
         aligned16(A2) && aligned16(B2t);
}

int gp_gemm_nt2(gp_ctx* ctx, const float* A, const float* Bt, const float* A2, const float* B2t, int64_t M, int N, int K,
                float* out, int a_bf16, int b_bf16, int out_bf16) {
  GP_REQUIRE(ctx, A && Bt && A2 && B2t && out && M >= 0 && N > 0 && K > 0, "gemm_nt2: bad arguments");
  GP_REQUIRE(ctx, !out_bf16 || ctx->gemm_bf16, "gemm_nt2: a bf16 result needs the bf16-operand kernels");
  if (M == 0) return GP_OK;
  gp_epilogue e;
  e.out = out;
  e.bf16 = out_bf16 ? EPI_BF_OUT : 0u;
  if (!gp_gemm_nt2_fused(ctx, A, Bt, A2, B2t, M, N, K, a_bf16, b_bf16)) {
    GP_TRY(gp_gemm_nt(ctx, A, Bt, M, N, K, e, a_bf16, b_bf16));
    e.add_post = out;
    e.bf16 = out_bf16 ? (EPI_BF_OUT | EPI_BF_ADD_POST) : 0u;
    return gp_gemm_nt(ctx, A2, B2t, M, N, K, e, a_bf16, b_bf16);
  }
  gemm_args g{};
  g.A = A; g.B = Bt; g.A2 = A2; g.B2 = B2t; g.M = M; g.N = N; g.K = 2 * K; g.lda = K; g.ldb = K;
  g.a_bf16 = a_bf16;
  g.b_bf16 = b_bf16;
  g.vecA = g.vecB = 1;
  g.epi = e;
  g.vecC = epi_vec_ok(e, N);
  g.epi_kind = gp_epilogue_kind(g.epi, g.vecC);
  g.epi_mask = gp_epilogue_mask(g.epi, g.vecC);
  return dispatch_gemm<MODE_NT>(ctx, g, 1);
}

size_t gp_gemm_tn_scratch(int64_t rows, int M, int N) {
  tn_plan_t p = tn_plan(rows, M, N);   // the plan with the most splits: the buffer serves either one
  const size_t a = gp_align((size_t)p.splits * M * N * sizeof(float)) + gp_align((size_t)p.splits * p.tiles_m * N * sizeof(float));
  const size_t b = gp_align((size_t)gp_gemm_bf16_tn_dl_splits(rows, M, N) * M * N * sizeof(float));   // the bf16 kernel with its own plan
  return a > b ? a : b;
}

int gp_gemm_tn(gp_ctx* ctx, const float* A, const float* B, int64_t rows, int M, int N, float* out,
               float* colsum_out, float* part, size_t part_bytes, int a_bf16, int b_bf16) {
  GP_REQUIRE(ctx, !colsum_out || !(a_bf16 || b_bf16), "gemm_tn: column sums need fp32 operands");
  GP_REQUIRE(ctx, A && B && out && rows >= 0 && M > 0 && N > 0, "gemm_tn: bad arguments");
  if (rows == 0) {
    GP_HIP(ctx, (hipError_t)gp_zero_async(ctx->stream, out, sizeof(float) * M * N));
    if (colsum_out) GP_HIP(ctx, (hipError_t)gp_zero_async(ctx->stream, colsum_out, sizeof(float) * N));
    return GP_OK;
  }
  if (rows > INT32_MAX) return gp_fail(ctx, GP_INT32_OVERFLOW, "gemm_tn: too many rows");
  const bool vA = a_bf16 ? (M % 2 == 0 && ((uintptr_t)A & 3) == 0) : (M % 4 == 0) && aligned16(A);
  const bool vB = b_bf16 ? (N % 2 == 0 && ((uintptr_t)B & 3) == 0) : (N % 4 == 0) && aligned16(B);
  const bool light = !ctx->gemm_bf16 && ctx->f32_split && !a_bf16 && !b_bf16 && gp_gemm_split_tn_ok(M, N, vA, vB);
  const tn_plan_t p = tn_plan(rows, M, N, light);
  const size_t need = gp_gemm_tn_scratch(rows, M, N);
  if (!part || part_bytes < need) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "gemm_tn: scratch %zu < %zu", part_bytes, need);
  gemm_args g{};
  g.A = A; g.B = B; g.M = M; g.N = N; g.K = (int)rows; g.lda = M; g.ldb = N;
  g.a_bf16 = a_bf16;
  g.b_bf16 = b_bf16;
  // fp32 operand: 16-byte loads legal; bf16 operand (4-byte loads of column pairs): even extent, 4-byte aligned
  g.vecA = vA;
  g.vecB = vB;
  g.k_per_split = p.per;
  g.part = part;
  g.vecC = (N % 4 == 0) && aligned16(part) && ((size_t)M * N % 4 == 0);
  if (ctx->gemm_bf16 && !colsum_out) {
    const int s_dl = gp_gemm_bf16_tn_dl_splits(rows, M, N);
    if (s_dl > 0 && gp_gemm_bf16_tn_dl_ok(&g)) {
      GP_TRY(gp_gemm_bf16_tn_dl(ctx, &g, s_dl));
      return launch_reduce(ctx, part, s_dl, (int64_t)M * N, out, nullptr, 0, 0, nullptr);
    }
  }
  float* cpart = (float*)((char*)part + gp_align((size_t)p.splits * M * N * sizeof(float)));
  g.colsum_part = colsum_out ? cpart : nullptr;
  GP_TRY(dispatch_gemm<MODE_TN>(ctx, g, p.splits));
  const int64_t n1 = (int64_t)M * N, n2 = colsum_out ? N : 0;
  return launch_reduce(ctx, part, p.splits, n1, out, cpart, p.splits * p.tiles_m, n2, colsum_out);
}

static void colsum_plan(int64_t rows, int* blocks, int64_t* per) {
  int64_t b = (rows + 127) / 128;
  if (b > 1024) b = 1024;
  if (b < 1) b = 1;
  *per = (rows + b - 1) / b;
  *blocks = (int)((rows + *per - 1) / *per);
  if (*blocks < 1) *blocks = 1;
}

size_t gp_colsum_scratch(int64_t rows, int N) {
  int b; int64_t p;
  colsum_plan(rows, &b, &p);
  return gp_align((size_t)b * N * sizeof(float));
}

int gp_colsum(gp_ctx* ctx, const float* X, int64_t rows, int N, float* out, float* part, size_t part_bytes) {
  GP_REQUIRE(ctx, X && out && rows >= 0 && N > 0, "colsum: bad arguments");
  int blocks; int64_t per;
  colsum_plan(rows, &blocks, &per);
  size_t need = (size_t)blocks * N * sizeof(float);
  if (!part || part_bytes < need) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "colsum: scratch %zu < %zu", part_bytes, need);
  {
    gp_prof_scope prof(ctx, "colsum_part", 0.0, 4.0 * (double)rows * N);
    colsum_part_kernel<<<blocks, 256, 0, ctx->stream>>>(X, rows, N, per, part);
    GP_LAUNCH_CHECK(ctx, "colsum_part_kernel");
  }
  return gp_reduce_parts(ctx, part, blocks, N, out);
}

int gp_reduce_parts(gp_ctx* ctx, const float* part, int splits, int64_t n, float* out) {
  if (n == 0) return GP_OK;
  return launch_reduce(ctx, part, splits, n, out, nullptr, 0, 0, nullptr);
}

int gp_ew_dsilu_mul(gp_ctx* ctx, const float* g, const float* z, float* out, int64_t n) {
  if (n == 0) return GP_OK;
  gp_prof_scope prof(ctx, "ew_dsilu_mul", 0.0, 12.0 * (double)n);
  ew_dsilu_mul_kernel<<<nblk(n), 256, 0, ctx->stream>>>(g, z, out, n);
  GP_LAUNCH_CHECK(ctx, "ew_dsilu_mul_kernel");
  return GP_OK;
}

int gp_ew_gate_bwd(gp_ctx* ctx, const float* dxg, const float* z, const float* gate, float* dz, float* dgate, int64_t n) {
  if (n == 0) return GP_OK;
  gp_prof_scope prof(ctx, "ew_gate_bwd", 0.0, 20.0 * (double)n);
  ew_gate_bwd_kernel<<<nblk(n), 256, 0, ctx->stream>>>(dxg, z, gate, dz, dgate, n);
  GP_LAUNCH_CHECK(ctx, "ew_gate_bwd_kernel");
  return GP_OK;
}

int gp_ew_add3(gp_ctx* ctx, const float* a, const float* b, const float* c, float* out, int64_t n) {
  if (n == 0) return GP_OK;
  gp_prof_scope prof(ctx, "ew_add3", 0.0, (c ? 16.0 : 12.0) * (double)n);
  ew_add3_kernel<<<nblk(n), 256, 0, ctx->stream>>>(a, b, c, out, n);
  GP_LAUNCH_CHECK(ctx, "ew_add3_kernel");
  return GP_OK;
}

extern "C" int gp_linear_forward(gp_ctx* ctx, const float* x, const float* W, const float* b, int64_t rows,
                                 int32_t k, int32_t n, int32_t act, float* out) {
  if (!ctx) return GP_BAD_ARG;
  GP_REQUIRE(ctx, x && W && out && rows >= 0 && k > 0 && n > 0, "gp_linear_forward: bad arguments");
  GP_REQUIRE(ctx, act == 0 || act == 1, "gp_linear_forward: act must be 0 or 1");
  GP_HIP(ctx, hipSetDevice(ctx->device));
  gp_epilogue e;
  e.bias = b;
  e.act = act;
  e.out = out;
  return gp_gemm_nn(ctx, x, W, rows, n, k, e);
}

extern "C" int gp_linear_forward_bf16(gp_ctx* ctx, const float* x, const float* W, const float* b, int64_t rows,
                                      int32_t k, int32_t n, int32_t act, float* out) {
  if (!ctx) return GP_BAD_ARG;
  const bool prev = ctx->gemm_bf16;
  ctx->gemm_bf16 = true;
  const int rc = gp_linear_forward(ctx, x, W, b, rows, k, n, act, out);
  ctx->gemm_bf16 = prev;
  return rc;
}
