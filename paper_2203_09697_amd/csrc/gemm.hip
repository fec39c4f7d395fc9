// fp32 GEMM on the matrix cores (v_mfma_f32_32x32x2_f32) with fused epilogues, plus the small
// reductions and elementwise kernels the edge MLPs need (EdgeUpdate of paper Sec. 2.1 / 3.3).
//
// Tiling: a 256-thread workgroup (4 wavefronts of 64) owns a BM x BN tile of C; the K loop
// advances 16 at a time through LDS tiles As[k][m], Bs[k][n] (k-major, so the 32 lanes that
// feed one MFMA operand read consecutive LDS words).  Each wavefront owns (BM/WAVES_M) x
// (BN/WAVES_N) of the tile as 32x32 MFMA blocks.  The next K-slab is fetched into registers
// while the current one is multiplied.
#include <stdarg.h>

#include <type_traits>

#include "gemm.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int BK = 16;
constexpr int THREADS = 256;
enum { MODE_NN = 0, MODE_NT = 1, MODE_TN = 2 };

struct gemm_args {
  const float* A;
  const float* B;
  int64_t M;   // rows of C
  int N, K;    // cols of C, contraction length (TN: total rows to reduce)
  int64_t lda, ldb;
  int vecA, vecB;          // 16-byte vector loads are legal for this operand
  int64_t k_per_split;     // TN only
  float* part;             // TN only: [splits, M, N]
  gp_epilogue epi;
};

__device__ __forceinline__ void epilogue_store(const gp_epilogue& e, int64_t row, int col, int n, float v) {
  const int64_t o = row * n + col;
  if (e.bias) v += e.bias[col];
  if (e.add_pre) v += e.add_pre[o];
  if (e.save_pre) e.save_pre[o] = v;
  if (e.act == 1) v = silu_f(v);
  else if (e.act == 2) v *= dsilu_f(e.zsrc[o]);
  if (e.mul) v *= e.mul[o];
  if (e.add_post) v += e.add_post[o];
  v *= e.scale;
  if (e.out) e.out[o] = v;
  if (e.out2) e.out2[o] = v * dsilu_f(e.z2src[o]);
}

// Workgroup ids are dealt round-robin to the 8 XCDs; renumber them so that each XCD works on
// a contiguous range of tiles and neighbouring tiles (same A rows) share that XCD's L2.
__device__ __forceinline__ int xcd_remap(int bid, int n) {
  const int q = n >> 3, r = n & 7;
  const int x = bid & 7, i = bid >> 3;
  return x * q + (x < r ? x : r) + i;
}

// Source has the contraction index contiguous: tile of X rows by BK k's, stored transposed.
template <int X>
struct loader_kcontig {
  static constexpr int TOTAL = X * BK / 4;
  static constexpr int NV = (TOTAL + THREADS - 1) / THREADS;
  f32x4 r[NV];
  __device__ __forceinline__ void fetch(const float* __restrict__ src, int64_t ld, int64_t row0,
                                        int64_t n_rows, int k0, int k_end, int vec) {
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      const int row = idx >> 2, kq = (idx & 3) * 4;
      const int64_t gr = (TOTAL % THREADS == 0 || idx < TOTAL) ? row0 + row : n_rows;
      const int gk = k0 + kq;
      f32x4 v = {0.f, 0.f, 0.f, 0.f};
      if (gr < n_rows) {
        const float* p = src + gr * ld + gk;
        if (vec) {
          if (gk < k_end) v = *reinterpret_cast<const f32x4*>(p);
        } else {
#pragma unroll
          for (int c = 0; c < 4; ++c)
            if (gk + c < k_end) v[c] = p[c];
        }
      }
      r[it] = v;
    }
  }
  template <int LD>
  __device__ __forceinline__ void store(float* __restrict__ S) const {
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      const int row = idx >> 2, kq = (idx & 3) * 4;
      if (TOTAL % THREADS != 0 && idx >= TOTAL) continue;
#pragma unroll
      for (int c = 0; c < 4; ++c) S[(kq + c) * LD + row] = r[it][c];
    }
  }
};

// Source has the tile's m/n index contiguous: BK rows by X columns, stored as is.
template <int X>
struct loader_xcontig {
  static constexpr int TOTAL = X * BK / 4;
  static constexpr int NV = (TOTAL + THREADS - 1) / THREADS;
  f32x4 r[NV];
  __device__ __forceinline__ void fetch(const float* __restrict__ src, int64_t ld, int64_t x0,
                                        int64_t n_x, int64_t k0, int64_t k_end, int vec) {
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      const int k = idx / (X / 4), xq = (idx % (X / 4)) * 4;
      const int64_t gk = (TOTAL % THREADS == 0 || idx < TOTAL) ? k0 + k : k_end, gx = x0 + xq;
      f32x4 v = {0.f, 0.f, 0.f, 0.f};
      if (gk < k_end) {
        const float* p = src + gk * ld + gx;
        if (vec) {
          if (gx < n_x) v = *reinterpret_cast<const f32x4*>(p);
        } else {
#pragma unroll
          for (int c = 0; c < 4; ++c)
            if (gx + c < n_x) v[c] = p[c];
        }
      }
      r[it] = v;
    }
  }
  template <int LD>
  __device__ __forceinline__ void store(float* __restrict__ S) const {
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      const int k = idx / (X / 4), xq = (idx % (X / 4)) * 4;
      if (TOTAL % THREADS != 0 && idx >= TOTAL) continue;
      *reinterpret_cast<f32x4*>(&S[k * LD + xq]) = r[it];
    }
  }
};

template <int BM, int BN, int WAVES_M, int WAVES_N, int MODE>
__global__ void __launch_bounds__(THREADS)
gemm_f32_kernel(const gemm_args g) {
  static_assert(WAVES_M * WAVES_N == 4, "four wavefronts per workgroup");
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int MB = WM / 32, NB = WN / 32;
  constexpr bool A_KC = (MODE != MODE_TN);   // A source has k contiguous
  constexpr bool B_KC = (MODE == MODE_NT);
  constexpr int LDA = BM + (A_KC ? 2 : 4);
  constexpr int LDB = BN + (B_KC ? 2 : 4);
  __shared__ __attribute__((aligned(16))) float As[BK * LDA];
  __shared__ __attribute__((aligned(16))) float Bs[BK * LDB];

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

  f32x16 acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  typename std::conditional<A_KC, loader_kcontig<BM>, loader_xcontig<BM>>::type la;
  typename std::conditional<B_KC, loader_kcontig<BN>, loader_xcontig<BN>>::type lb;

  auto fetch = [&](int64_t k0) {
    if constexpr (A_KC) la.fetch(g.A, g.lda, m0, g.M, (int)k0, (int)k_end, g.vecA);
    else la.fetch(g.A, g.lda, m0, g.M, k0, k_end, g.vecA);
    if constexpr (B_KC) lb.fetch(g.B, g.ldb, n0, g.N, (int)k0, (int)k_end, g.vecB);
    else lb.fetch(g.B, g.ldb, n0, g.N, k0, k_end, g.vecB);
  };

  if (k_begin < k_end) {
    fetch(k_begin);
    la.template store<LDA>(As);
    lb.template store<LDB>(Bs);
  }
  __syncthreads();

  const int kh = lane >> 5, l32 = lane & 31;
  for (int64_t k0 = k_begin; k0 < k_end; k0 += BK) {
    const bool more = k0 + BK < k_end;
    if (more) fetch(k0 + BK);
#pragma unroll
    for (int kk = 0; kk < BK; kk += 2) {
      float a[MB], b[NB];
#pragma unroll
      for (int i = 0; i < MB; ++i) a[i] = As[(kk + kh) * LDA + wm0 + i * 32 + l32];
#pragma unroll
      for (int j = 0; j < NB; ++j) b[j] = Bs[(kk + kh) * LDB + wn0 + j * 32 + l32];
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
    if (more) {
      la.template store<LDA>(As);
      lb.template store<LDB>(Bs);
    }
    __syncthreads();
  }

  // C layout of the 32x32 block: register v of lane l holds row 8*(v/4) + 4*(l/32) + v%4, col l%32
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const int col = n0 + wn0 + j * 32 + l32;
      if (col >= g.N) continue;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t row = m0 + wm0 + i * 32 + (v >> 2) * 8 + kh * 4 + (v & 3);
        if (row >= g.M) continue;
        if (MODE == MODE_TN) g.part[((int64_t)blockIdx.y * g.M + row) * g.N + col] = acc[i][j][v];
        else epilogue_store(g.epi, row, col, g.N, acc[i][j][v]);
      }
    }
}

// out[i] = sum_z part[z*n + i]
__global__ void reduce_parts_kernel(const float* __restrict__ part, int splits, int64_t n, float* __restrict__ out) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float s = 0.f;
  for (int z = 0; z < splits; ++z) s += part[(int64_t)z * n + i];
  out[i] = s;
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

template <int BM, int BN, int WMS, int WNS, int MODE>
int launch_gemm(gp_ctx* ctx, gemm_args& g, int splits) {
  const int64_t tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
  if (tiles > INT32_MAX) return gp_fail(ctx, GP_BAD_ARG, "gemm: too many tiles");
  dim3 grid((unsigned)tiles, (unsigned)splits, 1);
  gemm_f32_kernel<BM, BN, WMS, WNS, MODE><<<grid, THREADS, 0, ctx->stream>>>(g);
  GP_LAUNCH_CHECK(ctx, "gemm_f32_kernel");
  return GP_OK;
}

template <int MODE>
int dispatch_gemm(gp_ctx* ctx, gemm_args& g, int splits) {
  if (g.N > 64) return launch_gemm<128, 128, 2, 2, MODE>(ctx, g, splits);
  if (g.N > 32) return launch_gemm<128, 64, 2, 2, MODE>(ctx, g, splits);
  return launch_gemm<128, 32, 4, 1, MODE>(ctx, g, splits);
}

int check_epi(gp_ctx* ctx, const gp_epilogue& e) {
  GP_REQUIRE(ctx, e.out || e.out2 || e.save_pre, "gemm: epilogue has no output");
  GP_REQUIRE(ctx, e.act != 2 || e.zsrc, "gemm: act=2 needs zsrc");
  GP_REQUIRE(ctx, !e.out2 || e.z2src, "gemm: out2 needs z2src");
  return GP_OK;
}

}  // namespace

int gp_gemm_nn(gp_ctx* ctx, const float* A, const float* B, int64_t M, int N, int K, const gp_epilogue& epi) {
  GP_REQUIRE(ctx, A && B && M >= 0 && N > 0 && K > 0, "gemm_nn: bad arguments");
  GP_TRY(check_epi(ctx, epi));
  if (M == 0) return GP_OK;
  gemm_args g{};
  g.A = A; g.B = B; g.M = M; g.N = N; g.K = K; g.lda = K; g.ldb = N;
  g.vecA = (K % 4 == 0) && aligned16(A);
  g.vecB = (N % 4 == 0) && aligned16(B);
  g.epi = epi;
  return dispatch_gemm<MODE_NN>(ctx, g, 1);
}

int gp_gemm_nt(gp_ctx* ctx, const float* A, const float* Bt, int64_t M, int N, int K, const gp_epilogue& epi) {
  GP_REQUIRE(ctx, A && Bt && M >= 0 && N > 0 && K > 0, "gemm_nt: bad arguments");
  GP_TRY(check_epi(ctx, epi));
  if (M == 0) return GP_OK;
  gemm_args g{};
  g.A = A; g.B = Bt; g.M = M; g.N = N; g.K = K; g.lda = K; g.ldb = K;
  g.vecA = (K % 4 == 0) && aligned16(A);
  g.vecB = (K % 4 == 0) && aligned16(Bt);
  g.epi = epi;
  return dispatch_gemm<MODE_NT>(ctx, g, 1);
}

static void tn_plan(int64_t rows, int M, int N, int* splits, int64_t* per) {
  // enough workgroups to cover the chip a few times over, each reducing at least 256 rows
  const int64_t tiles = (int64_t)((M + 127) / 128) * ((N + (N > 64 ? 127 : N > 32 ? 63 : 31)) / (N > 64 ? 128 : N > 32 ? 64 : 32));
  int64_t s = (1024 + tiles - 1) / tiles;
  int64_t max_s = (rows + 255) / 256;
  if (s > max_s) s = max_s;
  if (s < 1) s = 1;
  int64_t p = (rows + s - 1) / s;
  p = (p + BK - 1) / BK * BK;
  s = (rows + p - 1) / p;
  if (s < 1) s = 1;
  *splits = (int)s;
  *per = p;
}

size_t gp_gemm_tn_scratch(int64_t rows, int M, int N) {
  int s; int64_t p;
  tn_plan(rows, M, N, &s, &p);
  return gp_align((size_t)s * M * N * sizeof(float));
}

int gp_gemm_tn(gp_ctx* ctx, const float* A, const float* B, int64_t rows, int M, int N, float* out,
               float* part, size_t part_bytes) {
  GP_REQUIRE(ctx, A && B && out && rows >= 0 && M > 0 && N > 0, "gemm_tn: bad arguments");
  if (rows == 0) {
    GP_HIP(ctx, hipMemsetAsync(out, 0, sizeof(float) * M * N, ctx->stream));
    return GP_OK;
  }
  if (rows > INT32_MAX) return gp_fail(ctx, GP_INT32_OVERFLOW, "gemm_tn: too many rows");
  int splits; int64_t per;
  tn_plan(rows, M, N, &splits, &per);
  size_t need = (size_t)splits * M * N * sizeof(float);
  if (!part || part_bytes < need) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "gemm_tn: scratch %zu < %zu", part_bytes, need);
  gemm_args g{};
  g.A = A; g.B = B; g.M = M; g.N = N; g.K = (int)rows; g.lda = M; g.ldb = N;
  g.vecA = (M % 4 == 0) && aligned16(A);
  g.vecB = (N % 4 == 0) && aligned16(B);
  g.k_per_split = per;
  g.part = part;
  GP_TRY(dispatch_gemm<MODE_TN>(ctx, g, splits));
  reduce_parts_kernel<<<nblk((int64_t)M * N), 256, 0, ctx->stream>>>(part, splits, (int64_t)M * N, out);
  GP_LAUNCH_CHECK(ctx, "reduce_parts_kernel");
  return GP_OK;
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
  colsum_part_kernel<<<blocks, 256, 0, ctx->stream>>>(X, rows, N, per, part);
  GP_LAUNCH_CHECK(ctx, "colsum_part_kernel");
  reduce_parts_kernel<<<nblk(N), 256, 0, ctx->stream>>>(part, blocks, N, out);
  GP_LAUNCH_CHECK(ctx, "reduce_parts_kernel");
  return GP_OK;
}

int gp_reduce_parts(gp_ctx* ctx, const float* part, int splits, int64_t n, float* out) {
  if (n == 0) return GP_OK;
  reduce_parts_kernel<<<nblk(n), 256, 0, ctx->stream>>>(part, splits, n, out);
  GP_LAUNCH_CHECK(ctx, "reduce_parts_kernel");
  return GP_OK;
}

int gp_ew_dsilu_mul(gp_ctx* ctx, const float* g, const float* z, float* out, int64_t n) {
  if (n == 0) return GP_OK;
  ew_dsilu_mul_kernel<<<nblk(n), 256, 0, ctx->stream>>>(g, z, out, n);
  GP_LAUNCH_CHECK(ctx, "ew_dsilu_mul_kernel");
  return GP_OK;
}

int gp_ew_gate_bwd(gp_ctx* ctx, const float* dxg, const float* z, const float* gate, float* dz, float* dgate, int64_t n) {
  if (n == 0) return GP_OK;
  ew_gate_bwd_kernel<<<nblk(n), 256, 0, ctx->stream>>>(dxg, z, gate, dz, dgate, n);
  GP_LAUNCH_CHECK(ctx, "ew_gate_bwd_kernel");
  return GP_OK;
}

int gp_ew_add3(gp_ctx* ctx, const float* a, const float* b, const float* c, float* out, int64_t n) {
  if (n == 0) return GP_OK;
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
