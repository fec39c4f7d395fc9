// Streaming TripletUpdate + TripletAggr (paper Sec. 3.3) with a materialised per-triplet factor
// s[T,F]: HBM-bound kernels.  16-byte accesses: a row of F floats is covered by F/4 lanes, so
// one wavefront instruction moves 64/(F/4) rows; several row groups are kept in flight.
//   forward   a[e,:]  = sum_{t in seg_ji(e)} x[kj(t),:] * s[t,:]
//   backward  gx[e',:] = sum_{q in seg_kj(e')} ga[ji(q),:] * s[perm(q),:];  gs[t,:] = ga[ji(t),:] * x[kj(t),:]
// Per triplet the forward streams F*4 bytes of s and 4 bytes of index; x rows are re-used ~deg
// times and come from cache.
#include <stdarg.h>

#include "triplet.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int WPB = 4;
constexpr int UNR = 4;

__device__ __forceinline__ f32x4 ld4(const float* p) { return *reinterpret_cast<const f32x4*>(p); }
__device__ __forceinline__ void st4(float* p, f32x4 v) { *reinterpret_cast<f32x4*>(p) = v; }

// LPR = lanes per row = F/4 (power of two); RPI = rows per instruction = 64 / LPR
template <int LPR>
__device__ __forceinline__ f32x4 reduce_rows(f32x4 v) {
#pragma unroll
  for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
    for (int c = 0; c < 4; ++c) v[c] += __shfl_xor(v[c], off, 64);
  return v;
}

template <int LPR>
__global__ void __launch_bounds__(WPB * 64)
stream_fwd4_kernel(const int32_t* __restrict__ seg, const int32_t* __restrict__ idx_kj, const float* __restrict__ x,
                   const float* __restrict__ s, int64_t E, float* __restrict__ a) {
  constexpr int RPI = 64 / LPR, F = LPR * 4;
  const int lane = threadIdx.x & 63;
  const int64_t e = (int64_t)blockIdx.x * WPB + (threadIdx.x >> 6);
  if (e >= E) return;
  const int r = lane / LPR, c4 = (lane % LPR) * 4;
  const int64_t t0 = seg[e], t1 = seg[e + 1];
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int64_t t = t0 + r; t < t1; t += RPI * UNR) {
    f32x4 xv[UNR], sv[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int64_t tt = t + u * RPI;
      const bool ok = tt < t1;
      const int64_t tc = ok ? tt : t;
      const int64_t kj = idx_kj[tc];
      xv[u] = ld4(x + kj * F + c4);
      sv[u] = ld4(s + tc * F + c4);
      if (!ok) sv[u] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) acc += xv[u] * sv[u];
  }
  acc = reduce_rows<LPR>(acc);
  if (r == 0) st4(a + e * F + c4, acc);
}

template <int LPR>
__global__ void __launch_bounds__(WPB * 64)
stream_bwd_x4_kernel(const int32_t* __restrict__ seg_kj, const int32_t* __restrict__ idx_ji_kj,
                     const int32_t* __restrict__ perm_kj, const float* __restrict__ s, const float* __restrict__ ga,
                     int64_t E, float* __restrict__ gx) {
  constexpr int RPI = 64 / LPR, F = LPR * 4;
  const int lane = threadIdx.x & 63;
  const int64_t e = (int64_t)blockIdx.x * WPB + (threadIdx.x >> 6);
  if (e >= E) return;
  const int r = lane / LPR, c4 = (lane % LPR) * 4;
  const int64_t q0 = seg_kj[e], q1 = seg_kj[e + 1];
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int64_t q = q0 + r; q < q1; q += RPI * UNR) {
    f32x4 gv[UNR], sv[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int64_t qq = q + u * RPI;
      const bool ok = qq < q1;
      const int64_t qc = ok ? qq : q;
      gv[u] = ld4(ga + (int64_t)idx_ji_kj[qc] * F + c4);
      sv[u] = ld4(s + (int64_t)perm_kj[qc] * F + c4);
      if (!ok) sv[u] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) acc += gv[u] * sv[u];
  }
  acc = reduce_rows<LPR>(acc);
  if (r == 0) st4(gx + e * F + c4, acc);
}

template <int LPR>
__global__ void __launch_bounds__(WPB * 64)
stream_bwd_s4_kernel(const int32_t* __restrict__ seg, const int32_t* __restrict__ idx_kj, const float* __restrict__ x,
                     const float* __restrict__ ga, int64_t E, float* __restrict__ gs) {
  constexpr int RPI = 64 / LPR, F = LPR * 4;
  const int lane = threadIdx.x & 63;
  const int64_t e = (int64_t)blockIdx.x * WPB + (threadIdx.x >> 6);
  if (e >= E) return;
  const int r = lane / LPR, c4 = (lane % LPR) * 4;
  const f32x4 g = ld4(ga + e * F + c4);
  const int64_t t0 = seg[e], t1 = seg[e + 1];
  for (int64_t t = t0 + r; t < t1; t += RPI * UNR) {
    f32x4 xv[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int64_t tt = t + u * RPI;
      xv[u] = ld4(x + (int64_t)idx_kj[tt < t1 ? tt : t] * F + c4);
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int64_t tt = t + u * RPI;
      if (tt < t1) st4(gs + tt * F + c4, g * xv[u]);
    }
  }
}

inline unsigned blocks(int64_t E) { return (unsigned)((E + WPB - 1) / WPB); }
inline bool fast_ok(int F, const void* a, const void* b, const void* c) {
  const bool pow2 = F >= 4 && F <= 256 && (F & (F - 1)) == 0;
  return pow2 && ((((uintptr_t)a) | ((uintptr_t)b) | ((uintptr_t)c)) & 15) == 0;
}

}  // namespace

#define GP_STREAM_DISPATCH(F, KERNEL, ...)                                       \
  switch ((F) / 4) {                                                             \
    case 1: KERNEL<1><<<blocks(E), WPB * 64, 0, ctx->stream>>>(__VA_ARGS__); break;   \
    case 2: KERNEL<2><<<blocks(E), WPB * 64, 0, ctx->stream>>>(__VA_ARGS__); break;   \
    case 4: KERNEL<4><<<blocks(E), WPB * 64, 0, ctx->stream>>>(__VA_ARGS__); break;   \
    case 8: KERNEL<8><<<blocks(E), WPB * 64, 0, ctx->stream>>>(__VA_ARGS__); break;   \
    case 16: KERNEL<16><<<blocks(E), WPB * 64, 0, ctx->stream>>>(__VA_ARGS__); break; \
    case 32: KERNEL<32><<<blocks(E), WPB * 64, 0, ctx->stream>>>(__VA_ARGS__); break; \
    default: KERNEL<64><<<blocks(E), WPB * 64, 0, ctx->stream>>>(__VA_ARGS__); break; \
  }

// Return 1 if the vectorised kernels handled the call, 0 if the caller must use the generic ones.
int gp_stream_fwd_fast(gp_ctx* ctx, const gp_graph* g, int F, const float* x, const float* s, float* a) {
  if (!fast_ok(F, x, s, a)) return 0;
  const int64_t E = g->n_edges;
  GP_STREAM_DISPATCH(F, stream_fwd4_kernel, g->seg_ptr_ji, g->idx_kj, x, s, E, a);
  return 1;
}

int gp_stream_bwd_fast(gp_ctx* ctx, const gp_graph* g, const int32_t* perm_kj, int F, const float* x, const float* s,
                       const float* ga, float* gx, float* gs) {
  if (!fast_ok(F, x, s, ga) || !fast_ok(F, gx, gs, gs)) return 0;
  const int64_t E = g->n_edges;
  GP_STREAM_DISPATCH(F, stream_bwd_x4_kernel, g->seg_ptr_kj, g->idx_ji_kj, perm_kj, s, ga, E, gx);
  GP_STREAM_DISPATCH(F, stream_bwd_s4_kernel, g->seg_ptr_ji, g->idx_kj, x, ga, E, gs);
  return 1;
}
