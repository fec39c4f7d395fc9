// Gradient of the loss with respect to the triplet cosines for the bilinear block (needed for
// forces, paper Sec. 3.2): with U[e',l,o] = sum_c Rad[e',l,c] V[e',c,o],
//   dL/dcos(alpha_t) = sum_l Y_l0'(cos alpha_t) sum_o dz[ji(t),o] U[kj(t),l,o].
// One wavefront per source edge walks the kj-major triplet view, U of that edge held in registers.
#include <stdarg.h>

#include "triplet.h"

namespace {

constexpr int WPB = 4;
constexpr int ST = 8;
__device__ __constant__ float Y_NORM_G[ST] = {
    0.28209479177387814f, 0.4886025119029199f, 0.6307831305050401f, 0.7463526651802308f,
    0.8462843753216345f, 0.9356025796273888f, 1.0171072362820548f, 1.0925484305920792f};  // sqrt((2l+1)/(4 pi))

__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// dY[l] = sqrt((2l+1)/(4 pi)) P_l'(c);  P'_{l+1} = P'_{l-1} + (2l+1) P_l
__device__ __forceinline__ void dy_l0(float c, int S, float* dY) {
  float P[ST], dP[ST];
  P[0] = 1.f; dP[0] = 0.f;
  P[1] = c;   dP[1] = 1.f;
#pragma unroll
  for (int l = 1; l < ST - 1; ++l) {
    P[l + 1] = ((float)(2 * l + 1) * c * P[l] - (float)l * P[l - 1]) / (float)(l + 1);
    dP[l + 1] = dP[l - 1] + (float)(2 * l + 1) * P[l];
  }
#pragma unroll
  for (int l = 0; l < ST; ++l) dY[l] = (l < S) ? Y_NORM_G[l] * dP[l] : 0.f;
}

// U[e, l, o] = sum_c Radt[(l*C+c)*E + e] * V[e, c*O + o].  A workgroup takes 64 consecutive edges and
// stages their slice of the transposed radial table in LDS (256 contiguous bytes per (l, c)); then one
// wavefront per edge, lanes over o.
constexpr int EU_EDGES = 64;

__global__ void __launch_bounds__(WPB* 64)
edge_U_kernel(const float* __restrict__ Radt, const float* __restrict__ V, int64_t E, int S, int C, int O,
              float* __restrict__ U) {
  extern __shared__ float rad_s[];   // [(l*C + c) * 64 + edge]
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int64_t e0 = (int64_t)blockIdx.x * EU_EDGES;
  for (int i = threadIdx.x; i < S * C * EU_EDGES; i += WPB * 64) {
    const int64_t e = e0 + (i & (EU_EDGES - 1));
    rad_s[i] = e < E ? Radt[(int64_t)(i / EU_EDGES) * E + e] : 0.f;
  }
  __syncthreads();
  for (int el = w; el < EU_EDGES && e0 + el < E; el += WPB) {
    const int64_t e = e0 + el;
    for (int o = lane; o < O; o += 64) {
      float acc[ST];
#pragma unroll
      for (int l = 0; l < ST; ++l) acc[l] = 0.f;
      for (int c = 0; c < C; ++c) {
        const float v = V[(e * C + c) * O + o];
#pragma unroll
        for (int l = 0; l < ST; ++l)
          if (l < S) acc[l] += rad_s[(l * C + c) * EU_EDGES + el] * v;
      }
#pragma unroll
      for (int l = 0; l < ST; ++l)
        if (l < S) U[(e * S + l) * O + o] = acc[l];
    }
  }
}

// FPL = ceil(O / 64) features per lane
template <int FPL>
__global__ void __launch_bounds__(WPB* 64)
trip_dcos_kernel(const int32_t* __restrict__ seg_kj, const int32_t* __restrict__ idx_ji_kj,
                 const float* __restrict__ cos_kj, const float* __restrict__ U, const float* __restrict__ dz,
                 int64_t E, int O, int S, int accumulate, float* __restrict__ gc_kj) {
  __shared__ float dY_s[WPB][64][ST];
  __shared__ int ji_s[WPB][64];
  __shared__ float res_s[WPB][64];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t e = (int64_t)blockIdx.x * WPB + w;
  if (e >= E) return;
  float Ur[ST][FPL];
#pragma unroll
  for (int l = 0; l < ST; ++l)
#pragma unroll
    for (int i = 0; i < FPL; ++i) {
      const int o = lane + i * 64;
      Ur[l][i] = (l < S && o < O) ? U[(e * S + l) * O + o] : 0.f;
    }
  const int q0 = seg_kj[e], q1 = seg_kj[e + 1];
  for (int base = q0; base < q1; base += 64) {
    const int n = min(64, q1 - base);
    if (lane < n) {
      float dY[ST];
      dy_l0(cos_kj[base + lane], S, dY);
#pragma unroll
      for (int l = 0; l < ST; ++l) dY_s[w][lane][l] = dY[l];
      ji_s[w][lane] = idx_ji_kj[base + lane];
    }
    wave_lds_sync();
    for (int tt = 0; tt < n; ++tt) {
      const int64_t ji = ji_s[w][tt];
      float part = 0.f;
#pragma unroll
      for (int i = 0; i < FPL; ++i) {
        const int o = lane + i * 64;
        float wv = 0.f;
#pragma unroll
        for (int l = 0; l < ST; ++l) wv += dY_s[w][tt][l] * Ur[l][i];
        if (o < O) part += dz[ji * O + o] * wv;
      }
      part = wave_sum(part);
      if (lane == 0) res_s[w][tt] = part;
    }
    wave_lds_sync();
    if (lane < n) {
      const float r = res_s[w][lane];
      if (accumulate) gc_kj[base + lane] += r;
      else gc_kj[base + lane] = r;
    }
    wave_lds_sync();
  }
}

}  // namespace

int gp_tripG_edge_U(gp_ctx* ctx, const float* Radt, const float* V, int64_t E, int S, int C, int O, float* U) {
  if (E == 0) return GP_OK;
  GP_REQUIRE(ctx, Radt && V && U && S >= 1 && S <= ST && C >= 1 && O >= 1, "edge_U: bad arguments");
  gp_prof_scope prof(ctx, "tripG_edge_U", 2.0 * E * S * C * O, 4.0 * E * (S * C + S * O + C * O));
  edge_U_kernel<<<(unsigned)((E + EU_EDGES - 1) / EU_EDGES), WPB * 64, (size_t)S * C * EU_EDGES * sizeof(float), ctx->stream>>>(
      Radt, V, E, S, C, O, U);
  GP_LAUNCH_CHECK(ctx, "edge_U_kernel");
  return GP_OK;
}

int gp_tripG_grad_cos(gp_ctx* ctx, const gp_graph* g, const float* cos_alpha_kj, const float* U, const float* dz,
                      int O, int S, int accumulate, float* grad_cos_kj) {
  GP_REQUIRE(ctx, g, "grad_cos: graph is NULL");
  const int64_t E = g->n_edges;
  if (E == 0 || g->n_triplets == 0) return GP_OK;
  GP_REQUIRE(ctx, g->seg_ptr_kj && g->idx_ji_kj && cos_alpha_kj && U && dz && grad_cos_kj, "grad_cos: NULL pointer");
  if (O < 1 || O > 256 || S < 1 || S > ST) return gp_fail(ctx, GP_UNSUPPORTED_DIMS, "grad_cos: emb_bil=%d num_spherical=%d unsupported", O, S);
  gp_prof_scope prof(ctx, "tripG_grad_cos", (double)g->n_triplets * 2.0 * (S + 1) * O, (double)g->n_triplets * 12.0 + 4.0 * E * S * O);
  const unsigned blocks = (unsigned)((E + WPB - 1) / WPB);
#define CALL_DCOS(FPL)                                                                                          \
  trip_dcos_kernel<FPL><<<blocks, WPB * 64, 0, ctx->stream>>>(g->seg_ptr_kj, g->idx_ji_kj, cos_alpha_kj, U, dz, E, O, \
                                                             S, accumulate, grad_cos_kj)
  if (O <= 64) CALL_DCOS(1);
  else if (O <= 128) CALL_DCOS(2);
  else CALL_DCOS(4);
#undef CALL_DCOS
  GP_LAUNCH_CHECK(ctx, "trip_dcos_kernel");
  return GP_OK;
}
