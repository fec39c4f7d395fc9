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
constexpr int EU_EDGES = 32;   // edges per workgroup (14 KB of LDS; 64: 4 % slower)
constexpr int EU_UNR = 1;      // edges of a wavefront in flight together (2: 40 % slower, the 32 bf16 values in flight cost registers)

constexpr int EU_CMAX = 16;   // largest emb_cbf

// The slice of the transposed radial table for EU_EDGES consecutive edges, [(l*C + c) * EU_EDGES + edge], into LDS.  All loads
// of a thread are issued before the first LDS write (a rolled loop would expose one memory round trip per pass).
__device__ __forceinline__ void stage_radial_slice(const float* __restrict__ Radt, int64_t E, int64_t e0, int rows, float* rad_s) {
  constexpr int PASSES = ST * EU_CMAX * EU_EDGES / (WPB * 64);
  float r[PASSES];
  const int n = rows * EU_EDGES;
#pragma unroll
  for (int k = 0; k < PASSES; ++k) {
    const int i = threadIdx.x + k * WPB * 64;
    const int ic = i < n ? i : n - 1;
    const int64_t e = e0 + (ic & (EU_EDGES - 1));
    r[k] = Radt[(int64_t)(ic / EU_EDGES) * E + (e < E ? e : E - 1)];
  }
#pragma unroll
  for (int k = 0; k < PASSES; ++k) {
    const int i = threadIdx.x + k * WPB * 64;
    if (i < n) rad_s[i] = e0 + (i & (EU_EDGES - 1)) < E ? r[k] : 0.f;
  }
}

// VT: storage type of V (fp32, or bf16 as written by the epilogue of the GEMM that produces it)
// OUT16: U is written as bf16 [E][8][O] (rows l >= S zero), the operand layout of the one-pass grad-cos kernel
template <class VT, bool OUT16>
__global__ void __launch_bounds__(WPB* 64)
edge_U_kernel(const float* __restrict__ Radt, const VT* __restrict__ V, int64_t E, int S, int C, int O,
              float* __restrict__ U) {
  extern __shared__ float rad_s[];   // [(l*C + c) * EU_EDGES + edge]
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int64_t e0 = (int64_t)blockIdx.x * EU_EDGES;
  stage_radial_slice(Radt, E, e0, S * C, rad_s);
  __syncthreads();
  // EU_UNR edges of a wavefront at a time, all their loads first (clamped indices: no branch around a load): the
  // memory round trip, and the wait for the previous stores that comes with it, is paid once per EU_UNR edges
  for (int el0 = w; el0 < EU_EDGES && e0 + el0 < E; el0 += EU_UNR * WPB) {
    for (int o = lane; o < O; o += 64) {
      VT v[EU_UNR][EU_CMAX];
#pragma unroll
      for (int u = 0; u < EU_UNR; ++u) {
        const int el = el0 + u * WPB;
        const int64_t e = (el < EU_EDGES && e0 + el < E) ? e0 + el : e0 + el0;
#pragma unroll
        for (int c = 0; c < EU_CMAX; ++c) v[u][c] = V[(e * C + (c < C ? c : C - 1)) * O + o];
      }
#pragma unroll
      for (int u = 0; u < EU_UNR; ++u) {
        const int el = el0 + u * WPB;
        if (el >= EU_EDGES || e0 + el >= E) break;
        const int64_t e = e0 + el;
        float acc[ST];
#pragma unroll
        for (int l = 0; l < ST; ++l) acc[l] = 0.f;
#pragma unroll
        for (int c = 0; c < EU_CMAX; ++c)
          if (c < C) {
            const float vc = (float)v[u][c];
#pragma unroll
            for (int l = 0; l < ST; ++l)
              if (l < S) acc[l] += rad_s[(l * C + c) * EU_EDGES + el] * vc;
          }
        if constexpr (OUT16) {
          static_assert(ST == 8, "eight rows per edge");
          __bf16* U16 = reinterpret_cast<__bf16*>(U);
#pragma unroll
          for (int l = 0; l < ST; ++l) U16[(e * 8 + l) * O + o] = (__bf16)acc[l];
        } else {
#pragma unroll
          for (int l = 0; l < ST; ++l)
            if (l < S) U[(e * S + l) * O + o] = acc[l];
        }
      }
    }
  }
}

// U in the operand layout of the one-pass grad-cos kernel, bf16 [E][8][O], from V stored as bf16: the edge's V block
// (C x O, contiguous) is fetched once by the wavefront, 16 bytes per lane, through its LDS slice; a lane then owns one
// (l, 8 consecutive o) piece of the edge's 8 x O result (contiguous too) and writes it with one 16-byte store.  The
// kernel above takes 2-byte loads per lane and writes 128-byte rows: 0.59 ms at 3e5 edges against 0.3 ms here.
template <int O>
__global__ void __launch_bounds__(WPB* 64)
edge_U16_kernel(const float* __restrict__ Radt, const __bf16* __restrict__ V, int64_t E, int S, int C, __bf16* __restrict__ U16) {
  typedef __bf16 h8 __attribute__((ext_vector_type(8)));
  constexpr int CH = O / 8;                       // 16-byte pieces per row
  extern __shared__ float rad_s[];                // [(l*C + c) * EU_EDGES + edge]
  __shared__ __attribute__((aligned(16))) __bf16 V_s[WPB][2][EU_CMAX * O];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int64_t e0 = (int64_t)blockIdx.x * EU_EDGES;
  stage_radial_slice(Radt, E, e0, S * C, rad_s);
  __syncthreads();
  const int n_piece = C * CH;                     // pieces of the edge's V block
  auto fetch = [&](int el, h8 (&v)[(EU_CMAX * CH + 63) / 64]) __attribute__((always_inline)) {
    const int64_t e = e0 + el < E ? e0 + el : E - 1;
#pragma unroll
    for (int k = 0; k < (EU_CMAX * CH + 63) / 64; ++k) {
      const int i = lane + 64 * k;
      v[k] = *reinterpret_cast<const h8*>(V + (e * C) * O + 8 * (i < n_piece ? i : 0));
    }
  };
  h8 vn[(EU_CMAX * CH + 63) / 64];
  if (e0 + w < E) fetch(w, vn);
  int buf = 0;
  for (int el = w; el < EU_EDGES && e0 + el < E; el += WPB, buf ^= 1) {
    __bf16* vs = V_s[w][buf];
#pragma unroll
    for (int k = 0; k < (EU_CMAX * CH + 63) / 64; ++k) {
      const int i = lane + 64 * k;
      if (i < n_piece) *reinterpret_cast<h8*>(vs + 8 * i) = vn[k];
    }
    if (el + WPB < EU_EDGES && e0 + el + WPB < E) fetch(el + WPB, vn);   // the next edge's block is on its way during the sums
    wave_lds_sync();
    const int64_t e = e0 + el;
    for (int item = lane; item < 8 * CH; item += 64) {
      const int l = item / CH, oc = item % CH;
      float acc[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = 0.f;
      if (l < S) {
        for (int c = 0; c < C; ++c) {
          const float r = rad_s[(l * C + c) * EU_EDGES + el];
          const h8 v = *reinterpret_cast<const h8*>(vs + c * O + 8 * oc);
#pragma unroll
          for (int i = 0; i < 8; ++i) acc[i] += r * (float)v[i];
        }
      }
      h8 out;
#pragma unroll
      for (int i = 0; i < 8; ++i) out[i] = (__bf16)acc[i];
      *reinterpret_cast<h8*>(U16 + (e * 8 + l) * O + 8 * oc) = out;
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
      Ur[l][i] = U[(e * S + (l < S ? l : S - 1)) * O + (o < O ? o : 0)] * ((l < S && o < O) ? 1.f : 0.f);   // unconditional load
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

int gp_tripG_edge_U(gp_ctx* ctx, const float* Radt, const float* V, int64_t E, int S, int C, int O, float* U, int v_half, int out16) {
  if (E == 0) return GP_OK;
  GP_REQUIRE(ctx, Radt && V && U && S >= 1 && S <= ST && C >= 1 && C <= EU_CMAX && O >= 1, "edge_U: bad arguments");
  gp_prof_scope prof(ctx, "tripG_edge_U", 2.0 * E * S * C * O, 4.0 * E * (S * C + S * O) + (v_half ? 2.0 : 4.0) * E * C * O);
  const unsigned blocks = (unsigned)((E + EU_EDGES - 1) / EU_EDGES);
  const size_t lds = (size_t)S * C * EU_EDGES * sizeof(float);
  if (out16 && v_half && (O == 32 || O == 64 || O == 128) && (reinterpret_cast<uintptr_t>(V) & 15) == 0 && (reinterpret_cast<uintptr_t>(U) & 15) == 0) {
    const __bf16* Vh = reinterpret_cast<const __bf16*>(V);
    __bf16* Uh = reinterpret_cast<__bf16*>(U);
    if (O == 32) edge_U16_kernel<32><<<blocks, WPB * 64, lds, ctx->stream>>>(Radt, Vh, E, S, C, Uh);
    else if (O == 64) edge_U16_kernel<64><<<blocks, WPB * 64, lds, ctx->stream>>>(Radt, Vh, E, S, C, Uh);
    else edge_U16_kernel<128><<<blocks, WPB * 64, lds, ctx->stream>>>(Radt, Vh, E, S, C, Uh);
  } else if (out16) {
    if (v_half) edge_U_kernel<__bf16, true><<<blocks, WPB * 64, lds, ctx->stream>>>(Radt, reinterpret_cast<const __bf16*>(V), E, S, C, O, U);
    else edge_U_kernel<float, true><<<blocks, WPB * 64, lds, ctx->stream>>>(Radt, V, E, S, C, O, U);
  } else if (v_half) edge_U_kernel<__bf16, false><<<blocks, WPB * 64, lds, ctx->stream>>>(Radt, reinterpret_cast<const __bf16*>(V), E, S, C, O, U);
  else edge_U_kernel<float, false><<<blocks, WPB * 64, lds, ctx->stream>>>(Radt, V, E, S, C, O, U);
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
