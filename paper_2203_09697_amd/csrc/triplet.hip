// TripletUpdate + TripletAggr (paper Sec. 3.3: Hadamard product of the gathered, down-projected
// message m_kj with the projected spherical basis, summed over k in N_j \ {i} into edge j->i),
// forward and backward, variant D.
//
// Mapping: one wavefront per segment (a target edge in the forward pass, a source edge in the
// backward pass); lanes run over the feature dimension so every gathered row is one coalesced
// read; for rows narrower than 64 features the wavefront splits into 64/LPR groups that take
// alternate triplets and are combined by a butterfly at the end.  Reductions follow the sorted
// segment order, there are no atomics, results are bit-reproducible run to run.
#include <stdarg.h>

#include "gemm.h"
#include "triplet.h"

namespace {

constexpr int WPB = 4;        // wavefronts per workgroup
constexpr int ST = 8;         // max num_spherical
constexpr int UNR = 4;        // gathered rows kept in flight per group
__device__ __constant__ float Y_NORM[ST] = {
    0.28209479177387814f, 0.4886025119029199f, 0.6307831305050401f, 0.7463526651802308f,
    0.8462843753216345f, 0.9356025796273888f, 1.0171072362820548f, 1.0925484305920792f};  // sqrt((2l+1)/(4 pi))

// wavefront-local ordering of LDS traffic (no other wavefront touches this wave's slice)
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Y[l] = sqrt((2l+1)/(4 pi)) P_l(c), l < S; zero above
__device__ __forceinline__ void y_l0(float c, int S, float* Y) {
  float p0 = 1.0f, p1 = c;
#pragma unroll
  for (int l = 0; l < ST; ++l) {
    float P = (l == 0) ? 1.0f : p1;
    Y[l] = (l < S) ? Y_NORM[l] * P : 0.0f;
    if (l >= 1) {
      float p2 = ((float)(2 * l + 1) * c * p1 - (float)l * p0) / (float)(l + 1);
      p0 = p1;
      p1 = p2;
    }
  }
}

template <int FPL>
__device__ __forceinline__ void butterfly(float (&v)[FPL], int lpr) {
  for (int off = lpr; off < WAVE; off <<= 1)
#pragma unroll
    for (int i = 0; i < FPL; ++i) v[i] += __shfl_xor(v[i], off, WAVE);
}

// ------------------------------------------------------------------ per-edge radial projection
__global__ void project_radial_kernel(const float* __restrict__ rad, const float* __restrict__ W1, int64_t E,
                                      int S, int R, int B, float* __restrict__ Qt) {
  // one workgroup per 64 edges: their rad rows are one contiguous chunk, staged in LDS so that
  // both the read of rad and the transposed write of Qt are coalesced
  extern __shared__ float rad_s[];                 // [64][S*R + 1]
  const int SR = S * R, LD = SR + 1;
  const int64_t e0 = (int64_t)blockIdx.x * 64;
  const int ne = (int)min((int64_t)64, E - e0);
  for (int i = threadIdx.x; i < ne * SR; i += blockDim.x) rad_s[(i / SR) * LD + (i % SR)] = rad[e0 * SR + i];
  __syncthreads();
  for (int o = threadIdx.x; o < 64 * S * B; o += blockDim.x) {
    const int el = o & 63, lb = o >> 6;
    if (el >= ne) continue;
    const int b = lb % B, l = lb / B;
    const float* r = rad_s + el * LD + l * R;
    float s = 0.f;
    for (int n = 0; n < R; ++n) s += r[n] * W1[(l * R + n) * B + b];
    Qt[(int64_t)lb * E + e0 + el] = s;
  }
}

// ------------------------------------------------------------------ fused forward
template <int BT, int LPR, int FPL>
__global__ void __launch_bounds__(WPB* WAVE)
tripD_fwd_kernel(const int32_t* __restrict__ seg, const int32_t* __restrict__ idx_kj,
                 const float* __restrict__ cos_alpha, const float* __restrict__ x,
                 const float* __restrict__ Q, const float* __restrict__ W2, int64_t E, int F, int S, int B,
                 float* __restrict__ a, float* __restrict__ Bacc) {
  constexpr int G = WAVE / LPR;
  __shared__ float p_s[WPB][WAVE][BT];
  __shared__ int kj_s[WPB][WAVE];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t e = (int64_t)blockIdx.x * WPB + w;
  if (e >= E) return;
  const int grp = lane / LPR, fl = lane % LPR;
  float acc[BT][FPL];
#pragma unroll
  for (int b = 0; b < BT; ++b)
#pragma unroll
    for (int i = 0; i < FPL; ++i) acc[b][i] = 0.f;
  const int t0 = seg[e], t1 = seg[e + 1];
  for (int base = t0; base < t1; base += WAVE) {
    const int n = min(WAVE, t1 - base);
    if (lane < n) {
      const int t = base + lane;
      const int kj = idx_kj[t];
      float Y[ST];
      y_l0(cos_alpha[t], S, Y);
      // Q is stored transposed, Qt[(l*B+b)*E + e]: the lanes of a segment hold (almost)
      // consecutive source edges, so each of these loads is one or two cache lines per wavefront
      const float* q = Q + kj;
#pragma unroll
      for (int b = 0; b < BT; ++b) {
        float p = 0.f;
        if (b < B)
          for (int l = 0; l < S; ++l) p += Y[l] * q[(int64_t)(l * B + b) * E];
        p_s[w][lane][b] = p;
      }
      kj_s[w][lane] = kj;
    }
    wave_lds_sync();
    // UNR gathered rows are requested before any is consumed, to keep loads in flight
    for (int tt = grp; tt < n; tt += UNR * G) {
      float xv[UNR][FPL];
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const int id = tt + u * G;
        const int64_t kj = kj_s[w][id < n ? id : tt];
#pragma unroll
        for (int i = 0; i < FPL; ++i) {
          const int f = fl + i * WAVE;
          // (the unconditional form of the backward kernel measured 20 % slower here, with up to 16 accumulator rows)
          xv[u][i] = (f < F && id < n) ? x[kj * F + f] : 0.f;
        }
      }
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const int id = tt + u * G;
        if (id < n) {
#pragma unroll
          for (int i = 0; i < FPL; ++i)
#pragma unroll
            for (int b = 0; b < BT; ++b) acc[b][i] += p_s[w][id][b] * xv[u][i];
        }
      }
    }
    wave_lds_sync();
  }
#pragma unroll
  for (int b = 0; b < BT; ++b) butterfly<FPL>(acc[b], LPR);
  if (grp == 0) {
#pragma unroll
    for (int i = 0; i < FPL; ++i) {
      const int f = fl + i * WAVE;
      if (f < F) {
        float s = 0.f;
#pragma unroll
        for (int b = 0; b < BT; ++b)
          if (b < B) {
            if (W2) s += W2[b * F + f] * acc[b][i];
            Bacc[(e * B + b) * F + f] = acc[b][i];
          }
        if (W2) a[e * F + f] = s;   // W2 == NULL: bilinear form, only the accumulator is wanted
      }
    }
  }
}

// ------------------------------------------------------------------ fused backward (kj-major)
template <int LPR, int FPL>
__global__ void __launch_bounds__(WPB* WAVE)
tripD_bwd_kernel(const int32_t* __restrict__ seg_kj, const int32_t* __restrict__ idx_ji_kj,
                 const float* __restrict__ cos_kj, const float* __restrict__ x, const float* __restrict__ Q,
                 const float* __restrict__ W2, const float* __restrict__ ga, const float* __restrict__ z,
                 int64_t E, int F, int S, int B, float* __restrict__ gx, float* __restrict__ gQ) {
  constexpr int G = WAVE / LPR;
  extern __shared__ float dyn_s[];
  __shared__ float Y_s[WPB][WAVE][ST];
  __shared__ int ji_s[WPB][WAVE];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t e = (int64_t)blockIdx.x * WPB + w;
  if (e >= E) return;
  const int LDU = F + 1;
  float* u_s = dyn_s + (size_t)w * ST * LDU;
  const int grp = lane / LPR, fl = lane % LPR;
  float H[ST][FPL];
#pragma unroll
  for (int l = 0; l < ST; ++l)
#pragma unroll
    for (int i = 0; i < FPL; ++i) H[l][i] = 0.f;
  const int q0 = seg_kj[e], q1 = seg_kj[e + 1];
  for (int base = q0; base < q1; base += WAVE) {
    const int n = min(WAVE, q1 - base);
    if (lane < n) {
      float Y[ST];
      y_l0(cos_kj[base + lane], S, Y);
#pragma unroll
      for (int l = 0; l < ST; ++l) Y_s[w][lane][l] = Y[l];
      ji_s[w][lane] = idx_ji_kj[base + lane];
    }
    wave_lds_sync();
    for (int tt = grp; tt < n; tt += UNR * G) {
      float gv[UNR][FPL];
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const int id = tt + u * G;
        const int64_t ji = ji_s[w][id < n ? id : tt];
#pragma unroll
        for (int i = 0; i < FPL; ++i) {
          const int f = fl + i * WAVE;
          // clamped column and a 0/1 factor instead of a select around the load: a load that is only needed on one
          // side of a branch gets moved there and waited for on its own
          gv[u][i] = ga[ji * F + (f < F ? f : 0)] * ((f < F && id < n) ? 1.f : 0.f);
        }
      }
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const int id = tt + u * G;
        if (id < n) {
#pragma unroll
          for (int i = 0; i < FPL; ++i)
#pragma unroll
            for (int l = 0; l < ST; ++l) H[l][i] += Y_s[w][id][l] * gv[u][i];
        }
      }
    }
    wave_lds_sync();
  }
#pragma unroll
  for (int l = 0; l < ST; ++l) butterfly<FPL>(H[l], LPR);
  // every group now holds the full sums; group 0 finishes the edge
  if (!Q) {
    // H-only mode (bilinear variant): gx receives H[e, l, f]
    if (grp == 0)
#pragma unroll
      for (int i = 0; i < FPL; ++i) {
        const int f = fl + i * WAVE;
        if (f < F)
#pragma unroll
          for (int l = 0; l < ST; ++l)
            if (l < S) gx[(e * S + l) * F + f] = H[l][i];
      }
    return;
  }
  const float* q = Q + e;   // transposed table: element (l,b) of this edge at q[(l*B+b)*E]
  if (grp == 0) {
#pragma unroll
    for (int i = 0; i < FPL; ++i) {
      const int f = fl + i * WAVE;
      if (f < F) {
        float dx = 0.f;
        for (int b = 0; b < B; ++b) {
          float D = 0.f;
#pragma unroll
          for (int l = 0; l < ST; ++l)
            if (l < S) D += q[(int64_t)(l * B + b) * E] * H[l][i];
          dx += W2[b * F + f] * D;
        }
        if (z) dx *= dsilu_f(z[e * F + f]);
        gx[e * F + f] = dx;
        const float xv = x[e * F + f];
#pragma unroll
        for (int l = 0; l < ST; ++l) u_s[l * LDU + f] = xv * H[l][i];
      }
    }
  }
  wave_lds_sync();
  for (int idx = lane; idx < S * B; idx += WAVE) {
    const int l = idx / B, b = idx % B;
    float s = 0.f;
    for (int f = 0; f < F; ++f) s += W2[b * F + f] * u_s[l * LDU + f];
    gQ[e * S * B + idx] = s;
  }
}

// ------------------------------------------------------------------ weight-gradient partial sums
__global__ void w2grad_part_kernel(const float* __restrict__ ga, const float* __restrict__ Bacc, int64_t E,
                                   int F, int B, int64_t per, float* __restrict__ part) {
  const int64_t e0 = (int64_t)blockIdx.x * per, e1 = min(E, e0 + per);
  for (int idx = threadIdx.x; idx < B * F; idx += blockDim.x) {
    const int b = idx / F, f = idx % F;
    float s = 0.f;
    for (int64_t e = e0; e < e1; ++e) s += ga[e * F + f] * Bacc[(e * B + b) * F + f];
    part[(int64_t)blockIdx.x * B * F + idx] = s;
  }
}

__global__ void w1grad_part_kernel(const float* __restrict__ rad, const float* __restrict__ gQ, int64_t E, int S,
                                   int R, int B, int64_t per, float* __restrict__ part) {
  const int64_t e0 = (int64_t)blockIdx.x * per, e1 = min(E, e0 + per);
  const int n_out = S * R * B;
  for (int idx = threadIdx.x; idx < n_out; idx += blockDim.x) {
    const int b = idx % B, ln = idx / B, l = ln / R;
    float s = 0.f;
    for (int64_t e = e0; e < e1; ++e) s += rad[e * S * R + ln] * gQ[(e * S + l) * B + b];
    part[(int64_t)blockIdx.x * n_out + idx] = s;
  }
}

// ------------------------------------------------------------------ streaming forms
template <int LPR, int FPL>
__global__ void __launch_bounds__(WPB* WAVE)
stream_fwd_kernel(const int32_t* __restrict__ seg, const int32_t* __restrict__ idx_kj, const float* __restrict__ x,
                  const float* __restrict__ s, int64_t E, int F, float* __restrict__ a) {
  constexpr int G = WAVE / LPR;
  const int lane = threadIdx.x & 63;
  const int64_t e = (int64_t)blockIdx.x * WPB + (threadIdx.x >> 6);
  if (e >= E) return;
  const int grp = lane / LPR, fl = lane % LPR;
  float acc[FPL];
#pragma unroll
  for (int i = 0; i < FPL; ++i) acc[i] = 0.f;
  const int t1 = seg[e + 1];
  for (int64_t t = seg[e] + grp; t < t1; t += G) {
    const int64_t kj = idx_kj[t];
#pragma unroll
    for (int i = 0; i < FPL; ++i) {
      const int f = fl + i * WAVE;
      if (f < F) acc[i] += x[kj * F + f] * s[t * F + f];
    }
  }
  butterfly<FPL>(acc, LPR);
  if (grp == 0)
#pragma unroll
    for (int i = 0; i < FPL; ++i) {
      const int f = fl + i * WAVE;
      if (f < F) a[e * F + f] = acc[i];
    }
}

template <int LPR, int FPL>
__global__ void __launch_bounds__(WPB* WAVE)
stream_bwd_x_kernel(const int32_t* __restrict__ seg_kj, const int32_t* __restrict__ idx_ji_kj,
                    const int32_t* __restrict__ perm_kj, const float* __restrict__ s, const float* __restrict__ ga,
                    int64_t E, int F, float* __restrict__ gx) {
  constexpr int G = WAVE / LPR;
  const int lane = threadIdx.x & 63;
  const int64_t e = (int64_t)blockIdx.x * WPB + (threadIdx.x >> 6);
  if (e >= E) return;
  const int grp = lane / LPR, fl = lane % LPR;
  float acc[FPL];
#pragma unroll
  for (int i = 0; i < FPL; ++i) acc[i] = 0.f;
  const int q1 = seg_kj[e + 1];
  for (int64_t q = seg_kj[e] + grp; q < q1; q += G) {
    const int64_t ji = idx_ji_kj[q], t = perm_kj[q];
#pragma unroll
    for (int i = 0; i < FPL; ++i) {
      const int f = fl + i * WAVE;
      if (f < F) acc[i] += ga[ji * F + f] * s[t * F + f];
    }
  }
  butterfly<FPL>(acc, LPR);
  if (grp == 0)
#pragma unroll
    for (int i = 0; i < FPL; ++i) {
      const int f = fl + i * WAVE;
      if (f < F) gx[e * F + f] = acc[i];
    }
}

template <int LPR, int FPL>
__global__ void __launch_bounds__(WPB* WAVE)
stream_bwd_s_kernel(const int32_t* __restrict__ seg, const int32_t* __restrict__ idx_kj, const float* __restrict__ x,
                    const float* __restrict__ ga, int64_t E, int F, float* __restrict__ gs) {
  constexpr int G = WAVE / LPR;
  const int lane = threadIdx.x & 63;
  const int64_t e = (int64_t)blockIdx.x * WPB + (threadIdx.x >> 6);
  if (e >= E) return;
  const int grp = lane / LPR, fl = lane % LPR;
  float g[FPL];
#pragma unroll
  for (int i = 0; i < FPL; ++i) {
    const int f = fl + i * WAVE;
    g[i] = (f < F) ? ga[e * F + f] : 0.f;
  }
  const int t1 = seg[e + 1];
  for (int64_t t = seg[e] + grp; t < t1; t += G) {
    const int64_t kj = idx_kj[t];
#pragma unroll
    for (int i = 0; i < FPL; ++i) {
      const int f = fl + i * WAVE;
      if (f < F) gs[t * F + f] = g[i] * x[kj * F + f];
    }
  }
}

inline unsigned seg_blocks(int64_t E) { return (unsigned)((E + WPB - 1) / WPB); }

// pick (LPR, FPL) for a feature width and call fn.template operator()<LPR, FPL>()
#define GP_DISPATCH_WIDTH(F, CALL)                      \
  do {                                                  \
    if ((F) <= 16) { CALL(16, 1); }                     \
    else if ((F) <= 32) { CALL(32, 1); }                \
    else if ((F) <= 64) { CALL(64, 1); }                \
    else if ((F) <= 128) { CALL(64, 2); }               \
    else { CALL(64, 4); }                               \
  } while (0)

void slab_plan(int64_t E, int* blocks, int64_t* per) {
  int64_t b = (E + 63) / 64;
  if (b > 1024) b = 1024;
  if (b < 1) b = 1;
  *per = (E + b - 1) / b;
  if (*per < 1) *per = 1;
  *blocks = (int)((E + *per - 1) / *per);
  if (*blocks < 1) *blocks = 1;
}

int check_graph(gp_ctx* ctx, const gp_graph* g, bool need_ji, bool need_kj) {
  GP_REQUIRE(ctx, g, "graph is NULL");
  GP_REQUIRE(ctx, g->n_edges >= 0 && g->n_triplets >= 0, "graph: negative size");
  if (g->n_edges > INT32_MAX - 1 || g->n_triplets > INT32_MAX) return gp_fail(ctx, GP_INT32_OVERFLOW, "graph: sizes exceed int32");
  if (g->n_edges == 0) return GP_OK;
  if (need_ji) GP_REQUIRE(ctx, g->seg_ptr_ji && (g->n_triplets == 0 || g->idx_kj), "graph: ji-major arrays missing");
  if (need_kj) GP_REQUIRE(ctx, g->seg_ptr_kj && (g->n_triplets == 0 || g->idx_ji_kj), "graph: kj-major arrays missing");
  return GP_OK;
}

}  // namespace

int gp_tripD_project_radial(gp_ctx* ctx, const float* rad, const float* W1, int64_t E, int S, int R, int B, float* Q) {
  if (E == 0) return GP_OK;
  const size_t lds = (size_t)64 * (S * R + 1) * sizeof(float);
  project_radial_kernel<<<(unsigned)((E + 63) / 64), 256, lds, ctx->stream>>>(rad, W1, E, S, R, B, Q);
  GP_LAUNCH_CHECK(ctx, "project_radial_kernel");
  return GP_OK;
}

int gp_tripD_forward(gp_ctx* ctx, const gp_graph* g, const float* cos_alpha, const float* x, const float* Q,
                     const float* W2, int F, int S, int B, float* a, float* Bacc) {
  GP_TRY(check_graph(ctx, g, true, false));
  const int64_t E = g->n_edges;
  if (E == 0) return GP_OK;
  if (F < 1 || F > 256 || S < 1 || S > ST || B < 1 || B > 16)
    return gp_fail(ctx, GP_UNSUPPORTED_DIMS, "triplet D forward: int_emb=%d num_spherical=%d basis_emb=%d unsupported", F, S, B);
  GP_REQUIRE(ctx, x && Q && Bacc && (!W2 || a) && (g->n_triplets == 0 || cos_alpha), "triplet forward: NULL pointer");
  const double Td = (double)g->n_triplets, Ed = (double)E;
  gp_prof_scope prof(ctx, W2 ? "tripD_fwd" : "tripG_fwd", Td * 2.0 * (S * B + B * F) + Ed * 2.0 * B * F,
                     Td * 8.0 + Ed * 4.0 * (F + S * B + B * F + F) + Ed * 4.0);
#define CALL_FWD(LPR, FPL)                                                                                       \
  do {                                                                                                           \
    if (B <= 4) tripD_fwd_kernel<4, LPR, FPL><<<seg_blocks(E), WPB * WAVE, 0, ctx->stream>>>(                    \
        g->seg_ptr_ji, g->idx_kj, cos_alpha, x, Q, W2, E, F, S, B, a, Bacc);                                     \
    else if (B <= 8) tripD_fwd_kernel<8, LPR, FPL><<<seg_blocks(E), WPB * WAVE, 0, ctx->stream>>>(               \
        g->seg_ptr_ji, g->idx_kj, cos_alpha, x, Q, W2, E, F, S, B, a, Bacc);                                     \
    else tripD_fwd_kernel<16, LPR, FPL><<<seg_blocks(E), WPB * WAVE, 0, ctx->stream>>>(                          \
        g->seg_ptr_ji, g->idx_kj, cos_alpha, x, Q, W2, E, F, S, B, a, Bacc);                                     \
  } while (0)
  GP_DISPATCH_WIDTH(F, CALL_FWD);
#undef CALL_FWD
  GP_LAUNCH_CHECK(ctx, "tripD_fwd_kernel");
  return GP_OK;
}

int gp_tripD_backward(gp_ctx* ctx, const gp_graph* g, const float* cos_alpha_kj, const float* x, const float* Q,
                      const float* W2, const float* grad_a, const float* z, int F, int S, int B, float* grad_x,
                      float* grad_Q) {
  GP_TRY(check_graph(ctx, g, false, true));
  const int64_t E = g->n_edges;
  if (E == 0) return GP_OK;
  if (F < 1 || F > 256 || S < 1 || S > ST || B < 1 || B > 16)
    return gp_fail(ctx, GP_UNSUPPORTED_DIMS, "triplet D backward: int_emb=%d num_spherical=%d basis_emb=%d unsupported", F, S, B);
  GP_REQUIRE(ctx, grad_a && grad_x && (!Q || (x && W2 && grad_Q)) && (g->n_triplets == 0 || cos_alpha_kj),
             "triplet backward: NULL pointer");
  const size_t dyn = (size_t)WPB * ST * (F + 1) * sizeof(float);
  const double Td = (double)g->n_triplets, Ed = (double)E;
  gp_prof_scope prof(ctx, Q ? "tripD_bwd" : "trip_bwd_H", Td * 2.0 * S * F + Ed * 2.0 * (S * B * F * 2 + B * F),
                     Td * 8.0 + Ed * 4.0 * (F * 4 + S * B * 2) + Ed * 4.0);
#define CALL_BWD(LPR, FPL)                                                                      \
  tripD_bwd_kernel<LPR, FPL><<<seg_blocks(E), WPB * WAVE, dyn, ctx->stream>>>(                  \
      g->seg_ptr_kj, g->idx_ji_kj, cos_alpha_kj, x, Q, W2, grad_a, z, E, F, S, B, grad_x, grad_Q)
  GP_DISPATCH_WIDTH(F, CALL_BWD);
#undef CALL_BWD
  GP_LAUNCH_CHECK(ctx, "tripD_bwd_kernel");
  return GP_OK;
}

size_t gp_tripD_wgrad_scratch(int64_t E, int F, int S, int R, int B) {
  int blocks; int64_t per;
  slab_plan(E, &blocks, &per);
  size_t n = (size_t)(B * F > S * R * B ? B * F : S * R * B);
  return gp_align((size_t)blocks * n * sizeof(float));
}

int gp_tripD_weight_grads(gp_ctx* ctx, const float* grad_a, const float* Bacc, const float* rad, const float* grad_Q,
                          int64_t E, int F, int S, int R, int B, float* grad_W2, float* grad_W1, float* part,
                          size_t part_bytes) {
  int blocks; int64_t per;
  slab_plan(E, &blocks, &per);
  if (!part || part_bytes < gp_tripD_wgrad_scratch(E, F, S, R, B))
    return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "triplet D weight grads: scratch too small");
  if (E == 0) {
    GP_HIP(ctx, (hipError_t)gp_zero_async(ctx->stream, grad_W2, sizeof(float) * B * F));
    GP_HIP(ctx, (hipError_t)gp_zero_async(ctx->stream, grad_W1, sizeof(float) * S * R * B));
    return GP_OK;
  }
  if (Bacc) {   // NULL: grad_W2 comes from the matrix-core backward kernel
    w2grad_part_kernel<<<blocks, 256, 0, ctx->stream>>>(grad_a, Bacc, E, F, B, per, part);
    GP_LAUNCH_CHECK(ctx, "w2grad_part_kernel");
    GP_TRY(gp_reduce_parts(ctx, part, blocks, (int64_t)B * F, grad_W2));
  }
  w1grad_part_kernel<<<blocks, 256, 0, ctx->stream>>>(rad, grad_Q, E, S, R, B, per, part);
  GP_LAUNCH_CHECK(ctx, "w1grad_part_kernel");
  GP_TRY(gp_reduce_parts(ctx, part, blocks, (int64_t)S * R * B, grad_W1));
  return GP_OK;
}

extern "C" int gp_triplet_aggregate_fwd(gp_ctx* ctx, const gp_graph* graph, int32_t width, const float* x,
                                        const float* s, float* a) {
  if (!ctx) return GP_BAD_ARG;
  GP_TRY(check_graph(ctx, graph, true, false));
  const int64_t E = graph->n_edges;
  const int F = width;
  if (F < 1 || F > 256) return gp_fail(ctx, GP_UNSUPPORTED_DIMS, "gp_triplet_aggregate_fwd: width %d not in 1..256", F);
  if (E == 0) return GP_OK;
  GP_REQUIRE(ctx, x && a && (graph->n_triplets == 0 || s), "gp_triplet_aggregate_fwd: NULL pointer");
  GP_HIP(ctx, hipSetDevice(ctx->device));
  gp_prof_scope prof(ctx, "triplet_stream_fwd", 2.0 * graph->n_triplets * F,
                     (double)graph->n_triplets * (4.0 * F + 4.0) + (double)E * (8.0 * F + 4.0));
  if (gp_stream_fwd_fast(ctx, graph, F, x, s, a)) {
    GP_LAUNCH_CHECK(ctx, "stream_fwd4_kernel");
    return GP_OK;
  }
#define CALL_S(LPR, FPL) \
  stream_fwd_kernel<LPR, FPL><<<seg_blocks(E), WPB * WAVE, 0, ctx->stream>>>(graph->seg_ptr_ji, graph->idx_kj, x, s, E, F, a)
  GP_DISPATCH_WIDTH(F, CALL_S);
#undef CALL_S
  GP_LAUNCH_CHECK(ctx, "stream_fwd_kernel");
  return GP_OK;
}

extern "C" int gp_triplet_aggregate_bwd(gp_ctx* ctx, const gp_graph* graph, const int32_t* perm_kj, int32_t width,
                                        const float* x, const float* s, const float* grad_a, float* grad_x,
                                        float* grad_s) {
  if (!ctx) return GP_BAD_ARG;
  GP_TRY(check_graph(ctx, graph, true, true));
  const int64_t E = graph->n_edges;
  const int F = width;
  if (F < 1 || F > 256) return gp_fail(ctx, GP_UNSUPPORTED_DIMS, "gp_triplet_aggregate_bwd: width %d not in 1..256", F);
  if (E == 0) return GP_OK;
  GP_REQUIRE(ctx, x && grad_a && grad_x && (graph->n_triplets == 0 || (s && grad_s && perm_kj)),
             "gp_triplet_aggregate_bwd: NULL pointer");
  GP_HIP(ctx, hipSetDevice(ctx->device));
  gp_prof_scope prof(ctx, "triplet_stream_bwd", 3.0 * graph->n_triplets * F,
                     (double)graph->n_triplets * (12.0 * F + 16.0) + (double)E * (12.0 * F + 8.0));
  if (graph->n_triplets > 0 && gp_stream_bwd_fast(ctx, graph, perm_kj, F, x, s, grad_a, grad_x, grad_s)) {
    GP_LAUNCH_CHECK(ctx, "stream_bwd4 kernels");
    return GP_OK;
  }
#define CALL_S(LPR, FPL)                                                                                          \
  do {                                                                                                            \
    stream_bwd_x_kernel<LPR, FPL><<<seg_blocks(E), WPB * WAVE, 0, ctx->stream>>>(                                 \
        graph->seg_ptr_kj, graph->idx_ji_kj, perm_kj, s, grad_a, E, F, grad_x);                                   \
    stream_bwd_s_kernel<LPR, FPL><<<seg_blocks(E), WPB * WAVE, 0, ctx->stream>>>(graph->seg_ptr_ji, graph->idx_kj, \
                                                                                 x, grad_a, E, F, grad_s);        \
  } while (0)
  GP_DISPATCH_WIDTH(F, CALL_S);
#undef CALL_S
  GP_LAUNCH_CHECK(ctx, "stream_bwd kernels");
  return GP_OK;
}

// ================================================================== variant G per-edge pieces
namespace {

// A workgroup takes 64 consecutive edges: their slice of the transposed radial table is 256
// contiguous bytes per (l, c), staged in LDS once; then one wavefront per edge, lanes over o.
constexpr int EG_EDGES = 32;   // edges per workgroup (14 KB of LDS: 8 wavefronts per SIMD fit); 64 measured 1 % slower
constexpr int EG_UNR = 2;      // edges of a wavefront in flight together; 4 measured slower (registers)

__global__ void __launch_bounds__(WPB* WAVE)
edge_G_kernel(const float* __restrict__ Radt, const float* __restrict__ H, int64_t E, int S, int C, int O,
              int out_half, float* __restrict__ Gout) {
  extern __shared__ float dyn_s[];   // rad_s[(l*C + c) * 64 + edge]
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int64_t e0 = (int64_t)blockIdx.x * EG_EDGES;
  {
    // all loads of a thread before the first LDS write: a rolled loop would expose one memory round trip per pass
    constexpr int PASSES = ST * 16 * EG_EDGES / (WPB * WAVE);   // emb_cbf <= 16
    float r[PASSES];
    const int n = S * C * EG_EDGES;
#pragma unroll
    for (int k = 0; k < PASSES; ++k) {
      const int i = threadIdx.x + k * WPB * WAVE;
      const int ic = i < n ? i : n - 1;
      const int64_t e = e0 + (ic & (EG_EDGES - 1));
      r[k] = Radt[(int64_t)(ic / EG_EDGES) * E + (e < E ? e : E - 1)];
    }
#pragma unroll
    for (int k = 0; k < PASSES; ++k) {
      const int i = threadIdx.x + k * WPB * WAVE;
      if (i < n) dyn_s[i] = e0 + (i & (EG_EDGES - 1)) < E ? r[k] : 0.f;
    }
  }
  __syncthreads();
  // EG_UNR edges of a wavefront at a time: their H rows are requested together, so the memory round trip (and the
  // wait for the previous stores, which complete through the same counter) is paid once per EG_UNR edges
  for (int el0 = w; el0 < EG_EDGES && e0 + el0 < E; el0 += EG_UNR * WPB) {
    for (int o = lane; o < O; o += WAVE) {
      float h[EG_UNR][ST];
#pragma unroll
      for (int u = 0; u < EG_UNR; ++u) {
        const int el = el0 + u * WPB;
        const int64_t e = (el < EG_EDGES && e0 + el < E) ? e0 + el : e0 + el0;   // a valid row either way
#pragma unroll
        for (int l = 0; l < ST; ++l) h[u][l] = H[(e * S + (l < S ? l : S - 1)) * O + o];
      }
#pragma unroll
      for (int u = 0; u < EG_UNR; ++u) {
        const int el = el0 + u * WPB;
        if (el >= EG_EDGES || e0 + el >= E) break;
        const int64_t e = e0 + el;
        for (int c = 0; c < C; ++c) {
          float s = 0.f;
#pragma unroll
          for (int l = 0; l < ST; ++l)
            if (l < S) s += dyn_s[(l * C + c) * EG_EDGES + el] * h[u][l];
          if (out_half) reinterpret_cast<__bf16*>(Gout)[(e * C + c) * O + o] = (__bf16)s;
          else Gout[(e * C + c) * O + o] = s;
        }
      }
    }
  }
}

// The same product written as bf16 for O = 32, 64 or 128: the edge's S x O block of H (fp32, contiguous) goes once
// through the wavefront's LDS slice, a lane owns (c, 8 consecutive o) pieces of the edge's C x O result (contiguous)
// and writes each with one 16-byte store instead of C stores of 2 bytes per lane.
template <int O, class HT>   // HT: storage of H (float or __bf16)
__global__ void __launch_bounds__(WPB* WAVE)
edge_G16_kernel(const float* __restrict__ Radt, const HT* __restrict__ H, int64_t E, int S, int C, __bf16* __restrict__ Gout) {
  typedef __bf16 h8 __attribute__((ext_vector_type(8)));
  typedef float f4 __attribute__((ext_vector_type(4)));
  constexpr int CH = O / 8;
  constexpr int PE = 16 / (int)sizeof(HT);             // elements per 16-byte piece
  constexpr int NV = (ST * O / PE + WAVE - 1) / WAVE;  // 16-byte pieces of the H block per lane
  extern __shared__ float dyn_s[];                     // rad_s[(l*C + c) * EG_EDGES + edge]
  __shared__ __attribute__((aligned(16))) float H_s[WPB][2][ST * O];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int64_t e0 = (int64_t)blockIdx.x * EG_EDGES;
  {
    constexpr int PASSES = ST * 16 * EG_EDGES / (WPB * WAVE);
    float r[PASSES];
    const int n = S * C * EG_EDGES;
#pragma unroll
    for (int k = 0; k < PASSES; ++k) {
      const int i = threadIdx.x + k * WPB * WAVE;
      const int ic = i < n ? i : n - 1;
      const int64_t e = e0 + (ic & (EG_EDGES - 1));
      r[k] = Radt[(int64_t)(ic / EG_EDGES) * E + (e < E ? e : E - 1)];
    }
#pragma unroll
    for (int k = 0; k < PASSES; ++k) {
      const int i = threadIdx.x + k * WPB * WAVE;
      if (i < n) dyn_s[i] = e0 + (i & (EG_EDGES - 1)) < E ? r[k] : 0.f;
    }
  }
  __syncthreads();
  const int n_piece = S * O / PE;
  auto fetch = [&](int el, f4 (&v)[NV]) __attribute__((always_inline)) {
    const int64_t e = e0 + el < E ? e0 + el : E - 1;
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      const int i = lane + WAVE * k;
      v[k] = *reinterpret_cast<const f4*>(H + e * S * O + PE * (i < n_piece ? i : 0));
    }
  };
  f4 vn[NV];
  if (e0 + w < E) fetch(w, vn);
  int buf = 0;
  for (int el = w; el < EG_EDGES && e0 + el < E; el += WPB, buf ^= 1) {
    float* hs = H_s[w][buf];
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      const int i = lane + WAVE * k;
      if (i < n_piece) {
        if constexpr (sizeof(HT) == 4) *reinterpret_cast<f4*>(hs + 4 * i) = vn[k];
        else {   // 8 bf16 values: widened on their way into the slice
          const h8 h = __builtin_bit_cast(h8, vn[k]);
          *reinterpret_cast<f4*>(hs + 8 * i) = f4{(float)h[0], (float)h[1], (float)h[2], (float)h[3]};
          *reinterpret_cast<f4*>(hs + 8 * i + 4) = f4{(float)h[4], (float)h[5], (float)h[6], (float)h[7]};
        }
      }
    }
    if (el + WPB < EG_EDGES && e0 + el + WPB < E) fetch(el + WPB, vn);
    wave_lds_sync();
    const int64_t e = e0 + el;
    for (int item = lane; item < C * CH; item += WAVE) {
      const int c = item / CH, oc = item % CH;
      float acc[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = 0.f;
      for (int l = 0; l < S; ++l) {
        const float r = dyn_s[(l * C + c) * EG_EDGES + el];
        const f4 a = *reinterpret_cast<const f4*>(hs + l * O + 8 * oc), b = *reinterpret_cast<const f4*>(hs + l * O + 8 * oc + 4);
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] += r * a[i], acc[4 + i] += r * b[i];
      }
      h8 out;
#pragma unroll
      for (int i = 0; i < 8; ++i) out[i] = (__bf16)acc[i];
      *reinterpret_cast<h8*>(Gout + (e * C + c) * O + 8 * oc) = out;
    }
  }
}

__global__ void __launch_bounds__(WPB* WAVE)
edge_dRad_kernel(const float* __restrict__ V, const float* __restrict__ H, int64_t E, int S, int C, int O,
                 float* __restrict__ dRad) {
  extern __shared__ float dyn_s[];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t e = (int64_t)blockIdx.x * WPB + w;
  if (e >= E) return;
  const int LD = O + 1;
  float* V_s = dyn_s + (size_t)w * (C + S) * LD;
  float* H_s = V_s + (size_t)C * LD;
  for (int i = lane; i < C * O; i += WAVE) V_s[(i / O) * LD + (i % O)] = V[e * C * O + i];
  for (int i = lane; i < S * O; i += WAVE) H_s[(i / O) * LD + (i % O)] = H[e * S * O + i];
  wave_lds_sync();
  for (int idx = lane; idx < S * C; idx += WAVE) {
    const int l = idx / C, c = idx % C;
    float s = 0.f;
    for (int o = 0; o < O; ++o) s += V_s[c * LD + o] * H_s[l * LD + o];
    dRad[e * S * C + idx] = s;
  }
}

// dRad[e, l, c] = sum_o V[e, c, o] H[e, l, o] without LDS, for C <= 16 and O = 4 OQ: lane = (c, quarter q of the o
// range).  A lane loads its OQ values of V[c, :] (the wavefront reads the edge's C x O block contiguously) and the
// same OQ columns of the S rows of H (16 lanes share each address), all requested before the first use; the four
// partial sums of a c are combined by two lane exchanges.  VT: storage type of V.
constexpr int DQ_EPW = 1;   // edges per wavefront (4 measured 2 % slower: starting the wavefronts is not the limit)
template <int OQ, class VT, class HT>   // storage of V and of H (float or __bf16)
__global__ void __launch_bounds__(WPB* WAVE)
edge_dRad_q_kernel(const VT* __restrict__ V, const HT* __restrict__ H, int64_t E, int S, int C, float* __restrict__ dRad) {
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  constexpr int O = 4 * OQ;
  __shared__ __attribute__((aligned(16))) float H_s[WPB][ST * O];
  const int c = lane >> 2, q = lane & 3;
  for (int64_t e = ((int64_t)blockIdx.x * WPB + w) * DQ_EPW, e_end = e + DQ_EPW < E ? e + DQ_EPW : E; e < e_end; ++e) {
  const VT* vp = V + (e * C + (c < C ? c : C - 1)) * O + q * OQ;
  float v[OQ];
  if (sizeof(VT) == 2) {
    typedef __bf16 h8 __attribute__((ext_vector_type(8)));
#pragma unroll
    for (int i = 0; i < OQ; i += 8) {
      const h8 t = *reinterpret_cast<const h8*>(vp + i);
#pragma unroll
      for (int k = 0; k < 8; ++k) v[i + k] = (float)t[k];
    }
  } else {
    typedef float f4 __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int i = 0; i < OQ; i += 4) {
      const f4 t = *reinterpret_cast<const f4*>(reinterpret_cast<const float*>(vp) + i);
#pragma unroll
      for (int k = 0; k < 4; ++k) v[i + k] = t[k];
    }
  }
  // the S x O block of H goes through the wavefront's LDS slice: fetched once (S O / 4 sixteen-byte loads spread over
  // the lanes) instead of by each of the 16 lanes that share a quarter, which kept the address path busy 16 times over
  {
    typedef float f4 __attribute__((ext_vector_type(4)));
    constexpr int PE = 16 / (int)sizeof(HT);   // elements per 16-byte piece
    const HT* hp = H + e * S * O;
#pragma unroll
    for (int k = 0; k < (ST * O / PE + WAVE - 1) / WAVE; ++k) {
      const int idx = lane + k * WAVE;
      const f4 t = *reinterpret_cast<const f4*>(hp + PE * (idx < S * O / PE ? idx : 0));
      if (idx < S * O / PE) {
        if constexpr (sizeof(HT) == 4) *reinterpret_cast<f4*>(&H_s[w][4 * idx]) = t;
        else {
          typedef __bf16 h8 __attribute__((ext_vector_type(8)));
          const h8 h = __builtin_bit_cast(h8, t);
          *reinterpret_cast<f4*>(&H_s[w][8 * idx]) = f4{(float)h[0], (float)h[1], (float)h[2], (float)h[3]};
          *reinterpret_cast<f4*>(&H_s[w][8 * idx + 4]) = f4{(float)h[4], (float)h[5], (float)h[6], (float)h[7]};
        }
      }
    }
  }
  wave_lds_sync();
  float part[ST];
#pragma unroll
  for (int l = 0; l < ST; ++l) {
    part[l] = 0.f;
    typedef float f4 __attribute__((ext_vector_type(4)));
    const float* hp = &H_s[w][(l < S ? l : S - 1) * O + q * OQ];
#pragma unroll
    for (int i = 0; i < OQ; i += 4) {
      const f4 t = *reinterpret_cast<const f4*>(hp + i);
#pragma unroll
      for (int k = 0; k < 4; ++k) part[l] += v[i + k] * t[k];
    }
  }
  wave_lds_sync();   // the slice is rewritten for the next edge
#pragma unroll
  for (int l = 0; l < ST; ++l) {
    part[l] += __shfl_xor(part[l], 1);
    part[l] += __shfl_xor(part[l], 2);
  }
  if (q == 0 && c < C) {
#pragma unroll
    for (int l = 0; l < ST; ++l)
      if (l < S) dRad[e * S * C + l * C + c] = part[l];
  }
  }
}

__global__ void permute3_kernel(const float* __restrict__ src, int n0, int n1, int n2, int p0, int p1, int p2,
                                float* __restrict__ dst) {
  const int n[3] = {n0, n1, n2};
  const int total = n0 * n1 * n2;
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int d2 = n[p2], d1 = n[p1];
  const int c = i % d2, b = (i / d2) % d1, a = i / (d2 * d1);
  int idx[3];
  idx[p0] = a; idx[p1] = b; idx[p2] = c;
  dst[i] = src[(idx[0] * n1 + idx[1]) * n2 + idx[2]];
}

__global__ void ew_dsilu2_kernel(const float* __restrict__ g, float s, const float* __restrict__ z1,
                                 const float* __restrict__ z2, float* __restrict__ d1, float* __restrict__ d2,
                                 int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const float v = g[i] * s;
  d1[i] = v * dsilu_f(z1[i]);
  d2[i] = v * dsilu_f(z2[i]);
}

}  // namespace

bool gp_tripG_edge_takes_half_H(int C, int O) { return C >= 1 && C <= 16 && (O == 32 || O == 64 || O == 128); }

int gp_tripG_edge_G(gp_ctx* ctx, const float* Radt, const float* H, int64_t E, int S, int C, int O, float* Gout, int out_half,
                    int h_half) {
  if (E == 0) return GP_OK;
  GP_REQUIRE(ctx, Radt && H && Gout && S >= 1 && S <= ST && C >= 1 && C <= 16 && O >= 1, "edge_G: bad arguments");
  gp_prof_scope prof(ctx, "tripG_edge_G", 2.0 * E * S * C * O,
                     4.0 * E * S * C + (h_half ? 2.0 : 4.0) * E * S * O + (out_half ? 2.0 : 4.0) * E * C * O);
  const unsigned blocks = (unsigned)((E + EG_EDGES - 1) / EG_EDGES);
  const size_t lds = (size_t)S * C * EG_EDGES * sizeof(float);
  if (out_half && (O == 32 || O == 64 || O == 128) && ((reinterpret_cast<uintptr_t>(H) | reinterpret_cast<uintptr_t>(Gout)) & 15) == 0) {
    __bf16* Gh = reinterpret_cast<__bf16*>(Gout);
    const __bf16* Hh = reinterpret_cast<const __bf16*>(H);
#define GP_EG16(OW)                                                                                          \
  do {                                                                                                       \
    if (h_half) edge_G16_kernel<OW, __bf16><<<blocks, WPB * WAVE, lds, ctx->stream>>>(Radt, Hh, E, S, C, Gh); \
    else edge_G16_kernel<OW, float><<<blocks, WPB * WAVE, lds, ctx->stream>>>(Radt, H, E, S, C, Gh);         \
  } while (0)
    if (O == 32) GP_EG16(32);
    else if (O == 64) GP_EG16(64);
    else GP_EG16(128);
#undef GP_EG16
  } else {
    if (h_half) return gp_fail(ctx, GP_UNSUPPORTED_DIMS, "edge_G: a bf16 H needs a bf16 result, a width of 32, 64 or 128 and 16-byte aligned arrays");
    edge_G_kernel<<<blocks, WPB * WAVE, lds, ctx->stream>>>(Radt, H, E, S, C, O, out_half, Gout);
  }
  GP_LAUNCH_CHECK(ctx, "edge_G_kernel");
  return GP_OK;
}

int gp_tripG_edge_dRad(gp_ctx* ctx, const float* V, const float* H, int64_t E, int S, int C, int O, float* dRad, int v_half,
                       int h_half) {
  if (E == 0) return GP_OK;
  GP_REQUIRE(ctx, V && H && dRad && S >= 1 && S <= ST && C >= 1 && O >= 1, "edge_dRad: bad arguments");
  gp_prof_scope prof(ctx, "tripG_edge_dRad", 2.0 * E * S * C * O,
                     4.0 * E * S * C + (h_half ? 2.0 : 4.0) * E * S * O + (v_half ? 2.0 : 4.0) * E * C * O);
  // 16-byte loads need 16-byte aligned rows: true for the widths below when the bases are (fp32 V and H: O % 4,
  // bf16 V: O % 8)
  const bool aligned = (((uintptr_t)V | (uintptr_t)H) & 15) == 0;
  if (C <= 16 && aligned && (O == 32 || O == 64 || O == 128)) {
    const __bf16* Vh = reinterpret_cast<const __bf16*>(V);
    const __bf16* Hh = reinterpret_cast<const __bf16*>(H);
    const unsigned dq_blocks = (unsigned)((E + WPB * DQ_EPW - 1) / (WPB * DQ_EPW));
#define GP_DRAD(OQ)                                                                                           \
  do {                                                                                                        \
    if (v_half && h_half) edge_dRad_q_kernel<OQ, __bf16, __bf16><<<dq_blocks, WPB * WAVE, 0, ctx->stream>>>(Vh, Hh, E, S, C, dRad); \
    else if (v_half) edge_dRad_q_kernel<OQ, __bf16, float><<<dq_blocks, WPB * WAVE, 0, ctx->stream>>>(Vh, H, E, S, C, dRad); \
    else if (h_half) edge_dRad_q_kernel<OQ, float, __bf16><<<dq_blocks, WPB * WAVE, 0, ctx->stream>>>(V, Hh, E, S, C, dRad); \
    else edge_dRad_q_kernel<OQ, float, float><<<dq_blocks, WPB * WAVE, 0, ctx->stream>>>(V, H, E, S, C, dRad);    \
  } while (0)
    if (O == 32) GP_DRAD(8);
    else if (O == 64) GP_DRAD(16);
    else GP_DRAD(32);
#undef GP_DRAD
    GP_LAUNCH_CHECK(ctx, "edge_dRad_q_kernel");
    return GP_OK;
  }
  if (v_half || h_half) return gp_fail(ctx, GP_UNSUPPORTED_DIMS, "edge_dRad: bf16 V or H needs emb_cbf <= 16 and a width of 32, 64 or 128");
  const size_t lds = (size_t)WPB * (C + S) * (O + 1) * sizeof(float);
  if (lds > 64 * 1024) return gp_fail(ctx, GP_UNSUPPORTED_DIMS, "edge_dRad: (emb_cbf+num_spherical)*emb_bil too large");
  edge_dRad_kernel<<<seg_blocks(E), WPB * WAVE, lds, ctx->stream>>>(V, H, E, S, C, O, dRad);
  GP_LAUNCH_CHECK(ctx, "edge_dRad_kernel");
  return GP_OK;
}

int gp_permute3(gp_ctx* ctx, const float* src, int n0, int n1, int n2, int p0, int p1, int p2, float* dst) {
  GP_REQUIRE(ctx, src && dst && n0 > 0 && n1 > 0 && n2 > 0, "permute3: bad arguments");
  GP_REQUIRE(ctx, ((1 << p0) | (1 << p1) | (1 << p2)) == 7, "permute3: not a permutation");
  const int total = n0 * n1 * n2;
  permute3_kernel<<<(total + 255) / 256, 256, 0, ctx->stream>>>(src, n0, n1, n2, p0, p1, p2, dst);
  GP_LAUNCH_CHECK(ctx, "permute3_kernel");
  return GP_OK;
}

int gp_ew_dsilu2(gp_ctx* ctx, const float* g, float s, const float* z1, const float* z2, float* d1, float* d2,
                 int64_t n) {
  if (n == 0) return GP_OK;
  gp_prof_scope prof(ctx, "ew_dsilu2", 0.0, 20.0 * (double)n);
  ew_dsilu2_kernel<<<(unsigned)((n + 255) / 256), 256, 0, ctx->stream>>>(g, s, z1, z2, d1, d2, n);
  GP_LAUNCH_CHECK(ctx, "ew_dsilu2_kernel");
  return GP_OK;
}
