// TripletUpdate + TripletAggr of the bilinear block (paper Sec. 3.4) on the matrix cores.
//
//   A[e, c, f] = sum_{t in seg(e)} y_t[c] x[kj(t), f],   y_t[c] = sum_l Y_l0(cos alpha_t) Rad[kj(t), l, c]
//
// Grouped by centre atom j (the atom shared by the two edges of a triplet): every target edge
// e = (j->i) sums over the same rows of x, the in-edges of j, which are the contiguous rows
// r0 .. r0+d-1 of the edge list (it is sorted by target atom).  So for one atom
//
//   A[e] (C x F) = Y[e]^T (C x d) . X_j (d x F),   Y[e][p, c] = y_t[c] for t = (row r0+p -> e), 0 if k = i
//
// i.e. one dense product with M = (out-edges of j) x C rows, K = d, N = F; X_j is staged once in
// LDS (bf16, transposed) and shared by all out-edges.  Two kernels:
//
//   tripG_y_kernel     writes Y in bf16, already in the register layout of the MFMA A operand:
//                      per edge e a block Yb[pg][c][8] (pg = group of 8 positions), starting at
//                      position offset seg_ptr_ji[e] + 16 e (room for padding d to a multiple
//                      of 16).  A thread owns 8 positions x 2 values of c and keeps the radial
//                      rows it needs (8 x S x 2 values) in registers while it walks the edges.
//   tripG_mfma_kernel  v_mfma_f32_32x32x16_bf16: a wavefront owns 4 edges (2 row blocks of
//                      2 edges x 16 c) by all F columns; A fragments come straight from Yb
//                      (16 bytes per lane, read once), B fragments from LDS.
//
// Operands are rounded to bf16, sums are fp32.  Needs the centre-atom lists of gp_graph.
#include <stdarg.h>

#include "triplet.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int ST = 8;        // max num_spherical
constexpr int CP = 16;       // rows per edge in an MFMA tile = max emb_cbf
constexpr int PARTS = 8;     // at most this many workgroups share one centre atom
constexpr int EPP = 64;      // target edges per workgroup
constexpr int YT = 256;      // threads of the y kernel
constexpr int MT = 512;      // threads of the contraction kernel
constexpr int KU = 4;        // k-steps of A fragments loaded ahead
constexpr size_t LDS_MAX = 160 * 1024;

__device__ __constant__ float Y_NORM_M[ST] = {
    0.28209479177387814f, 0.4886025119029199f, 0.6307831305050401f, 0.7463526651802308f,
    0.8462843753216345f, 0.9356025796273888f, 1.0171072362820548f, 1.0925484305920792f};  // sqrt((2l+1)/(4 pi))

// The share of one workgroup: centre atom j = blockIdx.x / PARTS, its in-edge rows r0 .. r0+d-1
// (Kp = d rounded up to 16) and the slice [eb, ee) of its out-edge list.
struct part_t {
  int r0, d, Kp, o0, eb, ee;
};

// false (for every thread of the workgroup alike) if this workgroup has nothing to do
__device__ __forceinline__ bool centre_part(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ out_ptr,
                                            int kp_cap, part_t& P) {
  const int j = blockIdx.x / PARTS, part = blockIdx.x % PARTS;
  P.r0 = row_ptr[j];
  P.d = row_ptr[j + 1] - P.r0;
  P.Kp = (P.d + 15) & ~15;
  P.o0 = out_ptr[j];
  const int dout = out_ptr[j + 1] - P.o0;
  if (dout <= 0 || P.Kp > kp_cap) return false;
  int nparts = (dout + EPP - 1) / EPP;
  nparts = nparts < PARTS ? nparts : PARTS;
  if (part >= nparts) return false;
  const int len = (((dout + nparts - 1) / nparts) + 3) & ~3;
  P.eb = part * len;
  P.ee = P.eb + len < dout ? P.eb + len : dout;
  return P.eb < P.ee;
}

__device__ __forceinline__ int64_t y_offset(int seg, int e) {   // in bf16 elements
  return ((int64_t)seg + 16 * (int64_t)e) * CP;
}

template <int SM>   // loops over l run to SM >= num_spherical (rows above num_spherical are zero)
__global__ void __launch_bounds__(YT)
tripG_y_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ out_ptr,
               const int32_t* __restrict__ out_list, const int32_t* __restrict__ seg_ptr_ji,
               const int32_t* __restrict__ idx_kj, const float* __restrict__ cos_alpha,
               const float* __restrict__ Radt, int64_t E, int S, int C, int kp_cap, __bf16* __restrict__ Yb) {
  part_t P;
  if (!centre_part(row_ptr, out_ptr, kp_cap, P)) return;
  __shared__ int s_e[64], s_seg[64], s_cnt[64], s_gap[64];
  const int n_pg = P.Kp / 8;
  const int cp = threadIdx.x & 7;
  for (int pg0 = 0; pg0 < n_pg; pg0 += YT / 8) {
    const int pg = pg0 + (threadIdx.x >> 3);
    const bool active = pg < n_pg;
    float rad[SM][2][8];
#pragma unroll
    for (int l = 0; l < SM; ++l)
#pragma unroll
      for (int cc = 0; cc < 2; ++cc)
#pragma unroll
        for (int pi = 0; pi < 8; ++pi) {
          const int p = 8 * pg + pi, c = 2 * cp + cc;
          const bool ok = active && l < S && c < C && p < P.d;
          rad[l][cc][pi] = ok ? Radt[(int64_t)(l * C + c) * E + P.r0 + p] : 0.f;
        }
    for (int c0 = P.eb; c0 < P.ee; c0 += 64) {
      __syncthreads();
      if (threadIdx.x < 64 && c0 + (int)threadIdx.x < P.ee) {
        const int e = out_list[P.o0 + c0 + threadIdx.x];
        const int seg = seg_ptr_ji[e], cnt = seg_ptr_ji[e + 1] - seg;
        // the segment lists rows r0, r0+1, ... with (at most) the row coming from atom i left
        // out: first slot whose row is not r0 + slot
        int lo = 0, hi = cnt;
        while (lo < hi) {
          const int mid = (lo + hi) >> 1;
          if (idx_kj[seg + mid] == P.r0 + mid) lo = mid + 1;
          else hi = mid;
        }
        s_e[threadIdx.x] = e;
        s_seg[threadIdx.x] = seg;
        s_cnt[threadIdx.x] = cnt;
        s_gap[threadIdx.x] = lo;
      }
      __syncthreads();
      const int n = P.ee - c0 < 64 ? P.ee - c0 : 64;
      if (!active) continue;
      for (int ei = 0; ei < n; ++ei) {
        const int e = s_e[ei], seg = s_seg[ei], cnt = s_cnt[ei], gap = s_gap[ei];
        float y[2][8];
#pragma unroll
        for (int pi = 0; pi < 8; ++pi) {
          const int p = 8 * pg + pi;
          const int q = p - (p > gap ? 1 : 0);
          const bool valid = p != gap && q < cnt;
          const float cs = valid ? cos_alpha[seg + q] : 0.f;
          float p0 = 1.f, p1 = cs;
          float a0 = Y_NORM_M[0] * rad[0][0][pi], a1 = Y_NORM_M[0] * rad[0][1][pi];
#pragma unroll
          for (int l = 1; l < SM; ++l) {
            const float yl = Y_NORM_M[l] * p1;
            a0 += yl * rad[l][0][pi];
            a1 += yl * rad[l][1][pi];
            const float p2 = ((float)(2 * l + 1) * cs * p1 - (float)l * p0) * (1.0f / (float)(l + 1));
            p0 = p1;
            p1 = p2;
          }
          y[0][pi] = valid ? a0 : 0.f;
          y[1][pi] = valid ? a1 : 0.f;
        }
        __bf16* dst = Yb + y_offset(seg, e) + (int64_t)pg * (CP * 8) + (2 * cp) * 8;
#pragma unroll
        for (int cc = 0; cc < 2; ++cc) {
          bf16x8 v;
#pragma unroll
          for (int pi = 0; pi < 8; ++pi) v[pi] = (__bf16)y[cc][pi];
          *reinterpret_cast<bf16x8*>(dst + 8 * cc) = v;
        }
      }
    }
  }
}

template <int CB>   // F = 32 CB
__global__ void __launch_bounds__(MT)
tripG_mfma_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ out_ptr,
                  const int32_t* __restrict__ out_list, const int32_t* __restrict__ seg_ptr_ji,
                  const float* __restrict__ x, const __bf16* __restrict__ Yb, int C, int kp_cap,
                  float* __restrict__ A) {
  constexpr int F = 32 * CB;
  part_t P;
  if (!centre_part(row_ptr, out_ptr, kp_cap, P)) return;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  __bf16* XT = reinterpret_cast<__bf16*>(smem_raw);   // XT[f][p], row stride LDP
  // LDP/8 is odd, so the 16-byte reads of 8 lanes with consecutive f fall into 8 different bank groups
  const int LDP = P.Kp + 8;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

  // stage X_j: a wavefront takes a tile of 16 positions x 32 features; a lane converts two rows of
  // 4 features and writes 4 packed position pairs
  const int tiles_p = P.Kp / 16;
  for (int t = wave; t < tiles_p * CB; t += MT / 64) {
    const int pp = (t % tiles_p) * 8 + (lane & 7), fq = (t / tiles_p) * 8 + (lane >> 3);
    const int p0 = 2 * pp;
    f32x4 v0 = {0.f, 0.f, 0.f, 0.f}, v1 = {0.f, 0.f, 0.f, 0.f};
    if (p0 < P.d) v0 = *reinterpret_cast<const f32x4*>(x + (int64_t)(P.r0 + p0) * F + 4 * fq);
    if (p0 + 1 < P.d) v1 = *reinterpret_cast<const f32x4*>(x + (int64_t)(P.r0 + p0 + 1) * F + 4 * fq);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      bf16x2 pr;
      pr[0] = (__bf16)v0[i];
      pr[1] = (__bf16)v1[i];
      *reinterpret_cast<bf16x2*>(&XT[(4 * fq + i) * LDP + p0]) = pr;
    }
  }
  __syncthreads();

  const int kh = lane >> 5, l32 = lane & 31;
  const int nks = P.Kp / 16;
  const int n_e = P.ee - P.eb;
  for (int grp = wave; grp * 4 < n_e; grp += MT / 64) {
    int e4[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int idx = grp * 4 + k;
      e4[k] = out_list[P.o0 + P.eb + (idx < n_e ? idx : n_e - 1)];
    }
    // A operand: row l32 = (edge l32/16 of the row block, c = l32%16), k = 8 kh .. 8 kh + 7
    const __bf16* ya[2];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
      const int e = (l32 >> 4) ? e4[2 * rb + 1] : e4[2 * rb];
      ya[rb] = Yb + y_offset(seg_ptr_ji[e], e) + kh * (CP * 8) + (l32 & 15) * 8;
    }
    f32x16 acc[2][CB];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[rb][cb][v] = 0.f;

    if (nks > 0) {
      bf16x8 an[KU][2];
      auto load_chunk = [&](int ks0) {
#pragma unroll
        for (int u = 0; u < KU; ++u) {
          const int ks = ks0 + u < nks ? ks0 + u : nks - 1;
#pragma unroll
          for (int rb = 0; rb < 2; ++rb) an[u][rb] = *reinterpret_cast<const bf16x8*>(ya[rb] + (int64_t)ks * (2 * CP * 8));
        }
      };
      load_chunk(0);
      for (int ks0 = 0; ks0 < nks; ks0 += KU) {
        bf16x8 ac[KU][2];
#pragma unroll
        for (int u = 0; u < KU; ++u)
#pragma unroll
          for (int rb = 0; rb < 2; ++rb) ac[u][rb] = an[u][rb];
        if (ks0 + KU < nks) load_chunk(ks0 + KU);
#pragma unroll
        for (int u = 0; u < KU; ++u) {
          if (ks0 + u < nks) {
            bf16x8 b[CB];
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
              b[cb] = *reinterpret_cast<const bf16x8*>(&XT[(cb * 32 + l32) * LDP + (ks0 + u) * 16 + kh * 8]);
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
              for (int cb = 0; cb < CB; ++cb)
                acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ac[u][rb], b[cb], acc[rb][cb], 0, 0, 0);
          }
        }
      }
    }

    // accumulator register v of lane (kh, l32): row 8 (v/4) + 4 kh + v%4, column l32
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int k = 2 * rb + (v >> 3);                       // edge of the group (uniform)
        const int c = 8 * ((v >> 2) & 1) + 4 * kh + (v & 3);
        if (grp * 4 + k >= n_e || c >= C) continue;
        float* dst = A + ((int64_t)e4[k] * C + c) * F + l32;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) dst[cb * 32] = acc[rb][cb][v];
      }
  }
}

int kp_of(const gp_graph* g) { return (g->max_in_degree + 15) & ~15; }

}  // namespace

size_t gp_tripG_mfma_scratch(int64_t E, int64_t T) { return gp_align((size_t)(T + 16 * E) * CP * sizeof(__bf16)); }

bool gp_tripG_mfma_usable(const gp_graph* g, int F, int S, int C) {
  if (!g || !g->row_ptr || !g->out_ptr || !g->out_list || g->n_atoms <= 0 || g->max_in_degree <= 0) return false;
  if (g->n_atoms > INT32_MAX / PARTS) return false;
  if (F % 32 != 0 || F < 32 || F > 128 || C < 1 || C > CP || S < 1 || S > ST) return false;
  return (size_t)F * (kp_of(g) + 8) * sizeof(__bf16) <= LDS_MAX;
}

int gp_tripG_forward_mfma(gp_ctx* ctx, const gp_graph* g, const float* cos_alpha, const float* x, const float* Radt,
                          int F, int S, int C, float* A, void* ybuf, size_t ybytes) {
  const int64_t E = g->n_edges, T = g->n_triplets;
  if (E == 0) return GP_OK;
  GP_REQUIRE(ctx, gp_tripG_mfma_usable(g, F, S, C), "triplet G (matrix-core form): graph lists or widths not supported");
  GP_REQUIRE(ctx, g->seg_ptr_ji && (T == 0 || (g->idx_kj && cos_alpha)) && x && Radt && A && ybuf, "triplet G forward: NULL pointer");
  if (ybytes < gp_tripG_mfma_scratch(E, T)) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "triplet G forward: y buffer too small");
  const int kp_cap = kp_of(g);
  const unsigned grid = (unsigned)(g->n_atoms * PARTS);
  const double Td = (double)T, Ed = (double)E;
  __bf16* Yb = static_cast<__bf16*>(ybuf);
  {
    gp_prof_scope prof(ctx, "tripG_y", Td * (2.0 * S * C + 4.0 * S), (Td + 16.0 * Ed) * CP * 2.0 + Td * 8.0 + Ed * 4.0 * S * C);
    if (S <= 7)
      tripG_y_kernel<7><<<grid, YT, 0, ctx->stream>>>(g->row_ptr, g->out_ptr, g->out_list, g->seg_ptr_ji, g->idx_kj,
                                                       cos_alpha, Radt, E, S, C, kp_cap, Yb);
    else
      tripG_y_kernel<8><<<grid, YT, 0, ctx->stream>>>(g->row_ptr, g->out_ptr, g->out_list, g->seg_ptr_ji, g->idx_kj,
                                                       cos_alpha, Radt, E, S, C, kp_cap, Yb);
    GP_LAUNCH_CHECK(ctx, "tripG_y_kernel");
  }
  {
    const size_t lds = (size_t)F * (kp_cap + 8) * sizeof(__bf16);
    gp_prof_scope prof(ctx, "tripG_mfma_fwd", Td * 2.0 * C * F, (Td + 16.0 * Ed) * CP * 2.0 + Ed * 4.0 * (F + (double)C * F));
#define GP_TRIPG_LAUNCH(CB)                                                                                       \
  do {                                                                                                            \
    static size_t lds_set = 0;                                                                                    \
    if (lds > lds_set) {                                                                                          \
      GP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&tripG_mfma_kernel<CB>),                      \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));                     \
      lds_set = lds;                                                                                              \
    }                                                                                                             \
    tripG_mfma_kernel<CB><<<grid, MT, lds, ctx->stream>>>(g->row_ptr, g->out_ptr, g->out_list, g->seg_ptr_ji, x,  \
                                                          Yb, C, kp_cap, A);                                      \
  } while (0)
    switch (F / 32) {
      case 1: GP_TRIPG_LAUNCH(1); break;
      case 2: GP_TRIPG_LAUNCH(2); break;
      case 3: GP_TRIPG_LAUNCH(3); break;
      default: GP_TRIPG_LAUNCH(4); break;
    }
#undef GP_TRIPG_LAUNCH
    GP_LAUNCH_CHECK(ctx, "tripG_mfma_kernel");
  }
  return GP_OK;
}
