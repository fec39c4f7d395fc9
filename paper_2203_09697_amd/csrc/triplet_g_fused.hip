// TripletUpdate + TripletAggr of the bilinear block (paper Sec. 3.4) in one pass: nothing of size T is written.
//
//   A[e, c, f] = sum_{t in seg(e)} y_t[c] x[kj(t), f],   y_t[c] = sum_l Y_l0(cos alpha_t) Rad[kj(t), l, c]
//
// Grouped by centre atom j as in triplet_g_mfma.hip: for all out-edges e = (j->i) the sum runs over the same rows
// of x, the in-edges p = 0 .. d-1 of j.  Per in-edge row and c the Legendre sum is a polynomial of degree S-1 in
// cos alpha whose coefficients depend on the row only, so a triplet's y is one Horner evaluation.  The kernel
// evaluates the operand y in registers, in the lane layout of the matrix-core instruction, from the cosines
// (4 bytes per triplet, the only per-triplet data it reads) and feeds v_mfma_f32_16x16x32_bf16:
//
//   D[f, c] += X^T[f, p] . Y[p, c]        rows f (16 per tile), contraction over 32 in-edge rows, columns c (16)
//
// so that a lane (p-quarter kq, column c) needs the coefficients of (8 rows, c) only, whichever edge it works on:
// they are read once per 32 rows and reused for the 4 out-edges a wavefront owns.  Work item = (centre atom, group
// of 32 out-edges): 8 wavefronts x 4 edges, walking the atom's rows in slabs of 64 through two LDS buffers.  A slab
// holds X^T (bf16), the coefficient table (fp32) and the cosines of the group's 32 edges; the first two are plain
// copies of what a pre-pass lays out per atom (16-byte global->LDS loads, no registers), the cosines are staged
// through registers with the segment's one missing row (k = i) already skipped.
//
// Operands are rounded to bf16, sums are fp32, the polynomial is evaluated in fp32.
#include <stdarg.h>

#include "centre_atom.h"
#include "triplet.h"

namespace {

typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(1))) void* global_void_ptr;

constexpr int GE = 32;          // out-edges per work item
constexpr int SLAB = 64;        // in-edge rows per slab
constexpr int PADJ = 72;        // padded row space per atom: base_j = roundup8(row_ptr[j]) + PADJ j leaves room for
                                // rounding every atom's rows up to a whole slab (d + 63) on an 8-aligned base (+ 7)
constexpr int COEF_ROW = 128;   // floats per padded row of the coefficient table: [half][c 16][4]
constexpr int FT = 512;         // threads of the main kernel

__host__ __device__ inline int64_t padded_base(int r0, int64_t j) { return (((int64_t)r0 + 7) & ~(int64_t)7) + PADJ * j; }
inline int64_t padded_rows(int64_t E, int64_t N) { return ((E + 7) & ~(int64_t)7) + PADJ * N + SLAB; }

__device__ __forceinline__ int swz(int f) { return f ^ ((f >> 3) & 7); }   // 16-byte slot of feature f inside a p-block

// grp_ptr[j] = number of work items of the atoms before j; grp_atom[w] = atom of work item w.  One workgroup.
__global__ void __launch_bounds__(1024)
fused_groups_kernel(const int32_t* __restrict__ out_ptr, int n_atoms, int32_t* __restrict__ grp_ptr, int32_t* __restrict__ grp_atom) {
  __shared__ int32_t wave_tot[16];
  __shared__ int32_t carry;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  if (tid == 0) carry = 0;
  __syncthreads();
  for (int base = 0; base < n_atoms; base += 1024) {
    const int j = base + tid;
    const int v = j < n_atoms ? (out_ptr[j + 1] - out_ptr[j] + GE - 1) / GE : 0;
    int incl = v;
    for (int o = 1; o < 64; o <<= 1) {
      const int u = __shfl_up(incl, o, 64);
      if (lane >= o) incl += u;
    }
    if (lane == 63) wave_tot[w] = incl;
    __syncthreads();
    int before = carry;
    for (int k = 0; k < w; ++k) before += wave_tot[k];
    if (j < n_atoms) {
      grp_ptr[j] = before + incl - v;
      for (int k = 0; k < v; ++k) grp_atom[before + incl - v + k] = j;
    }
    __syncthreads();
    if (tid == 1023) carry = before + incl;
    __syncthreads();
  }
  if (tid == 0) grp_ptr[n_atoms] = carry;
}

// Pre-pass, one workgroup per (atom j, 64 of its padded rows): X^T in bf16 as [p-block of 8 rows][f][8], the
// coefficients of the powers of cos alpha as [row][half][c][4] (rows past the atom's last one and columns past C are
// zero, so padded rows contribute nothing), and, from the workgroups of the first 64 rows, the position `gap` of the
// row each out-edge's segment leaves out (its length if none).
template <int SM>
__global__ void __launch_bounds__(256)
fused_pack_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ out_ptr, const int32_t* __restrict__ out_list,
                  const int32_t* __restrict__ seg_ptr_ji, const int32_t* __restrict__ idx_kj, const float* __restrict__ x,
                  const float* __restrict__ Radt, int64_t E, int S, int C, int F, __bf16* __restrict__ xb,
                  float* __restrict__ coef, int32_t* __restrict__ gap) {
  const int j = blockIdx.x;
  const int r0 = row_ptr[j], d = row_ptr[j + 1] - r0;
  const int p0 = SLAB * (int)blockIdx.y;
  if (blockIdx.y == 0) {
    const int o0 = out_ptr[j], dout = out_ptr[j + 1] - o0;
    for (int t = threadIdx.x; t < dout; t += 256) {
      const int e = out_list[o0 + t];
      const int seg = seg_ptr_ji[e], cnt = seg_ptr_ji[e + 1] - seg;
      gap[e] = first_mismatch(idx_kj + seg, cnt, [=](int slot) { return r0 + slot; });
    }
  }
  if (p0 >= ((d + SLAB - 1) & ~(SLAB - 1))) return;
  const int64_t base = padded_base(r0, j) + p0;
  // X^T: item (p-block pb, feature f); consecutive threads take consecutive f of the same rows
  for (int it = threadIdx.x; it < (SLAB / 8) * F; it += 256) {
    const int pb = it / F, f = it % F;
    bf16x8 v;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int p = p0 + 8 * pb + i;
      const float xv = x[(int64_t)(r0 + (p < d ? p : 0)) * F + f];   // clamped row, zeroed below: the load stays unconditional
      v[i] = (__bf16)(p < d ? xv : 0.f);
    }
    *reinterpret_cast<bf16x8*>(xb + ((base / 8 + pb) * F + f) * 8) = v;
  }
  // coefficients: item (row p, column c); consecutive threads take consecutive rows of one (l, c) line of Radt
  for (int it = threadIdx.x; it < SLAB * CP; it += 256) {
    const int pl = it % SLAB, c = it / SLAB, p = p0 + pl;
    const bool ok = p < d && c < C;
    float rl[SM];
#pragma unroll
    for (int l = 0; l < SM; ++l)
      rl[l] = Radt[(int64_t)((l < S ? l : 0) * C + (c < C ? c : 0)) * E + r0 + (p < d ? p : 0)] * ((ok && l < S) ? Y_NORM_M[l] : 0.f);
    float m[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      float sum = 0.f;
#pragma unroll
      for (int l = k; l < SM; l += 2) sum += leg_mono(l, k) * rl[l];
      m[k] = sum;
    }
    float* dst = coef + (base + pl) * COEF_ROW + c * 4;
    *reinterpret_cast<f32x4*>(dst) = f32x4{m[0], m[1], m[2], m[3]};
    *reinterpret_cast<f32x4*>(dst + 64) = f32x4{m[4], m[5], m[6], m[7]};
  }
}

__device__ __forceinline__ void wait_vm0() { __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8)); }   // vmcnt(0) only

template <int NT, int SM>   // F = 16 NT (NT = 2, 4, 8); SM = number of polynomial coefficients kept (>= num_spherical)
__global__ void __launch_bounds__(FT, 1)
tripG_fused_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ out_ptr, const int32_t* __restrict__ out_list,
                   const int32_t* __restrict__ seg_ptr_ji, const float* __restrict__ cos_alpha, const __bf16* __restrict__ xb,
                   const float* __restrict__ coef, const int32_t* __restrict__ gap_of, const int32_t* __restrict__ grp_ptr,
                   const int32_t* __restrict__ grp_atom, int n_atoms, int C, int out_half, float* __restrict__ A) {
  constexpr int F = 16 * NT;
  constexpr int XT_B = SLAB / 8 * F * 16, CF_B = SLAB * COEF_ROW * 4, CS_B = GE * SLAB * 4, BUF_B = XT_B + CF_B + CS_B;
  constexpr int XT_LOADS = XT_B / 1024, CF_LOADS = CF_B / 1024;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int s_e[GE], s_seg[GE], s_gap[GE];

  // work item: (atom, group of GE out-edges), numbered atom-major; each XCD takes a contiguous range
  const int total = grp_ptr[n_atoms];
  const int q8 = total >> 3, r8 = total & 7, xcd = (int)blockIdx.x & 7, ith = (int)blockIdx.x >> 3;
  if (ith >= q8 + (xcd < r8 ? 1 : 0)) return;
  const int w = xcd * q8 + (xcd < r8 ? xcd : r8) + ith;
  const int j = grp_atom[w];
  const int part = w - grp_ptr[j];
  const int r0 = row_ptr[j], d = row_ptr[j + 1] - r0;
  const int o0 = out_ptr[j] + GE * part;
  const int n_e = out_ptr[j + 1] - o0 < GE ? out_ptr[j + 1] - o0 : GE;
  const int64_t base = padded_base(r0, j);
  const int n_slab = (d + SLAB - 1) / SLAB;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kq = lane >> 4, c = lane & 15;

  auto stage_async = [&](int slab, int buf) __attribute__((always_inline)) {
    unsigned char* dst = smem + buf * BUF_B;
    const int64_t row0 = base + (int64_t)SLAB * slab;
#pragma unroll
    for (int L = 0; L < (XT_LOADS + 7) / 8; ++L) {
      const int ld = wv + 8 * L;   // uniform
      if (ld < XT_LOADS) {
        const int piece = ld * 64 + lane, pb = piece / F, f = swz(piece % F);
        const __bf16* src = xb + ((row0 / 8 + pb) * F + f) * 8;
        __builtin_amdgcn_global_load_lds((global_void_ptr)src, (lds_void_ptr)(dst + ld * 1024), 16, 0, 0);
      }
    }
#pragma unroll
    for (int L = 0; L < CF_LOADS / 8; ++L) {
      const int ld = wv + 8 * L;
      const int piece = ld * 64 + lane, h = piece >> 10, p = (piece & 1023) >> 4, cc = piece & 15;
      const float* src = coef + (row0 + p) * COEF_ROW + h * 64 + cc * 4;
      __builtin_amdgcn_global_load_lds((global_void_ptr)src, (lds_void_ptr)(dst + XT_B + ld * 1024), 16, 0, 0);
    }
  };
  // cosines of the group's edges for one slab: thread (edge tid / 16, rows 4 (tid % 16) .. + 3); the row the segment
  // leaves out is marked 2, rows past the atom's last one give 0 (their coefficients are zero)
  const int c_el = tid >> 4, c_p = 4 * (tid & 15);
  auto load_cos = [&](int slab, float (&v)[4]) __attribute__((always_inline)) {
    const int seg = s_seg[c_el], gap = s_gap[c_el];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int P = SLAB * slab + c_p + i;
      const bool ok = P < d && P != gap && c_el < n_e;
      const float cv = cos_alpha[ok ? seg + P - (P > gap ? 1 : 0) : 0];   // index 0 exists: not launched for T = 0
      v[i] = ok ? cv : (P == gap ? 2.f : 0.f);
    }
  };
  auto write_cos = [&](int buf, const float (&v)[4]) __attribute__((always_inline)) {
    *reinterpret_cast<f32x4*>(smem + buf * BUF_B + XT_B + CF_B + (c_el * SLAB + c_p) * 4) = f32x4{v[0], v[1], v[2], v[3]};
  };

  if (n_slab > 0) stage_async(0, 0);
  if (tid < GE) {
    const bool ok = tid < n_e;
    const int e = out_list[o0 + (ok ? tid : 0)];
    s_e[tid] = ok ? e : -1;
    s_seg[tid] = seg_ptr_ji[e];
    s_gap[tid] = ok ? gap_of[e] : -1;
  }
  __syncthreads();
  float cosr[4];
  if (n_slab > 0) {
    load_cos(0, cosr);
    wait_vm0();
    write_cos(0, cosr);
  }
  __syncthreads();

  f32x4 acc[4][NT];
#pragma unroll
  for (int e4 = 0; e4 < 4; ++e4)
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[e4][t] = f32x4{0.f, 0.f, 0.f, 0.f};

  int gap4[4];
#pragma unroll
  for (int e4 = 0; e4 < 4; ++e4) gap4[e4] = __builtin_amdgcn_readfirstlane(s_gap[4 * wv + e4]);

  for (int s = 0; s < n_slab; ++s) {
    const int b = s & 1;
    const bool more = s + 1 < n_slab;
    if (more) {
      stage_async(s + 1, b ^ 1);
      load_cos(s + 1, cosr);
    }
    const unsigned char* buf = smem + b * BUF_B;
    const float* coefS = reinterpret_cast<const float*>(buf + XT_B);
    const float* cosS = reinterpret_cast<const float*>(buf + XT_B + CF_B);
#pragma unroll
    for (int ks = 0; ks < SLAB / 32; ++ks) {
      const int P0 = SLAB * s + 32 * ks;
      if (P0 < d) {
        float cf[8][8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int p = 32 * ks + 8 * kq + i;
          const f32x4 lo = *reinterpret_cast<const f32x4*>(coefS + (p * 16 + c) * 4);
          const f32x4 hi = *reinterpret_cast<const f32x4*>(coefS + 4096 + (p * 16 + c) * 4);
#pragma unroll
          for (int k = 0; k < 4; ++k) cf[i][k] = lo[k], cf[i][4 + k] = hi[k];
        }
        bf16x8 yb[4];
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
          const float* cp = cosS + (4 * wv + e4) * SLAB + 32 * ks + 8 * kq;
          const f32x4 c0 = *reinterpret_cast<const f32x4*>(cp), c1 = *reinterpret_cast<const f32x4*>(cp + 4);
          float xv[8] = {c0[0], c0[1], c0[2], c0[3], c1[0], c1[1], c1[2], c1[3]};
          const bool masked = gap4[e4] >= P0 && gap4[e4] < P0 + 32;   // uniform: this step holds the row the segment leaves out
          if (masked) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
              const bool ok = xv[i] <= 1.5f;
              const float xx = ok ? xv[i] : 0.f;
              float y = cf[i][SM - 1];
#pragma unroll
              for (int k = SM - 2; k >= 0; --k) y = y * xx + cf[i][k];
              yb[e4][i] = (__bf16)(ok ? y : 0.f);
            }
          } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
              float y = cf[i][SM - 1];
#pragma unroll
              for (int k = SM - 2; k >= 0; --k) y = y * xv[i] + cf[i][k];
              yb[e4][i] = (__bf16)y;
            }
          }
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          const bf16x8 xa = *reinterpret_cast<const bf16x8*>(buf + (((4 * ks + kq) * F + swz(NT * c + t)) << 4));
#pragma unroll
          for (int e4 = 0; e4 < 4; ++e4)
            acc[e4][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, yb[e4], acc[e4][t], 0, 0, 0);
        }
      }
    }
    if (more) {
      wait_vm0();
      write_cos(b ^ 1, cosr);
    }
    __syncthreads();
  }

  // accumulator register i of tile t in lane (g = kq, c): feature NT (4 g + i) + t, i.e. 4 NT consecutive features
#pragma unroll
  for (int e4 = 0; e4 < 4; ++e4) {
    const int el = 4 * wv + e4;
    if (el >= n_e || c >= C) continue;
    const int64_t at = ((int64_t)s_e[el] * C + c) * F + 4 * NT * kq;
    if (out_half) {
      __bf16* dst = reinterpret_cast<__bf16*>(A) + at;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if constexpr (NT == 8) {
          bf16x8 v;
#pragma unroll
          for (int t = 0; t < 8; ++t) v[t] = (__bf16)acc[e4][t][i];
          *reinterpret_cast<bf16x8*>(dst + 8 * i) = v;
        } else {
#pragma unroll
          for (int t = 0; t < NT; t += 2) {
            bf16x2 v;
            v[0] = (__bf16)acc[e4][t][i];
            v[1] = (__bf16)acc[e4][t + 1][i];
            *reinterpret_cast<bf16x2*>(dst + NT * i + t) = v;
          }
        }
      }
    } else {
      float* dst = A + at;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int t = 0; t < NT; t += 2) {
          typedef float f32x2 __attribute__((ext_vector_type(2)));
          *reinterpret_cast<f32x2*>(dst + NT * i + t) = f32x2{acc[e4][t][i], acc[e4][t + 1][i]};
        }
    }
  }
}

struct fused_ws {
  __bf16* xb;
  float* coef;
  int32_t *gap, *grp_ptr, *grp_atom;
};
size_t carve_fused(void* p, int64_t N, int64_t E, int F, fused_ws* w) {
  gp_carver c(p);
  const int64_t rows = padded_rows(E, N);
  w->xb = c.take<__bf16>((size_t)rows * F);
  w->coef = c.take<float>((size_t)rows * COEF_ROW);
  w->gap = c.take<int32_t>((size_t)E);
  w->grp_ptr = c.take<int32_t>((size_t)N + 1);
  w->grp_atom = c.take<int32_t>((size_t)(E / GE + N + 1));
  return c.off;
}

}  // namespace

size_t gp_tripG_fused_scratch(int64_t N, int64_t E, int F) {
  fused_ws w;
  return carve_fused(nullptr, N, E, F, &w);
}

bool gp_tripG_fused_usable(const gp_graph* g, int F, int S, int C) {
  if (!g || !g->row_ptr || !g->out_ptr || !g->out_list || g->n_atoms <= 0 || g->n_triplets <= 0) return false;
  if (g->n_atoms > INT32_MAX / 64 || g->n_edges / GE + g->n_atoms > INT32_MAX / 2) return false;
  if (g->max_in_degree <= 0 || g->max_out_degree <= 0) return false;
  return (F == 32 || F == 64 || F == 128) && C >= 1 && C <= CP && S >= 1 && S <= ST;
}

int gp_tripG_forward_fused(gp_ctx* ctx, const gp_graph* g, const float* cos_alpha, const float* x, const float* Radt,
                           int F, int S, int C, float* A, void* ws, size_t ws_bytes, int out_half) {
  const int64_t E = g->n_edges, T = g->n_triplets, N = g->n_atoms;
  if (E == 0) return GP_OK;
  GP_REQUIRE(ctx, gp_tripG_fused_usable(g, F, S, C), "triplet G (fused matrix-core form): graph lists or widths not supported");
  GP_REQUIRE(ctx, g->seg_ptr_ji && g->idx_kj && cos_alpha && x && Radt && A && ws, "triplet G forward: NULL pointer");
  fused_ws w;
  if (ws_bytes < carve_fused(ws, N, E, F, &w)) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "triplet G forward: workspace too small");
  hipStream_t st = ctx->stream;
  const double Td = (double)T, Ed = (double)E;
  {
    gp_prof_scope prof(ctx, "tripG_pack", Ed * 2.0 * S * 8 * CP, Ed * (4.0 * F + 4.0 * S * C + 2.0 * F + 4.0 * COEF_ROW + 8.0));
    fused_groups_kernel<<<1, 1024, 0, st>>>(g->out_ptr, (int)N, w.grp_ptr, w.grp_atom);
    const dim3 grid((unsigned)N, (unsigned)((g->max_in_degree + SLAB - 1) / SLAB));
    if (S <= 7)
      fused_pack_kernel<7><<<grid, 256, 0, st>>>(g->row_ptr, g->out_ptr, g->out_list, g->seg_ptr_ji, g->idx_kj, x, Radt, E, S, C, F,
                                                 w.xb, w.coef, w.gap);
    else
      fused_pack_kernel<8><<<grid, 256, 0, st>>>(g->row_ptr, g->out_ptr, g->out_list, g->seg_ptr_ji, g->idx_kj, x, Radt, E, S, C, F,
                                                 w.xb, w.coef, w.gap);
    GP_LAUNCH_CHECK(ctx, "fused_pack_kernel");
  }
  {
    gp_prof_scope prof(ctx, "tripG_fused_fwd", Td * (2.0 * C * F + 2.0 * S * C), Td * 4.0 + Ed * ((out_half ? 2.0 : 4.0) * C * F + 2.0 * F + 4.0 * COEF_ROW));
    const unsigned grid = (unsigned)(E / GE + N);   // an upper bound of the number of work items; the rest exit at once
#define GP_FUSED_LAUNCH(NT, SM)                                                                                          \
  do {                                                                                                                   \
    constexpr size_t lds = 2 * ((size_t)SLAB / 8 * 16 * NT * 16 + (size_t)SLAB * COEF_ROW * 4 + (size_t)GE * SLAB * 4);  \
    static bool raised = false;                                                                                          \
    if (!raised) {                                                                                                       \
      GP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&tripG_fused_kernel<NT, SM>),                        \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));                            \
      raised = true;                                                                                                     \
    }                                                                                                                    \
    tripG_fused_kernel<NT, SM><<<grid, FT, lds, st>>>(g->row_ptr, g->out_ptr, g->out_list, g->seg_ptr_ji, cos_alpha,     \
                                                      w.xb, w.coef, w.gap, w.grp_ptr, w.grp_atom, (int)N, C, out_half, A); \
  } while (0)
    if (S <= 7) {
      if (F == 128) GP_FUSED_LAUNCH(8, 7);
      else if (F == 64) GP_FUSED_LAUNCH(4, 7);
      else GP_FUSED_LAUNCH(2, 7);
    } else {
      if (F == 128) GP_FUSED_LAUNCH(8, 8);
      else if (F == 64) GP_FUSED_LAUNCH(4, 8);
      else GP_FUSED_LAUNCH(2, 8);
    }
#undef GP_FUSED_LAUNCH
    GP_LAUNCH_CHECK(ctx, "tripG_fused_kernel");
  }
  return GP_OK;
}
