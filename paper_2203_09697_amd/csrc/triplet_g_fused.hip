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

constexpr int GE = 16;          // out-edges per work item (4 wavefronts x 4 edges)
constexpr int SLAB = 32;        // in-edge rows per slab (one step of the matrix-core contraction)
constexpr int COEF_ROW = 128;   // floats per padded row of the coefficient table: [half][c 16][4]
constexpr int FT = 256;         // threads of the main kernel

// Work items (atom, group of GE out-edges), numbered atom-major: item[w] = {first padded row of the atom, its number
// of in-edge rows, out-list position of the group's first edge, edges in the group}; n_items[0] = their number.
// One workgroup (a scan over the atoms).
__global__ void __launch_bounds__(1024)
fused_items_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ out_ptr, int n_atoms,
                   int32_t* __restrict__ n_items, int32_t* __restrict__ item) {
  __shared__ int32_t wave_tot[16];
  __shared__ int32_t carry;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  if (tid == 0) carry = 0;
  __syncthreads();
  for (int base = 0; base < n_atoms; base += 1024) {
    const int j = base + tid;
    const int o0 = j < n_atoms ? out_ptr[j] : 0, dout = j < n_atoms ? out_ptr[j + 1] - o0 : 0;
    const int v = (dout + GE - 1) / GE;
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
      const int r0 = row_ptr[j], d = row_ptr[j + 1] - r0;
      const int first = before + incl - v;
      for (int k = 0; k < v; ++k) {
        int32_t* it = item + 4 * (int64_t)(first + k);
        it[0] = (int32_t)padded_base(r0, j);
        it[1] = d;
        it[2] = o0 + GE * k;
        it[3] = dout - GE * k < GE ? dout - GE * k : GE;
      }
    }
    __syncthreads();
    if (tid == 1023) carry = before + incl;
    __syncthreads();
  }
  if (tid == 0) n_items[0] = carry;
}

// Pre-pass, one workgroup per (atom j, 64 of its padded rows), in two kernels.  First X^T in bf16 as [p-block of 8 rows][f][8]
// (no LDS, so many workgroups per compute unit; inside the second kernel its stores held back the loads of the radial
// part, which complete through the same counter).  Rows past the atom's last one are zero: padded rows contribute nothing.
__global__ void __launch_bounds__(256)
fused_pack_x_kernel(const int32_t* __restrict__ row_ptr, const float* __restrict__ x, int F, const int32_t* __restrict__ rows,
                    __bf16* __restrict__ xb) {
  const int j = blockIdx.x;
  const int r0 = row_ptr[j], d = row_ptr[j + 1] - r0;
  const int p0 = ROWPAD * (int)blockIdx.y;
  if (p0 >= ((d + ROWPAD - 1) & ~(ROWPAD - 1))) return;
  const int64_t base = padded_base(r0, j) + p0;
  // item (p-block pb, feature f); consecutive threads take consecutive f of the same rows
  for (int it = threadIdx.x; it < (ROWPAD / 8) * F; it += 256) {
    const int pb = it / F, f = it % F;
    bf16x8 v;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int p = p0 + 8 * pb + i;
      const int q = r0 + (p < d ? p : 0);                            // clamped row, zeroed below: the load stays unconditional
      const float xv = x[(int64_t)(rows ? rows[q] : q) * F + f];
      v[i] = (__bf16)(p < d ? xv : 0.f);
    }
    *reinterpret_cast<bf16x8*>(xb + ((base / 8 + pb) * F + f) * 8) = v;
  }
}

// The out-edge table of the pre-pass, one thread per out-edge (grid: atoms x blocks of 256 out-edges): {edge id, start of its
// segment, position of the row the segment leaves out (the number of rows if none), rows in the segment}; the search for
// the left-out row is a chain of dependent loads, which the other two kernels no longer wait behind.
__global__ void __launch_bounds__(256)
fused_pack_info_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ out_ptr, const int32_t* __restrict__ out_list,
                       const int32_t* __restrict__ seg_ptr_ji, const int32_t* __restrict__ idx_kj, const int32_t* __restrict__ rows,
                       int32_t* __restrict__ edge_info) {
  const int j = blockIdx.x;
  const int r0 = row_ptr[j];
  const int o0 = out_ptr[j], dout = out_ptr[j + 1] - o0;
  const int t = 256 * (int)blockIdx.y + threadIdx.x;
  if (t >= dout) return;
  const int e = out_list[o0 + t];
  const int seg = seg_ptr_ji[e], cnt = seg_ptr_ji[e + 1] - seg;
  const int gap = first_mismatch(idx_kj + seg, cnt, [=](int slot) { return rows ? rows[r0 + slot] : r0 + slot; });
  int32_t* dst = edge_info + 4 * (int64_t)(o0 + t);
  dst[0] = e;
  dst[1] = seg;
  dst[2] = gap;                   // = cnt = the number of rows when no row is left out
  dst[3] = cnt;
}

// Third kernel, the first one's grid: the coefficients of the powers of cos alpha as [row][half][c][4] (rows past the atom's last one
// and columns past C are zero), or with RADB the radial values themselves.
template <int SM, bool RADB = false>
__global__ void __launch_bounds__(256)
fused_pack_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ out_ptr, const int32_t* __restrict__ out_list,
                  const int32_t* __restrict__ seg_ptr_ji, const int32_t* __restrict__ idx_kj, const float* __restrict__ x,
                  const float* __restrict__ Radt, int64_t E, int S, int C, int F, const int32_t* __restrict__ rows,
                  __bf16* __restrict__ xb, float* __restrict__ coef, int32_t* __restrict__ edge_info) {
  const int j = blockIdx.x;
  const int r0 = row_ptr[j], d = row_ptr[j + 1] - r0;
  const int p0 = ROWPAD * (int)blockIdx.y;
  if (p0 >= ((d + ROWPAD - 1) & ~(ROWPAD - 1))) return;
  const int64_t base = padded_base(r0, j) + p0;
  // coefficients.  Radt is read with consecutive threads on consecutive rows of one (l, c) line and parked in LDS;
  // the table is then written with consecutive threads on consecutive c of one row, i.e. in whole 256-byte runs
  // (written straight from the first order, every 16-byte store went to a line of its own: 0.24 -> 0.1 ms at 3e5 edges).
  __shared__ float s_r[SM * CP * (ROWPAD + 1)];
  for (int it = threadIdx.x; it < ROWPAD * CP; it += 256) {
    const int pl = it % ROWPAD, c = it / ROWPAD, p = p0 + pl;
    const bool ok = p < d && c < C;
#pragma unroll
    for (int l = 0; l < SM; ++l)
      s_r[(l * CP + c) * (ROWPAD + 1) + pl] =
          Radt[(int64_t)((l < S ? l : 0) * C + (c < C ? c : 0)) * E + r0 + (p < d ? p : 0)] * ((ok && l < S) ? Y_NORM_M[l] : 0.f);
  }
  __syncthreads();
  for (int it = threadIdx.x; it < ROWPAD * CP; it += 256) {
    const int c = it % CP, pl = it / CP;
    float rl[SM];
#pragma unroll
    for (int l = 0; l < SM; ++l) rl[l] = s_r[(l * CP + c) * (ROWPAD + 1) + pl];
    if constexpr (RADB) {
      // the normalised radial values themselves, bf16 [row][c][8 l]: the kernel forms y with the matrix cores
      bf16x8 v;
#pragma unroll
      for (int l = 0; l < 8; ++l) v[l] = (__bf16)(l < SM ? rl[l < SM ? l : 0] : 0.f);
      *reinterpret_cast<bf16x8*>(reinterpret_cast<__bf16*>(coef) + ((base + pl) * CP + c) * 8) = v;
      continue;
    }
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

// Two workgroups of 4 wavefronts share a compute unit (the registers allow 8 wavefronts): they work on different
// items and drift apart, so one's staging, stores and prologue run beside the other's arithmetic.
template <int NT, int SM>   // F = 16 NT (NT = 2, 4, 8); SM = number of polynomial coefficients kept (>= num_spherical)
__global__ void __launch_bounds__(FT, 2)
tripG_fused_kernel(const float* __restrict__ cos_alpha, int64_t T, const __bf16* __restrict__ xb, const float* __restrict__ coef,
                   const int32_t* __restrict__ edge_info, const int32_t* __restrict__ n_items, const int32_t* __restrict__ item,
                   int C, int out_half, float* __restrict__ A) {
  constexpr int F = 16 * NT;
  constexpr int XT_B = SLAB / 8 * F * 16, CF_B = SLAB * COEF_ROW * 4, CS_B = GE * SLAB * 4, BUF_B = XT_B + CF_B + CS_B;
  constexpr int XT_LOADS = XT_B / 1024, CF_LOADS = CF_B / 1024, CS_LOADS = CS_B / 256;
  static_assert(CF_LOADS % 4 == 0 && CS_LOADS % 4 == 0, "the loads of a slab are dealt evenly to the 4 wavefronts");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int s_e[GE], s_seg[GE], s_gap[GE];

  // work items are numbered atom-major; each XCD (workgroup ids are dealt round-robin to the 8 XCDs) takes a contiguous
  // range of them, so the groups of one atom, which stage the same rows, run side by side on one L2
  const int total = n_items[0];
  const int q8 = total >> 3, r8 = total & 7, xcd = (int)blockIdx.x & 7, ith = (int)blockIdx.x >> 3;
  if (ith >= q8 + (xcd < r8 ? 1 : 0)) return;
  const int w = xcd * q8 + (xcd < r8 ? xcd : r8) + ith;
  const int4 it = *reinterpret_cast<const int4*>(item + 4 * (int64_t)w);
  const int64_t base = it.x;
  const int d = it.y, o0 = it.z, n_e = it.w;
  const int n_slab = (d + SLAB - 1) / SLAB;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kq = lane >> 4, c = lane & 15;

  // per-lane parts of the source offsets (the same for every slab and load); the rest is uniform
  // X^T: a load covers 4 consecutive (p-block, tile) pairs, 16 rows each: pair 4 ld + lane / 16
  const int xt_lane = ((kq / NT) * F + NT * rowperm(c) + kq % NT) * 8;   // bf16 elements
  const int cf_lane = (lane >> 4) * COEF_ROW + (lane & 15) * 4;          // floats: row lane/16 of the load's 4 rows, column lane%16
  auto stage_tables = [&](int slab, int buf) __attribute__((always_inline)) {
    unsigned char* dst = smem + buf * BUF_B;
    const int64_t row0 = base + (int64_t)SLAB * slab;
#pragma unroll
    for (int L = 0; L < (XT_LOADS + 3) / 4; ++L) {
      // uniform; a wavefront without a load of its own repeats the last one, so that every wavefront issues the same
      // number of loads per slab and can wait for "all but the newest slab's"
      const int ld = wv + 4 * L < XT_LOADS ? wv + 4 * L : XT_LOADS - 1;
      const __bf16* src = xb + ((row0 / 8 + (4 * ld) / NT) * F + (4 * ld) % NT) * 8 + xt_lane;
      __builtin_amdgcn_global_load_lds((global_void_ptr)src, (lds_void_ptr)(dst + ld * 1024), 16, 0, 0);
    }
#pragma unroll
    for (int L = 0; L < CF_LOADS / 4; ++L) {
      const int ld = wv + 4 * L;   // pieces 64 ld ..: half ld / 8, rows 4 (ld % 8) .. + 3, columns 0..15
      const float* src = coef + (row0 + 4 * (ld & 7)) * COEF_ROW + (ld >> 3) * 64 + cf_lane;
      __builtin_amdgcn_global_load_lds((global_void_ptr)src, (lds_void_ptr)(dst + XT_B + ld * 1024), 16, 0, 0);
    }
  };

  constexpr int PW = (XT_LOADS + 3) / 4 + CF_LOADS / 4 + CS_LOADS / 4;   // loads per wavefront and slab
  if (n_slab > 0) stage_tables(0, 0);
  if (tid < GE) {
    const int4 ei = *reinterpret_cast<const int4*>(edge_info + 4 * (int64_t)(o0 + (tid < n_e ? tid : 0)));
    s_e[tid] = tid < n_e ? ei.x : -1;
    s_seg[tid] = ei.y;
    s_gap[tid] = tid < n_e ? ei.z : -1;
  }
  __syncthreads();
  // Cosines: 4-byte global->LDS loads, a wavefront's load covers 2 edges x 32 rows.  Row P of the atom is slot P, or
  // P - 1 behind the row the segment leaves out, of the edge's segment; the left-out row itself and rows past the
  // atom's last one fetch some valid cosine that is never used (the former is zeroed below, the latter have zero
  // coefficients).
  int cs_seg[CS_LOADS / 4], cs_gap[CS_LOADS / 4];
#pragma unroll
  for (int L = 0; L < CS_LOADS / 4; ++L) {
    const int el = 2 * (wv + 4 * L) + (lane >> 5);
    cs_seg[L] = s_seg[el];
    cs_gap[L] = s_gap[el];
  }
  auto stage_cos = [&](int slab, int buf) __attribute__((always_inline)) {
    unsigned char* dst = smem + buf * BUF_B + XT_B + CF_B;
#pragma unroll
    for (int L = 0; L < CS_LOADS / 4; ++L) {
      const int ld = wv + 4 * L;
      const int P = SLAB * slab + (lane & 31);
      int64_t idx = (int64_t)cs_seg[L] + P - (P > cs_gap[L] ? 1 : 0);
      idx = idx < 0 ? 0 : (idx < T ? idx : T - 1);   // edges past the group's last one, the end of the array
      __builtin_amdgcn_global_load_lds((global_void_ptr)(cos_alpha + idx), (lds_void_ptr)(dst + ld * 256), 4, 0, 0);
    }
  };
  if (n_slab > 0) stage_cos(0, 0);
  if (n_slab > 1) {
    stage_tables(1, 1);
    stage_cos(1, 1);
  }

  f32x4 acc[4][NT];
#pragma unroll
  for (int e4 = 0; e4 < 4; ++e4)
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[e4][t] = f32x4{0.f, 0.f, 0.f, 0.f};
  int gap4[4];
#pragma unroll
  for (int e4 = 0; e4 < 4; ++e4) gap4[e4] = __builtin_amdgcn_readfirstlane(s_gap[4 * wv + e4]);
  if (n_slab > 1) wait_vmcnt<PW>();   // slab 0 has landed (this wavefront's part; the barrier covers the others')
  else wait_vm0();
  __syncthreads();

  int b = 0;   // ring of STAGES buffers: slab s in buffer s % STAGES, slabs s + 1 and s + 2 on their way
  for (int s = 0; s < n_slab; ++s) {
    const int b2 = b >= 1 ? b - 1 : STAGES - 1;   // (s + 2) % STAGES
    const bool more = s + 2 < n_slab;
    if (more) {
      stage_tables(s + 2, b2);
      stage_cos(s + 2, b2);
    }
    const unsigned char* buf = smem + b * BUF_B;
    const float* coefS = reinterpret_cast<const float*>(buf + XT_B);
    const float* cosS = reinterpret_cast<const float*>(buf + XT_B + CF_B);
    const int P0 = SLAB * s;
    float cf[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int p = 8 * kq + i;
      const f32x4 lo = *reinterpret_cast<const f32x4*>(coefS + (p * 16 + c) * 4);
      const f32x4 hi = *reinterpret_cast<const f32x4*>(coefS + SLAB * 64 + (p * 16 + c) * 4);
#pragma unroll
      for (int k = 0; k < 4; ++k) cf[i][k] = lo[k], cf[i][4 + k] = hi[k];
    }
    bf16x8 yb[4];
#pragma unroll
    for (int e4 = 0; e4 < 4; ++e4) {
      const float* cp = cosS + (4 * wv + e4) * SLAB + 8 * kq;
      const f32x4 c0 = *reinterpret_cast<const f32x4*>(cp), c1 = *reinterpret_cast<const f32x4*>(cp + 4);
      const float xv[8] = {c0[0], c0[1], c0[2], c0[3], c1[0], c1[1], c1[2], c1[3]};
      float y[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float v = cf[i][SM - 1];
#pragma unroll
        for (int k = SM - 2; k >= 0; --k) v = v * xv[i] + cf[i][k];
        y[i] = v;
      }
      if (gap4[e4] >= P0 && gap4[e4] < P0 + SLAB) {   // uniform: this slab holds the row the segment leaves out (k = i)
        const int gl = gap4[e4] - P0 - 8 * kq;
#pragma unroll
        for (int i = 0; i < 8; ++i) y[i] = gl == i ? 0.f : y[i];
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) yb[e4][i] = (__bf16)y[i];
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const bf16x8 xa = *reinterpret_cast<const bf16x8*>(buf + ((kq * F + t * 16 + c) << 4));
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4)
        acc[e4][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, yb[e4], acc[e4][t], 0, 0, 0);
    }
    if (more) wait_vmcnt<PW>();   // slab s + 1 has landed, slab s + 2 may still be under way
    else wait_vm0();
    __syncthreads();
    b = b == STAGES - 1 ? 0 : b + 1;
  }

  // accumulator register i of tile t in lane (g = kq, c): feature NT (4 i + g) + t
#pragma unroll
  for (int e4 = 0; e4 < 4; ++e4) {
    const int el = 4 * wv + e4;
    if (el >= n_e || c >= C) continue;
    const int64_t at = ((int64_t)s_e[el] * C + c) * F + NT * kq;
    if (out_half) {
      __bf16* dst = reinterpret_cast<__bf16*>(A) + at;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if constexpr (NT == 8) {
          bf16x8 v;
#pragma unroll
          for (int t = 0; t < 8; ++t) v[t] = (__bf16)acc[e4][t][i];
          *reinterpret_cast<bf16x8*>(dst + 32 * i) = v;
        } else {
#pragma unroll
          for (int t = 0; t < NT; t += 2) {
            bf16x2 v;
            v[0] = (__bf16)acc[e4][t][i];
            v[1] = (__bf16)acc[e4][t + 1][i];
            *reinterpret_cast<bf16x2*>(dst + 4 * NT * i + t) = v;
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
          *reinterpret_cast<f32x2*>(dst + 4 * NT * i + t) = f32x2{acc[e4][t][i], acc[e4][t + 1][i]};
        }
    }
  }
}

// The same sum with y itself formed on the matrix cores.  For 4 rows p_q (q = 0..3) and the wavefront's 4 out-edges e',
//
//   y[p_q, e', c] = sum_l P_l(cos alpha(p_q, e')) R[p_q, l, c]        (R: normalised radial values, bf16)
//
// is one v_mfma_f32_16x16x32_bf16 with rows (q, e'), contraction index (q', l) and an operand that is zero unless q' = q:
// lane (kq, r = (q, e')) supplies the 8 Legendre values of its pair when kq = q and zeros otherwise, lane (kq, c) of the
// other operand the 8 radial values of row p_kq.  Taking p_q = 8 q + j in the j-th of 8 such products, lane (g, c) ends up
// with y[8 g + j, e' = i, c] in result register i of product j: for every edge i exactly the 8 consecutive rows it must
// supply to the second product D[f, c] += X^T[f, p] Y[p, c].  A quarter of the first product's arithmetic is used, but
// the vector units, where the one-pass kernel above spends most of its time (7 multiply-adds per value y), are left with
// the Legendre recurrence of the wavefront's 128 (row, edge) pairs per slab: two pairs per lane, handed to the lanes that
// feed the products through a slice of LDS the wavefront owns (its LDS operations complete in order: no barrier).
template <int NT>
__global__ void __launch_bounds__(FT, 2)
tripG_fusedM_kernel(const float* __restrict__ cos_alpha, int64_t T, const __bf16* __restrict__ xb, const __bf16* __restrict__ radb,
                    const int32_t* __restrict__ edge_info, const int32_t* __restrict__ n_items, const int32_t* __restrict__ item,
                    int C, int S, int out_half, float* __restrict__ A) {
  constexpr int F = 16 * NT;
  constexpr int XT_B = SLAB / 8 * F * 16, RB_B = SLAB * CP * 16, CS_B = GE * SLAB * 4, BUF_B = XT_B + RB_B + CS_B;
  constexpr int XT_LOADS = XT_B / 1024, RB_LOADS = RB_B / 1024, CS_LOADS = CS_B / 256;
  static_assert(RB_LOADS % 4 == 0 && CS_LOADS % 4 == 0 && CP == 16, "the loads of a slab are dealt evenly to the 4 wavefronts");
  constexpr int PAIR_B = 4 * SLAB * 16;   // a wavefront's pairs of one slab, 8 bf16 each: [row % 8][row / 8][edge]
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int s_e[GE], s_seg[GE], s_gap[GE];
  unsigned char* pairS = smem + STAGES * BUF_B;   // 4 slices of PAIR_B bytes, then PAIR_B bytes of zeros

  const int total = n_items[0];
  const int q8 = total >> 3, r8 = total & 7, xcd = (int)blockIdx.x & 7, ith = (int)blockIdx.x >> 3;
  if (ith >= q8 + (xcd < r8 ? 1 : 0)) return;
  const int w = xcd * q8 + (xcd < r8 ? xcd : r8) + ith;
  const int4 it = *reinterpret_cast<const int4*>(item + 4 * (int64_t)w);
  const int64_t base = it.x;
  const int d = it.y, o0 = it.z, n_e = it.w;
  const int n_slab = (d + SLAB - 1) / SLAB;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kq = lane >> 4, c = lane & 15;

  const int xt_lane = ((kq / NT) * F + NT * rowperm(c) + kq % NT) * 8;   // bf16 elements (see the kernel above)
  auto stage_tables = [&](int slab, int buf) __attribute__((always_inline)) {
    unsigned char* dst = smem + buf * BUF_B;
    const int64_t row0 = base + (int64_t)SLAB * slab;
#pragma unroll
    for (int L = 0; L < (XT_LOADS + 3) / 4; ++L) {
      const int ld = wv + 4 * L < XT_LOADS ? wv + 4 * L : XT_LOADS - 1;
      const __bf16* src = xb + ((row0 / 8 + (4 * ld) / NT) * F + (4 * ld) % NT) * 8 + xt_lane;
      __builtin_amdgcn_global_load_lds((global_void_ptr)src, (lds_void_ptr)(dst + ld * 1024), 16, 0, 0);
    }
#pragma unroll
    for (int L = 0; L < RB_LOADS / 4; ++L) {
      const int ld = wv + 4 * L;   // rows 4 ld .. 4 ld + 3: 1 KB, contiguous in the table
      const __bf16* src = radb + (row0 + 4 * ld) * (CP * 8) + lane * 8;
      __builtin_amdgcn_global_load_lds((global_void_ptr)src, (lds_void_ptr)(dst + XT_B + ld * 1024), 16, 0, 0);
    }
  };
  constexpr int PW = (XT_LOADS + 3) / 4 + RB_LOADS / 4 + CS_LOADS / 4;
  if (n_slab > 0) stage_tables(0, 0);
  reinterpret_cast<uint64_t*>(pairS + 4 * PAIR_B)[tid] = 0ull;
  if (tid < GE) {
    const int4 ei = *reinterpret_cast<const int4*>(edge_info + 4 * (int64_t)(o0 + (tid < n_e ? tid : 0)));
    s_e[tid] = tid < n_e ? ei.x : -1;
    s_seg[tid] = ei.y;
    s_gap[tid] = tid < n_e ? ei.z : -1;
  }
  __syncthreads();
  int cs_seg[CS_LOADS / 4], cs_gap[CS_LOADS / 4];
#pragma unroll
  for (int L = 0; L < CS_LOADS / 4; ++L) {
    const int el = 2 * (wv + 4 * L) + (lane >> 5);
    cs_seg[L] = s_seg[el];
    cs_gap[L] = s_gap[el];
  }
  auto stage_cos = [&](int slab, int buf) __attribute__((always_inline)) {
    unsigned char* dst = smem + buf * BUF_B + XT_B + RB_B;
#pragma unroll
    for (int L = 0; L < CS_LOADS / 4; ++L) {
      const int ld = wv + 4 * L;
      const int P = SLAB * slab + (lane & 31);
      int64_t idx = (int64_t)cs_seg[L] + P - (P > cs_gap[L] ? 1 : 0);
      idx = idx < 0 ? 0 : (idx < T ? idx : T - 1);
      __builtin_amdgcn_global_load_lds((global_void_ptr)(cos_alpha + idx), (lds_void_ptr)(dst + ld * 256), 4, 0, 0);
    }
  };
  if (n_slab > 0) stage_cos(0, 0);
  if (n_slab > 1) {
    stage_tables(1, 1);
    stage_cos(1, 1);
  }

  f32x4 acc[4][NT];
#pragma unroll
  for (int e4 = 0; e4 < 4; ++e4)
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[e4][t] = f32x4{0.f, 0.f, 0.f, 0.f};
  // Legendre values: this lane evaluates the pairs (rows r_p and r_p + 4, edge e_p) and stores them at positions lane
  // and lane + 64 of the slice ...
  const int e_p = lane & 3, r_p = 8 * ((lane >> 2) & 3) + (lane >> 4);
  const int my_gap = s_gap[4 * wv + e_p] - r_p;   // the left-out row relative to the lane's first row of slab 0
  unsigned char* pair_wr = pairS + wv * PAIR_B + lane * 16;
  // ... and feeds the first products as lane (kq, r = (q, e')): the pair (row 8 q + j, e') when q = kq, zeros otherwise
  const unsigned char* pair_rd = (c >> 2) == kq ? pairS + wv * PAIR_B + (4 * kq + (c & 3)) * 16 : pairS + 4 * PAIR_B;
  if (n_slab > 1) wait_vmcnt<PW>();
  else wait_vm0();
  __syncthreads();

  int b = 0;
  for (int s = 0; s < n_slab; ++s) {
    const int b2 = b >= 1 ? b - 1 : STAGES - 1;
    const bool more = s + 2 < n_slab;
    if (more) {
      stage_tables(s + 2, b2);
      stage_cos(s + 2, b2);
    }
    const unsigned char* buf = smem + b * BUF_B;
    const unsigned char* radS = buf + XT_B;
    const float* cosS = reinterpret_cast<const float*>(buf + XT_B + RB_B);
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const float* cp = cosS + (4 * wv + e_p) * SLAB + r_p;
    const f32x2 cx = {cp[0], cp[4]};
    const int gl = my_gap - SLAB * s;   // 0 or 4 if the left-out row is this lane's first or second
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      // Legendre polynomials P_0..P_7 of the pair's cosine (the normalisation sits in the radial table)
      const float x = cx[h];
      float P[8];
      P[0] = 1.f;
      P[1] = x;
#pragma unroll
      for (int l = 1; l < 7; ++l) P[l + 1] = ((float)(2 * l + 1) / (float)(l + 1)) * x * P[l] - ((float)l / (float)(l + 1)) * P[l - 1];
      union {
        bf16x8 h8;
        u32x4 w;
      } pk;
#pragma unroll
      for (int l = 0; l < 8; ++l) pk.h8[l] = (__bf16)P[l];
      if (gl == 4 * h) pk.w = u32x4{0u, 0u, 0u, 0u};
      *reinterpret_cast<u32x4*>(pair_wr + 1024 * h) = pk.w;
    }
    bf16x8 yb[4];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const bf16x8 rb = *reinterpret_cast<const bf16x8*>(radS + (((8 * kq + j) * CP + c) << 4));
      const bf16x8 pa = *reinterpret_cast<const bf16x8*>(pair_rd + 256 * j);
      const f32x4 y = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa, rb, f32x4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
#pragma unroll
      for (int i = 0; i < 4; ++i) yb[i][j] = (__bf16)y[i];
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const bf16x8 xa = *reinterpret_cast<const bf16x8*>(buf + ((kq * F + t * 16 + c) << 4));
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4)
        acc[e4][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, yb[e4], acc[e4][t], 0, 0, 0);
    }
    if (more) wait_vmcnt<PW>();
    else wait_vm0();
    __syncthreads();
    b = b == STAGES - 1 ? 0 : b + 1;
  }

  // accumulator register i of tile t in lane (g = kq, c): feature NT (4 i + g) + t
#pragma unroll
  for (int e4 = 0; e4 < 4; ++e4) {
    const int el = 4 * wv + e4;
    if (el >= n_e || c >= C) continue;
    const int64_t at = ((int64_t)s_e[el] * C + c) * F + NT * kq;
    if (out_half) {
      __bf16* dst = reinterpret_cast<__bf16*>(A) + at;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if constexpr (NT == 8) {
          bf16x8 v;
#pragma unroll
          for (int t = 0; t < 8; ++t) v[t] = (__bf16)acc[e4][t][i];
          *reinterpret_cast<bf16x8*>(dst + 32 * i) = v;
        } else {
#pragma unroll
          for (int t = 0; t < NT; t += 2) {
            bf16x2 v;
            v[0] = (__bf16)acc[e4][t][i];
            v[1] = (__bf16)acc[e4][t + 1][i];
            *reinterpret_cast<bf16x2*>(dst + 4 * NT * i + t) = v;
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
          *reinterpret_cast<f32x2*>(dst + 4 * NT * i + t) = f32x2{acc[e4][t][i], acc[e4][t + 1][i]};
        }
    }
  }
}

struct fused_ws {
  __bf16* xb;
  float* coef;
  int32_t *edge_info, *n_items, *item;
};
size_t carve_fused(void* p, int64_t N, int64_t E, int F, fused_ws* w) {
  gp_carver c(p);
  const int64_t rows = padded_rows(E, N);
  w->xb = c.take<__bf16>((size_t)rows * F);
  w->coef = c.take<float>((size_t)rows * COEF_ROW);
  w->edge_info = c.take<int32_t>(4 * (size_t)E);
  w->n_items = c.take<int32_t>(4);
  w->item = c.take<int32_t>(4 * (size_t)(E / GE + N + 1));
  return c.off;
}

}  // namespace

size_t gp_tripG_fused_scratch(int64_t N, int64_t E, int F) {
  fused_ws w;
  return carve_fused(nullptr, N, E, F, &w);
}

bool gp_tripG_fused_usable(const gp_graph* g, int F, int S, int C) {
  if (!g || !g->row_ptr || !g->out_ptr || !g->out_list || g->n_atoms <= 0 || g->n_triplets <= 0) return false;
  if (g->n_edges + (int64_t)PADJ * g->n_atoms + ROWPAD + 8 > INT32_MAX || g->n_edges / GE + g->n_atoms > INT32_MAX / 8) return false;
  if (g->max_in_degree <= 0 || g->max_out_degree <= 0) return false;
  return (F == 32 || F == 64 || F == 128) && C >= 1 && C <= CP && S >= 1 && S <= ST;
}

int gp_tripG_forward_fused(gp_ctx* ctx, const gp_graph* g, const float* cos_alpha, const float* x, const float* Radt,
                           int F, int S, int C, float* A, void* ws, size_t ws_bytes, int out_half, const int32_t* rows_list) {
  const int64_t E = g->n_edges, T = g->n_triplets, N = g->n_atoms;
  if (E == 0) return GP_OK;
  GP_REQUIRE(ctx, gp_tripG_fused_usable(g, F, S, C), "triplet G (fused matrix-core form): graph lists or widths not supported");
  GP_REQUIRE(ctx, g->seg_ptr_ji && g->idx_kj && cos_alpha && x && Radt && A && ws, "triplet G forward: NULL pointer");
  fused_ws w;
  if (ws_bytes < carve_fused(ws, N, E, F, &w)) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "triplet G forward: workspace too small");
  hipStream_t st = ctx->stream;
  const double Td = (double)T, Ed = (double)E;
  const bool y_mfma = ctx->trip_mfma != 3;   // mode 3: the earlier one-pass kernel that evaluates y on the vector units
  {
    gp_prof_scope prof(ctx, "tripG_pack", Ed * 2.0 * S * 8 * CP, Ed * (4.0 * F + 4.0 * S * C + 2.0 * F + 4.0 * COEF_ROW + 8.0));
    fused_items_kernel<<<1, 1024, 0, st>>>(g->row_ptr, g->out_ptr, (int)N, w.n_items, w.item);
    const dim3 grid((unsigned)N, (unsigned)((g->max_in_degree + ROWPAD - 1) / ROWPAD));
    fused_pack_x_kernel<<<grid, 256, 0, st>>>(g->row_ptr, x, F, rows_list, w.xb);
    fused_pack_info_kernel<<<dim3((unsigned)N, (unsigned)((g->max_out_degree + 255) / 256)), 256, 0, st>>>(
        g->row_ptr, g->out_ptr, g->out_list, g->seg_ptr_ji, g->idx_kj, rows_list, w.edge_info);
    if (y_mfma)
      fused_pack_kernel<8, true><<<grid, 256, 0, st>>>(g->row_ptr, g->out_ptr, g->out_list, g->seg_ptr_ji, g->idx_kj, x, Radt, E, S, C,
                                                       F, rows_list, w.xb, w.coef, w.edge_info);
    else if (S <= 7)
      fused_pack_kernel<7><<<grid, 256, 0, st>>>(g->row_ptr, g->out_ptr, g->out_list, g->seg_ptr_ji, g->idx_kj, x, Radt, E, S, C, F,
                                                 rows_list, w.xb, w.coef, w.edge_info);
    else
      fused_pack_kernel<8><<<grid, 256, 0, st>>>(g->row_ptr, g->out_ptr, g->out_list, g->seg_ptr_ji, g->idx_kj, x, Radt, E, S, C, F,
                                                 rows_list, w.xb, w.coef, w.edge_info);
    GP_LAUNCH_CHECK(ctx, "fused_pack_kernel");
  }
  {
    gp_prof_scope prof(ctx, "tripG_fused_fwd", Td * (2.0 * C * F + 2.0 * S * C), Td * 4.0 + Ed * ((out_half ? 2.0 : 4.0) * C * F + 2.0 * F + 4.0 * COEF_ROW));
    const unsigned grid = (unsigned)(E / GE + N);   // an upper bound of the number of work items; the rest exit at once
#define GP_FUSEDM_LAUNCH(NT)                                                                                             \
  do {                                                                                                                   \
    constexpr size_t lds = STAGES * ((size_t)SLAB / 8 * 16 * NT * 16 + (size_t)SLAB * CP * 16 + (size_t)GE * SLAB * 4) +  \
                           5 * (size_t)4 * SLAB * 16; /* + the wavefronts' Legendre pairs and the zeros */              \
    static_assert(2 * (lds + 256) <= 160 * 1024, "two workgroups per compute unit");                                     \
    static bool raised = false;                                                                                          \
    if (!raised && lds > 64 * 1024) {                                                                                    \
      GP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&tripG_fusedM_kernel<NT>),                           \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));                            \
      raised = true;                                                                                                     \
    }                                                                                                                    \
    tripG_fusedM_kernel<NT><<<grid, FT, lds, st>>>(cos_alpha, T, w.xb, reinterpret_cast<const __bf16*>(w.coef), w.edge_info,  \
                                                   w.n_items, w.item, C, S, out_half, A);                                \
  } while (0)
    if (y_mfma) {
      if (F == 128) GP_FUSEDM_LAUNCH(8);
      else if (F == 64) GP_FUSEDM_LAUNCH(4);
      else GP_FUSEDM_LAUNCH(2);
      GP_LAUNCH_CHECK(ctx, "tripG_fusedM_kernel");
      return GP_OK;
    }
#undef GP_FUSEDM_LAUNCH
#define GP_FUSED_LAUNCH(NT, SM)                                                                                          \
  do {                                                                                                                   \
    constexpr size_t lds = STAGES * ((size_t)SLAB / 8 * 16 * NT * 16 + (size_t)SLAB * COEF_ROW * 4 + (size_t)GE * SLAB * 4); \
    static_assert(2 * (lds + 256) <= 160 * 1024, "two workgroups per compute unit");                                     \
    static bool raised = false;                                                                                          \
    if (!raised && lds > 64 * 1024) {                                                                                    \
      GP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&tripG_fused_kernel<NT, SM>),                        \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));                            \
      raised = true;                                                                                                     \
    }                                                                                                                    \
    tripG_fused_kernel<NT, SM><<<grid, FT, lds, st>>>(cos_alpha, T, w.xb, w.coef, w.edge_info, w.n_items, w.item, C,     \
                                                      out_half, A);                                                      \
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
