// Backward triplet sum of the bilinear block (paper Sec. 3.4) per centre atom, staged like the one-pass forward kernel:
//
//   H[e', l, o] = sum_{t: kj(t)=e'} Y_l0(cos alpha_t) dz[ji(t), o]
//
// For centre atom j every in-edge row e' = (k->j) sums over the same out-edges e = (j->i) of j (positions n in its
// out-list), so H of the atom is one dense product with rows (in-edge, l), contraction over n and columns o.  As in
// triplet_g_fused.hip the product runs transposed on v_mfma_f32_16x16x32_bf16,
//
//   D[o, (p, l)] += dz^T[o, n] . Y[n, (p, l)]      rows o (16 per tile), contraction over 32 out-edges, columns 2 rows x 8 l
//
// with dz^T of the atom's out-edges laid out by a pre-pass (bf16, blocks of 8 positions) and streamed through an LDS
// ring by global->LDS loads together with the cosines of the group's rows (kj-major order, 4-byte loads that skip
// the position each row's segment leaves out), and the operand Y evaluated in registers: a lane keeps one l, so
// Y_l0 is one short even/odd polynomial of the cosine.  Work item = (centre atom, group of 32 in-edge rows):
// 4 wavefronts x 4 fragments of 2 rows; several items fit a compute unit (64 accumulator registers, 24 KB of LDS).
#include <stdarg.h>

#include "centre_atom.h"
#include "triplet.h"

namespace {

constexpr int HR = 32;          // in-edge rows per work item
constexpr int HRT = 4;          // fragments (2 rows x 8 l) per wavefront
constexpr int HSLAB = 32;       // out-edge positions per slab (one step of the contraction)

// Y_l0(x) = x^(l%2) (q0 + q1 x^2 + q2 x^4 + q3 x^6): Legendre polynomials in even/odd form (normalised in the kernel)
__device__ __constant__ float LEG_EO[ST][4] = {
    {1.f, 0.f, 0.f, 0.f},
    {1.f, 0.f, 0.f, 0.f},
    {-0.5f, 1.5f, 0.f, 0.f},
    {-1.5f, 2.5f, 0.f, 0.f},
    {0.375f, -3.75f, 4.375f, 0.f},
    {1.875f, -8.75f, 7.875f, 0.f},
    {-0.3125f, 6.5625f, -19.6875f, 14.4375f},
    {-2.1875f, 19.6875f, -43.3125f, 26.8125f}};

// Work items (atom, group of HR in-edge rows), atom-major: item[w] = {first padded out-list position of the atom, its
// number of out-edges, edge id of the group's first row, rows in the group}; n_items[0] = their number.
__global__ void __launch_bounds__(1024)
fusedH_items_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ out_ptr, int n_atoms,
                    int32_t* __restrict__ n_items, int32_t* __restrict__ item) {
  __shared__ int32_t wave_tot[16];
  __shared__ int32_t carry;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  if (tid == 0) carry = 0;
  __syncthreads();
  for (int base = 0; base < n_atoms; base += 1024) {
    const int j = base + tid;
    const int r0 = j < n_atoms ? row_ptr[j] : 0, d = j < n_atoms ? row_ptr[j + 1] - r0 : 0;
    const int v = (d + HR - 1) / HR;
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
      const int ob = out_ptr[j], dout = out_ptr[j + 1] - ob;
      for (int k = 0; k < v; ++k) {
        int32_t* it = item + 4 * (int64_t)(before + incl - v + k);
        it[0] = (int32_t)padded_base(ob, j);
        it[1] = dout;
        it[2] = r0 + HR * k;
        it[3] = d - HR * k < HR ? d - HR * k : HR;
      }
    }
    __syncthreads();
    if (tid == 1023) carry = before + incl;
    __syncthreads();
  }
  if (tid == 0) n_items[0] = carry;
}

// Pre-pass, one workgroup per (atom j, 64 of its padded out-list positions): dz of the out-edges in bf16 as
// [block of 8 positions][o][8] (positions past the atom's last out-edge are zero, so they contribute nothing whatever
// cosine is read for them), and, from the workgroups of the first 64 positions, for every in-edge row e' of the atom
// {start of its kj-major segment, position of the out-edge the segment leaves out (the number of out-edges if none)}.
__global__ void __launch_bounds__(256)
fusedH_pack_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ out_ptr, const int32_t* __restrict__ out_list,
                   const int32_t* __restrict__ seg_ptr_kj, const int32_t* __restrict__ idx_ji_kj, const float* __restrict__ dz,
                   int O, const int32_t* __restrict__ rows, __bf16* __restrict__ dzb, int32_t* __restrict__ row_info) {
  const int j = blockIdx.x;
  const int ob = out_ptr[j], dout = out_ptr[j + 1] - ob;
  const int n0 = ROWPAD * (int)blockIdx.y;
  const int32_t* outs = out_list + ob;
  if (blockIdx.y == 0) {
    const int r0 = row_ptr[j], d = row_ptr[j + 1] - r0;
    for (int p = threadIdx.x; p < d; p += 256) {
      const int e = rows ? rows[r0 + p] : r0 + p;
      const int seg = seg_ptr_kj[e], cnt = seg_ptr_kj[e + 1] - seg;
      row_info[2 * (int64_t)(r0 + p)] = seg;
      row_info[2 * (int64_t)(r0 + p) + 1] = first_mismatch(idx_ji_kj + seg, cnt, [=](int slot) { return outs[slot]; });
    }
  }
  if (n0 >= ((dout + ROWPAD - 1) & ~(ROWPAD - 1))) return;
  const int64_t base = padded_base(ob, j) + n0;
  for (int it = threadIdx.x; it < (ROWPAD / 8) * O; it += 256) {
    const int nb = it / O, o = it % O;
    bf16x8 v;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int n = n0 + 8 * nb + i;
      const float zv = dz[(int64_t)outs[n < dout ? n : 0] * O + o];   // clamped position, zeroed below: unconditional loads
      v[i] = (__bf16)(n < dout ? zv : 0.f);
    }
    *reinterpret_cast<bf16x8*>(dzb + ((base / 8 + nb) * O + o) * 8) = v;
  }
}

template <int NT>   // O = 16 NT (NT = 2, 4, 8)
// 3 workgroups per compute unit (2 at O = 128): with fewer registers a few values spill, and a spill reload inside the
// loop waits for every load in flight
__global__ void __launch_bounds__(256, NT == 8 ? 2 : 3)
tripG_H_fused_kernel(const float* __restrict__ cos_kj, int64_t T, const __bf16* __restrict__ dzb, const int32_t* __restrict__ row_info,
                     const int32_t* __restrict__ n_items, const int32_t* __restrict__ item, int S,
                     const int32_t* __restrict__ rows, int out_half, float* __restrict__ H) {
  constexpr int O = 16 * NT;
  constexpr int Z_B = HSLAB / 8 * O * 16;            // dz^T of a slab: 4 position blocks x O x 8 bf16
  constexpr int CS_B = HR * HSLAB * 4;               // cosines of the group's rows for a slab
  constexpr int BUF_B = Z_B + CS_B;
  constexpr int Z_LOADS = Z_B / 1024, CS_LOADS = CS_B / 256;
  constexpr int PW = (Z_LOADS + 3) / 4 + CS_LOADS / 4;   // loads per wavefront and slab
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int total = n_items[0];
  const int q8 = total >> 3, r8 = total & 7, xcd = (int)blockIdx.x & 7, ith = (int)blockIdx.x >> 3;
  if (ith >= q8 + (xcd < r8 ? 1 : 0)) return;
  const int w = xcd * q8 + (xcd < r8 ? xcd : r8) + ith;
  const int4 it = *reinterpret_cast<const int4*>(item + 4 * (int64_t)w);
  const int64_t base = it.x;
  const int dout = it.y, e0 = it.z, n_rows = it.w;
  const int n_slab = (dout + HSLAB - 1) / HSLAB;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kq = lane >> 4, c = lane & 15;
  const int p2 = c >> 3, l = c & 7;

  // Cosines: 4-byte global->LDS loads, a wavefront's load covers 2 rows x 32 positions.  Position n of the atom's
  // out-list is slot n, or n - 1 behind the position the row's segment leaves out, of the row's kj-major segment;
  // the left-out position itself and positions past the last out-edge fetch some valid cosine that is never used
  // (the former is zeroed below, the latter meet zero rows of dz^T).
  int cs_seg[CS_LOADS / 4], cs_gap[CS_LOADS / 4];
#pragma unroll
  for (int L = 0; L < CS_LOADS / 4; ++L) {
    const int pl = 2 * (wv + 4 * L) + (lane >> 5);
    const int64_t e = e0 + (pl < n_rows ? pl : n_rows - 1);
    cs_seg[L] = row_info[2 * e];
    cs_gap[L] = row_info[2 * e + 1];
  }
  // dz^T of a slab: a load covers 4 consecutive (position block, tile) pairs, 16 rows each (see triplet_g_fused.hip)
  const int z_lane = ((kq / NT) * O + NT * rowperm(c) + kq % NT) * 8;
  auto stage = [&](int slab, int buf) __attribute__((always_inline)) {
    unsigned char* dst = smem + buf * BUF_B;
    const int64_t row0 = base + (int64_t)HSLAB * slab;
#pragma unroll
    for (int L = 0; L < (Z_LOADS + 3) / 4; ++L) {
      const int ld = wv + 4 * L < Z_LOADS ? wv + 4 * L : Z_LOADS - 1;   // a wavefront without a load of its own repeats the last
      const __bf16* src = dzb + ((row0 / 8 + (4 * ld) / NT) * O + (4 * ld) % NT) * 8 + z_lane;
      __builtin_amdgcn_global_load_lds((global_void_ptr)src, (lds_void_ptr)(dst + ld * 1024), 16, 0, 0);
    }
#pragma unroll
    for (int L = 0; L < CS_LOADS / 4; ++L) {
      const int ld = wv + 4 * L;
      const int n = HSLAB * slab + (lane & 31);
      int64_t idx = (int64_t)cs_seg[L] + n - (n > cs_gap[L] ? 1 : 0);
      idx = idx < T ? idx : T - 1;
      __builtin_amdgcn_global_load_lds((global_void_ptr)(cos_kj + idx), (lds_void_ptr)(dst + Z_B + ld * 256), 4, 0, 0);
    }
  };
  if (n_slab > 0) stage(0, 0);
  if (n_slab > 1) stage(1, 1);

  // the lane's polynomial and its rows: fragment rt of this wavefront holds rows 8 wv + 2 rt + p2 of the group
  float q[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) q[i] = l < S ? Y_NORM_M[l] * LEG_EO[l][i] : 0.f;
  const bool odd = l & 1;
  int gap[HRT];
#pragma unroll
  for (int rt = 0; rt < HRT; ++rt) {
    const int pl = 8 * wv + 2 * rt + p2;
    const int64_t e = e0 + (pl < n_rows ? pl : n_rows - 1);   // clamped: rows past the group's end are computed, not stored
    gap[rt] = row_info[2 * e + 1] - 8 * kq;                   // relative to the lane's first position of slab 0
  }

  f32x4 acc[HRT][NT];
#pragma unroll
  for (int rt = 0; rt < HRT; ++rt)
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[rt][t] = f32x4{0.f, 0.f, 0.f, 0.f};

  if (n_slab > 1) wait_vmcnt<PW>();   // slab 0 has landed (this wavefront's part; the barrier covers the others')
  else wait_vm0();
  __syncthreads();

  int b = 0;
  for (int s = 0; s < n_slab; ++s) {
    const int b2 = b >= 1 ? b - 1 : STAGES - 1;
    const bool more = s + 2 < n_slab;
    if (more) stage(s + 2, b2);
    const unsigned char* buf = smem + b * BUF_B;
    const float* cosS = reinterpret_cast<const float*>(buf + Z_B);
    bf16x8 yb[HRT];
#pragma unroll
    for (int rt = 0; rt < HRT; ++rt) {
      const float* cp = cosS + (8 * wv + 2 * rt + p2) * HSLAB + 8 * kq;
      const f32x4 c0 = *reinterpret_cast<const f32x4*>(cp), c1 = *reinterpret_cast<const f32x4*>(cp + 4);
      const float xv[8] = {c0[0], c0[1], c0[2], c0[3], c1[0], c1[1], c1[2], c1[3]};
      const int gl = gap[rt] - HSLAB * s;   // position of the left-out out-edge among this lane's 8, if in 0..7
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float x = xv[i], t2 = x * x;
        const float y = (odd ? x : 1.f) * (q[0] + t2 * (q[1] + t2 * (q[2] + t2 * q[3])));
        yb[rt][i] = (__bf16)(gl == i ? 0.f : y);
      }
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const bf16x8 za = *reinterpret_cast<const bf16x8*>(buf + ((kq * O + t * 16 + c) << 4));
#pragma unroll
      for (int rt = 0; rt < HRT; ++rt)
        acc[rt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(za, yb[rt], acc[rt][t], 0, 0, 0);
    }
    if (more) wait_vmcnt<PW>();   // slab s + 1 has landed, slab s + 2 may still be under way
    else wait_vm0();
    __syncthreads();
    b = b == STAGES - 1 ? 0 : b + 1;
  }

  // accumulator register i of tile t in lane (g = kq, c = (p2, l)): column o = NT (4 i + g) + t of row (p2, l)
  if (l < S) {
#pragma unroll
    for (int rt = 0; rt < HRT; ++rt) {
      const int pl = 8 * wv + 2 * rt + p2;
      if (pl >= n_rows) continue;
      const int e_out = rows ? rows[e0 + pl] : e0 + pl;
      float* dst = H + ((int64_t)e_out * S + l) * O + NT * kq;
      if (out_half) {   // H as bf16 (its readers are the two per-edge products): the same elements, half the bytes
        __bf16* dh = reinterpret_cast<__bf16*>(H) + ((int64_t)e_out * S + l) * O + NT * kq;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int t = 0; t < NT; t += 2) {
            typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
            bf16x2 v;
            v[0] = (__bf16)acc[rt][t][i];
            v[1] = (__bf16)acc[rt][t + 1][i];
            *reinterpret_cast<bf16x2*>(dh + 4 * NT * i + t) = v;
          }
        continue;
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if constexpr (NT == 4 || NT == 8) {
#pragma unroll
          for (int t = 0; t < NT; t += 4)
            *reinterpret_cast<f32x4*>(dst + 4 * NT * i + t) = f32x4{acc[rt][t][i], acc[rt][t + 1][i], acc[rt][t + 2][i], acc[rt][t + 3][i]};
        } else {
          typedef float f32x2 __attribute__((ext_vector_type(2)));
          *reinterpret_cast<f32x2*>(dst + 4 * NT * i) = f32x2{acc[rt][0][i], acc[rt][1][i]};
        }
      }
    }
  }
}

// ---- grad cos alpha in the same per-(atom, 32 rows) decomposition:
//
//   grad_cos[t = (e', e)] (+)= sum_l Y_l0'(cos alpha_t) W[(e', l), n(e)],   W = U_j dz_out^T  (contraction over o)
//
// Every wavefront works alone on 8 in-edge rows of the item (two 32x32x16 products of (4 rows x 8 l) by 32 out-list
// positions per step); nothing is staged in LDS: the operand fragments of its rows (U, bf16, [edge][8][O]) stay in
// registers for the whole item, those of the out-edges come per step from a bf16 copy of dz in out-list order (rows
// of one atom: read by all wavefronts that work on it, hence from the caches), the cosines and the values to add to
// are read, and the results written, in runs of 32 consecutive triplets.  No LDS and about 130 registers let a dozen
// wavefronts per compute unit hide the latency of those loads; the kernel that keeps an atom's out-edges in LDS runs
// four.
__global__ void __launch_bounds__(256)
dcos_pack_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ out_ptr, const int32_t* __restrict__ out_list,
                 const int32_t* __restrict__ seg_ptr_kj, const int32_t* __restrict__ idx_ji_kj, const float* __restrict__ dz,
                 int O, __bf16* __restrict__ dzr, int32_t* __restrict__ row_info) {
  const int j = blockIdx.x;
  const int ob = out_ptr[j], dout = out_ptr[j + 1] - ob;
  const int n0 = ROWPAD * (int)blockIdx.y;
  const int32_t* outs = out_list + ob;
  if (blockIdx.y == 0) {
    const int r0 = row_ptr[j], d = row_ptr[j + 1] - r0;
    for (int p = threadIdx.x; p < d; p += 256) {
      const int seg = seg_ptr_kj[r0 + p], cnt = seg_ptr_kj[r0 + p + 1] - seg;
      row_info[2 * (int64_t)(r0 + p)] = seg;
      row_info[2 * (int64_t)(r0 + p) + 1] = first_mismatch(idx_ji_kj + seg, cnt, [=](int slot) { return outs[slot]; });
    }
  }
  if (n0 >= ((dout + ROWPAD - 1) & ~(ROWPAD - 1))) return;
  const int64_t base = padded_base(ob, j) + n0;
  const int ch = O / 8;
  for (int it = threadIdx.x; it < ROWPAD * ch; it += 256) {
    const int n = n0 + it / ch, oc = (it % ch) * 8;
    const bool ok = n < dout;
    const float* src = dz + (int64_t)outs[ok ? n : 0] * O + oc;   // clamped position times a 0/1 factor: unconditional loads
    const f32x4 v0 = *reinterpret_cast<const f32x4*>(src) * (ok ? 1.f : 0.f);
    const f32x4 v1 = *reinterpret_cast<const f32x4*>(src + 4) * (ok ? 1.f : 0.f);
    bf16x8 v;
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = (__bf16)v0[i], v[4 + i] = (__bf16)v1[i];
    *reinterpret_cast<bf16x8*>(dzr + (base + it / ch) * O + oc) = v;
  }
}

// U[e, l, o] fp32 ([E, S, O]) -> bf16 [E][8][O], rows l >= S zero
__global__ void u16_kernel(const float* __restrict__ U, int64_t E, int S, int O, __bf16* __restrict__ U16) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // (e, l, o / 4)
  const int q = O / 4;
  if (i >= E * 8 * q) return;
  const int64_t e = i / (8 * q);
  const int l = (int)(i / q) & 7, o = (int)(i % q) * 4;
  typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
  bf16x4 v = {(__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f};
  if (l < S) {
    const f32x4 u = *reinterpret_cast<const f32x4*>(U + (e * S + l) * O + o);
#pragma unroll
    for (int c = 0; c < 4; ++c) v[c] = (__bf16)u[c];
  }
  *reinterpret_cast<bf16x4*>(U16 + (e * 8 + l) * O + o) = v;
}

template <int KS>   // O = 16 KS (KS = 2, 4, 8)
__global__ void __launch_bounds__(256, KS == 8 ? 2 : 3)
tripG_dcos_fused_kernel(const float* __restrict__ cos_kj, int64_t T, const __bf16* __restrict__ U16, const __bf16* __restrict__ dzr,
                        const int32_t* __restrict__ row_info, const int32_t* __restrict__ n_items, const int32_t* __restrict__ item,
                        int S, int accumulate, float* __restrict__ grad_cos_kj) {
  constexpr int O = 16 * KS;
  const int total = n_items[0];
  const int q8 = total >> 3, r8 = total & 7, xcd = (int)blockIdx.x & 7, ith = (int)blockIdx.x >> 3;
  if (ith >= q8 + (xcd < r8 ? 1 : 0)) return;
  const int w = xcd * q8 + (xcd < r8 ? xcd : r8) + ith;
  const int4 it = *reinterpret_cast<const int4*>(item + 4 * (int64_t)w);
  const int64_t base = it.x;
  const int dout = it.y, e0 = it.z, n_rows = it.w;
  const int lane = threadIdx.x & 63;
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (8 * wv >= n_rows) return;          // wavefronts are independent: no barrier below
  const int kh = lane >> 5, l32 = lane & 31;

  // operand fragments of the wavefront's rows: MFMA row l32 = (row pl = l32 / 8 of the fragment, l = l32 % 8)
  bf16x8 a[2][KS];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt) {
    const int p = 8 * wv + 4 * rt + (l32 >> 3);
    const __bf16* src = U16 + ((int64_t)(e0 + (p < n_rows ? p : n_rows - 1)) * 8 + (l32 & 7)) * O + 8 * kh;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) a[rt][ks] = *reinterpret_cast<const bf16x8*>(src + 16 * ks);
  }
  // segment start and left-out position of the 8 rows (uniform: scalar registers); rows past the group's end repeat
  // its last row and are never stored
  int seg[8], gap[8];
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const int p = 8 * wv + r;
    const int64_t e = e0 + (p < n_rows ? p : n_rows - 1);
    seg[r] = row_info[2 * e];
    gap[r] = p < n_rows ? row_info[2 * e + 1] : -1 - dout;   // a row past the end: no position is valid (see `valid`)
  }
  // Y_l0'(x) for this lane's four l = 4 kh + i as polynomials in x^2 (times x for even l): from
  // P_l = x^(l%2) sum_c q_c x^(2c), P_l' = sum_c (2c + l%2) q_c x^(2c + l%2 - 1)
  float dq[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int lq = 4 * kh + i;
    const float nrm = lq < S ? Y_NORM_M[lq] : 0.f;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      if (i & 1) dq[i][c] = nrm * (float)(2 * c + 1) * LEG_EO[lq][c];
      else dq[i][c] = c < 3 ? nrm * (float)(2 * c + 2) * LEG_EO[lq][c + 1] : 0.f;
    }
  }

  const int n_slab = (dout + 31) >> 5;
  // position n of the out-list is slot n, or n - 1 behind the left-out position, of row r's segment
  auto fetch = [&](int nb, bf16x8 (&b)[KS], float (&xs)[8], float (&old)[8]) __attribute__((always_inline)) {
    const int n = nb * 32 + l32;
    const __bf16* src = dzr + (base + n) * O + 8 * kh;   // rows up to the next multiple of 64 exist and are zero
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) b[ks] = *reinterpret_cast<const bf16x8*>(src + 16 * ks);
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const bool valid = n < dout && n != gap[r] && gap[r] >= 0;
      const int64_t at = valid ? (int64_t)seg[r] + n - (n > gap[r] ? 1 : 0) : 0;   // unconditional loads, index 0 when unused
      xs[r] = cos_kj[at];
      old[r] = accumulate ? grad_cos_kj[at] : 0.f;
    }
  };
  bf16x8 b_n[KS];
  float xs_n[8], old_n[8];
  fetch(0, b_n, xs_n, old_n);
  for (int nb = 0; nb < n_slab; ++nb) {
    bf16x8 b[KS];
    float xs[8], old[8];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) b[ks] = b_n[ks];
#pragma unroll
    for (int r = 0; r < 8; ++r) xs[r] = xs_n[r], old[r] = old_n[r];
    if (nb + 1 < n_slab) fetch(nb + 1, b_n, xs_n, old_n);
    const int n = nb * 32 + l32;
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
      f32x16 acc;
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[rt][ks], b[ks], acc, 0, 0, 0);
      // accumulator register 4 pl + i of lane (kh, n): row pl of the fragment, l = 4 kh + i
#pragma unroll
      for (int pl = 0; pl < 4; ++pl) {
        const int r = 4 * rt + pl;
        const float x = xs[r], t2 = x * x;
        float part = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float wgt = dq[i][0] + t2 * (dq[i][1] + t2 * (dq[i][2] + t2 * dq[i][3]));
          part += acc[4 * pl + i] * ((i & 1) ? wgt : x * wgt);   // l even: odd derivative
        }
        const float tot = part + __shfl_xor(part, 32, 64);
        const bool valid = n < dout && n != gap[r] && gap[r] >= 0;
        if (valid && kh == (pl >> 1)) grad_cos_kj[(int64_t)seg[r] + n - (n > gap[r] ? 1 : 0)] = old[r] + tot;
      }
    }
  }
}

struct dcos_ws {
  __bf16 *dzr, *u16;
  int32_t *row_info, *n_items, *item;
};
size_t carve_dcos(void* p, int64_t N, int64_t E, int O, bool with_u16, dcos_ws* w) {
  gp_carver c(p);
  w->dzr = c.take<__bf16>((size_t)padded_rows(E, N) * O);
  w->u16 = c.take<__bf16>(with_u16 ? (size_t)E * 8 * O : 0);
  w->row_info = c.take<int32_t>(2 * (size_t)E);
  w->n_items = c.take<int32_t>(4);
  w->item = c.take<int32_t>(4 * (size_t)(E / HR + N + 1));
  return c.off;
}

struct fusedH_ws {
  __bf16* dzb;
  int32_t *row_info, *n_items, *item;
};
size_t carve_fusedH(void* p, int64_t N, int64_t E, int O, fusedH_ws* w) {
  gp_carver c(p);
  w->dzb = c.take<__bf16>((size_t)padded_rows(E, N) * O);
  w->row_info = c.take<int32_t>(2 * (size_t)E);
  w->n_items = c.take<int32_t>(4);
  w->item = c.take<int32_t>(4 * (size_t)(E / HR + N + 1));
  return c.off;
}

}  // namespace

size_t gp_tripG_H_fused_scratch(int64_t N, int64_t E, int O) {
  fusedH_ws w;
  return carve_fusedH(nullptr, N, E, O, &w);
}

bool gp_tripG_H_fused_usable(const gp_graph* g, int O, int S) {
  if (!g || !g->row_ptr || !g->out_ptr || !g->out_list || g->n_atoms <= 0 || g->n_triplets < 16) return false;
  if (!g->seg_ptr_kj || !g->idx_ji_kj || g->max_in_degree <= 0 || g->max_out_degree <= 0) return false;
  if (g->n_edges + (int64_t)PADJ * g->n_atoms + ROWPAD + 8 > INT32_MAX || g->n_edges / HR + g->n_atoms > INT32_MAX / 8) return false;
  return (O == 32 || O == 64 || O == 128) && S >= 1 && S <= ST;
}

int gp_tripG_backward_H_fused(gp_ctx* ctx, const gp_graph* g, const float* cos_alpha_kj, const float* dz, int O, int S, float* H,
                              void* ws, size_t ws_bytes, const int32_t* row_list, int out_half) {
  const int64_t E = g->n_edges, T = g->n_triplets, N = g->n_atoms;
  if (E == 0) return GP_OK;
  GP_REQUIRE(ctx, gp_tripG_H_fused_usable(g, O, S), "triplet G backward (one-pass matrix-core form): graph lists or widths not supported");
  GP_REQUIRE(ctx, cos_alpha_kj && dz && H && ws, "triplet G backward: NULL pointer");
  fusedH_ws w;
  if (ws_bytes < carve_fusedH(ws, N, E, O, &w)) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "triplet G backward: workspace too small");
  hipStream_t st = ctx->stream;
  {
    gp_prof_scope prof(ctx, "tripG_H_pack", 0.0, (double)E * (4.0 * O + 2.0 * O + 16.0));
    fusedH_items_kernel<<<1, 1024, 0, st>>>(g->row_ptr, g->out_ptr, (int)N, w.n_items, w.item);
    const dim3 grid((unsigned)N, (unsigned)((g->max_out_degree + ROWPAD - 1) / ROWPAD));
    fusedH_pack_kernel<<<grid, 256, 0, st>>>(g->row_ptr, g->out_ptr, g->out_list, g->seg_ptr_kj, g->idx_ji_kj, dz, O, row_list, w.dzb, w.row_info);
    GP_LAUNCH_CHECK(ctx, "fusedH_pack_kernel");
  }
  gp_prof_scope prof(ctx, "tripG_H_fused", (double)T * 2.0 * 8 * O, (double)T * 4.0 + (double)E * (2.0 * O + 4.0 * S * O));
  const unsigned grid = (unsigned)(E / HR + N);   // an upper bound of the number of work items; the rest exit at once
#define GP_H_LAUNCH(NT) \
  tripG_H_fused_kernel<NT><<<grid, 256, STAGES * (HSLAB / 8 * 16 * NT * 16 + HR * HSLAB * 4), st>>>(cos_alpha_kj, T, w.dzb, w.row_info, w.n_items, w.item, S, row_list, out_half, H)
  if (O == 128) GP_H_LAUNCH(8);
  else if (O == 64) GP_H_LAUNCH(4);
  else GP_H_LAUNCH(2);
#undef GP_H_LAUNCH
  GP_LAUNCH_CHECK(ctx, "tripG_H_fused_kernel");
  return GP_OK;
}

size_t gp_tripG_dcos_fused_scratch(int64_t N, int64_t E, int O, int with_u16) {
  dcos_ws w;
  return carve_dcos(nullptr, N, E, O, with_u16 != 0, &w);
}

int gp_tripG_grad_cos_fused(gp_ctx* ctx, const gp_graph* g, const float* cos_alpha_kj, const void* U, int u_is_bf16_padded,
                            const float* dz, int O, int S, int accumulate, float* grad_cos_kj, void* ws, size_t ws_bytes) {
  const int64_t E = g->n_edges, T = g->n_triplets, N = g->n_atoms;
  if (E == 0 || T == 0) return GP_OK;
  GP_REQUIRE(ctx, gp_tripG_H_fused_usable(g, O, S), "grad_cos (one-pass matrix-core form): graph lists or widths not supported");
  GP_REQUIRE(ctx, cos_alpha_kj && U && dz && grad_cos_kj && ws, "grad_cos: NULL pointer");
  dcos_ws w;
  if (ws_bytes < carve_dcos(ws, N, E, O, !u_is_bf16_padded, &w)) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "grad_cos: workspace too small");
  hipStream_t st = ctx->stream;
  const __bf16* U16 = reinterpret_cast<const __bf16*>(U);
  {
    gp_prof_scope prof(ctx, "tripG_dcos_pack", 0.0, (double)E * (4.0 * O + 2.0 * O + 16.0));
    if (!u_is_bf16_padded) {
      const int64_t n = E * 8 * (O / 4);
      u16_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(reinterpret_cast<const float*>(U), E, S, O, w.u16);
      GP_LAUNCH_CHECK(ctx, "u16_kernel");
      U16 = w.u16;
    }
    fusedH_items_kernel<<<1, 1024, 0, st>>>(g->row_ptr, g->out_ptr, (int)N, w.n_items, w.item);
    const dim3 grid((unsigned)N, (unsigned)((g->max_out_degree + ROWPAD - 1) / ROWPAD));
    dcos_pack_kernel<<<grid, 256, 0, st>>>(g->row_ptr, g->out_ptr, g->out_list, g->seg_ptr_kj, g->idx_ji_kj, dz, O, w.dzr, w.row_info);
    GP_LAUNCH_CHECK(ctx, "dcos_pack_kernel");
  }
  gp_prof_scope prof(ctx, "tripG_dcos_fused", (double)T * 2.0 * 8 * O, (double)T * (accumulate ? 12.0 : 8.0) + (double)E * (2.0 * O + 16.0 * O));
  const unsigned grid = (unsigned)(E / HR + N);   // an upper bound of the number of work items; the rest exit at once
  if (O == 128) tripG_dcos_fused_kernel<8><<<grid, 256, 0, st>>>(cos_alpha_kj, T, U16, w.dzr, w.row_info, w.n_items, w.item, S, accumulate, grad_cos_kj);
  else if (O == 64) tripG_dcos_fused_kernel<4><<<grid, 256, 0, st>>>(cos_alpha_kj, T, U16, w.dzr, w.row_info, w.n_items, w.item, S, accumulate, grad_cos_kj);
  else tripG_dcos_fused_kernel<2><<<grid, 256, 0, st>>>(cos_alpha_kj, T, U16, w.dzr, w.row_info, w.n_items, w.item, S, accumulate, grad_cos_kj);
  GP_LAUNCH_CHECK(ctx, "tripG_dcos_fused_kernel");
  return GP_OK;
}
