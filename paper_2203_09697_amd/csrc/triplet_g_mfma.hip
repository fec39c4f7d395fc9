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
//                      of 16).  A thread owns 8 positions x 2 values of c (c, c+8) and keeps the radial
//                      rows it needs (8 x S x 2 values) in registers while it walks the edges.
//   tripG_mfma_kernel  v_mfma_f32_32x32x16_bf16: a wavefront owns 4 edges (2 row blocks of
//                      2 edges x 16 c) by all F columns; A fragments come straight from Yb
//                      (16 bytes per lane, read once), B fragments from LDS.
//
// Operands are rounded to bf16, sums are fp32.  Needs the centre-atom lists of gp_graph.
#include <stdarg.h>

#include "gemm.h"
#include "triplet.h"

#include "centre_atom.h"

namespace {

__device__ __forceinline__ int64_t y_offset(int seg, int e) {   // in bf16 elements
  return ((int64_t)seg + 16 * (int64_t)e) * CP;
}


template <int SM>   // loops over l run to SM >= num_spherical (rows above num_spherical are zero)
__global__ void __launch_bounds__(YT, 3)   // three workgroups per CU: 168 registers (a few spilled) beat two at 192
tripG_y_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ out_ptr,
               const int32_t* __restrict__ out_list, const int32_t* __restrict__ seg_ptr_ji,
               const int32_t* __restrict__ idx_kj, const float* __restrict__ cos_alpha,
               const float* __restrict__ Radt, int64_t E, int S, int C, int kp_cap, int parts,
               const int32_t* __restrict__ row_list, int rad_by_pos, __bf16* __restrict__ Yb) {
  part_t P;
  if (!centre_part(row_ptr, out_ptr, kp_cap, parts, P)) return;
  __shared__ int s_e[64], s_seg[64], s_cnt[64], s_gap[64];
  const int n_pg = P.Kp / 8;
  const int cp = threadIdx.x & 7;
  const int n_slots = (int)(blockDim.x >> 3);   // groups of 8 threads; a group owns 8 positions of all 16 c
  for (int pg0 = 0; pg0 < n_pg; pg0 += n_slots) {
    // A pass with fewer position groups left than thread groups splits each position group's edges among
    // several thread groups (edges e_off, e_off + e_step, ...), so that the last pass keeps the block busy.
    const int left = n_pg - pg0, slot = threadIdx.x >> 3;
    const int e_step = left >= n_slots ? 1 : n_slots / left;
    const int e_off = left >= n_slots ? 0 : slot / left;
    const int pg = pg0 + (left >= n_slots ? slot : slot % left);
    const bool active = e_off < e_step;
    int row_e[8];   // edge ids of the thread's 8 positions (clamped to the atom's last row)
#pragma unroll
    for (int pi = 0; pi < 8; ++pi) {
      const int pos = P.r0 + (8 * pg + pi < P.d ? 8 * pg + pi : P.d - 1);
      row_e[pi] = rad_by_pos ? pos : row_edge(row_list, pos);   // rad_by_pos: the radial table was gathered into list order
    }
    float rad[SM][2][8];
#pragma unroll
    for (int l = 0; l < SM; ++l)
#pragma unroll
      for (int cc = 0; cc < 2; ++cc)
#pragma unroll
        for (int pi = 0; pi < 8; ++pi) {
          const int p = 8 * pg + pi, c = cp + 8 * cc;
          const bool ok = active && l < S && c < C && p < P.d;
          // pre-multiplied by the normalisation of Y_l0
          // unconditional load from a clamped (valid) address: no branch around it
          const float rv = Radt[(int64_t)((l < S ? l : S - 1) * C + (c < C ? c : C - 1)) * E + row_e[pi]];
          rad[l][cc][pi] = rv * (ok ? Y_NORM_M[l] : 0.f);   // the product uses rv on every path: the load cannot sink under a branch
        }
    // From the Legendre expansion sum_l rad[l] P_l(x) to powers of x, once per position and c: the polynomial is then
    // evaluated per triplet by Horner's rule, SM - 1 multiply-adds instead of a recurrence plus SM of them.  (The
    // result is rounded to bf16; the cancellation in the power basis costs a few units of fp32 rounding.)
#pragma unroll
    for (int cc = 0; cc < 2; ++cc)
#pragma unroll
      for (int pi = 0; pi < 8; ++pi) {
        float m[SM];
#pragma unroll
        for (int k = 0; k < SM; ++k) {
          float sum = 0.f;
#pragma unroll
          for (int l = k; l < SM; l += 2) sum += leg_mono(l, k) * rad[l][cc][pi];
          m[k] = sum;
        }
#pragma unroll
        for (int k = 0; k < SM; ++k) rad[k][cc][pi] = m[k];
      }
    for (int c0 = P.eb; c0 < P.ee; c0 += 64) {
      __syncthreads();
      if (threadIdx.x < 64 && c0 + (int)threadIdx.x < P.ee) {
        const int e = out_list[P.o0 + c0 + threadIdx.x];
        const int seg = seg_ptr_ji[e], cnt = seg_ptr_ji[e + 1] - seg;
        // the segment lists rows r0, r0+1, ... with (at most) the row coming from atom i left
        // out: first slot whose row is not r0 + slot
        const int r0 = P.r0;
        const int lo = first_mismatch(idx_kj + seg, cnt, [=](int slot) { return row_edge(row_list, r0 + slot); });
        s_e[threadIdx.x] = e;
        s_seg[threadIdx.x] = seg;
        s_cnt[threadIdx.x] = cnt;
        s_gap[threadIdx.x] = lo;
      }
      __syncthreads();
      const int n = P.ee - c0 < 64 ? P.ee - c0 : 64;
      if (!active) continue;
      // Cosines of the 8 positions for edge ei of the chunk (0 and an unset mask bit where there is no triplet).  The 8
      // threads of a position group need the same 8 cosines: thread cp fetches those of the group's edge number
      // k0 + cp, and the group hands them round with lane exchanges while it works through 8 edges.  Loads and
      // stores complete through one counter on this target, so a wait for loads also waits for every store issued
      // before: one wait per 8 edges instead of one per edge.
      if (e_off >= n) continue;
      const int n_mine = (n - e_off + e_step - 1) / e_step;   // edges e_off, e_off + e_step, ... < n
      auto load_cos = [&](int k, float (&cs)[8], unsigned& vmask) __attribute__((always_inline)) {
        const int ei = e_off + (k < n_mine ? k : n_mine - 1) * e_step;   // clamped: loads stay unconditional
        const int seg = s_seg[ei], cnt = s_cnt[ei], gap = s_gap[ei];
        vmask = 0;
#pragma unroll
        for (int pi = 0; pi < 8; ++pi) {
          const int p = 8 * pg + pi;
          const int q = p - (p > gap ? 1 : 0);
          const bool valid = p != gap && q < cnt;
          cs[pi] = cos_alpha[valid ? seg + q : 0];   // index 0 exists: the kernel is not launched for T = 0
          vmask |= (valid ? 1u : 0u) << pi;
        }
      };
      float cs_next[8];
      unsigned vm_next;
      load_cos(cp, cs_next, vm_next);
      for (int k0 = 0; k0 < n_mine; k0 += 8) {
        float cs_mine[8];
        const unsigned vm_mine = vm_next;
#pragma unroll
        for (int pi = 0; pi < 8; ++pi) cs_mine[pi] = cs_next[pi];
        if (k0 + 8 < n_mine) load_cos(k0 + 8 + cp, cs_next, vm_next);   // in flight during the 8 edges below
        const int jn = n_mine - k0 < 8 ? n_mine - k0 : 8;
#pragma unroll 1
        for (int jj = 0; jj < jn; ++jj) {
          const int src = (int)(threadIdx.x & 63 & ~7) | jj;
          const unsigned vm = (unsigned)__shfl((int)vm_mine, src);
          const int ei = e_off + (k0 + jj) * e_step;
          float y[2][8];
#pragma unroll
          for (int pi = 0; pi < 8; ++pi) {
            const bool valid = (vm >> pi) & 1u;
            const float x = __shfl(cs_mine[pi], src);
            float a0 = rad[SM - 1][0][pi], a1 = rad[SM - 1][1][pi];
#pragma unroll
            for (int k = SM - 2; k >= 0; --k) {
              a0 = a0 * x + rad[k][0][pi];
              a1 = a1 * x + rad[k][1][pi];
            }
            y[0][pi] = valid ? a0 : 0.f;   // no triplet: zero row of the operand
            y[1][pi] = valid ? a1 : 0.f;
          }
          // c = cp and cp + 8: the 8 threads of a position group write 128 contiguous bytes per store
          __bf16* dst = Yb + y_offset(s_seg[ei], s_e[ei]) + (int64_t)pg * (CP * 8) + cp * 8;
#pragma unroll
          for (int cc = 0; cc < 2; ++cc) {
            bf16x8 v;
#pragma unroll
            for (int pi = 0; pi < 8; ++pi) v[pi] = (__bf16)y[cc][pi];
            *reinterpret_cast<bf16x8*>(dst + 64 * cc) = v;
          }
        }
      }
    }
  }
}

// ---- variant D (Hadamard form, fp32): Bacc[e, b, f] = sum_{t in seg(e)} p_t[b] x[kj(t), f],
// p_t[b] = sum_l Y_l0(cos alpha_t) Q[kj(t), l, b], and a[e, f] = sum_b W2[b, f] Bacc[e, b, f].
// The same regrouping by centre atom j: rows (out-edge e, b), contraction over the in-edge rows p of j, columns f,
// on the fp32 matrix cores (v_mfma_f32_32x32x2_f32: lane l feeds row / column l % 32 at k = l / 32).  X_j and the
// atom's slice of Q (pre-multiplied by the normalisation of Y_l0 and the leading coefficient of P_l) are staged
// in LDS once; the left operand p_t[b] is evaluated in registers from the cosine, one value per lane and MFMA,
// so nothing of size T is stored.  A wavefront owns 4 out-edges (32 rows) by all F columns.
constexpr int DB = 8;            // basis_emb of the kernel
constexpr int LDQ = 64;          // floats per in-edge row of the staged Q: [l][b] (unpadded, like X)

template <int NT>   // F = 32 NT
__global__ void __launch_bounds__(256)
tripD_mfma_fwd_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ out_ptr,
                      const int32_t* __restrict__ out_list, const int32_t* __restrict__ seg_ptr_ji,
                      const int32_t* __restrict__ idx_kj, const float* __restrict__ cos_alpha,
                      const float* __restrict__ x, const float* __restrict__ Qt, const float* __restrict__ W2, int64_t E,
                      int S, int kp_cap, int parts, float* __restrict__ a_out, float* __restrict__ Bacc) {
  constexpr int F = 32 * NT, LDX = F;   // row stride of the staged X (padding against the 2-way bank conflict of the
                                        // two k halves measured 8 % slower: it costs a workgroup per CU)
  part_t P;
  if (!centre_part(row_ptr, out_ptr, kp_cap, parts, P)) return;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  float* X_s = reinterpret_cast<float*>(smem_raw);   // [Kp][LDX]
  float* Q_s = X_s + (size_t)P.Kp * LDX;             // [Kp][LDQ]
  __shared__ int s_e[64], s_seg[64], s_cnt[64], s_gap[64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll 4
  for (int i = threadIdx.x; i < P.Kp * (F / 4); i += 256) {
    const int p = i / (F / 4), f4 = (i % (F / 4)) * 4;
    // clamped row times a 0/1 factor: the load stays outside any branch, and four of them are under way together
    const f32x4 v = *reinterpret_cast<const f32x4*>(x + (int64_t)(P.r0 + (p < P.d ? p : 0)) * F + f4) * (p < P.d ? 1.f : 0.f);
    *reinterpret_cast<f32x4*>(&X_s[p * LDX + f4]) = v;
  }
  // Q of the atom's rows, converted from the Legendre expansion sum_l Y_l0(x) Q[l, b] to powers of x (coefficient k of
  // column b at k * 8 + b), so that the left operand is one Horner evaluation per triplet and b.  A thread takes
  // (row p, column b): its 8 loads (clamped addresses, a 0 factor outside the table) are under way together.
#pragma unroll 2
  for (int i = threadIdx.x; i < P.Kp * DB; i += 256) {
    const int p = i % P.Kp, b = i / P.Kp;           // consecutive threads: consecutive rows of one (l, b) line of Qt
    float ql[ST];
#pragma unroll
    for (int l = 0; l < ST; ++l)
      ql[l] = Qt[(int64_t)((l < S ? l : 0) * DB + b) * E + P.r0 + (p < P.d ? p : 0)] * ((p < P.d && l < S) ? Y_NORM_M[l] : 0.f);
#pragma unroll
    for (int k = 0; k < ST; ++k) {
      float sum = 0.f;
#pragma unroll
      for (int l = k; l < ST; l += 2) sum += leg_mono(l, k) * ql[l];
      Q_s[p * LDQ + k * DB + b] = sum;
    }
  }
  const int kh = lane >> 5, l32 = lane & 31;
  const int e_loc = l32 >> 3, b = l32 & 7;
  for (int c0 = P.eb; c0 < P.ee; c0 += 64) {
    __syncthreads();
    if (threadIdx.x < 64 && c0 + (int)threadIdx.x < P.ee) {
      const int e = out_list[P.o0 + c0 + threadIdx.x];
      const int seg = seg_ptr_ji[e], cnt = seg_ptr_ji[e + 1] - seg;
      // the segment lists rows r0, r0+1, ... with (at most) the row coming from atom i left out: first slot
      // whose row is not r0 + slot
      const int r0 = P.r0;
      const int lo = first_mismatch(idx_kj + seg, cnt, [=](int slot) { return r0 + slot; });
      s_e[threadIdx.x] = e;
      s_seg[threadIdx.x] = seg;
      s_cnt[threadIdx.x] = cnt;
      s_gap[threadIdx.x] = lo;
    }
    __syncthreads();
    const int n = P.ee - c0 < 64 ? P.ee - c0 : 64;
    for (int g0 = 4 * wave; g0 < n; g0 += 16) {
      const int ei = g0 + e_loc;
      const bool e_ok = ei < n;
      const int eic = e_ok ? ei : n - 1;
      const int seg = s_seg[eic], cnt = s_cnt[eic], gap = s_gap[eic];
      f32x16 acc[NT];
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
      // cosines of 8 k-steps at a time (2 marks "no triplet"), fetched one batch ahead of their use
      auto load_c = [&](int kp0, float (&c)[8]) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int p = 2 * (kp0 + u) + kh;
          const int slot = p - (p > gap ? 1 : 0);
          const bool ok = e_ok && kp0 < P.Kp / 2 && p < P.d && p != gap && slot < cnt;
          const float cv = cos_alpha[ok ? seg + slot : 0];   // unconditional load, index 0 when unused
          c[u] = ok ? cv : 2.f;
        }
      };
      float cn[8];
      load_c(0, cn);
      for (int kp0 = 0; kp0 < P.Kp / 2; kp0 += 8) {   // Kp is a multiple of 16
        float cs[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) cs[u] = cn[u];
        load_c(kp0 + 8, cn);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int p = 2 * (kp0 + u) + kh;
          const float* q = Q_s + p * LDQ + b;
          const bool ok = cs[u] <= 1.5f;
          const float cv = ok ? cs[u] : 0.f;
          float av = q[(ST - 1) * DB];
#pragma unroll
          for (int k = ST - 2; k >= 0; --k) av = av * cv + q[k * DB];
          av = ok ? av : 0.f;
#pragma unroll
          for (int t = 0; t < NT; ++t)
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, X_s[p * LDX + t * 32 + l32], acc[t], 0, 0, 0);
        }
      }
      // accumulator register v of lane (kh, l32): row 8 (v / 4) + 4 kh + v % 4 = (edge v / 4 of the group, b = 4 kh + v % 4),
      // column l32 of the block
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const int f = t * 32 + l32;
        float w2[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w2[i] = W2[(4 * kh + i) * F + f];
#pragma unroll
        for (int eg = 0; eg < 4; ++eg) {
          const bool ok_e = g0 + eg < n;
          const int64_t e = s_e[ok_e ? g0 + eg : n - 1];
          float sum = 0.f;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float v = acc[t][4 * eg + i];
            sum += w2[i] * v;
            if (ok_e && Bacc) Bacc[(e * DB + 4 * kh + i) * F + f] = v;
          }
          sum += __shfl_xor(sum, 32);
          if (ok_e && kh == 0) a_out[e * F + f] = sum;
        }
      }
    }
  }
}

template <int CB>   // F = 32 CB
__global__ void __launch_bounds__(MT)
tripG_mfma_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ out_ptr,
                  const int32_t* __restrict__ out_list, const int32_t* __restrict__ seg_ptr_ji,
                  const float* __restrict__ x, const __bf16* __restrict__ Yb, int C, int kp_cap, int parts, int out_half,
                  const int32_t* __restrict__ row_list, float* __restrict__ A) {
  constexpr int F = 32 * CB;
  part_t P;
  if (!centre_part(row_ptr, out_ptr, kp_cap, parts, P)) return;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  __bf16* XT = reinterpret_cast<__bf16*>(smem_raw);   // XT[f][p], row stride LDP
  // LDP/8 is odd, so the 16-byte reads of 8 lanes with consecutive f fall into 8 different bank groups
  const int LDP = P.Kp + 8;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

  // stage X_j: a wavefront takes a tile of 16 positions x 32 features; a lane converts two rows of
  // 4 features and writes 4 packed position pairs
  const int tiles_p = P.Kp / 16;
  // loads from clamped rows times a 0/1 factor (a select around a load would move the load under a branch and have
  // it waited for alone); unrolled so that the loads of several tiles are under way together
#pragma unroll 4
  for (int t = wave; t < tiles_p * CB; t += (int)(blockDim.x >> 6)) {
    const int pp = (t % tiles_p) * 8 + (lane & 7), fq = (t / tiles_p) * 8 + (lane >> 3);
    const int p0 = 2 * pp;
    const bool ok0 = p0 < P.d, ok1 = p0 + 1 < P.d;
    const f32x4 v0 = *reinterpret_cast<const f32x4*>(x + (int64_t)row_edge(row_list, P.r0 + (ok0 ? p0 : 0)) * F + 4 * fq) * (ok0 ? 1.f : 0.f);
    const f32x4 v1 = *reinterpret_cast<const f32x4*>(x + (int64_t)row_edge(row_list, P.r0 + (ok1 ? p0 + 1 : 0)) * F + 4 * fq) * (ok1 ? 1.f : 0.f);
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
  for (int grp = wave; grp * 4 < n_e; grp += (int)(blockDim.x >> 6)) {
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
        const int64_t at = ((int64_t)e4[k] * C + c) * F + l32;
        if (out_half) {
#pragma unroll
          for (int cb = 0; cb < CB; ++cb) reinterpret_cast<__bf16*>(A)[at + cb * 32] = (__bf16)acc[rb][cb][v];
        } else {
#pragma unroll
          for (int cb = 0; cb < CB; ++cb) A[at + cb * 32] = acc[rb][cb][v];
        }
      }
  }
}

// ---- backward (kj-major): rows are the in-edges of the centre atom, the sum runs over its out-edges ----
//
// For in-edge row p of atom j (edge e' = r0 + p) the kj-major segment lists the out-edges of j in
// the order of out_list, with (at most) the edge that returns to the source atom of e' left out.
struct rowinfo_t {
  int seg, cnt, gap;
};

__device__ __forceinline__ rowinfo_t row_info(const int32_t* __restrict__ seg_ptr_kj, const int32_t* __restrict__ idx_ji_kj,
                                              const int32_t* __restrict__ outs, int e) {
  rowinfo_t r;
  r.seg = seg_ptr_kj[e];
  r.cnt = seg_ptr_kj[e + 1] - r.seg;
  // first slot whose target edge is not the out-edge at the same position
  r.gap = first_mismatch(idx_ji_kj + r.seg, r.cnt, [=](int slot) { return outs[slot]; });
  return r;
}

// Share of a workgroup: centre atom j, `per` row groups of 8 in-edge rows each from group gb on
struct rows_t {
  int r0, d, o0, dout, gb, ge;
};
constexpr int GPW = 8;   // row groups per workgroup aimed at (two per wavefront; 4: variant-D backward kernel 0.130 -> 0.155 ms)

__device__ __forceinline__ bool centre_rows(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ out_ptr,
                                            int parts, rows_t& P) {
  int j, part;
  atom_and_part(parts, j, part);
  P.r0 = row_ptr[j];
  P.d = row_ptr[j + 1] - P.r0;
  P.o0 = out_ptr[j];
  P.dout = out_ptr[j + 1] - P.o0;
  if (P.d <= 0) return false;
  const int groups = (P.d + 7) / 8;
  int nparts = (groups + GPW - 1) / GPW;
  nparts = nparts < parts ? nparts : parts;
  if (part >= nparts) return false;
  const int len = (groups + nparts - 1) / nparts;
  P.gb = part * len;
  P.ge = P.gb + len < groups ? P.gb + len : groups;
  return P.gb < P.ge;
}

// Segment start, length and gap of every in-edge row of the workgroup's share, found once by the first threads
// (one binary search each, all under way together and while the other threads stage their operand) instead of once
// per row group by every lane.  rt holds 3 * cap ints, cap >= the rows of the share (share_rows on the host); the
// caller synchronises before reading it.
__host__ __device__ constexpr size_t row_tab_bytes(int cap) { return ((size_t)3 * cap * sizeof(int) + 15) & ~(size_t)15; }
__device__ __forceinline__ void fill_row_table(const int32_t* __restrict__ seg_ptr_kj, const int32_t* __restrict__ idx_ji_kj,
                                               const int32_t* __restrict__ outs, const rows_t& P, int* rt, int cap,
                                               const int32_t* __restrict__ row_list = nullptr) {
  const int row0 = P.gb * 8;
  const int nrows = (P.ge * 8 < P.d ? P.ge * 8 : P.d) - row0;
  for (int r = threadIdx.x; r < nrows && r < cap; r += blockDim.x) {   // cap >= nrows by construction of the launch
    const rowinfo_t ri = row_info(seg_ptr_kj, idx_ji_kj, outs, row_edge(row_list, P.r0 + row0 + r));
    rt[r] = ri.seg;
    rt[cap + r] = ri.cnt;
    rt[2 * cap + r] = ri.gap;
  }
}
// row p of the atom (p >= P.gb * 8; rows past the end of the list give the last row's entry, which the callers mask)
__device__ __forceinline__ rowinfo_t table_row(const int* rt, int cap, const rows_t& P, int p) {
  const int r = (p < P.d ? p : P.d - 1) - P.gb * 8;
  rowinfo_t ri;
  ri.seg = rt[r];
  ri.cnt = rt[cap + r];
  ri.gap = rt[2 * cap + r];
  return ri;
}

// Y_l0(x) = x^(l%2) (q0 + q1 x^2 + q2 x^4 + q3 x^6): Legendre polynomials in even/odd form,
// normalised by sqrt((2l+1)/(4 pi))
__device__ __constant__ float LEG_Q[ST][4] = {
    {1.f, 0.f, 0.f, 0.f},
    {1.f, 0.f, 0.f, 0.f},
    {-0.5f, 1.5f, 0.f, 0.f},
    {-1.5f, 2.5f, 0.f, 0.f},
    {0.375f, -3.75f, 4.375f, 0.f},
    {1.875f, -8.75f, 7.875f, 0.f},
    {-0.3125f, 6.5625f, -19.6875f, 14.4375f},
    {-2.1875f, 19.6875f, -43.3125f, 26.8125f}};

// H[e', l, o] = sum_{t: kj(t)=e'} Y_l0(cos alpha_t) dz[ji(t), o].  MFMA rows are (4 in-edge rows) x (l = 0..7),
// the contraction runs over the out-edge positions n, columns are o.  A fragments are evaluated in
// registers (a lane keeps one l, so Y_l0 is one short polynomial); dz of the out-edges is staged
// transposed in LDS.
template <int CB>   // O = 32 CB
__global__ void __launch_bounds__(256)
tripG_mfma_H_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ out_ptr,
                    const int32_t* __restrict__ out_list, const int32_t* __restrict__ seg_ptr_kj,
                    const int32_t* __restrict__ idx_ji_kj, const float* __restrict__ cos_kj,
                    const float* __restrict__ dz, int S, int kn_cap, int parts, int rows_cap,
                    const int32_t* __restrict__ row_list, float* __restrict__ H) {
  constexpr int O = 32 * CB;
  rows_t P;
  if (!centre_rows(row_ptr, out_ptr, parts, P)) return;
  const int Kn = (P.dout + 15) & ~15;
  if (Kn > kn_cap) return;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  int* row_tab = reinterpret_cast<int*>(smem_raw);
  __bf16* ZT = reinterpret_cast<__bf16*>(smem_raw + row_tab_bytes(rows_cap));   // ZT[o][n], row stride LDN
  const int LDN = Kn + 8;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int32_t* outs = out_list + P.o0;
  fill_row_table(seg_ptr_kj, idx_ji_kj, outs, P, row_tab, rows_cap, row_list);

  const int tiles_n = Kn / 16;
#pragma unroll 4
  for (int t = wave; t < tiles_n * CB; t += 4) {
    const int np = (t % tiles_n) * 8 + (lane & 7), oq = (t / tiles_n) * 8 + (lane >> 3);
    const int n0 = 2 * np;
    // the loop runs only if the atom has out-edges; loads from clamped positions times a 0/1 factor, see above
    const bool ok0 = n0 < P.dout, ok1 = n0 + 1 < P.dout;
    const f32x4 v0 = *reinterpret_cast<const f32x4*>(dz + (int64_t)outs[ok0 ? n0 : 0] * O + 4 * oq) * (ok0 ? 1.f : 0.f);
    const f32x4 v1 = *reinterpret_cast<const f32x4*>(dz + (int64_t)outs[ok1 ? n0 + 1 : 0] * O + 4 * oq) * (ok1 ? 1.f : 0.f);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      bf16x2 pr;
      pr[0] = (__bf16)v0[i];
      pr[1] = (__bf16)v1[i];
      *reinterpret_cast<bf16x2*>(&ZT[(4 * oq + i) * LDN + n0]) = pr;
    }
  }
  __syncthreads();

  const int kh = lane >> 5, l32 = lane & 31;
  const int l = l32 & 7;
  float q[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) q[i] = l < S ? Y_NORM_M[l] * LEG_Q[l][i] : 0.f;
  const bool odd = l & 1;
  const int nks = Kn / 16;

  for (int grp = P.gb + wave; grp < P.ge; grp += 4) {
    rowinfo_t ri[2];
    bool pv[2];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
      const int p = grp * 8 + rb * 4 + (l32 >> 3);
      pv[rb] = p < P.d;
      ri[rb] = table_row(row_tab, rows_cap, P, p);
    }
    f32x16 acc[2][CB];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[rb][cb][v] = 0.f;

    // cosines of k-step ks for both row blocks (2 marks "no triplet"); fetched two k-steps ahead
    auto load_x = [&](int ks, float (&x)[2][8]) {
#pragma unroll
      for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int n = ks * 16 + kh * 8 + i;
          const int slot = n - (n > ri[rb].gap ? 1 : 0);
          const bool valid = ks < nks && pv[rb] && n != ri[rb].gap && slot < ri[rb].cnt;
          const float cv = cos_kj[valid ? ri[rb].seg + slot : 0];   // unconditional load, index 0 when unused
          x[rb][i] = valid ? cv : 2.f;
        }
    };
    auto step = [&](int ks, const float (&xc)[2][8]) {
      bf16x8 a[2], b[CB];
#pragma unroll
      for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const bool valid = xc[rb][i] <= 1.5f;
          const float x = valid ? xc[rb][i] : 0.f;
          const float t2 = x * x;
          const float y = (odd ? x : 1.f) * (q[0] + t2 * (q[1] + t2 * (q[2] + t2 * q[3])));
          a[rb][i] = (__bf16)(valid ? y : 0.f);
        }
#pragma unroll
      for (int cb = 0; cb < CB; ++cb)
        b[cb] = *reinterpret_cast<const bf16x8*>(&ZT[(cb * 32 + l32) * LDN + ks * 16 + kh * 8]);
#pragma unroll
      for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
          acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[rb], b[cb], acc[rb][cb], 0, 0, 0);
    };
    float xn0[2][8], xn1[2][8];
    load_x(0, xn0);
    load_x(1, xn1);
    for (int ks = 0; ks < nks; ks += 2) {
      float xc0[2][8], xc1[2][8];
#pragma unroll
      for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int i = 0; i < 8; ++i) xc0[rb][i] = xn0[rb][i], xc1[rb][i] = xn1[rb][i];
      load_x(ks + 2, xn0);
      load_x(ks + 3, xn1);
      step(ks, xc0);
      if (ks + 1 < nks) step(ks + 1, xc1);
    }

    // accumulator register v of lane (kh, l32): row 8 (v/4) + 4 kh + v%4 = (in-edge row v/4 of the block, l = 4 kh + v%4)
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int p = grp * 8 + rb * 4 + (v >> 2), lo = 4 * kh + (v & 3);
        if (p >= P.d || lo >= S) continue;
        float* dst = H + ((int64_t)row_edge(row_list, P.r0 + p) * S + lo) * O + l32;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) dst[cb * 32] = acc[rb][cb][v];
      }
  }
}

// Backward of the Hadamard form (variant D) for one centre atom on the fp32 matrix cores.
//   H[e', l, f]   = sum_n Y_l0(cos alpha_(e', n)) ga[out(n), f]          MFMA rows (4 in-edge rows) x (l = 0..7),
//                                                                        contraction over the out-edge positions n
//   D[e', b, f]   = sum_l Q[e', l, b] H[e', l, f]
//   gx[e', f]     = SiLU'(z[e', f]) sum_b W2[b, f] D[e', b, f]
//   gQ[e', l, b]  = sum_f W2[b, f] x[e', f] H[e', l, f]
//   gW2[b, f]     = sum_e' x[e', f] D[e', b, f]                          (one partial sum per workgroup)
// which is the chain rule of a[e, f] = sum_t x[kj(t), f] sum_b W2[b, f] sum_l Y_l0(cos alpha_t) Q[kj(t), l, b] regrouped
// by the source edge e' = kj(t).  ga of the out-edges is staged in LDS once per workgroup; Y_l0 is evaluated in
// registers (a lane keeps one l); nothing of size T or E x B x F is read or written.
template <int NT>   // F = 32 NT
__global__ void __launch_bounds__(256, 2)   // three workgroups per CU would spill
tripD_mfma_bwd_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ out_ptr,
                      const int32_t* __restrict__ out_list, const int32_t* __restrict__ seg_ptr_kj,
                      const int32_t* __restrict__ idx_ji_kj, const float* __restrict__ cos_kj,
                      const float* __restrict__ x, const float* __restrict__ Qt, const float* __restrict__ W2,
                      const float* __restrict__ ga, const float* __restrict__ z, int64_t E, int S, int kn_cap,
                      int parts, int rows_cap, float* __restrict__ gx, float* __restrict__ gQ, float* __restrict__ w2part) {
  constexpr int F = 32 * NT, LDZ = F + 32;   // the two k halves of a wavefront read disjoint banks
  constexpr int LDU = F + 4;
  float* wp = w2part + (int64_t)blockIdx.x * DB * F;
  rows_t P;
  const bool work = centre_rows(row_ptr, out_ptr, parts, P);
  const int Kn = work ? (P.dout + 15) & ~15 : 0;
  if (!work || Kn > kn_cap) {
    for (int i = threadIdx.x; i < DB * F; i += 256) wp[i] = 0.f;
    return;
  }
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  int* row_tab = reinterpret_cast<int*>(smem_raw);
  float* Q_w = reinterpret_cast<float*>(smem_raw + row_tab_bytes(rows_cap));   // per wavefront: [4 rows][LDQ], element (l, b) at l * 8 + b
  float* U_w = Q_w + 4 * 4 * LDQ;                    // per wavefront: x H of one row, [8 l][LDU]
  float* Z_s = U_w + 4 * 8 * LDU;                    // [Kn][LDZ]; reused for the weight-gradient partial sums
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int32_t* outs = out_list + P.o0;
  fill_row_table(seg_ptr_kj, idx_ji_kj, outs, P, row_tab, rows_cap);
#pragma unroll 4
  for (int i = threadIdx.x; i < Kn * (F / 4); i += 256) {   // Kn > 0 only if the atom has out-edges
    const int n = i / (F / 4), f4 = (i % (F / 4)) * 4;
    const bool ok = n < P.dout;
    const f32x4 v = *reinterpret_cast<const f32x4*>(ga + (int64_t)outs[ok ? n : 0] * F + f4) * (ok ? 1.f : 0.f);
    *reinterpret_cast<f32x4*>(&Z_s[n * LDZ + f4]) = v;
  }
  __syncthreads();

  const int kh = lane >> 5, l32 = lane & 31;
  const int l = l32 & 7;
  float q[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) q[i] = l < S ? Y_NORM_M[l] * LEG_Q[l][i] : 0.f;
  const bool odd = l & 1;
  float w2[DB][NT], dw2[DB][NT];
#pragma unroll
  for (int b = 0; b < DB; ++b)
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      w2[b][t] = W2[b * F + t * 32 + l32];
      dw2[b][t] = 0.f;
    }
  float* Qw = Q_w + wave * 4 * LDQ;
  float* Uw = U_w + wave * 8 * LDU;
  float w2s[4 * NT];   // W2[b = lane / 8][slice lane % 8 of the columns]
#pragma unroll
  for (int k = 0; k < 4 * NT; ++k) w2s[k] = W2[(lane >> 3) * F + (lane & 7) * (4 * NT) + k];
  const int nb = Kn / 16;   // batches of 8 k-steps (16 out-edge positions)

  // a wavefront takes 4 in-edge rows (32 MFMA rows) at a time
  for (int sg = 2 * P.gb + wave; sg < 2 * P.ge && sg * 4 < P.d; sg += 4) {
    const int pa = sg * 4 + (l32 >> 3);
    const bool pv = pa < P.d;
    const rowinfo_t ri = table_row(row_tab, rows_cap, P, pa);
    // Q of the 4 rows: lane (row lane % 4, b = (lane / 4) % 8, l half lane / 32) fetches 4 values of l; they go to LDS
    // after the main loop
    float qv[4];
    {
      const int p = sg * 4 + (lane & 3), b = (lane >> 2) & 7;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int lq = 4 * kh + i;
        qv[i] = Qt[(int64_t)((lq < S ? lq : S - 1) * DB + b) * E + P.r0 + (p < P.d ? p : P.d - 1)] * ((p < P.d && lq < S) ? 1.f : 0.f);
      }
    }
    // x and z of the 4 rows, for the epilogue
    float xv[4][NT], zv[4][NT];
#pragma unroll
    for (int eg = 0; eg < 4; ++eg) {
      const int p = sg * 4 + eg;
      const int64_t e = P.r0 + (p < P.d ? p : P.d - 1);
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        xv[eg][t] = x[e * F + t * 32 + l32] * (p < P.d ? 1.f : 0.f);   // e is clamped to a valid row
        zv[eg][t] = z ? z[e * F + t * 32 + l32] : 0.f;
      }
    }
    f32x16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;

    // cosines of batch bt (2 marks "no triplet"), fetched one batch ahead
    auto load_c = [&](int bt, float (&c)[8]) __attribute__((always_inline)) {
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int n = bt * 16 + 2 * u + kh;
        const int slot = n - (n > ri.gap ? 1 : 0);
        const bool valid = bt < nb && pv && n != ri.gap && slot < ri.cnt;
        const float cv = cos_kj[valid ? ri.seg + slot : 0];   // unconditional load, index 0 when unused
        c[u] = valid ? cv : 2.f;
      }
    };
    float cn[8];
    load_c(0, cn);
    for (int bt = 0; bt < nb; ++bt) {
      float cc[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) cc[u] = cn[u];
      load_c(bt + 1, cn);
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const bool valid = cc[u] <= 1.5f;
        const float cv = valid ? cc[u] : 0.f;
        const float t2 = cv * cv;
        const float yv = (odd ? cv : 1.f) * (q[0] + t2 * (q[1] + t2 * (q[2] + t2 * q[3])));
        const float y = valid ? yv : 0.f;
        const float* zr = Z_s + (bt * 16 + 2 * u + kh) * LDZ + l32;
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(y, zr[t * 32], acc[t], 0, 0, 0);
      }
    }

    wave_lds_sync();   // the previous pass's reads of Qw are done
    {
      const int pr = lane & 3, b = (lane >> 2) & 7;
#pragma unroll
      for (int i = 0; i < 4; ++i) Qw[pr * LDQ + (4 * kh + i) * DB + b] = qv[i];
    }
    wave_lds_sync();

    // accumulator register v of lane (kh, l32): row 8 (v/4) + 4 kh + v%4 = (in-edge row v/4 of the pass, l = 4 kh + v%4),
    // column l32 of the block
#pragma unroll
    for (int eg = 0; eg < 4; ++eg) {
      const int p = sg * 4 + eg;
      const bool ok = p < P.d;
      const int64_t e = P.r0 + (ok ? p : P.d - 1);
      float D[DB][NT];
#pragma unroll
      for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int t = 0; t < NT; ++t) D[b][t] = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float* qr = Qw + eg * LDQ + (4 * kh + i) * DB;
        const f32x4 qa = *reinterpret_cast<const f32x4*>(qr), qb = *reinterpret_cast<const f32x4*>(qr + 4);
        const float qq[DB] = {qa[0], qa[1], qa[2], qa[3], qb[0], qb[1], qb[2], qb[3]};
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          const float h = acc[t][4 * eg + i];
          Uw[(4 * kh + i) * LDU + t * 32 + l32] = xv[eg][t] * h;
#pragma unroll
          for (int b = 0; b < DB; ++b) D[b][t] += qq[b] * h;
        }
      }
      float dxp[NT];
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        float sum = 0.f;
#pragma unroll
        for (int b = 0; b < DB; ++b) {
          sum += w2[b][t] * D[b][t];
          dw2[b][t] += xv[eg][t] * D[b][t];
        }
        dxp[t] = sum + __shfl_xor(sum, 32);
      }
      if (ok && kh == 0) {
#pragma unroll
        for (int t = 0; t < NT; ++t) gx[e * F + t * 32 + l32] = z ? dxp[t] * dsilu_f(zv[eg][t]) : dxp[t];
      }
      // gQ[l, b] = sum_f W2[b, f] U[l, f]: lane (b = lane / 8, slice fs = lane % 8 of the columns) forms its part of all
      // 8 sums, then the 8 lanes of a b exchange them, halving the number of values each time; lane fs ends with l = fs
      wave_lds_sync();
      float gq[8];
#pragma unroll
      for (int lq = 0; lq < 8; ++lq) {
        const float* ur = Uw + lq * LDU + (lane & 7) * (4 * NT);
        float sum = 0.f;
#pragma unroll
        for (int k4 = 0; k4 < NT; ++k4) {
          const f32x4 uv = *reinterpret_cast<const f32x4*>(ur + 4 * k4);
#pragma unroll
          for (int c = 0; c < 4; ++c) sum += w2s[4 * k4 + c] * uv[c];
        }
        gq[lq] = sum;
      }
#pragma unroll
      for (int m = 4, half = 4; m >= 1; m >>= 1, half >>= 1) {
        const bool up = (lane & m) != 0;
#pragma unroll
        for (int i = 0; i < half; ++i) {
          const float send = up ? gq[i] : gq[i + half];
          const float keep = up ? gq[i + half] : gq[i];
          gq[i] = keep + __shfl_xor(send, m);
        }
      }
      if (ok && (lane & 7) < S) gQ[(e * S + (lane & 7)) * DB + (lane >> 3)] = gq[0];
      wave_lds_sync();   // Uw is rewritten for the next row
      __builtin_amdgcn_sched_barrier(0);   // keep the four rows' epilogues apart: interleaved they need twice the registers
    }
  }

  // weight-gradient partial sum of the workgroup: 8 slots (wavefront, k half), summed in a fixed order
  __syncthreads();
  float* red = Z_s;
#pragma unroll
  for (int b = 0; b < DB; ++b)
#pragma unroll
    for (int t = 0; t < NT; ++t) red[((wave * 2 + kh) * DB + b) * F + t * 32 + l32] = dw2[b][t];
  __syncthreads();
  for (int i = threadIdx.x; i < DB * F; i += 256) {
    float sum = red[i];
#pragma unroll
    for (int k = 1; k < 8; ++k) sum += red[k * DB * F + i];
    wp[i] = sum;
  }
}

// grad_cos_kj[slot of (e', e)] (+)= sum_l Y_l0'(cos) W[(e', l), e],  W = U_j . dz_out^T  (rows (in-edge row, l),
// columns out-edge positions n, contraction over o).  U rows go straight from memory to A fragments,
// dz of the out-edges is staged in LDS (bf16); the derivative weights are applied to the accumulators.
template <int KS>   // O = 16 KS
__global__ void __launch_bounds__(256)
tripG_mfma_dcos_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ out_ptr,
                       const int32_t* __restrict__ out_list, const int32_t* __restrict__ seg_ptr_kj,
                       const int32_t* __restrict__ idx_ji_kj, const float* __restrict__ cos_kj,
                       const float* __restrict__ U, const float* __restrict__ dz, int S, int kn_cap, int parts, int rows_cap, int accumulate,
                       float* __restrict__ grad_cos_kj) {
  constexpr int O = 16 * KS, LDO = O + 8;
  rows_t P;
  if (!centre_rows(row_ptr, out_ptr, parts, P)) return;
  const int Kn = (P.dout + 31) & ~31;
  if (Kn > kn_cap || P.dout == 0) return;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  int* row_tab = reinterpret_cast<int*>(smem_raw);
  __bf16* ZB = reinterpret_cast<__bf16*>(smem_raw + row_tab_bytes(rows_cap));   // ZB[n][o], row stride LDO
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int32_t* outs = out_list + P.o0;
  fill_row_table(seg_ptr_kj, idx_ji_kj, outs, P, row_tab, rows_cap);

#pragma unroll 4
  for (int it = threadIdx.x; it < Kn * (O / 8); it += 256) {   // P.dout > 0 here
    const int n = it / (O / 8), oc = (it % (O / 8)) * 8;
    const bool ok = n < P.dout;
    const float* src = dz + (int64_t)outs[ok ? n : 0] * O + oc;   // clamped position times a 0/1 factor
    const f32x4 v0 = *reinterpret_cast<const f32x4*>(src) * (ok ? 1.f : 0.f);
    const f32x4 v1 = *reinterpret_cast<const f32x4*>(src + 4) * (ok ? 1.f : 0.f);
    bf16x8 v;
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = (__bf16)v0[i], v[4 + i] = (__bf16)v1[i];
    *reinterpret_cast<bf16x8*>(&ZB[n * LDO + oc]) = v;
  }
  __syncthreads();

  const int kh = lane >> 5, l32 = lane & 31;
  const int l = l32 & 7;
  // Y_l0'(x) for this lane's four l = 4 kh + i as polynomials in x^2 (times x for even l): from
  // P_l = x^(l%2) sum_i q_i x^(2i), P_l' = sum_i (2i + l%2) q_i x^(2i + l%2 - 1)
  float dq[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int lq = 4 * kh + i;
    const float nrm = lq < S ? Y_NORM_M[lq] : 0.f;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      if (i & 1) dq[i][c] = nrm * (float)(2 * c + 1) * LEG_Q[lq][c];
      else dq[i][c] = c < 3 ? nrm * (float)(2 * c + 2) * LEG_Q[lq][c + 1] : 0.f;
    }
  }
  for (int grp = P.gb + wave; grp < P.ge; grp += 4) {
    // A fragments: row (in-edge row l32/8 of the block, l), 8 consecutive o per k-step
    bf16x8 a[2][KS];
    rowinfo_t mine[2];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
      const int p = grp * 8 + rb * 4 + (l32 >> 3);
      const bool ok = p < P.d && l < S;
      const int e = P.r0 + (p < P.d ? p : P.d - 1);
      mine[rb] = table_row(row_tab, rows_cap, P, p);
      const float* src = U + ((int64_t)e * S + (l < S ? l : 0)) * O + kh * 8;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const f32x4 v0 = *reinterpret_cast<const f32x4*>(src + ks * 16), v1 = *reinterpret_cast<const f32x4*>(src + ks * 16 + 4);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          a[rb][ks][i] = (__bf16)(ok ? v0[i] : 0.f);
          a[rb][ks][4 + i] = (__bf16)(ok ? v1[i] : 0.f);
        }
      }
    }
    // row information of in-edge row pl of a block sits in lanes 8 pl .. 8 pl + 7
    int rseg[2][4], rcnt[2][4], rgap[2][4];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int pl = 0; pl < 4; ++pl) {
        rseg[rb][pl] = __shfl(mine[rb].seg, pl * 8, 64);
        rgap[rb][pl] = __shfl(mine[rb].gap, pl * 8, 64);
        // rows past the end of the atom's list take part in nothing
        rcnt[rb][pl] = grp * 8 + rb * 4 + pl < P.d ? __shfl(mine[rb].cnt, pl * 8, 64) : 0;
      }
    // cosines (and, when accumulating, the values to add to) of this lane's column for the 8 rows;
    // fetched one column block ahead so that the loads overlap the products
    auto fetch = [&](int nb, float (&xs)[2][4], float (&old)[2][4]) {
      const int n = nb * 32 + l32;
#pragma unroll
      for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int pl = 0; pl < 4; ++pl) {
          const int slot = n - (n > rgap[rb][pl] ? 1 : 0);
          const bool valid = n != rgap[rb][pl] && slot < rcnt[rb][pl];
          const int at = valid ? rseg[rb][pl] + slot : 0;   // unconditional loads, index 0 when unused
          const float cv = cos_kj[at], ov = accumulate ? grad_cos_kj[at] : 0.f;
          xs[rb][pl] = valid ? cv : 0.f;
          old[rb][pl] = valid ? ov : 0.f;
        }
    };
    float xs_n[2][4], old_n[2][4];
    fetch(0, xs_n, old_n);
    for (int nb = 0; nb < Kn / 32; ++nb) {
      float xs[2][4], old[2][4];
#pragma unroll
      for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int pl = 0; pl < 4; ++pl) xs[rb][pl] = xs_n[rb][pl], old[rb][pl] = old_n[rb][pl];
      if (nb + 1 < Kn / 32) fetch(nb + 1, xs_n, old_n);
      f32x16 acc[2];
#pragma unroll
      for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[rb][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 b = *reinterpret_cast<const bf16x8*>(&ZB[(nb * 32 + l32) * LDO + ks * 16 + kh * 8]);
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[rb][ks], b, acc[rb], 0, 0, 0);
      }
      const int n = nb * 32 + l32;   // this lane's column
#pragma unroll
      for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int pl = 0; pl < 4; ++pl) {
          const int slot = n - (n > rgap[rb][pl] ? 1 : 0);
          const bool valid = n != rgap[rb][pl] && slot < rcnt[rb][pl];
          const float x = xs[rb][pl], t2 = x * x;
          float part = 0.f;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float w = dq[i][0] + t2 * (dq[i][1] + t2 * (dq[i][2] + t2 * dq[i][3]));
            part += acc[rb][4 * pl + i] * ((i & 1) ? w : x * w);   // l = 4 kh + i even: odd derivative
          }
          const float total = part + __shfl_xor(part, 32, 64);
          if (valid && kh == (pl >> 1)) grad_cos_kj[rseg[rb][pl] + slot] = old[rb][pl] + total;
        }
    }
  }
}

int kp_of(const gp_graph* g) { return (g->max_in_degree + 15) & ~15; }
// Workgroups per centre atom: as many as the atom with the most out-edges (forward kernels: PART_EDGES edges each) or
// in-edges (backward kernels: GPW groups of 8 rows each) needs, at most PARTS.  Launching PARTS everywhere
// would leave most workgroups without work, and starting a workgroup is not free (1280 atoms x 8: 0.2 ms).
// (Shares of 32 rather than 64 out-edges: variant-D forward kernel 0.106 -> 0.080 ms at configuration 2, y kernel and
// contraction 0.094 + 0.114 -> 0.076 + 0.083 ms at configuration 3; 16: the same.  Configuration 4 has 8 parts either way.)
constexpr int PART_EDGES = 32;
int parts_out(const gp_graph* g) { const int n = (g->max_out_degree + PART_EDGES - 1) / PART_EDGES; return n < 1 ? 1 : n > PARTS ? PARTS : n; }
int parts_in(const gp_graph* g);
// Most in-edge rows in one workgroup's share (centre_rows).  An atom with up to GPW groups is one share; a larger one
// is cut into shares of at most GPW groups unless the number of parts is capped, and then the largest atom has the
// largest share.  (Not simply the largest atom's share: with 9 groups in 2 parts it has 40 rows, an atom of 7 groups 56.)
int share_rows(const gp_graph* g) {
  const int groups = (g->max_in_degree + 7) / 8, parts = parts_in(g);
  const int whole = groups < GPW ? groups : GPW, cut = (groups + parts - 1) / parts;
  return 8 * (whole > cut ? whole : cut);
}
int parts_in(const gp_graph* g) { const int n = (g->max_in_degree + 8 * GPW - 1) / (8 * GPW); return n < 1 ? 1 : n > PARTS_IN ? PARTS_IN : n; }
int kn_of(const gp_graph* g) { return (g->max_out_degree + 31) & ~31; }
// dz of the out-edges (bf16, transposed)
size_t lds_H(int O, int kn) { return (size_t)(kn + 8) * O * sizeof(__bf16); }

}  // namespace

size_t gp_tripG_mfma_scratch(int64_t E, int64_t T) { return gp_align((size_t)(T + 16 * E) * CP * sizeof(__bf16)); }

bool gp_tripG_mfma_usable(const gp_graph* g, int F, int S, int C) {
  if (!g || !g->row_ptr || !g->out_ptr || !g->out_list || g->n_atoms <= 0 || g->max_in_degree <= 0) return false;
  if (g->n_triplets <= 0) return false;   // the kernels read cos_alpha[0] for absent triplets
  if (g->n_atoms > INT32_MAX / PARTS_IN) return false;
  if (F % 32 != 0 || F < 32 || F > 128 || C < 1 || C > CP || S < 1 || S > ST) return false;
  return (size_t)F * (kp_of(g) + 8) * sizeof(__bf16) <= LDS_MAX;
}

bool gp_tripD_mfma_usable(const gp_graph* g, int F, int S, int B) {
  if (!g || !g->row_ptr || !g->out_ptr || !g->out_list || g->n_atoms <= 0 || g->max_in_degree <= 0) return false;
  if (g->n_triplets <= 0) return false;   // the kernel reads cos_alpha[0] for absent triplets
  if (g->n_atoms > INT32_MAX / PARTS_IN) return false;
  if (B != DB || F % 32 != 0 || F < 32 || F > 128 || S < 1 || S > ST) return false;
  return (size_t)kp_of(g) * (F + LDQ) * sizeof(float) <= 64 * 1024;
}

int gp_tripD_forward_mfma(gp_ctx* ctx, const gp_graph* g, const float* cos_alpha, const float* x, const float* Qt,
                          const float* W2, int F, int S, int B, float* a, float* Bacc) {
  const int64_t E = g->n_edges, T = g->n_triplets;
  if (E == 0) return GP_OK;
  GP_REQUIRE(ctx, gp_tripD_mfma_usable(g, F, S, B), "triplet D (matrix-core form): graph lists or widths not supported");
  GP_REQUIRE(ctx, g->seg_ptr_ji && g->idx_kj && cos_alpha && x && Qt && W2 && a, "triplet D forward: NULL pointer");
  const int kp_cap = kp_of(g), parts = parts_out(g);
  const unsigned grid = (unsigned)(g->n_atoms * parts);
  const size_t lds = (size_t)kp_cap * (F + LDQ) * sizeof(float);
  const double Td = (double)T, Ed = (double)E;
  gp_prof_scope prof(ctx, "tripD_mfma_fwd", Td * 2.0 * (S * B + B * F) + Ed * 2.0 * B * F,
                     Td * 8.0 + Ed * 4.0 * (F + S * B + (Bacc ? B * F : 0) + F) + Ed * 4.0);
#define GP_D_FWD(NT)                                                                                              \
  tripD_mfma_fwd_kernel<NT><<<grid, 256, lds, ctx->stream>>>(g->row_ptr, g->out_ptr, g->out_list, g->seg_ptr_ji, \
                                                             g->idx_kj, cos_alpha, x, Qt, W2, E, S, kp_cap, parts, a, Bacc)
  if (F == 32) GP_D_FWD(1);
  else if (F == 64) GP_D_FWD(2);
  else if (F == 96) GP_D_FWD(3);
  else GP_D_FWD(4);
#undef GP_D_FWD
  GP_LAUNCH_CHECK(ctx, "tripD_mfma_fwd_kernel");
  return GP_OK;
}

int gp_tripG_forward_mfma(gp_ctx* ctx, const gp_graph* g, const float* cos_alpha, const float* x, const float* Radt,
                          int F, int S, int C, float* A, void* ybuf, size_t ybytes, int out_half, const int32_t* row_list,
                          int rad_by_pos) {
  const int64_t E = g->n_edges, T = g->n_triplets;
  if (E == 0) return GP_OK;
  GP_REQUIRE(ctx, gp_tripG_mfma_usable(g, F, S, C), "triplet G (matrix-core form): graph lists or widths not supported");
  GP_REQUIRE(ctx, g->seg_ptr_ji && (T == 0 || (g->idx_kj && cos_alpha)) && x && Radt && A && ybuf, "triplet G forward: NULL pointer");
  if (ybytes < gp_tripG_mfma_scratch(E, T)) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "triplet G forward: y buffer too small");
  const int kp_cap = kp_of(g), parts = parts_out(g);
  const unsigned grid = (unsigned)(g->n_atoms * parts);
  const double Td = (double)T, Ed = (double)E;
  __bf16* Yb = static_cast<__bf16*>(ybuf);
  {
    gp_prof_scope prof(ctx, "tripG_y", Td * (2.0 * S * C + 4.0 * S), (Td + 16.0 * Ed) * CP * 2.0 + Td * 8.0 + Ed * 4.0 * S * C);
    const int yt = kp_cap >= YT ? YT : (kp_cap + 63) & ~63;
    if (S <= 7)
      tripG_y_kernel<7><<<grid, yt, 0, ctx->stream>>>(g->row_ptr, g->out_ptr, g->out_list, g->seg_ptr_ji, g->idx_kj,
                                                       cos_alpha, Radt, E, S, C, kp_cap, parts, row_list, rad_by_pos, Yb);
    else
      tripG_y_kernel<8><<<grid, yt, 0, ctx->stream>>>(g->row_ptr, g->out_ptr, g->out_list, g->seg_ptr_ji, g->idx_kj,
                                                       cos_alpha, Radt, E, S, C, kp_cap, parts, row_list, rad_by_pos, Yb);
    GP_LAUNCH_CHECK(ctx, "tripG_y_kernel");
  }
  {
    const size_t lds = (size_t)F * (kp_cap + 8) * sizeof(__bf16);
    // registers allow 8 wavefronts per CU: two workgroups of 256 threads if their X tiles fit side by side
    const int mt = lds <= LDS_MAX / 2 ? 256 : MT;
    gp_prof_scope prof(ctx, "tripG_mfma_fwd", Td * 2.0 * C * F, (Td + 16.0 * Ed) * CP * 2.0 + Ed * (4.0 * F + (out_half ? 2.0 : 4.0) * C * F));
#define GP_TRIPG_LAUNCH(CB)                                                                                       \
  do {                                                                                                            \
    static size_t lds_set = 0;                                                                                    \
    if (lds > lds_set) {                                                                                          \
      GP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&tripG_mfma_kernel<CB>),                      \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));                     \
      lds_set = lds;                                                                                              \
    }                                                                                                             \
    tripG_mfma_kernel<CB><<<grid, mt, lds, ctx->stream>>>(g->row_ptr, g->out_ptr, g->out_list, g->seg_ptr_ji, x,  \
                                                          Yb, C, kp_cap, parts, out_half, row_list, A);           \
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

namespace {
size_t lds_D_bwd(int F, int kn) {
  const size_t zs = (size_t)kn * (F + 32), red = (size_t)8 * DB * F;
  return (4 * 4 * LDQ + 4 * 8 * (F + 4) + (zs > red ? zs : red)) * sizeof(float);
}
}  // namespace

bool gp_tripD_mfma_bwd_usable(const gp_graph* g, int F, int S, int B) {
  if (!g || !g->row_ptr || !g->out_ptr || !g->out_list || g->n_atoms <= 0 || g->max_out_degree <= 0) return false;
  if (g->n_triplets <= 0) return false;   // the kernel reads cos_alpha_kj[0] for absent triplets
  if (!g->seg_ptr_kj || !g->idx_ji_kj || g->n_atoms > INT32_MAX / PARTS_IN) return false;
  if (B != DB || F % 32 != 0 || F < 32 || F > 128 || S < 1 || S > ST) return false;
  const int kn = (g->max_out_degree + 15) & ~15;
  return lds_D_bwd(F, kn) + row_tab_bytes(share_rows(g)) <= 64 * 1024;
}

size_t gp_tripD_mfma_bwd_scratch(const gp_graph* g, int F) {
  return gp_align((size_t)g->n_atoms * parts_in(g) * DB * F * sizeof(float));
}

int gp_tripD_backward_mfma(gp_ctx* ctx, const gp_graph* g, const float* cos_alpha_kj, const float* x, const float* Qt,
                           const float* W2, const float* grad_a, const float* z, int F, int S, int B, float* grad_x,
                           float* grad_Q, float* grad_W2, float* part, size_t part_bytes) {
  const int64_t E = g->n_edges, T = g->n_triplets;
  if (E == 0) return GP_OK;
  GP_REQUIRE(ctx, gp_tripD_mfma_bwd_usable(g, F, S, B), "triplet D backward (matrix-core form): graph lists or widths not supported");
  GP_REQUIRE(ctx, cos_alpha_kj && x && Qt && W2 && grad_a && grad_x && grad_Q && grad_W2, "triplet D backward: NULL pointer");
  if (!part || part_bytes < gp_tripD_mfma_bwd_scratch(g, F))
    return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "triplet D backward: scratch too small");
  const int kn_cap = (g->max_out_degree + 15) & ~15, parts = parts_in(g), rows_cap = share_rows(g);
  const unsigned grid = (unsigned)(g->n_atoms * parts);
  const size_t lds = lds_D_bwd(F, kn_cap) + row_tab_bytes(rows_cap);
  const double Td = (double)T, Ed = (double)E;
  {
    gp_prof_scope prof(ctx, "tripD_mfma_bwd", Td * 2.0 * 8 * F + Ed * 2.0 * (3.0 * 8 * DB * F + 2.0 * DB * F),
                       Td * 4.0 + Ed * 4.0 * (4.0 * F + 2.0 * S * DB));
#define GP_D_BWD(NT)                                                                                                 \
  tripD_mfma_bwd_kernel<NT><<<grid, 256, lds, ctx->stream>>>(g->row_ptr, g->out_ptr, g->out_list, g->seg_ptr_kj,    \
                                                             g->idx_ji_kj, cos_alpha_kj, x, Qt, W2, grad_a, z, E, S, \
                                                             kn_cap, parts, rows_cap, grad_x, grad_Q, part)
    if (F == 32) GP_D_BWD(1);
    else if (F == 64) GP_D_BWD(2);
    else if (F == 96) GP_D_BWD(3);
    else GP_D_BWD(4);
#undef GP_D_BWD
    GP_LAUNCH_CHECK(ctx, "tripD_mfma_bwd_kernel");
  }
  return gp_reduce_parts(ctx, part, (int)grid, (int64_t)DB * F, grad_W2);
}

bool gp_tripG_mfma_bwd_usable(const gp_graph* g, int O, int S) {
  if (!g || !g->row_ptr || !g->out_ptr || !g->out_list || g->n_atoms <= 0 || g->max_out_degree <= 0) return false;
  if (g->n_triplets <= 0) return false;   // the kernels read cos_alpha_kj[0] for absent triplets
  if (!g->seg_ptr_kj || !g->idx_ji_kj || g->n_atoms > INT32_MAX / PARTS_IN) return false;
  if (O % 32 != 0 || O < 32 || O > 128 || S < 1 || S > ST) return false;
  const size_t tab = row_tab_bytes(share_rows(g));   // the kernels' row table
  return lds_H(O, kn_of(g)) + tab <= LDS_MAX && (size_t)kn_of(g) * (O + 8) * sizeof(__bf16) + tab <= LDS_MAX;
}

bool gp_tripG_mfma_H_usable(const gp_graph* g, int O, int S) {
  if (!g || !g->row_ptr || !g->out_ptr || !g->out_list || g->n_atoms <= 0 || g->max_out_degree <= 0) return false;
  if (g->n_triplets <= 0) return false;
  if (!g->seg_ptr_kj || !g->idx_ji_kj || g->n_atoms > INT32_MAX / PARTS_IN) return false;
  if (O % 32 != 0 || O < 32 || O > 128 || S < 1 || S > ST) return false;
  return lds_H(O, kn_of(g)) + row_tab_bytes(share_rows(g)) <= LDS_MAX;
}

int gp_tripG_backward_H_mfma(gp_ctx* ctx, const gp_graph* g, const float* cos_alpha_kj, const float* dz, int O, int S,
                             float* H, const int32_t* row_list) {
  const int64_t E = g->n_edges, T = g->n_triplets;
  if (E == 0) return GP_OK;
  GP_REQUIRE(ctx, gp_tripG_mfma_H_usable(g, O, S), "triplet G backward (matrix-core form): graph lists or widths not supported");
  GP_REQUIRE(ctx, dz && H && (T == 0 || cos_alpha_kj), "triplet G backward: NULL pointer");
  const int kn_cap = kn_of(g), parts = parts_in(g);
  const unsigned grid = (unsigned)(g->n_atoms * parts);
  const int rows_cap = share_rows(g);
  const size_t lds = lds_H(O, kn_cap) + row_tab_bytes(rows_cap);
  gp_prof_scope prof(ctx, "tripG_mfma_H", (double)T * 2.0 * 8 * O, (double)T * 4.0 + 4.0 * E * (O + (double)S * O));
#define GP_TRIPG_LAUNCH(CB)                                                                                          \
  do {                                                                                                               \
    static size_t lds_set = 0;                                                                                       \
    if (lds > lds_set) {                                                                                             \
      GP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&tripG_mfma_H_kernel<CB>),                       \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));                        \
      lds_set = lds;                                                                                                 \
    }                                                                                                                \
    tripG_mfma_H_kernel<CB><<<grid, 256, lds, ctx->stream>>>(g->row_ptr, g->out_ptr, g->out_list, g->seg_ptr_kj,     \
                                                             g->idx_ji_kj, cos_alpha_kj, dz, S, kn_cap, parts,       \
                                                             rows_cap, row_list, H);                                 \
  } while (0)
  switch (O / 32) {
    case 1: GP_TRIPG_LAUNCH(1); break;
    case 2: GP_TRIPG_LAUNCH(2); break;
    case 3: GP_TRIPG_LAUNCH(3); break;
    default: GP_TRIPG_LAUNCH(4); break;
  }
#undef GP_TRIPG_LAUNCH
  GP_LAUNCH_CHECK(ctx, "tripG_mfma_H_kernel");
  return GP_OK;
}

int gp_tripG_grad_cos_mfma(gp_ctx* ctx, const gp_graph* g, const float* cos_alpha_kj, const float* U, const float* dz,
                           int O, int S, int accumulate, float* grad_cos_kj) {
  const int64_t E = g->n_edges, T = g->n_triplets;
  if (E == 0 || T == 0) return GP_OK;
  GP_REQUIRE(ctx, gp_tripG_mfma_bwd_usable(g, O, S), "grad_cos (matrix-core form): graph lists or widths not supported");
  GP_REQUIRE(ctx, cos_alpha_kj && U && dz && grad_cos_kj, "grad_cos: NULL pointer");
  const int kn_cap = kn_of(g), parts = parts_in(g);
  const unsigned grid = (unsigned)(g->n_atoms * parts);
  const int rows_cap = share_rows(g);
  const size_t lds = (size_t)kn_cap * (O + 8) * sizeof(__bf16) + row_tab_bytes(rows_cap);
  gp_prof_scope prof(ctx, "tripG_mfma_dcos", (double)T * 2.0 * 8 * O, (double)T * 12.0 + 4.0 * E * (O + (double)S * O));
#define GP_TRIPG_LAUNCH(KS)                                                                                          \
  do {                                                                                                               \
    static size_t lds_set = 0;                                                                                       \
    if (lds > lds_set) {                                                                                             \
      GP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&tripG_mfma_dcos_kernel<KS>),                    \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));                        \
      lds_set = lds;                                                                                                 \
    }                                                                                                                \
    tripG_mfma_dcos_kernel<KS><<<grid, 256, lds, ctx->stream>>>(g->row_ptr, g->out_ptr, g->out_list, g->seg_ptr_kj,  \
                                                                g->idx_ji_kj, cos_alpha_kj, U, dz, S, kn_cap, parts, \
                                                                rows_cap, accumulate, grad_cos_kj);                            \
  } while (0)
  switch (O / 32) {
    case 1: GP_TRIPG_LAUNCH(2); break;
    case 2: GP_TRIPG_LAUNCH(4); break;
    case 3: GP_TRIPG_LAUNCH(6); break;
    default: GP_TRIPG_LAUNCH(8); break;
  }
#undef GP_TRIPG_LAUNCH
  GP_LAUNCH_CHECK(ctx, "tripG_mfma_dcos_kernel");
  return GP_OK;
}
