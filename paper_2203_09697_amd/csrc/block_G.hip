// Interaction block, variant G (paper Sec. 3.4: bilinear layer in place of the Hadamard product,
// operations ordered so that nothing of size T x width is stored), forward and backward.
//
//   x    = act(m W_ba) * (g (W_rbfS W_rbfB));  x = act(x W_down)                [E, F]
//   Rad  = g . W_c                                                             [E, S, C]
//   y_t  = sum_l Y_l0(cos alpha_t) Rad[kj(t), l, :]                             [T, C]  (never stored)
//   A_e  = sum_{t in seg(e)} y_t (x) x[kj(t)]                                   [E, C, F]
//   z    = A . W_bil                                                           [E, O]
//   m'   = (act(m W_skip) + act(z W_up)) / sqrt(2)
//
// Backward: with H[e',l,o] = sum_{t: kj(t)=e'} Y_l(t) dz[ji(t),o] (one pass over the kj-major
// triplet view), G[e',c,o] = sum_l Rad[e',l,c] H[e',l,o] gives dx = G . W_bil^T, and
// V[e',c,o] = sum_f W_bil[c,f,o] x[e',f] gives dRad[e',l,c] = sum_o V[e',c,o] H[e',l,o].
#include <stdarg.h>

#include <algorithm>

#include "aux_stream.h"
#include "gemm.h"
#include "triplet.h"

namespace {

constexpr float INV_SQRT2 = 0.70710678118654752440f;

bool half_storage(const gp_dims* d);

struct saved_G {
  float *z_ba, *gate, *xg, *z_dn, *x, *Radt, *A, *z, *z_up, *z_skip, *Wrbf, *WcT;
  float* B1;   // radial factor at the target edge only: B1[e,l,f] = sum_t Y_l(t) x[kj(t),f]
  float* z_ac; // symmetric blocks only: pre-activation of the second up-projection [E, H]
  __bf16* m_h; // bf16 storage only: the block's input messages rounded to bf16 [E, H] (operand of four GEMMs)
};

size_t carve_saved_G(void* p, const gp_dims* d, int64_t E, saved_G* s) {
  gp_carver c(p);
  const size_t H = d->emb, F = d->int_emb, C = d->emb_cbf, O = d->emb_bil, S = d->num_spherical, R = d->num_radial;
  s->z_ba = c.take<float>(E * H);
  s->gate = c.take<float>(E * H);
  s->xg = c.take<float>(E * H);
  s->z_dn = c.take<float>(E * F);
  s->x = c.take<float>(E * F);
  s->Radt = c.take<float>(S * C * E);
  s->A = c.take<float>(E * C * F);
  s->z = c.take<float>(E * O);
  s->z_up = c.take<float>(E * H);
  s->z_skip = c.take<float>(E * H);
  s->Wrbf = c.take<float>(R * H);
  s->WcT = c.take<float>(S * C * R);
  s->B1 = c.take<float>(d->radial_at_target ? E * S * F : 0);
  s->z_ac = c.take<float>(d->symmetric ? E * H : 0);
  s->m_h = c.take<__bf16>(half_storage(d) ? E * H : 0);
  return c.off;
}

struct scratch_G {
  float* eh[4];                  // [E, H]
  float *dz, *Hd, *Gm, *V, *dRad, *dzdn, *U;
  float *WbilP, *WbilV, *dWrbf, *dWcP;
  float* part;
  float* part_aux;   // split-K partials of the GEMMs issued on the side stream
  size_t part_bytes;
  void* ybuf;        // per-triplet y in bf16 for the matrix-core triplet kernels (bf16 blocks only)
  size_t ybytes;
  float *dA, *dB1, *gc_ji;   // radial factor at the target edge only: [E,C,F], [E,S,F], [T]
  int32_t* iota;             // ... and bf16: 0, 1, ..., E-1 (the in-edges of an atom as a list, for the mirrored views)
  float* Radt_out;           // ... and the radial table with its columns in out-list order [S*C, E]
  float* eh5;                // symmetric blocks only: a fifth [E, H] buffer
  // bf16 storage only: weight matrices rounded to bf16 once per call, so that both operands of the large
  // GEMMs are copied to LDS without conversion
  __bf16 *W_ba_h, *W_skip_h, *W_down_h, *W_up_h, *W_bil_h, *WbilP_h, *W_up_ac_h;
  float* df;         // backward, low-rank gate: gradient of the [E, emb_rbf] factor g W_rbfS
  __bf16* WbilV_h;   // backward: the [f, (c,o)] copy of W_bil
  __bf16* x_h;   // backward: the saved x rounded to bf16, an operand of the global->LDS GEMM kernel
};

size_t part_bytes_G(const gp_dims* d, int64_t E) {
  const int H = d->emb, F = d->int_emb, C = d->emb_cbf, O = d->emb_bil, S = d->num_spherical, R = d->num_radial;
  size_t m = gp_gemm_tn_scratch(E, H, H);
  m = std::max(m, gp_gemm_tn_scratch(E, O, H));
  m = std::max(m, gp_gemm_tn_scratch(E, C * F, O));
  m = std::max(m, gp_gemm_tn_scratch(E, R, S * C));
  m = std::max(m, gp_gemm_tn_scratch(E, H, F));
  m = std::max(m, gp_gemm_tn_scratch(E, R, H));
  m = std::max(m, gp_gemm_tn_scratch(R, d->emb_rbf, H));
  m = std::max(m, gp_gemm_tn_scratch(E, d->emb_rbf, H));
  m = std::max(m, gp_gemm_tn_scratch(E, R, d->emb_rbf));
  return m;
}

size_t carve_scratch_G(void* p, const gp_dims* d, int64_t N, int64_t E, int64_t T, scratch_G* s) {
  gp_carver c(p);
  const size_t H = d->emb, F = d->int_emb, C = d->emb_cbf, O = d->emb_bil, S = d->num_spherical, R = d->num_radial;
  for (int i = 0; i < 4; ++i) s->eh[i] = c.take<float>(E * H);
  s->dz = c.take<float>(E * O);
  s->Hd = c.take<float>(E * S * O);
  s->Gm = c.take<float>(E * C * O);
  s->V = c.take<float>(E * C * O);
  s->dRad = c.take<float>(E * S * C);
  s->dzdn = c.take<float>(E * F);
  s->U = c.take<float>(E * std::max<size_t>(S, 4) * O);   // fp32 [E, S, O], or bf16 [E, 8, O] for the one-pass grad-cos kernel
  s->WbilP = c.take<float>(C * O * F);
  s->WbilV = c.take<float>(F * C * O);
  s->dWrbf = c.take<float>(R * H);
  s->dWcP = c.take<float>(R * S * C);
  s->part_bytes = part_bytes_G(d, E);
  s->part = (float*)c.take<char>(s->part_bytes);
  s->part_aux = (float*)c.take<char>(s->part_bytes);
  // scratch of the matrix-core triplet kernels: the per-triplet y buffer of the two-kernel form, or the per-atom
  // operand tables of the fused form (N > 0: the graph carries its lists by centre atom)
  s->ybytes = d->dtype == GP_BF16_F32ACC ? std::max(gp_tripG_mfma_scratch(E, T), N > 0 ? std::max({gp_tripG_fused_scratch(N, E, std::max(d->int_emb, d->emb_bil)), gp_tripG_H_fused_scratch(N, E, std::max(d->int_emb, d->emb_bil)), gp_tripG_dcos_fused_scratch(N, E, d->emb_bil, 0)}) : (size_t)0) : 0;
  s->ybuf = c.take<char>(s->ybytes);
  const bool rt = d->radial_at_target != 0;
  s->dA = c.take<float>(rt ? E * C * F : 0);
  s->dB1 = c.take<float>(rt ? E * S * F : 0);
  s->gc_ji = c.take<float>(rt ? (size_t)T : 0);
  s->iota = c.take<int32_t>(rt && d->dtype == GP_BF16_F32ACC ? E : 0);
  s->Radt_out = c.take<float>(rt && d->dtype == GP_BF16_F32ACC ? S * C * E : 0);
  s->eh5 = c.take<float>(d->symmetric ? E * H : 0);
  const bool hs = half_storage(d);
  s->W_ba_h = c.take<__bf16>(hs ? H * H : 0);
  s->W_skip_h = c.take<__bf16>(hs ? H * H : 0);
  s->W_down_h = c.take<__bf16>(hs ? H * F : 0);
  s->W_up_h = c.take<__bf16>(hs ? O * H : 0);
  s->W_bil_h = c.take<__bf16>(hs ? C * F * O : 0);
  s->WbilP_h = c.take<__bf16>(hs ? C * O * F : 0);
  s->W_up_ac_h = c.take<__bf16>(hs && d->symmetric ? O * H : 0);
  s->df = c.take<float>(hs ? E * (size_t)d->emb_rbf : 0);
  s->WbilV_h = c.take<__bf16>(hs ? F * C * O : 0);
  s->x_h = c.take<__bf16>(hs ? E * F : 0);
  return c.off;
}

int check_dims_G(gp_ctx* ctx, const gp_dims* d) {
  GP_REQUIRE(ctx, d, "dims is NULL");
  if (d->variant != GP_VARIANT_G) return gp_fail(ctx, GP_UNSUPPORTED_DIMS, "variant %d is not the bilinear block", d->variant);
  if (d->emb < 1 || d->emb > 4096 || d->int_emb < 1 || d->int_emb > 256 || d->emb_cbf < 1 || d->emb_cbf > 16 ||
      d->emb_bil < 1 || d->emb_bil > 128 || d->emb_rbf < 1 || d->emb_rbf > 256 || d->num_spherical < 1 ||
      d->num_spherical > 8 || d->num_radial < 2 || d->num_radial > 1024)
    return gp_fail(ctx, GP_UNSUPPORTED_DIMS,
                   "variant G supports emb<=4096, emb_trip<=256, emb_cbf<=16, emb_bil<=128, emb_rbf<=256, "
                   "num_spherical<=8, num_radial<=1024 (got %d,%d,%d,%d,%d,%d,%d)", d->emb, d->int_emb, d->emb_cbf,
                   d->emb_bil, d->emb_rbf, d->num_spherical, d->num_radial);
  return GP_OK;
}

// The triplet kernels walk one of the two sorted views of the triplet list.  Handing them a graph
// whose two views are exchanged makes the kernel written for "sum over the triplets of a source
// edge" sum over the triplets of a target edge and vice versa (used when the radial factor sits
// at the target edge: every formula is the mirror image of the source-edge form).
gp_graph mirrored(const gp_graph* g) {
  gp_graph m = *g;
  m.idx_kj = g->idx_ji_kj;
  m.seg_ptr_ji = g->seg_ptr_kj;
  m.idx_ji_kj = g->idx_kj;
  m.seg_ptr_kj = g->seg_ptr_ji;
  m.n_atoms = 0;   // the lists by centre atom do not describe the mirrored views
  m.row_ptr = m.out_ptr = m.out_list = nullptr;
  return m;
}

// The lists by centre atom for the mirrored views: the rows of an atom (the edges whose features are gathered) are
// its out-edges, in out_list order, and the edges it accumulates into are its in-edges, which have consecutive ids
// (iota = 0, 1, ... serves as their list).  The matrix-core kernels take the row list as a separate argument.
gp_graph mirrored_lists(const gp_graph* g, const int32_t* iota) {
  gp_graph m = mirrored(g);
  m.n_atoms = g->n_atoms;
  m.row_ptr = g->out_ptr;
  m.out_ptr = g->row_ptr;
  m.out_list = iota;
  m.max_in_degree = g->max_out_degree;
  m.max_out_degree = g->max_in_degree;
  return m;
}

// dst[r, q] = src[r, list[q]] for the rows r = blockIdx.y of an [rows, n] matrix
__global__ void gather_cols_kernel(const float* __restrict__ src, const int32_t* __restrict__ list, int64_t n, float* __restrict__ dst) {
  const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (q < n) dst[(int64_t)blockIdx.y * n + q] = src[(int64_t)blockIdx.y * n + list[q]];
}

__global__ void iota_kernel(int32_t* __restrict__ out, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = (int32_t)i;
}

typedef __bf16 h4 __attribute__((ext_vector_type(4)));
typedef float f4 __attribute__((ext_vector_type(4)));
// four consecutive elements of an fp32 or bf16 array (index a multiple of 4, base 16- / 8-byte aligned)
__device__ __forceinline__ f4 load4(const float* p, int64_t i) { return *reinterpret_cast<const f4*>(p + i); }
__device__ __forceinline__ f4 load4(const __bf16* p, int64_t i) {
  const h4 h = *reinterpret_cast<const h4*>(p + i);
  return f4{(float)h[0], (float)h[1], (float)h[2], (float)h[3]};
}
__device__ __forceinline__ void store4(float* p, int64_t i, f4 v) { *reinterpret_cast<f4*>(p + i) = v; }
__device__ __forceinline__ void store4(__bf16* p, int64_t i, f4 v) {
  *reinterpret_cast<h4*>(p + i) = h4{(__bf16)v[0], (__bf16)v[1], (__bf16)v[2], (__bf16)v[3]};
}

// Symmetric message passing, forward: t[e,:] = sqrt(2) t[e,:] + u_ac[id_swap[e],:] (second term 0 without an
// opposite edge); the up-projection GEMM then stores (act(.) + t) / 2.  ST: storage type of t and u_ac.
template <class ST>
__global__ void sym_mix_kernel(ST* __restrict__ t, const ST* __restrict__ u_ac, const int32_t* __restrict__ id_swap,
                               int64_t E, int H) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= E * H) return;
  const int sw = id_swap[i / H];
  t[i] = (ST)(1.41421356237309504880f * (float)t[i] + (sw >= 0 ? (float)u_ac[(int64_t)sw * H + (i % H)] : 0.f));
}
// backward: d_up = g/2 silu'(z_up), d_skip = g/sqrt(2) silu'(z_skip), d_ac[e] = g[id_swap[e]]/2 silu'(z_ac[e]) (0 if none)
template <class ST>
__global__ void sym_bwd_kernel(const float* __restrict__ g, const ST* __restrict__ z_up, const ST* __restrict__ z_skip,
                               const ST* __restrict__ z_ac, const int32_t* __restrict__ id_swap, int64_t E, int H,
                               ST* __restrict__ d_up, ST* __restrict__ d_skip, ST* __restrict__ d_ac) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= E * H) return;
  const float gv = g[i];
  d_up[i] = (ST)(0.5f * gv * dsilu_f((float)z_up[i]));
  d_skip[i] = (ST)(0.70710678118654752440f * gv * dsilu_f((float)z_skip[i]));
  const int sw = id_swap[i / H];
  d_ac[i] = (ST)(sw >= 0 ? 0.5f * g[(int64_t)sw * H + (i % H)] * dsilu_f((float)z_ac[i]) : 0.f);
}
// the same two steps on 4 consecutive features per thread (H % 4 == 0)
template <class ST>
__global__ void sym_mix4_kernel(ST* __restrict__ t, const ST* __restrict__ u_ac, const int32_t* __restrict__ id_swap,
                                int64_t E, int H) {
  const int64_t i = 4 * ((int64_t)blockIdx.x * blockDim.x + threadIdx.x);
  if (i >= E * H) return;
  const int sw = id_swap[i / H];
  f4 v = 1.41421356237309504880f * load4(t, i);
  if (sw >= 0) v += load4(u_ac, (int64_t)sw * H + (i % H));
  store4(t, i, v);
}
template <class ST>
__global__ void sym_bwd4_kernel(const float* __restrict__ g, const ST* __restrict__ z_up, const ST* __restrict__ z_skip,
                                const ST* __restrict__ z_ac, const int32_t* __restrict__ id_swap, int64_t E, int H,
                                ST* __restrict__ d_up, ST* __restrict__ d_skip, ST* __restrict__ d_ac) {
  const int64_t i = 4 * ((int64_t)blockIdx.x * blockDim.x + threadIdx.x);
  if (i >= E * H) return;
  const f4 gv = load4(g, i), zu = load4(z_up, i), zs = load4(z_skip, i), za = load4(z_ac, i);
  const int sw = id_swap[i / H];
  f4 gs = {0.f, 0.f, 0.f, 0.f};
  if (sw >= 0) gs = load4(g, (int64_t)sw * H + (i % H));
  f4 du, ds, da;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    du[c] = 0.5f * gv[c] * dsilu_f(zu[c]);
    ds[c] = 0.70710678118654752440f * gv[c] * dsilu_f(zs[c]);
    da[c] = 0.5f * gs[c] * dsilu_f(za[c]);
  }
  store4(d_up, i, du);
  store4(d_skip, i, ds);
  store4(d_ac, i, da);
}

// ---- bf16 storage of the [E, emb] intermediates (bf16 blocks): elementwise kernels, 4 elements per thread

// d1 = g s silu'(z1), d2 = g s silu'(z2);  g fp32, everything else bf16
template <class GT>   // GT: storage of g (float, or __bf16 when the block above handed its input gradient over as bf16)
__global__ void dsilu2_half_kernel(const GT* __restrict__ g, float s, const __bf16* __restrict__ z1,
                                   const __bf16* __restrict__ z2, __bf16* __restrict__ d1, __bf16* __restrict__ d2,
                                   int64_t n) {
  const int64_t i = 4 * ((int64_t)blockIdx.x * blockDim.x + threadIdx.x);
  if (i >= n) return;
  if (i + 3 < n) {
    const f4 gv = load4(g, i);
    const h4 a = *reinterpret_cast<const h4*>(z1 + i), b = *reinterpret_cast<const h4*>(z2 + i);
    h4 o1, o2;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      o1[c] = (__bf16)(gv[c] * s * dsilu_f((float)a[c]));
      o2[c] = (__bf16)(gv[c] * s * dsilu_f((float)b[c]));
    }
    *reinterpret_cast<h4*>(d1 + i) = o1;
    *reinterpret_cast<h4*>(d2 + i) = o2;
  } else {
    for (int64_t k = i; k < n; ++k) {
      d1[k] = (__bf16)((float)g[k] * s * dsilu_f((float)z1[k]));
      d2[k] = (__bf16)((float)g[k] * s * dsilu_f((float)z2[k]));
    }
  }
}

// dz = dxg gate silu'(z), dgate = dxg silu(z);  all bf16
__global__ void gate_bwd_half_kernel(const __bf16* __restrict__ dxg, const __bf16* __restrict__ z,
                                     const __bf16* __restrict__ gate, __bf16* __restrict__ dz, __bf16* __restrict__ dgate,
                                     int64_t n) {
  const int64_t i = 4 * ((int64_t)blockIdx.x * blockDim.x + threadIdx.x);
  if (i >= n) return;
  if (i + 3 < n) {
    const h4 d = *reinterpret_cast<const h4*>(dxg + i), zz = *reinterpret_cast<const h4*>(z + i),
             gt = *reinterpret_cast<const h4*>(gate + i);
    h4 o1, o2;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const float dv = (float)d[c], zv = (float)zz[c];
      o1[c] = (__bf16)(dv * (float)gt[c] * dsilu_f(zv));
      o2[c] = (__bf16)(dv * silu_f(zv));
    }
    *reinterpret_cast<h4*>(dz + i) = o1;
    *reinterpret_cast<h4*>(dgate + i) = o2;
  } else {
    for (int64_t k = i; k < n; ++k) {
      const float dv = (float)dxg[k], zv = (float)z[k];
      dz[k] = (__bf16)(dv * (float)gate[k] * dsilu_f(zv));
      dgate[k] = (__bf16)(dv * silu_f(zv));
    }
  }
}

// The same with the gate evaluated in place from its two factors, gate[e, h] = sum_k g[e, k] Wrbf[k, h] with
// g [E, R], Wrbf [R, H], R <= 16 (in fp32; the forward GEMM's epilogue multiplied by the same sum of bf16-rounded
// factors, a difference below the rounding of the bf16 results), instead of read: a
// thread keeps the R x 4 weights of its 4 columns in registers and walks GATE_ROWS rows, whose R values are uniform
// across the workgroup.
constexpr int GATE_ROWS = 64;
__global__ void __launch_bounds__(256)
gate_bwd_lr_kernel(const __bf16* __restrict__ dxg, const __bf16* __restrict__ z, const float* __restrict__ g,
                   const float* __restrict__ Wrbf, int64_t E, int H, int R, __bf16* __restrict__ dz, __bf16* __restrict__ dgate) {
  const int col = 4 * ((int)blockIdx.y * 256 + (int)threadIdx.x);
  if (col >= H) return;
  float wk[16][4];
#pragma unroll
  for (int k = 0; k < 16; ++k) {
    const f4 w4 = *reinterpret_cast<const f4*>(Wrbf + (int64_t)(k < R ? k : 0) * H + col);
#pragma unroll
    for (int c = 0; c < 4; ++c) wk[k][c] = k < R ? w4[c] : 0.f;
  }
  const int64_t r0 = (int64_t)blockIdx.x * GATE_ROWS;
  const int64_t r1 = r0 + GATE_ROWS < E ? r0 + GATE_ROWS : E;
#pragma unroll 4
  for (int64_t row = r0; row < r1; ++row) {
    const int64_t i = row * H + col;
    const h4 d = *reinterpret_cast<const h4*>(dxg + i), zz = *reinterpret_cast<const h4*>(z + i);
    const float* gr = g + row * R;
    float gt[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      const float gk = k < R ? gr[k] : 0.f;
#pragma unroll
      for (int c = 0; c < 4; ++c) gt[c] += gk * wk[k][c];
    }
    h4 o1, o2;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      // one sigmoid for silu and its derivative
      const float dv = (float)d[c], zv = (float)zz[c], sg = sigmoid_f(zv);
      o1[c] = (__bf16)(dv * gt[c] * (sg * (1.0f + zv * (1.0f - sg))));
      o2[c] = (__bf16)(dv * zv * sg);
    }
    *reinterpret_cast<h4*>(dz + i) = o1;
    *reinterpret_cast<h4*>(dgate + i) = o2;
  }
}

// out = bf16(in), 4 elements per thread
__global__ void to_half_kernel(const float* __restrict__ in, __bf16* __restrict__ out, int64_t n) {
  const int64_t i = 4 * ((int64_t)blockIdx.x * blockDim.x + threadIdx.x);
  if (i >= n) return;
  if (i + 3 < n) {
    const f4 v = *reinterpret_cast<const f4*>(in + i);
    h4 o;
#pragma unroll
    for (int c = 0; c < 4; ++c) o[c] = (__bf16)v[c];
    *reinterpret_cast<h4*>(out + i) = o;
  } else {
    for (int64_t k = i; k < n; ++k) out[k] = (__bf16)in[k];
  }
}

// Several small fp32 -> bf16 conversions in one launch: blockIdx.y names the job, blockIdx.x one 32 x 32
// tile of one of its `batch` consecutive [rows, cols] matrices.  A job writes each matrix transposed
// (batches consecutive again), or as it stands with row stride dst_ld and batch stride dst_batch.
struct half_job {
  const float* src;
  __bf16* dst;
  int rows, cols, batch, transpose, dst_ld, dst_batch;
};
constexpr int HALF_JOBS_MAX = 8;
struct half_jobs {
  half_job j[HALF_JOBS_MAX];
};
__global__ void to_half_jobs_kernel(half_jobs jobs) {
  __shared__ float t[32][33];
  const half_job jb = jobs.j[blockIdx.y];
  const int tc = (jb.cols + 31) / 32, tr = (jb.rows + 31) / 32;
  int tile = blockIdx.x;
  if (tile >= tc * tr * jb.batch) return;   // the whole workgroup
  const int b = tile / (tc * tr);
  tile %= tc * tr;
  const int r0 = (tile / tc) * 32, c0 = (tile % tc) * 32;
  const float* in = jb.src + (int64_t)b * jb.rows * jb.cols;
  if (!jb.transpose) {
    __bf16* out = jb.dst + (int64_t)b * jb.dst_batch;
    for (int i = threadIdx.y; i < 32; i += 8) {
      const int r = r0 + i, c = c0 + threadIdx.x;
      if (r < jb.rows && c < jb.cols) out[(int64_t)r * jb.dst_ld + c] = (__bf16)in[(int64_t)r * jb.cols + c];
    }
    return;
  }
  __bf16* out = jb.dst + (int64_t)b * jb.rows * jb.cols;
  for (int i = threadIdx.y; i < 32; i += 8) {
    const int r = r0 + i, c = c0 + threadIdx.x;
    t[i][threadIdx.x] = (r < jb.rows && c < jb.cols) ? in[(int64_t)r * jb.cols + c] : 0.f;
  }
  __syncthreads();
  for (int i = threadIdx.y; i < 32; i += 8) {
    const int c = c0 + i, r = r0 + threadIdx.x;
    if (c < jb.cols && r < jb.rows) out[(int64_t)c * jb.rows + r] = (__bf16)t[threadIdx.x][i];
  }
}

// Whether the [E, emb]-sized intermediates of a block are stored as bf16: bf16 blocks whose widths
// allow 16-byte rows of bf16.  They are consumed by bf16-operand GEMMs (which would round them
// anyway) or by elementwise activation derivatives.  The buffers keep their fp32 sizes.
bool half_storage(const gp_dims* d) {
  return d->dtype == GP_BF16_F32ACC && d->emb % 8 == 0 && (d->emb_cbf * d->emb_bil) % 8 == 0;
}

// dst[q] (+)= src[perm[q]]
__global__ void permute_add_kernel(const float* __restrict__ src, const int32_t* __restrict__ perm, int64_t n,
                                   int accumulate, float* __restrict__ dst) {
  const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (q >= n) return;
  const float v = src[perm[q]];
  dst[q] = accumulate ? dst[q] + v : v;
}

// The dense per-centre-atom form pays once an edge has enough triplets: measured at 42 triplets per edge
// (configuration 3) the forward pair of kernels wins (0.40 vs 0.52 ms) and the backward kernels lose (0.28 vs
// 0.15 ms); at 333 (configuration 4) both win by far.
constexpr double MFMA_FWD_DENSITY = 32.0, MFMA_BWD_DENSITY = 96.0;
bool want_trip_mfma(const gp_ctx* ctx, const gp_dims* d, const gp_graph* g, double min_density) {
  if (d->dtype != GP_BF16_F32ACC || ctx->trip_mfma == 0 || d->radial_at_target) return false;
  if (ctx->trip_mfma >= 1) return true;
  return g->n_edges > 0 && (double)g->n_triplets >= min_density * (double)g->n_edges;
}

// The same choice for blocks with the radial factor at the target edge, whose triplet sums run on the mirrored views
bool want_rt_mfma(const gp_ctx* ctx, const gp_dims* d, const gp_graph* g, double min_density) {
  if (d->dtype != GP_BF16_F32ACC || ctx->trip_mfma == 0 || !d->radial_at_target) return false;
  if (!g->row_ptr || !g->out_ptr || !g->out_list || g->n_atoms <= 0) return false;
  if (ctx->trip_mfma >= 1) return true;
  return g->n_edges > 0 && (double)g->n_triplets >= min_density * (double)g->n_edges;
}

// The accumulator A[E, C, F] is stored as bf16 when the matrix-core kernel writes it and bf16 storage is on: its
// only readers are two bf16-operand GEMMs.  Forward and backward must agree, so the triplet mode of the
// context must not change between the two calls of a step.
// The gate silu(m W_ba) is multiplied by, (g W_rbfS) W_rbfB, has rank emb_rbf: where the wide GEMM runs in the kernel that
// can evaluate such a factor in its epilogue, the [E, emb] gate matrix is never written or read (forward: a [E, emb_rbf]
// product instead of the [E, emb] one and one epilogue input stream less; backward: one input stream less).  The
// [E, emb_rbf] factor takes the gate's place in the saved buffer.  Forward and backward decide alike from the shapes.
bool lowrank_gate(const gp_ctx* ctx, const gp_dims* d, int64_t E) {
  return half_storage(d) && d->emb % 8 == 0 && d->int_emb % 2 == 0 && d->emb_bil % 2 == 0 && d->emb_rbf <= 16 &&
         gp_gemm_nt_takes_lowrank(ctx, E, d->emb, d->emb);
}

// z [E, emb_bil] is stored as bf16 where both of its GEMM operand roles allow 16-byte pieces
bool z_half(const gp_dims* d) { return half_storage(d) && d->int_emb % 2 == 0 && d->emb_bil % 8 == 0 && d->emb % 8 == 0; }

// bf16 copies of the weights are used when their row lengths allow paired loads
bool weights_half(const gp_dims* d) { return half_storage(d) && d->int_emb % 2 == 0 && d->emb_bil % 2 == 0; }

int to_half(gp_ctx* ctx, const float* in, __bf16* out, int64_t n) {
  gp_prof_scope prof(ctx, "to_half", 0.0, 6.0 * (double)n);
  to_half_kernel<<<(unsigned)((n / 4 + 256) / 256), 256, 0, ctx->stream>>>(in, out, n);
  GP_LAUNCH_CHECK(ctx, "to_half_kernel");
  return GP_OK;
}
// the bf16 copies of a block's weights, gathered and made by one launch
struct half_batch {
  gp_ctx* ctx;
  half_jobs jobs{};
  int n = 0, tiles = 0;
  double elems = 0.0;
  explicit half_batch(gp_ctx* c) : ctx(c) {}
  // dst = src (transpose == false) or its transpose, for each of `batch` consecutive [rows, cols] matrices;
  // dst_ld / dst_batch (elements, plain copies only) default to the dense layout
  const float* add(const float* src, __bf16* dst, int rows, int cols, bool transpose, int batch = 1, int dst_ld = 0,
                   int dst_batch = 0) {
    if (n < HALF_JOBS_MAX && rows > 0 && cols > 0 && batch > 0) {
      jobs.j[n++] = half_job{src, dst, rows, cols, batch, transpose ? 1 : 0, dst_ld ? dst_ld : cols,
                             dst_batch ? dst_batch : rows * cols};
      const int t = ((rows + 31) / 32) * ((cols + 31) / 32) * batch;
      tiles = t > tiles ? t : tiles;
      elems += (double)rows * cols * batch;
    } else if (rows > 0 && cols > 0 && batch > 0)
      n = HALF_JOBS_MAX + 1;   // reported by run()
    return reinterpret_cast<const float*>(dst);
  }
  int run() {
    if (n == 0) return GP_OK;
    GP_REQUIRE(ctx, n <= HALF_JOBS_MAX, "half_batch: more conversions than one launch takes");
    gp_prof_scope prof(ctx, "to_half", 0.0, 6.0 * elems);
    to_half_jobs_kernel<<<dim3((unsigned)tiles, (unsigned)n), dim3(32, 8), 0, ctx->stream>>>(jobs);
    GP_LAUNCH_CHECK(ctx, "to_half_jobs_kernel");
    return GP_OK;
  }
};

bool a_half(const gp_ctx* ctx, const gp_dims* d, const gp_graph* g) {
  if (!half_storage(d) || (d->emb_cbf * d->int_emb) % 8 != 0) return false;
  // radial factor at the target edge: A (and its gradient) is written by a per-edge product, whose 16-byte bf16 stores and
  // loads exist for these widths
  if (d->radial_at_target) return d->emb_cbf <= 16 && (d->int_emb == 32 || d->int_emb == 64 || d->int_emb == 128);
  return want_trip_mfma(ctx, d, g, MFMA_FWD_DENSITY) && gp_tripG_mfma_usable(g, d->int_emb, d->num_spherical, d->emb_cbf);
}

int check_weights_G(gp_ctx* ctx, const gp_dims* d, const gp_weights_G* w, const char* what) {
  GP_REQUIRE(ctx, w, "%s is NULL", what);
  GP_REQUIRE(ctx, !d->symmetric || w->W_up_ac, "%s: W_up_ac is needed by a symmetric block", what);
  GP_REQUIRE(ctx, w->W_ba && w->W_rbfS && w->W_rbfB && w->W_down && w->W_c && w->W_bil && w->W_up && w->W_skip,
             "%s has a NULL member", what);
  return GP_OK;
}

}  // namespace

size_t gp_block_G_saved_bytes(const gp_dims* d, int64_t E) {
  saved_G s;
  return carve_saved_G(nullptr, d, E, &s);
}
size_t gp_block_G_scratch_bytes(const gp_dims* d, int64_t N, int64_t E, int64_t T) {
  scratch_G s;
  return carve_scratch_G(nullptr, d, N, E, T, &s);
}

namespace {

// m_in_h / m_out_h: the block input / output is a bf16 matrix (a stack of bf16 blocks hands its messages over in the
// storage its GEMMs read them in; the values are those the fp32 hand-over would be rounded to)
int forward_G(gp_ctx* ctx, const gp_dims* dims, const gp_weights_G* w, const gp_graph* graph,
              const gp_basis* basis, const float* m_in, int m_in_h, float* m_out, int m_out_h, void* saved, size_t saved_bytes,
              void* scratch, size_t scratch_bytes) {
  if (!ctx) return GP_BAD_ARG;
  GP_TRY(check_dims_G(ctx, dims));
  GP_TRY(check_weights_G(ctx, dims, w, "weights"));
  GP_REQUIRE(ctx, graph && basis, "gp_block_forward_G: graph/basis is NULL");
  const int64_t E = graph->n_edges;
  GP_REQUIRE(ctx, E >= 0 && graph->n_triplets >= 0, "gp_block_forward_G: negative size");
  if (E == 0) return GP_OK;
  GP_REQUIRE(ctx, m_in && m_out && saved && scratch, "gp_block_forward_G: NULL pointer");
  GP_REQUIRE(ctx, basis->rbf && (graph->n_triplets == 0 || basis->cos_alpha), "gp_block_forward_G: basis arrays missing");
  GP_TRY(gp_take_deferred(ctx, "gp_block_forward_G"));
  saved_G s;
  scratch_G sc;
  if (saved_bytes < carve_saved_G(saved, dims, E, &s)) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "gp_block_forward_G: saved buffer too small");
  // a scratch buffer sized without the centre-atom lists (n_atoms = 0 in the query) is accepted: the fused triplet
  // kernel, whose tables depend on the number of atoms, is then not used
  if (scratch_bytes < carve_scratch_G(scratch, dims, graph->n_atoms, E, graph->n_triplets, &sc) &&
      scratch_bytes < carve_scratch_G(scratch, dims, 0, E, graph->n_triplets, &sc))
    return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "gp_block_forward_G: scratch too small");
  GP_HIP(ctx, hipSetDevice(ctx->device));
  gp_bf16_scope gemm_dtype(ctx, dims->dtype == GP_BF16_F32ACC);
  const int H = dims->emb, F = dims->int_emb, C = dims->emb_cbf, O = dims->emb_bil, S = dims->num_spherical,
            R = dims->num_radial, RB = dims->emb_rbf;
  const float* g = basis->rbf;
  gp_epilogue e;

  e = gp_epilogue(); e.out = s.Wrbf;
  GP_TRY(gp_gemm_nn(ctx, w->W_rbfS, w->W_rbfB, R, H, RB, e));                       // W_rbf = W_rbfS W_rbfB
  const bool hs = half_storage(dims);   // gate, z_ba, xg, z_skip, t_skip, z_up live in HBM as bf16
  const bool ah = a_half(ctx, dims, graph);
  ctx->fwd_flags[saved] = ah ? 1u : 0u;   // element type of the accumulator A: the backward call must read it the same way
  if (dims->dtype == GP_BF16_F32ACC && ctx->trip_mfma != 0) GP_TRY(gp_check_degrees(ctx, graph));
  const bool lrg = lowrank_gate(ctx, dims, E);
  if (lrg) {
    e = gp_epilogue(); e.out = s.gate;
    GP_TRY(gp_gemm_nn(ctx, g, w->W_rbfS, E, RB, R, e));                             // g W_rbfS [E, emb_rbf], fp32
  } else {
    e = gp_epilogue(); e.out = s.gate; e.bf16 = hs ? EPI_BF_OUT : 0u;
    GP_TRY(gp_gemm_nn(ctx, g, s.Wrbf, E, H, R, e));                                 // gate
  }
  GP_REQUIRE(ctx, !(m_in_h || m_out_h) || (hs && weights_half(dims)), "gp_block_forward_G_stacked: bf16 messages need a block that stores bf16 (see gp_block_G_stacks_bf16)");
  const float* m_op = m_in;   // the input messages as a GEMM operand
  if (m_in_h) {
    // already rounded; the backward call is handed the same matrix again
  } else if (hs) {
    GP_TRY(to_half(ctx, m_in, s.m_h, (int64_t)E * H));
    m_op = reinterpret_cast<const float*>(s.m_h);
  }
  const bool wh = weights_half(dims);
  int rc = GP_OK;
  // the two H x H weights as transposed bf16 copies: activations times a [N, K] weight is the form the
  // global->LDS GEMM kernel takes
  half_batch wcopy(ctx);   // one launch for all of them
  if (wh) {
    wcopy.add(w->W_ba, sc.W_ba_h, H, H, true);
    wcopy.add(w->W_skip, sc.W_skip_h, H, H, true);
  }
  const float* W_ba_T = reinterpret_cast<const float*>(sc.W_ba_h);
  const float* W_skip_T = reinterpret_cast<const float*>(sc.W_skip_h);
  // the two weights that contract a wide row into a narrow one likewise, where the activations are bf16
  const bool down_T = wh && hs && H % 8 == 0, bil_T = wh && ah;
  const float* W_down = wh ? wcopy.add(w->W_down, sc.W_down_h, H, F, down_T) : w->W_down;   // [F, H] with down_T
  const float* W_bil = bil_T ? wcopy.add(w->W_bil, sc.W_bil_h, C * F, O, true) : w->W_bil;  // [O, (c,f)]
  // and the up-projection(s) as [H, O] where z is bf16
  if (z_half(dims)) {
    wcopy.add(w->W_up, sc.W_up_h, O, H, true);
    if (dims->symmetric) wcopy.add(w->W_up_ac, sc.W_up_ac_h, O, H, true);
  }
  GP_TRY(wcopy.run());
  e = gp_epilogue(); e.save_pre = s.z_ba; e.act = 1; e.out = s.xg;
  if (lrg) e.lr_a = s.gate, e.lr_b = w->W_rbfB, e.lr_k = RB;
  else e.mul = s.gate;
  e.bf16 = hs ? (EPI_BF_SAVE_PRE | EPI_BF_MUL | EPI_BF_OUT) : 0u;
  if (wh) GP_TRY(gp_gemm_nt(ctx, m_op, W_ba_T, E, H, H, e, 1, 1));                  // xg
  else GP_TRY(gp_gemm_nn(ctx, m_op, w->W_ba, E, H, H, e, hs));
  e = gp_epilogue(); e.save_pre = s.z_dn; e.act = 1; e.out = s.x;
  if (down_T) GP_TRY(gp_gemm_nt(ctx, s.xg, W_down, E, F, H, e, 1, 1));              // x
  else GP_TRY(gp_gemm_nn(ctx, s.xg, W_down, E, F, H, e, hs, wh));
  GP_TRY(gp_permute3(ctx, w->W_c, S, R, C, 0, 2, 1, s.WcT));                        // WcT[(l,c), n]
  e = gp_epilogue(); e.out = s.Radt;
  GP_TRY(gp_gemm_nt(ctx, s.WcT, g, S * C, (int)E, R, e));                           // Radt[(l,c), e]
  if (dims->radial_at_target) {
    // A_e = Rad_e^T B1_e,  B1[e,l,f] = sum_{t in seg(e)} Y_l(t) x[kj(t),f]: the radial factor has left the sum
    GP_REQUIRE(ctx, graph->seg_ptr_kj && (graph->n_triplets == 0 || graph->idx_ji_kj), "gp_block_forward_G: kj-major view missing");
    const gp_graph gm = mirrored(graph);
    const gp_graph gml = mirrored_lists(graph, sc.iota);
    if (want_rt_mfma(ctx, dims, graph, MFMA_BWD_DENSITY) && gp_tripG_mfma_H_usable(&gml, F, S)) {
      iota_kernel<<<(unsigned)((E + 255) / 256), 256, 0, ctx->stream>>>(sc.iota, E);
      GP_LAUNCH_CHECK(ctx, "iota_kernel");
      if (ctx->trip_mfma != 2 && gp_tripG_H_fused_usable(&gml, F, S) && sc.ybytes >= gp_tripG_H_fused_scratch(graph->n_atoms, E, F))
        GP_TRY(gp_tripG_backward_H_fused(ctx, &gml, basis->cos_alpha, s.x, F, S, s.B1, sc.ybuf, sc.ybytes, graph->out_list));
      else
        GP_TRY(gp_tripG_backward_H_mfma(ctx, &gml, basis->cos_alpha, s.x, F, S, s.B1, graph->out_list));
    } else
      GP_TRY(gp_tripD_backward(ctx, &gm, basis->cos_alpha, nullptr, nullptr, nullptr, s.x, nullptr, F, S, 1, s.B1, nullptr));
    GP_TRY(gp_tripG_edge_G(ctx, s.Radt, s.B1, E, S, C, F, s.A, ah));
  } else if (want_trip_mfma(ctx, dims, graph, MFMA_FWD_DENSITY) && gp_tripG_mfma_usable(graph, F, S, C)) {
    // one pass with y evaluated in registers where the widths allow and the scratch holds its tables; the two-kernel
    // form with the per-triplet y buffer otherwise, or when asked for (mode 2)
    if (ctx->trip_mfma != 2 && gp_tripG_fused_usable(graph, F, S, C) && sc.ybytes >= gp_tripG_fused_scratch(graph->n_atoms, E, F))
      GP_TRY(gp_tripG_forward_fused(ctx, graph, basis->cos_alpha, s.x, s.Radt, F, S, C, s.A, sc.ybuf, sc.ybytes, ah));
    else
      GP_TRY(gp_tripG_forward_mfma(ctx, graph, basis->cos_alpha, s.x, s.Radt, F, S, C, s.A, sc.ybuf, sc.ybytes, ah));
  }
  else
    GP_TRY(gp_tripD_forward(ctx, graph, basis->cos_alpha, s.x, s.Radt, nullptr, F, S, C, nullptr, s.A));
  // z is an operand of the up-projections and of their weight gradients only: stored as bf16, like every other operand
  // of a bf16 block, it goes from memory to LDS without a conversion (z_half() says when)
  const bool zh = z_half(dims);
  e = gp_epilogue(); e.out = s.z; e.bf16 = zh ? EPI_BF_OUT : 0u;
  if (bil_T) GP_TRY(gp_gemm_nt(ctx, s.A, W_bil, E, O, C * F, e, 1, 1));             // z
  else GP_TRY(gp_gemm_nn(ctx, s.A, W_bil, E, O, C * F, e, ah, 0));
  float* t_skip = sc.eh[0];
  e = gp_epilogue(); e.save_pre = s.z_skip; e.act = 1; e.out = t_skip; e.bf16 = hs ? (EPI_BF_SAVE_PRE | EPI_BF_OUT) : 0u;
  if (wh) GP_TRY(gp_gemm_nt(ctx, m_op, W_skip_T, E, H, H, e, 1, 1));
  else GP_TRY(gp_gemm_nn(ctx, m_op, w->W_skip, E, H, H, e, hs));
  if (dims->symmetric) {
    // m' = (t_skip + (act(z W_up) + act(z W_up_ac)[id_swap]) / sqrt(2)) / sqrt(2) = (act(z W_up) + t) / 2,
    // t = sqrt(2) t_skip + act(z W_up_ac)[id_swap]
    GP_REQUIRE(ctx, graph->id_swap, "gp_block_forward_G: graph->id_swap is needed by a symmetric block");
    float* u_ac = sc.eh[1];
    e = gp_epilogue(); e.save_pre = s.z_ac; e.act = 1; e.out = u_ac; e.bf16 = hs ? (EPI_BF_SAVE_PRE | EPI_BF_OUT) : 0u;
    if (zh) {
      GP_TRY(gp_gemm_nt(ctx, s.z, reinterpret_cast<const float*>(sc.W_up_ac_h), E, H, O, e, 1, 1));
    } else
      GP_TRY(gp_gemm_nn(ctx, s.z, w->W_up_ac, E, H, O, e));
    {
      gp_prof_scope prof(ctx, "ew_sym_mix", 0.0, (hs ? 6.0 : 12.0) * (double)E * H);
      const unsigned blocks = (unsigned)(((int64_t)E * H + 255) / 256), blocks4 = (unsigned)(((int64_t)E * H / 4 + 255) / 256);
      if (hs) sym_mix4_kernel<__bf16><<<blocks4, 256, 0, ctx->stream>>>((__bf16*)t_skip, (const __bf16*)u_ac, graph->id_swap, E, H);
      else if (H % 4 == 0) sym_mix4_kernel<float><<<blocks4, 256, 0, ctx->stream>>>(t_skip, u_ac, graph->id_swap, E, H);
      else sym_mix_kernel<float><<<blocks, 256, 0, ctx->stream>>>(t_skip, u_ac, graph->id_swap, E, H);
      GP_LAUNCH_CHECK(ctx, "sym_mix_kernel");
    }
    e = gp_epilogue(); e.save_pre = s.z_up; e.act = 1; e.add_post = t_skip; e.scale = 0.5f; e.out = m_out;
    e.bf16 = hs ? (EPI_BF_SAVE_PRE | EPI_BF_ADD_POST | (m_out_h ? EPI_BF_OUT : 0u)) : 0u;
    if (zh) {
      GP_TRY(gp_gemm_nt(ctx, s.z, reinterpret_cast<const float*>(sc.W_up_h), E, H, O, e, 1, 1));
    } else
      GP_TRY(gp_gemm_nn(ctx, s.z, w->W_up, E, H, O, e));
    return GP_OK;
  }
  e = gp_epilogue(); e.save_pre = s.z_up; e.act = 1; e.add_post = t_skip; e.scale = INV_SQRT2; e.out = m_out;
  e.bf16 = hs ? (EPI_BF_SAVE_PRE | EPI_BF_ADD_POST | (m_out_h ? EPI_BF_OUT : 0u)) : 0u;
  if (zh) {
    GP_TRY(gp_gemm_nt(ctx, s.z, reinterpret_cast<const float*>(sc.W_up_h), E, H, O, e, 1, 1));
  } else
    GP_TRY(gp_gemm_nn(ctx, s.z, w->W_up, E, H, O, e));
  return GP_OK;
}

// m_in_h as in forward_G; gmo_h / gmi_h: the gradient coming in / going out is a bf16 matrix
int backward_G(gp_ctx* ctx, const gp_dims* dims, const gp_weights_G* w, const gp_graph* graph,
               const gp_basis* basis, const float* m_in, int m_in_h, const void* saved, size_t saved_bytes,
               const float* grad_m_out, int gmo_h, float* grad_m_in, int gmi_h, gp_weights_G* gw, float* grad_rbf,
               float* grad_cos_kj, int32_t accumulate_basis_grads, void* scratch, size_t scratch_bytes) {
  if (!ctx) return GP_BAD_ARG;
  GP_TRY(check_dims_G(ctx, dims));
  GP_TRY(check_weights_G(ctx, dims, w, "weights"));
  GP_TRY(check_weights_G(ctx, dims, gw, "grad_w"));
  GP_REQUIRE(ctx, graph && basis, "gp_block_backward_G: graph/basis is NULL");
  const int64_t E = graph->n_edges;
  GP_REQUIRE(ctx, E > 0 && graph->n_triplets >= 0, "gp_block_backward_G: empty edge list");
  GP_REQUIRE(ctx, m_in && grad_m_out && grad_m_in && saved && scratch, "gp_block_backward_G: NULL pointer");
  GP_REQUIRE(ctx, basis->rbf && (graph->n_triplets == 0 || basis->cos_alpha_kj), "gp_block_backward_G: basis arrays missing");
  GP_TRY(gp_take_deferred(ctx, "gp_block_backward_G"));
  saved_G s;
  scratch_G sc;
  if (saved_bytes < carve_saved_G(const_cast<void*>(saved), dims, E, &s)) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "gp_block_backward_G: saved buffer too small");
  if (scratch_bytes < carve_scratch_G(scratch, dims, graph->n_atoms, E, graph->n_triplets, &sc) &&
      scratch_bytes < carve_scratch_G(scratch, dims, 0, E, graph->n_triplets, &sc))
    return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "gp_block_backward_G: scratch too small");
  GP_HIP(ctx, hipSetDevice(ctx->device));
  gp_bf16_scope gemm_dtype(ctx, dims->dtype == GP_BF16_F32ACC);
  const int H = dims->emb, F = dims->int_emb, C = dims->emb_cbf, O = dims->emb_bil, S = dims->num_spherical,
            R = dims->num_radial, RB = dims->emb_rbf;
  const int64_t EH = E * H;
  const float* g = basis->rbf;
  const bool hs = half_storage(dims);   // saved z_ba, gate, xg, z_skip, z_up and the four buffers below are bf16
  float *d_up = sc.eh[0], *d_skip = sc.eh[1], *dxg = sc.eh[2], *dgate = sc.eh[3];
  gp_epilogue e;

  const bool wh = weights_half(dims);
  GP_REQUIRE(ctx, !(m_in_h || gmo_h || gmi_h) || (hs && wh), "gp_block_backward_G_stacked: bf16 messages need a block that stores bf16 (see gp_block_G_stacks_bf16)");
  GP_REQUIRE(ctx, !gmo_h || !dims->symmetric, "gp_block_backward_G_stacked: a symmetric block takes its incoming gradient as fp32");
  int rc = GP_OK;
  // the bf16 copies of the weights this pass multiplies by, one launch
  const bool dzdn_half = !dims->radial_at_target && hs && wh && F % 8 == 0;   // dz_dn stored as bf16 (below)
  const float *W_up = w->W_up, *W_skip = w->W_skip, *W_ba = w->W_ba, *W_up_ac = w->W_up_ac, *W_down = w->W_down;
  const float* WbilP = sc.WbilP;
  if (wh) {
    half_batch wcopy(ctx);
    W_up = wcopy.add(w->W_up, sc.W_up_h, O, H, false);
    W_skip = wcopy.add(w->W_skip, sc.W_skip_h, H, H, false);
    W_ba = wcopy.add(w->W_ba, sc.W_ba_h, H, H, false);
    if (dims->symmetric) W_up_ac = wcopy.add(w->W_up_ac, sc.W_up_ac_h, O, H, false);
    if (dzdn_half) W_down = wcopy.add(w->W_down, sc.W_down_h, H, F, false);
    // W_bil [c, f, o] as [(c,o), f]: C transposes
    if (!dims->radial_at_target) {
      WbilP = wcopy.add(w->W_bil, sc.WbilP_h, F, O, true, C);
      // and as [f, (c,o)]: matrix c lands at column c O of rows C O long
      if (dzdn_half && (C * O) % 8 == 0) wcopy.add(w->W_bil, sc.WbilV_h, F, O, false, C, C * O, O);
    } else if ((C * O) % 8 == 0)
      wcopy.add(w->W_bil, sc.WbilV_h, F, O, false, C, C * O, O);   // read where G' is bf16
    GP_TRY(wcopy.run());
  }
  gp_aux aux(ctx);   // the large weight-gradient GEMMs run on the side stream
  if (dims->symmetric) {
    GP_REQUIRE(ctx, graph->id_swap, "gp_block_backward_G: graph->id_swap is needed by a symmetric block");
    float* d_ac = sc.eh5;
    {
      gp_prof_scope prof(ctx, "ew_sym_bwd", 0.0, (hs ? 20.0 : 32.0) * (double)EH);
      const unsigned blocks = (unsigned)((EH + 255) / 256), blocks4 = (unsigned)((EH / 4 + 255) / 256);
      const bool vec4 = H % 4 == 0 && ((uintptr_t)grad_m_out & 15) == 0;   // the library's own buffers are 256-byte aligned
      if (hs && !vec4)
        sym_bwd_kernel<__bf16><<<blocks, 256, 0, ctx->stream>>>(grad_m_out, (const __bf16*)s.z_up, (const __bf16*)s.z_skip,
                                                               (const __bf16*)s.z_ac, graph->id_swap, E, H, (__bf16*)d_up,
                                                               (__bf16*)d_skip, (__bf16*)d_ac);
      else if (hs)
        sym_bwd4_kernel<__bf16><<<blocks4, 256, 0, ctx->stream>>>(grad_m_out, (const __bf16*)s.z_up, (const __bf16*)s.z_skip,
                                                                 (const __bf16*)s.z_ac, graph->id_swap, E, H, (__bf16*)d_up,
                                                                 (__bf16*)d_skip, (__bf16*)d_ac);
      else if (vec4)
        sym_bwd4_kernel<float><<<blocks4, 256, 0, ctx->stream>>>(grad_m_out, s.z_up, s.z_skip, s.z_ac, graph->id_swap, E, H, d_up,
                                                                d_skip, d_ac);
      else
        sym_bwd_kernel<float><<<blocks, 256, 0, ctx->stream>>>(grad_m_out, s.z_up, s.z_skip, s.z_ac, graph->id_swap, E, H, d_up,
                                                              d_skip, d_ac);
      GP_LAUNCH_CHECK(ctx, "sym_bwd_kernel");
    }
    GP_TRY(gp_gemm_tn(ctx, s.z, d_ac, E, O, H, gw->W_up_ac, nullptr, sc.part, sc.part_bytes, z_half(dims), hs));
    e = gp_epilogue(); e.out = sc.dz;
    GP_TRY(gp_gemm_nt(ctx, d_ac, W_up_ac, E, O, H, e, hs, wh));                     // dz (opposite-edge path)
  } else if (hs) {
    gp_prof_scope prof(ctx, "ew_dsilu2_half", 0.0, (gmo_h ? 10.0 : 12.0) * (double)EH);   // the gradient + 4 bf16 arrays
    if (gmo_h)
      dsilu2_half_kernel<__bf16><<<(unsigned)((EH / 4 + 256) / 256), 256, 0, ctx->stream>>>(
          reinterpret_cast<const __bf16*>(grad_m_out), INV_SQRT2, (const __bf16*)s.z_up, (const __bf16*)s.z_skip, (__bf16*)d_up, (__bf16*)d_skip, EH);
    else
      dsilu2_half_kernel<float><<<(unsigned)((EH / 4 + 256) / 256), 256, 0, ctx->stream>>>(
          grad_m_out, INV_SQRT2, (const __bf16*)s.z_up, (const __bf16*)s.z_skip, (__bf16*)d_up, (__bf16*)d_skip, EH);
    GP_LAUNCH_CHECK(ctx, "dsilu2_half_kernel");
  } else {
    GP_TRY(gp_ew_dsilu2(ctx, grad_m_out, INV_SQRT2, s.z_up, s.z_skip, d_up, d_skip, EH));
  }
  GP_TRY(aux.on_aux([&] { return gp_gemm_tn(ctx, s.z, d_up, E, O, H, gw->W_up, nullptr, sc.part_aux, sc.part_bytes, z_half(dims), hs); }, {d_up}));
  e = gp_epilogue(); e.out = sc.dz;
  if (dims->symmetric) e.add_post = sc.dz;
  GP_TRY(gp_gemm_nt(ctx, d_up, W_up, E, O, H, e, hs, wh));                          // dz
  const float* m_op = m_in_h ? m_in : hs ? reinterpret_cast<const float*>(s.m_h) : m_in;   // rounded copy written by the forward pass
  GP_TRY(aux.on_aux([&] { return gp_gemm_tn(ctx, m_op, d_skip, E, H, H, gw->W_skip, nullptr, sc.part_aux, sc.part_bytes, hs, hs); }, {}));
  // dm = d_skip W_skip^T + dz_ba W_ba^T.  With bf16 storage both products run as ONE GEMM at the end of the call (its
  // contraction walks both operand pairs), so dm is written once instead of written, read back and written again
  // (configuration 4: 0.79 + 1.19 ms -> 1.22 ms); d_skip stays untouched until then.
  const bool dm_fused = hs && wh;
  if (!dm_fused) {
    e = gp_epilogue(); e.out = grad_m_in;
    GP_TRY(gp_gemm_nt(ctx, d_skip, W_skip, E, H, H, e, hs, wh));                    // dm (skip path)
  }
  const bool ah = a_half(ctx, dims, graph);
  {
    const auto it = ctx->fwd_flags.find(saved);
    if (it != ctx->fwd_flags.end() && (it->second != 0u) != ah)
      return gp_fail(ctx, GP_BAD_ARG, "gp_block_backward_G: the forward call of this `saved` buffer stored the triplet accumulator as %s; "
                     "gp_set_triplet_mfma must not change between forward and backward", it->second ? "bf16" : "fp32");
  }
  GP_TRY(aux.on_aux([&] { return gp_gemm_tn(ctx, s.A, sc.dz, E, C * F, O, gw->W_bil, nullptr, sc.part_aux, sc.part_bytes, ah, 0); }, {}));
  if (dims->radial_at_target) {
    // mirror image of the source-edge form: G[e',c,o] = sum_{t: kj(t)=e'} y'_t[c] dz[ji(t),o] with
    // y'_t[c] = sum_l Y_l(t) Rad[ji(t),l,c] is the forward kernel on the mirrored views
    const gp_graph gm = mirrored(graph);
    const gp_graph gml = mirrored_lists(graph, sc.iota);
    bool gh = false;
    if (want_rt_mfma(ctx, dims, graph, MFMA_FWD_DENSITY) && gp_tripG_mfma_usable(&gml, O, S, C)) {
      iota_kernel<<<(unsigned)((E + 255) / 256), 256, 0, ctx->stream>>>(sc.iota, E);
      GP_LAUNCH_CHECK(ctx, "iota_kernel");
      // the radial table in out-list order, so that the threads of the y kernel read neighbouring columns
      gather_cols_kernel<<<dim3((unsigned)((E + 255) / 256), (unsigned)(S * C)), 256, 0, ctx->stream>>>(s.Radt, graph->out_list, E, sc.Radt_out);
      GP_LAUNCH_CHECK(ctx, "gather_cols_kernel");
      // G' is read by the next GEMM only: bf16 from the matrix-core kernels where that GEMM takes bf16 operands
      gh = hs && wh && (C * O) % 8 == 0;
      if (ctx->trip_mfma != 2 && gp_tripG_fused_usable(&gml, O, S, C) && sc.ybytes >= gp_tripG_fused_scratch(graph->n_atoms, E, O))
        GP_TRY(gp_tripG_forward_fused(ctx, &gml, basis->cos_alpha_kj, sc.dz, sc.Radt_out, O, S, C, sc.Gm, sc.ybuf, sc.ybytes, gh,
                                      graph->out_list));
      else
        GP_TRY(gp_tripG_forward_mfma(ctx, &gml, basis->cos_alpha_kj, sc.dz, sc.Radt_out, O, S, C, sc.Gm, sc.ybuf, sc.ybytes, gh,
                                     graph->out_list, 1));
    } else
      GP_TRY(gp_tripD_forward(ctx, &gm, basis->cos_alpha_kj, sc.dz, s.Radt, nullptr, O, S, C, nullptr, sc.Gm));
    e = gp_epilogue(); e.act = 2; e.zsrc = s.z_dn; e.out = sc.dzdn;
    if (gh) {
      GP_TRY(gp_gemm_nt(ctx, sc.Gm, reinterpret_cast<const float*>(sc.WbilV_h), E, F, C * O, e, 1, 1));   // dz_dn ([f, (c,o)] copy)
    } else {
      GP_TRY(gp_permute3(ctx, w->W_bil, C, F, O, 0, 2, 1, sc.WbilP));               // [(c,o), f]
      GP_TRY(gp_gemm_nn(ctx, sc.Gm, sc.WbilP, E, F, C * O, e));                     // dz_dn
    }
    GP_TRY(gp_permute3(ctx, w->W_bil, C, F, O, 2, 0, 1, sc.WbilV));                 // [o, (c,f)]
    e = gp_epilogue(); e.out = sc.dA; e.bf16 = ah ? EPI_BF_OUT : 0u;   // read by the per-edge products below only
    GP_TRY(gp_gemm_nn(ctx, sc.dz, sc.WbilV, E, C * F, O, e));                       // dA[e, (c,f)]
    GP_TRY(gp_tripG_edge_dRad(ctx, sc.dA, s.B1, E, S, C, F, sc.dRad, ah));          // dRad[e, (l,c)]
    if (grad_cos_kj && graph->n_triplets > 0) {
      GP_REQUIRE(ctx, graph->perm_kj, "gp_block_backward_G: graph->perm_kj is needed for grad_cos_kj with radial_at_target");
      GP_TRY(gp_tripG_edge_U(ctx, s.Radt, sc.dA, E, S, C, F, sc.dB1, ah));          // dB1[e,l,f]
      GP_TRY(gp_tripG_grad_cos(ctx, &gm, basis->cos_alpha, sc.dB1, s.x, F, S, 0, sc.gc_ji));   // ji-major order
      permute_add_kernel<<<(unsigned)((graph->n_triplets + 255) / 256), 256, 0, ctx->stream>>>(
          sc.gc_ji, graph->perm_kj, graph->n_triplets, accumulate_basis_grads, grad_cos_kj);
      GP_LAUNCH_CHECK(ctx, "permute_add_kernel");
    }
  } else {
  // one pass over the triplets (kj-major): H[e', l, o]
  const bool bwd_mfma = want_trip_mfma(ctx, dims, graph, MFMA_BWD_DENSITY) && gp_tripG_mfma_bwd_usable(graph, O, S);
  // H is read by the two per-edge products only: bf16 from the one-pass kernel where they take it so
  bool hh = false;
  if (bwd_mfma && ctx->trip_mfma != 2 && gp_tripG_H_fused_usable(graph, O, S) &&
      sc.ybytes >= gp_tripG_H_fused_scratch(graph->n_atoms, E, O)) {
    hh = hs && gp_tripG_edge_takes_half_H(C, O);
    GP_TRY(gp_tripG_backward_H_fused(ctx, graph, basis->cos_alpha_kj, sc.dz, O, S, sc.Hd, sc.ybuf, sc.ybytes, nullptr, hh));
  }
  else if (bwd_mfma)
    GP_TRY(gp_tripG_backward_H_mfma(ctx, graph, basis->cos_alpha_kj, sc.dz, O, S, sc.Hd));
  else
    GP_TRY(gp_tripD_backward(ctx, graph, basis->cos_alpha_kj, nullptr, nullptr, nullptr, sc.dz, nullptr, O, S, 1,
                             sc.Hd, nullptr));
  GP_TRY(gp_tripG_edge_G(ctx, s.Radt, sc.Hd, E, S, C, O, sc.Gm, hs, hh));           // G[e', (c,o)] (bf16 with hs)
  if (!wh) GP_TRY(gp_permute3(ctx, w->W_bil, C, F, O, 0, 2, 1, sc.WbilP));          // [(c,o), f]; the bf16 copy was made above
  // dz_dn is an operand of two GEMMs only: bf16 with bf16 storage and weights
  const bool dh = hs && wh && F % 8 == 0;
  e = gp_epilogue(); e.act = 2; e.zsrc = s.z_dn; e.out = sc.dzdn; e.bf16 = dh ? EPI_BF_OUT : 0u;
  if (dh && (C * O) % 8 == 0) {
    GP_TRY(gp_gemm_nt(ctx, sc.Gm, reinterpret_cast<const float*>(sc.WbilV_h), E, F, C * O, e, 1, 1));   // dz_dn ([f, (c,o)] copy)
  } else
    GP_TRY(gp_gemm_nn(ctx, sc.Gm, WbilP, E, F, C * O, e, hs, wh));                  // dz_dn
  // V is read by the two per-edge kernels below only: bf16 storage halves its traffic
  const bool vh = hs && (O == 32 || O == 64 || O == 128);
  e = gp_epilogue(); e.out = sc.V; e.bf16 = vh ? EPI_BF_OUT : 0u;
  if (dh) {
    // x times the [(c,o), f] copy of W_bil, both bf16 and k-contiguous: the form the global->LDS kernel takes
    GP_TRY(to_half(ctx, s.x, sc.x_h, (int64_t)E * F));
    GP_TRY(gp_gemm_nt(ctx, reinterpret_cast<const float*>(sc.x_h), WbilP, E, C * O, F, e, 1, 1));   // V[e', (c,o)]
  } else {
    GP_TRY(gp_permute3(ctx, w->W_bil, C, F, O, 1, 0, 2, sc.WbilV));                 // [f, (c,o)]
    GP_TRY(gp_gemm_nn(ctx, s.x, sc.WbilV, E, C * O, F, e));                         // V[e', (c,o)]
  }
  GP_TRY(gp_tripG_edge_dRad(ctx, sc.V, sc.Hd, E, S, C, O, sc.dRad, vh, hh));        // dRad[e', (l,c)]
  if (grad_cos_kj && graph->n_triplets > 0) {
    const bool dcos_fused = bwd_mfma && ctx->trip_mfma != 2 && gp_tripG_H_fused_usable(graph, O, S) &&
                            sc.ybytes >= gp_tripG_dcos_fused_scratch(graph->n_atoms, E, O, 0);
    GP_TRY(gp_tripG_edge_U(ctx, s.Radt, sc.V, E, S, C, O, sc.U, vh, dcos_fused));
    if (dcos_fused)
      GP_TRY(gp_tripG_grad_cos_fused(ctx, graph, basis->cos_alpha_kj, sc.U, 1, sc.dz, O, S, accumulate_basis_grads, grad_cos_kj,
                                     sc.ybuf, sc.ybytes));
    else if (bwd_mfma)
      GP_TRY(gp_tripG_grad_cos_mfma(ctx, graph, basis->cos_alpha_kj, sc.U, sc.dz, O, S, accumulate_basis_grads, grad_cos_kj));
    else
      GP_TRY(gp_tripG_grad_cos(ctx, graph, basis->cos_alpha_kj, sc.U, sc.dz, O, S, accumulate_basis_grads, grad_cos_kj));
  }
  }
  GP_TRY(gp_gemm_tn(ctx, g, sc.dRad, E, R, S * C, sc.dWcP, nullptr, sc.part, sc.part_bytes));   // [n, (l,c)]
  GP_TRY(gp_permute3(ctx, sc.dWcP, R, S, C, 1, 0, 2, gw->W_c));                     // -> [l, n, c]
  GP_TRY(aux.on_aux([&] { return gp_gemm_tn(ctx, s.xg, sc.dzdn, E, H, F, gw->W_down, nullptr, sc.part_aux, sc.part_bytes, hs, dzdn_half); }, {}));
  e = gp_epilogue(); e.out = dxg; e.bf16 = hs ? EPI_BF_OUT : 0u;
  if (dzdn_half) {
    GP_TRY(gp_gemm_nt(ctx, sc.dzdn, W_down, E, H, F, e, 1, 1));                     // dxg
  } else
    GP_TRY(gp_gemm_nt(ctx, sc.dzdn, w->W_down, E, H, F, e));                        // dxg
  float* dz_ba = d_up;   // d_up is no longer needed on this stream
  GP_TRY(aux.before_write(d_up));
  if (lowrank_gate(ctx, dims, E)) {
    gp_prof_scope prof(ctx, "ew_gate_bwd_lr", 2.0 * RB * (double)EH, 8.0 * (double)EH + 4.0 * RB * (double)E);   // 4 bf16 arrays
    gate_bwd_lr_kernel<<<dim3((unsigned)((E + GATE_ROWS - 1) / GATE_ROWS), (unsigned)((H + 1023) / 1024)), 256, 0, ctx->stream>>>(
        (const __bf16*)dxg, (const __bf16*)s.z_ba, s.gate, w->W_rbfB, E, H, RB, (__bf16*)dz_ba, (__bf16*)dgate);
    GP_LAUNCH_CHECK(ctx, "gate_bwd_lr_kernel");
  } else if (hs) {
    gp_prof_scope prof(ctx, "ew_gate_bwd_half", 0.0, 10.0 * (double)EH);   // 5 bf16 arrays
    gate_bwd_half_kernel<<<(unsigned)((EH / 4 + 256) / 256), 256, 0, ctx->stream>>>(
        (const __bf16*)dxg, (const __bf16*)s.z_ba, (const __bf16*)s.gate, (__bf16*)dz_ba, (__bf16*)dgate, EH);
    GP_LAUNCH_CHECK(ctx, "gate_bwd_half_kernel");
  } else {
    GP_TRY(gp_ew_gate_bwd(ctx, dxg, s.z_ba, s.gate, dz_ba, dgate, EH));
  }
  // Gradients of the gate's weights.  The gate is (g W_rbfS) W_rbfB, so with f = g W_rbfS stored (low-rank form) everything
  // follows from the narrow products df = dgate W_rbfB^T [E, emb_rbf] and f^T dgate, which read dgate once each, and the
  // gradient of the radial basis is df W_rbfS^T instead of a second full-width product dgate W_rbf^T; the general form goes
  // through the [R, emb] matrix g^T dgate (one full-width product: less traffic when the basis gradient is not asked for,
  // configuration 4: 0.31 vs 0.36 ms; with it 0.55 vs 0.40 ms).
  const bool lrg_b = lowrank_gate(ctx, dims, E) && grad_rbf != nullptr;
  if (lrg_b) {
    e = gp_epilogue(); e.out = sc.df;
    GP_TRY(gp_gemm_nt(ctx, dgate, w->W_rbfB, E, RB, H, e, hs, 0));                                          // df
    GP_TRY(gp_gemm_tn(ctx, s.gate, dgate, E, RB, H, gw->W_rbfB, nullptr, sc.part, sc.part_bytes, 0, hs));   // f^T dgate
    GP_TRY(gp_gemm_tn(ctx, g, sc.df, E, R, RB, gw->W_rbfS, nullptr, sc.part, sc.part_bytes));               // g^T df
  } else {
    GP_TRY(gp_gemm_tn(ctx, g, dgate, E, R, H, sc.dWrbf, nullptr, sc.part, sc.part_bytes, 0, hs));
    e = gp_epilogue(); e.out = gw->W_rbfS;
    GP_TRY(gp_gemm_nt(ctx, sc.dWrbf, w->W_rbfB, R, RB, H, e));
    GP_TRY(gp_gemm_tn(ctx, w->W_rbfS, sc.dWrbf, R, RB, H, gw->W_rbfB, nullptr, sc.part, sc.part_bytes));
  }
  GP_TRY(aux.on_aux([&] { return gp_gemm_tn(ctx, m_op, dz_ba, E, H, H, gw->W_ba, nullptr, sc.part_aux, sc.part_bytes, hs, hs); }, {}));
  if (dm_fused) {
    GP_TRY(gp_gemm_nt2(ctx, d_skip, W_skip, dz_ba, W_ba, E, H, H, grad_m_in, 1, 1, gmi_h));  // dm, both paths
  } else {
    e = gp_epilogue(); e.add_post = grad_m_in; e.out = grad_m_in;
    GP_TRY(gp_gemm_nt(ctx, dz_ba, W_ba, E, H, H, e, hs, wh));                       // dm += ba path
  }
  if (grad_rbf) {
    // dL/dg = dgate W_rbf^T + dRad . W_c  (both paths through the Gaussian basis)
    e = gp_epilogue(); e.out = grad_rbf;
    if (accumulate_basis_grads) e.add_post = grad_rbf;
    if (lrg_b) GP_TRY(gp_gemm_nt(ctx, sc.df, w->W_rbfS, E, R, RB, e));   // dgate W_rbf^T = df W_rbfS^T
    else GP_TRY(gp_gemm_nt(ctx, dgate, s.Wrbf, E, R, H, e, hs));
    e = gp_epilogue(); e.add_post = grad_rbf; e.out = grad_rbf;
    GP_TRY(gp_gemm_nn(ctx, sc.dRad, s.WcT, E, R, S * C, e));
  }
  return aux.join();
}

}  // namespace

extern "C" {

int gp_block_forward_G(gp_ctx* ctx, const gp_dims* dims, const gp_weights_G* w, const gp_graph* graph,
                       const gp_basis* basis, const float* m_in, float* m_out, void* saved, size_t saved_bytes,
                       void* scratch, size_t scratch_bytes) {
  return forward_G(ctx, dims, w, graph, basis, m_in, 0, m_out, 0, saved, saved_bytes, scratch, scratch_bytes);
}

int gp_block_backward_G(gp_ctx* ctx, const gp_dims* dims, const gp_weights_G* w, const gp_graph* graph,
                        const gp_basis* basis, const float* m_in, const void* saved, size_t saved_bytes,
                        const float* grad_m_out, float* grad_m_in, gp_weights_G* gw, float* grad_rbf,
                        float* grad_cos_kj, int32_t accumulate_basis_grads, void* scratch, size_t scratch_bytes) {
  return backward_G(ctx, dims, w, graph, basis, m_in, 0, saved, saved_bytes, grad_m_out, 0, grad_m_in, 0, gw, grad_rbf, grad_cos_kj,
                    accumulate_basis_grads, scratch, scratch_bytes);
}

int gp_block_G_stacks_bf16(const gp_dims* dims) {
  return dims && dims->variant == GP_VARIANT_G && half_storage(dims) && weights_half(dims) ? 1 : 0;
}

int gp_block_forward_G_stacked(gp_ctx* ctx, const gp_dims* dims, const gp_weights_G* w, const gp_graph* graph,
                               const gp_basis* basis, const void* m_in, int32_t m_in_bf16, void* m_out, int32_t m_out_bf16,
                               void* saved, size_t saved_bytes, void* scratch, size_t scratch_bytes) {
  return forward_G(ctx, dims, w, graph, basis, static_cast<const float*>(m_in), m_in_bf16 != 0, static_cast<float*>(m_out),
                   m_out_bf16 != 0, saved, saved_bytes, scratch, scratch_bytes);
}

int gp_block_backward_G_stacked(gp_ctx* ctx, const gp_dims* dims, const gp_weights_G* w, const gp_graph* graph,
                                const gp_basis* basis, const void* m_in, int32_t m_in_bf16, const void* saved, size_t saved_bytes,
                                const void* grad_m_out, int32_t grad_m_out_bf16, void* grad_m_in, int32_t grad_m_in_bf16,
                                gp_weights_G* gw, float* grad_rbf, float* grad_cos_kj, int32_t accumulate_basis_grads,
                                void* scratch, size_t scratch_bytes) {
  return backward_G(ctx, dims, w, graph, basis, static_cast<const float*>(m_in), m_in_bf16 != 0, saved, saved_bytes,
                    static_cast<const float*>(grad_m_out), grad_m_out_bf16 != 0, static_cast<float*>(grad_m_in), grad_m_in_bf16 != 0,
                    gw, grad_rbf, grad_cos_kj, accumulate_basis_grads, scratch, scratch_bytes);
}

}  // extern "C"