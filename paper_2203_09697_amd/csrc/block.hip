// Interaction block, variant D (paper Sec. 3.3): the EdgeUpdate MLPs around
// TripletUpdate/TripletAggr, forward and hand-derived backward.  Pure launch sequencing on the
// context's stream; every arithmetic step runs in the kernels of gemm.hip / triplet.hip.
//
//   x_ji = act(m W_ji + b_ji)
//   x_kj = act(m W_kj + b_kj) * (rbf (W_rbf1 W_rbf2));  x_kj = act(x_kj W_down)
//   a_e  = sum_{t in seg(e)} x_kj[kj(t)] * ((sbf_t W_sbf1) W_sbf2)
//   h    = x_ji + act(a W_up);  residual layers;  h = act(h W_lin + b_lin) + m;  residual layers
#include <stdarg.h>

#include <algorithm>

#include "aux_stream.h"
#include "gemm.h"
#include "triplet.h"

namespace {

struct res_saved {
  float *z1, *y1, *z2, *hout;
};

struct saved_D {
  float *z_ji, *z_kj, *gate, *xg, *z_dn, *x_kj, *Q, *Bacc, *a, *z_up, *h0, *z_lin, *h_lin, *Wrbf;
  res_saved before[GP_MAX_RES], after[GP_MAX_RES];
};

size_t carve_saved_D(void* p, const gp_dims* d, int64_t E, saved_D* s) {
  gp_carver c(p);
  const size_t H = d->emb, F = d->int_emb, B = d->basis_emb, S = d->num_spherical, R = d->num_radial;
  s->z_ji = c.take<float>(E * H);
  s->z_kj = c.take<float>(E * H);
  s->gate = c.take<float>(E * H);
  s->xg = c.take<float>(E * H);
  s->z_dn = c.take<float>(E * F);
  s->x_kj = c.take<float>(E * F);
  s->Q = c.take<float>(E * S * B);
  s->Bacc = c.take<float>(E * B * F);
  s->a = c.take<float>(E * F);
  s->z_up = c.take<float>(E * H);
  s->h0 = c.take<float>(E * H);
  s->z_lin = c.take<float>(E * H);
  s->h_lin = c.take<float>(E * H);
  s->Wrbf = c.take<float>(R * H);
  for (int r = 0; r < d->n_res_before; ++r) {
    s->before[r].z1 = c.take<float>(E * H);
    s->before[r].y1 = c.take<float>(E * H);
    s->before[r].z2 = c.take<float>(E * H);
    s->before[r].hout = c.take<float>(E * H);
  }
  for (int r = 0; r < d->n_res_after; ++r) {
    s->after[r].z1 = c.take<float>(E * H);
    s->after[r].y1 = c.take<float>(E * H);
    s->after[r].z2 = c.take<float>(E * H);
    s->after[r].hout = c.take<float>(E * H);   // the last one is unused: the block output goes to m_out
  }
  return c.off;
}

struct scratch_D {
  float* buf[7];     // [E,H] each
  float *dF1, *dF2;  // [E,F]
  float* dQ;         // [E,S*B]
  float* P;          // [E,S,F]: per-edge factor of the gradient with respect to cos(alpha) (basis gradients only)
  float* dWrbf;      // [R,H]
  float* part;
  float* part_aux;   // split-K partials of the GEMMs issued on the side stream
  size_t part_bytes;
};

size_t part_bytes_D(const gp_dims* d, int64_t E) {
  const int H = d->emb, F = d->int_emb, B = d->basis_emb, S = d->num_spherical, R = d->num_radial;
  size_t m = gp_gemm_tn_scratch(E, H, H);
  m = std::max(m, gp_gemm_tn_scratch(E, F, H));
  m = std::max(m, gp_gemm_tn_scratch(E, H, F));
  m = std::max(m, gp_gemm_tn_scratch(E, R, H));
  m = std::max(m, gp_gemm_tn_scratch(R, B, H));
  m = std::max(m, gp_colsum_scratch(E, H));
  m = std::max(m, gp_tripD_wgrad_scratch(E, F, S, R, B));
  return m;
}

// The matrix-core backward kernel also yields the gradient of W_sbf2, so the forward pass need not keep Bacc
// (E x basis_emb x int_emb floats).  Forward and backward must take the same decision: it depends only on the
// context's switch, the widths and the graph.
bool bwd_mfma_D(const gp_ctx* ctx, const gp_dims* d, const gp_graph* g) {
  if (ctx->trip_mfma == 0) return false;
  const int F = d->int_emb, S = d->num_spherical, B = d->basis_emb;
  return gp_tripD_mfma_usable(g, F, S, B) && gp_tripD_mfma_bwd_usable(g, F, S, B) &&
         gp_tripD_mfma_bwd_scratch(g, F) <= part_bytes_D(d, g->n_edges);
}

size_t carve_scratch_D(void* p, const gp_dims* d, int64_t E, scratch_D* s) {
  gp_carver c(p);
  const size_t H = d->emb, F = d->int_emb, B = d->basis_emb, S = d->num_spherical, R = d->num_radial;
  for (int i = 0; i < 7; ++i) s->buf[i] = c.take<float>(E * H);
  s->dF1 = c.take<float>(E * F);
  s->dF2 = c.take<float>(E * F);
  s->dQ = c.take<float>(E * S * B);
  s->P = c.take<float>(E * S * F);
  s->dWrbf = c.take<float>(R * H);
  s->part_bytes = part_bytes_D(d, E);
  s->part = (float*)c.take<char>(s->part_bytes);
  s->part_aux = (float*)c.take<char>(s->part_bytes);
  return c.off;
}

int check_dims_D(gp_ctx* ctx, const gp_dims* d) {
  GP_REQUIRE(ctx, d, "dims is NULL");
  if (d->variant != GP_VARIANT_D) return gp_fail(ctx, GP_UNSUPPORTED_DIMS, "variant %d is not the Hadamard block", d->variant);
  if (d->dtype != GP_F32) return gp_fail(ctx, GP_UNSUPPORTED_DIMS, "variant D is implemented in fp32 only");
  if (d->emb < 1 || d->emb > 4096 || d->int_emb < 1 || d->int_emb > 256 || d->basis_emb < 1 || d->basis_emb > 16 ||
      d->num_spherical < 1 || d->num_spherical > 8 || d->num_radial < 1 || d->num_radial > 16 ||
      d->n_res_before < 0 || d->n_res_before > GP_MAX_RES || d->n_res_after < 0 || d->n_res_after > GP_MAX_RES)
    return gp_fail(ctx, GP_UNSUPPORTED_DIMS,
                   "variant D supports emb<=4096, int_emb<=256, basis_emb<=16, num_spherical<=8, num_radial<=16, "
                   "residual layers<=%d (got %d,%d,%d,%d,%d,%d,%d)", GP_MAX_RES, d->emb, d->int_emb, d->basis_emb,
                   d->num_spherical, d->num_radial, d->n_res_before, d->n_res_after);
  return GP_OK;
}

int check_weights_D(gp_ctx* ctx, const gp_dims* d, const gp_weights_D* w, const char* what) {
  GP_REQUIRE(ctx, w, "%s is NULL", what);
  bool ok = w->W_ji && w->b_ji && w->W_kj && w->b_kj && w->W_rbf1 && w->W_rbf2 && w->W_down && w->W_sbf1 &&
            w->W_sbf2 && w->W_up && w->W_lin && w->b_lin;
  for (int r = 0; r < d->n_res_before; ++r)
    for (int q = 0; q < 4; ++q) ok = ok && w->res_before[r][q];
  for (int r = 0; r < d->n_res_after; ++r)
    for (int q = 0; q < 4; ++q) ok = ok && w->res_after[r][q];
  GP_REQUIRE(ctx, ok, "%s has a NULL member", what);
  return GP_OK;
}

// one residual layer forward: hout = hin + act(act(hin W1 + b1) W2 + b2)
int res_forward(gp_ctx* ctx, const float* hin, float* const* w, const res_saved& s, float* hout, int64_t E, int H) {
  gp_epilogue e1;
  e1.bias = w[1]; e1.save_pre = s.z1; e1.act = 1; e1.out = s.y1;
  GP_TRY(gp_gemm_nn(ctx, hin, w[0], E, H, H, e1));
  gp_epilogue e2;
  e2.bias = w[3]; e2.save_pre = s.z2; e2.act = 1; e2.add_post = hin; e2.out = hout;
  return gp_gemm_nn(ctx, s.y1, w[2], E, H, H, e2);
}

// One residual layer backward.  dz2 = dh * silu'(z2) is given (written by the producer of dh).
// dh_out = dh + d(hin through the layer); if z_next != NULL also dz_next = dh_out * silu'(z_next).
// The two weight-gradient GEMMs go to the side stream.
int res_backward(gp_ctx* ctx, gp_aux& aux, const float* hin, float* const* w, float* const* gw, const res_saved& s,
                 const float* dh, const float* dz2, float* dh_out, float* t2, const float* z_next, float* dz_next,
                 scratch_D& sc, int64_t E, int H) {
  GP_TRY(aux.on_aux([&] { return gp_gemm_tn(ctx, s.y1, dz2, E, H, H, gw[2], gw[3], sc.part_aux, sc.part_bytes); }, {dz2}));
  gp_epilogue e;
  e.act = 2; e.zsrc = s.z1; e.out = t2;
  GP_TRY(aux.before_write(t2));
  GP_TRY(gp_gemm_nt(ctx, dz2, w[2], E, H, H, e));                                       // dz1
  GP_TRY(aux.on_aux([&] { return gp_gemm_tn(ctx, hin, t2, E, H, H, gw[0], gw[1], sc.part_aux, sc.part_bytes); }, {t2}));
  gp_epilogue e2;
  e2.add_post = dh; e2.out = dh_out; e2.out2 = z_next ? dz_next : nullptr; e2.z2src = z_next;
  if (z_next) GP_TRY(aux.before_write(dz_next));
  return gp_gemm_nt(ctx, t2, w[0], E, H, H, e2);
}

}  // namespace

extern "C" {

int gp_block_workspace(const gp_dims* dims, int64_t n_atoms, int64_t n_edges, int64_t n_triplets, size_t* saved_bytes,
                       size_t* scratch_bytes) {
  if (!dims || !saved_bytes || !scratch_bytes || n_atoms < 0 || n_edges < 0 || n_triplets < 0) return GP_BAD_ARG;
  if (dims->variant == GP_VARIANT_D) {
    saved_D s;
    scratch_D sc;
    *saved_bytes = carve_saved_D(nullptr, dims, n_edges, &s);
    *scratch_bytes = carve_scratch_D(nullptr, dims, n_edges, &sc);
    return GP_OK;
  }
  if (dims->variant == GP_VARIANT_G) {
    *saved_bytes = gp_block_G_saved_bytes(dims, n_edges);
    *scratch_bytes = gp_block_G_scratch_bytes(dims, n_atoms, n_edges, n_triplets);
    return GP_OK;
  }
  return GP_UNSUPPORTED_DIMS;
}

int gp_block_forward_D(gp_ctx* ctx, const gp_dims* dims, const gp_weights_D* w, const gp_graph* graph,
                       const gp_basis* basis, const float* m_in, float* m_out, void* saved, size_t saved_bytes,
                       void* scratch, size_t scratch_bytes) {
  if (!ctx) return GP_BAD_ARG;
  GP_TRY(check_dims_D(ctx, dims));
  GP_TRY(check_weights_D(ctx, dims, w, "weights"));
  GP_REQUIRE(ctx, graph && basis, "gp_block_forward_D: graph/basis is NULL");
  const int64_t E = graph->n_edges;
  GP_REQUIRE(ctx, E >= 0 && graph->n_triplets >= 0, "gp_block_forward_D: negative size");
  if (E == 0) return GP_OK;
  GP_REQUIRE(ctx, m_in && m_out && saved && scratch, "gp_block_forward_D: NULL pointer");
  GP_REQUIRE(ctx, basis->rbf && basis->rad && (graph->n_triplets == 0 || basis->cos_alpha), "gp_block_forward_D: basis arrays missing");
  GP_TRY(gp_take_deferred(ctx, "gp_block_forward_D"));
  saved_D s;
  scratch_D sc;
  if (saved_bytes < carve_saved_D(saved, dims, E, &s)) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "gp_block_forward_D: saved buffer too small");
  if (scratch_bytes < carve_scratch_D(scratch, dims, E, &sc)) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "gp_block_forward_D: scratch too small");
  GP_HIP(ctx, hipSetDevice(ctx->device));
  const int H = dims->emb, F = dims->int_emb, B = dims->basis_emb, S = dims->num_spherical, R = dims->num_radial;
  float* x_ji = sc.buf[0];

  // Side stream, before the triplet sum: the projected radial table is needed only by the triplet kernel and the
  // projection of the target-edge message only by the epilogue of the up-projection, so both run next to the chain
  // that leads to the triplet sum.  After it: the layers act on every edge by itself, and a GEMM over all E rows at
  // these widths is one round of workgroups whose loading, multiplying and storing phases coincide; the rows are cut
  // in two and the halves run as two chains on the two streams, out of step with each other (configuration 2:
  // 9.70 -> 9.40 ms per step; cutting the chain before the triplet sum as well: 9.51 ms).
  constexpr int64_t SPLIT_MIN_ROWS = 2048;
  gp_aux aux(ctx);
  const int64_t half = ((E / 2 + 127) / 128) * 128;
  const bool split = aux.active() && E >= SPLIT_MIN_ROWS && half < E;
  gp_epilogue e;
  e.out = s.Wrbf;
  GP_TRY(gp_gemm_nn(ctx, w->W_rbf1, w->W_rbf2, R, H, B, e));
  auto project_radial = [&] { return gp_tripD_project_radial(ctx, basis->rad, w->W_sbf1, E, S, R, B, s.Q); };   // Q is [S*B, E]: not cut
  auto ji_rows = [&](int64_t r0, int64_t n) {
    const int64_t o = r0 * H;
    gp_epilogue q; q.bias = w->b_ji; q.save_pre = s.z_ji + o; q.act = 1; q.out = x_ji + o;
    return gp_gemm_nn(ctx, m_in + o, w->W_ji, n, H, H, q);
  };
  auto kj_rows = [&](int64_t r0, int64_t n) -> int {
    const int64_t o = r0 * H;
    gp_epilogue q; q.out = s.gate + o;
    GP_TRY(gp_gemm_nn(ctx, basis->rbf + r0 * R, s.Wrbf, n, H, R, q));
    q = gp_epilogue(); q.bias = w->b_kj; q.save_pre = s.z_kj + o; q.act = 1; q.mul = s.gate + o; q.out = s.xg + o;
    GP_TRY(gp_gemm_nn(ctx, m_in + o, w->W_kj, n, H, H, q));
    q = gp_epilogue(); q.save_pre = s.z_dn + r0 * F; q.act = 1; q.out = s.x_kj + r0 * F;
    return gp_gemm_nn(ctx, s.xg + o, w->W_down, n, F, H, q);
  };
  GP_TRY(aux.on_aux([&] { return project_radial(); }, {s.Q}));
  GP_TRY(aux.on_aux([&] { return ji_rows(0, E); }, {}));
  GP_TRY(kj_rows(0, E));
  GP_TRY(aux.before_write(s.Q));   // the projected radial table, written on the side stream
  const bool fwd_mfma = ctx->trip_mfma != 0 && gp_tripD_mfma_usable(graph, F, S, B);
  const bool keep_Bacc = !(fwd_mfma && bwd_mfma_D(ctx, dims, graph));
  ctx->fwd_flags[saved] = keep_Bacc ? 1u : 0u;   // the backward call must agree on whether Bacc was written
  if (fwd_mfma || bwd_mfma_D(ctx, dims, graph)) GP_TRY(gp_check_degrees(ctx, graph));
  if (fwd_mfma)
    GP_TRY(gp_tripD_forward_mfma(ctx, graph, basis->cos_alpha, s.x_kj, s.Q, w->W_sbf2, F, S, B, s.a, keep_Bacc ? s.Bacc : nullptr));
  else
    GP_TRY(gp_tripD_forward(ctx, graph, basis->cos_alpha, s.x_kj, s.Q, w->W_sbf2, F, S, B, s.a, s.Bacc));
  GP_TRY(aux.join());

  // rows [r0, r0 + n) of the layers after the triplet sum
  auto rows_forward = [&](int64_t r0, int64_t n) -> int {
    const int64_t o = r0 * H;
    auto at = [&](const res_saved& q) { return res_saved{q.z1 + o, q.y1 + o, q.z2 + o, q.hout + o}; };
    gp_epilogue eu; eu.save_pre = s.z_up + o; eu.act = 1; eu.add_post = x_ji + o; eu.out = s.h0 + o;
    GP_TRY(gp_gemm_nn(ctx, s.a + r0 * F, w->W_up, n, H, F, eu));
    const float* h = s.h0 + o;
    for (int r = 0; r < dims->n_res_before; ++r) {
      const res_saved q = at(s.before[r]);
      GP_TRY(res_forward(ctx, h, w->res_before[r], q, q.hout, n, H));
      h = q.hout;
    }
    float* lin_out = (dims->n_res_after == 0 ? m_out : s.h_lin) + o;
    gp_epilogue el; el.bias = w->b_lin; el.save_pre = s.z_lin + o; el.act = 1; el.add_post = m_in + o; el.out = lin_out;
    GP_TRY(gp_gemm_nn(ctx, h, w->W_lin, n, H, H, el));
    h = lin_out;
    for (int r = 0; r < dims->n_res_after; ++r) {
      const res_saved q = at(s.after[r]);
      float* out = (r == dims->n_res_after - 1) ? m_out + o : q.hout;
      GP_TRY(res_forward(ctx, h, w->res_after[r], q, out, n, H));
      h = out;
    }
    return GP_OK;
  };
  if (split) {
    GP_TRY(aux.on_aux([&] { return rows_forward(half, E - half); }, {}));
    GP_TRY(rows_forward(0, half));
    return aux.join();
  }
  return rows_forward(0, E);
}

}  // extern "C"

namespace {

// P[e, l, f] = x[e, f] sum_b W_sbf2[b, f] Q[e, l, b]: with it, dL/dcos(alpha_t) = sum_l Y_l0'(cos alpha_t) sum_f
// grad_a[ji(t), f] P[kj(t), l, f], the same contraction as the bilinear block's (U = P, dz = grad_a)
__global__ void cos_factor_kernel(const float* __restrict__ x, const float* __restrict__ W2, const float* __restrict__ Qt, int64_t E,
                                  int S, int B, int F, float* __restrict__ P) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // (e, l, f)
  if (i >= E * S * F) return;
  const int f = (int)(i % F), l = (int)((i / F) % S);
  const int64_t e = i / ((int64_t)F * S);
  float s = 0.f;
  for (int b = 0; b < B; ++b) s += W2[b * F + f] * Qt[(int64_t)(l * B + b) * E + e];
  P[i] = x[e * F + f] * s;
}

// grad_rad[e, l, n] (+)= sum_b grad_Q[e, l, b] W_sbf1[(l, n), b]   (Q[e, l, b] = sum_n rad[e, l, n] W_sbf1[(l, n), b])
__global__ void grad_rad_kernel(const float* __restrict__ gQ, const float* __restrict__ W1, int64_t E, int S, int R, int B,
                                int accumulate, float* __restrict__ grad_rad) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // (e, l, n)
  if (i >= E * S * R) return;
  const int n = (int)(i % R), l = (int)((i / R) % S);
  const int64_t e = i / ((int64_t)R * S);
  float s = 0.f;
  for (int b = 0; b < B; ++b) s += gQ[(e * S + l) * B + b] * W1[(l * R + n) * B + b];
  grad_rad[i] = accumulate ? grad_rad[i] + s : s;
}

int backward_D(gp_ctx* ctx, const gp_dims* dims, const gp_weights_D* w, const gp_graph* graph, const gp_basis* basis,
               const float* m_in, const void* saved, size_t saved_bytes, const float* grad_m_out, float* grad_m_in,
               gp_weights_D* gw, float* grad_rbf, float* grad_rad, float* grad_cos_kj, int accumulate_basis_grads,
               void* scratch, size_t scratch_bytes) {
  if (!ctx) return GP_BAD_ARG;
  GP_TRY(check_dims_D(ctx, dims));
  GP_TRY(check_weights_D(ctx, dims, w, "weights"));
  GP_TRY(check_weights_D(ctx, dims, gw, "grad_w"));
  GP_REQUIRE(ctx, graph && basis, "gp_block_backward_D: graph/basis is NULL");
  const int64_t E = graph->n_edges;
  GP_REQUIRE(ctx, E >= 0 && graph->n_triplets >= 0, "gp_block_backward_D: negative size");
  GP_REQUIRE(ctx, E > 0, "gp_block_backward_D: empty edge list");
  GP_REQUIRE(ctx, m_in && grad_m_out && grad_m_in && saved && scratch, "gp_block_backward_D: NULL pointer");
  GP_REQUIRE(ctx, basis->rbf && basis->rad && (graph->n_triplets == 0 || basis->cos_alpha_kj), "gp_block_backward_D: basis arrays missing");
  saved_D s;
  scratch_D sc;
  if (saved_bytes < carve_saved_D(const_cast<void*>(saved), dims, E, &s)) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "gp_block_backward_D: saved buffer too small");
  if (scratch_bytes < carve_scratch_D(scratch, dims, E, &sc)) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "gp_block_backward_D: scratch too small");
  GP_HIP(ctx, hipSetDevice(ctx->device));
  const int H = dims->emb, F = dims->int_emb, B = dims->basis_emb, S = dims->num_spherical, R = dims->num_radial;
  const int64_t EH = E * H;
  float *T1 = sc.buf[3], *T2 = sc.buf[4], *T3 = sc.buf[5], *dgate = sc.buf[6];
  // rotating buffers for dh; `keep` is a gradient that must survive (the skip into m)
  const float* dh = grad_m_out;
  const float* keep = nullptr;
  auto next_buf = [&]() -> float* {
    for (int i = 0; i < 3; ++i)
      if (sc.buf[i] != dh && sc.buf[i] != keep) return sc.buf[i];
    return nullptr;
  };

  gp_aux aux(ctx);
  // dz of the last activation in the block: the only elementwise pass that has no producer GEMM
  const float* z_first = dims->n_res_after > 0 ? s.after[dims->n_res_after - 1].z2 : s.z_lin;
  float* dzcur = T1;
  auto other_dz = [&]() -> float* { return dzcur == T1 ? T3 : T1; };
  GP_TRY(gp_ew_dsilu_mul(ctx, dh, z_first, dzcur, EH));

  // residual layers after the skip, last to first
  for (int r = dims->n_res_after - 1; r >= 0; --r) {
    const float* hin = (r == 0) ? s.h_lin : s.after[r - 1].hout;
    const float* z_next = (r > 0) ? s.after[r - 1].z2 : s.z_lin;
    float* out = next_buf();
    float* dznext = other_dz();
    GP_TRY(res_backward(ctx, aux, hin, w->res_after[r], gw->res_after[r], s.after[r], dh, dzcur, out, T2, z_next,
                        dznext, sc, E, H));
    dh = out;
    dzcur = dznext;
  }
  // h_lin = act(h W_lin + b_lin) + m;  dzcur = dz_lin
  keep = dh;
  {
    const float* hin = dims->n_res_before > 0 ? s.before[dims->n_res_before - 1].hout : s.h0;
    const float* z_next = dims->n_res_before > 0 ? s.before[dims->n_res_before - 1].z2 : s.z_up;
    GP_TRY(aux.on_aux([&] { return gp_gemm_tn(ctx, hin, dzcur, E, H, H, gw->W_lin, gw->b_lin, sc.part_aux, sc.part_bytes); },
                      {dzcur}));
    float* out = next_buf();
    float* dznext = other_dz();
    GP_TRY(aux.before_write(dznext));
    gp_epilogue e; e.out = out; e.out2 = dznext; e.z2src = z_next;
    GP_TRY(gp_gemm_nt(ctx, dzcur, w->W_lin, E, H, H, e));
    dh = out;
    dzcur = dznext;
  }
  for (int r = dims->n_res_before - 1; r >= 0; --r) {
    const float* hin = (r == 0) ? s.h0 : s.before[r - 1].hout;
    const float* z_next = (r > 0) ? s.before[r - 1].z2 : s.z_up;
    float* out = next_buf();
    float* dznext = other_dz();
    GP_TRY(res_backward(ctx, aux, hin, w->res_before[r], gw->res_before[r], s.before[r], dh, dzcur, out, T2, z_next,
                        dznext, sc, E, H));
    dh = out;
    dzcur = dznext;
  }
  // h0 = x_ji + act(a W_up);  dh = dh0, dzcur = dz_up
  // The branch through x_ji = act(m W_ji + b_ji) needs dh0 only: all of it (dz_ji, both gradients) runs on the side
  // stream next to the chain through the triplet sum, whose kernels leave much of the chip idle; its input gradient
  // is added by the epilogue of the last GEMM below.
  float* const dz_kj = dzcur;   // free again once the two GEMMs that read dz_up are done
  GP_TRY(aux.on_aux([&] { return gp_gemm_tn(ctx, s.a, dzcur, E, F, H, gw->W_up, nullptr, sc.part_aux, sc.part_bytes); },
                    {dzcur}));
  float* const dz_ji = other_dz();   // last read by side-stream work issued earlier, and written there: no wait needed
  float* const dm_ji = next_buf();
  GP_TRY(aux.on_aux(
      [&] {
        GP_TRY(gp_ew_dsilu_mul(ctx, dh, s.z_ji, dz_ji, EH));
        GP_TRY(gp_gemm_tn(ctx, m_in, dz_ji, E, H, H, gw->W_ji, gw->b_ji, sc.part_aux, sc.part_bytes));
        gp_epilogue e; e.out = dm_ji;
        return gp_gemm_nt(ctx, dz_ji, w->W_ji, E, H, H, e);
      },
      {dz_ji, dm_ji}));
  {
    gp_epilogue e; e.out = sc.dF1;
    GP_TRY(gp_gemm_nt(ctx, dzcur, w->W_up, E, F, H, e));                                     // da
  }
  // triplet interaction
  const bool bwd_mfma = bwd_mfma_D(ctx, dims, graph);
  {
    // the matrix-core backward kernel does without Bacc; the per-edge one needs what the forward call stored
    const auto it = ctx->fwd_flags.find(saved);
    if (!bwd_mfma && it != ctx->fwd_flags.end() && it->second == 0u)
      return gp_fail(ctx, GP_BAD_ARG, "gp_block_backward_D: the forward call of this `saved` buffer ran with the matrix-core triplet "
                     "kernels and kept no accumulator; gp_set_triplet_mfma must not change between forward and backward");
  }
  if (bwd_mfma)
    GP_TRY(gp_tripD_backward_mfma(ctx, graph, basis->cos_alpha_kj, s.x_kj, s.Q, w->W_sbf2, sc.dF1, s.z_dn, F, S, B,
                                  sc.dF2, sc.dQ, gw->W_sbf2, sc.part, sc.part_bytes));        // dz_dn, dQ, dW_sbf2
  else
    GP_TRY(gp_tripD_backward(ctx, graph, basis->cos_alpha_kj, s.x_kj, s.Q, w->W_sbf2, sc.dF1, s.z_dn, F, S, B,
                             sc.dF2, sc.dQ));                                                 // dz_dn, dQ
  // weight gradients that nothing below waits for: side stream (its own split-K buffer; its kernels run in order)
  GP_TRY(aux.on_aux(
      [&] {
        return gp_tripD_weight_grads(ctx, sc.dF1, bwd_mfma ? nullptr : s.Bacc, basis->rad, sc.dQ, E, F, S, R, B, gw->W_sbf2,
                                     gw->W_sbf1, sc.part_aux, sc.part_bytes);
      },
      {}));
  // gradients with respect to the basis (forces, Sec. 3.2): radial part of the spherical basis from grad_Q, cos(alpha)
  // through the per-edge factor P and the kernel the bilinear block uses for the same contraction
  if (grad_rad) {
    const int64_t n = E * S * R;
    grad_rad_kernel<<<(unsigned)((n + 255) / 256), 256, 0, ctx->stream>>>(sc.dQ, w->W_sbf1, E, S, R, B, accumulate_basis_grads, grad_rad);
    GP_LAUNCH_CHECK(ctx, "grad_rad_kernel");
  }
  if (grad_cos_kj && graph->n_triplets > 0) {
    const int64_t n = E * S * F;
    cos_factor_kernel<<<(unsigned)((n + 255) / 256), 256, 0, ctx->stream>>>(s.x_kj, w->W_sbf2, s.Q, E, S, B, F, sc.P);
    GP_LAUNCH_CHECK(ctx, "cos_factor_kernel");
    GP_TRY(gp_tripG_grad_cos(ctx, graph, basis->cos_alpha_kj, sc.P, sc.dF1, F, S, accumulate_basis_grads, grad_cos_kj));
  }
  GP_TRY(aux.on_aux([&] { return gp_gemm_tn(ctx, s.xg, sc.dF2, E, H, F, gw->W_down, nullptr, sc.part_aux, sc.part_bytes); },
                    {sc.dF2}));
  {
    GP_TRY(aux.before_write(T2));
    gp_epilogue e; e.out = T2;
    GP_TRY(gp_gemm_nt(ctx, sc.dF2, w->W_down, E, H, F, e));                                  // dxg
  }
  GP_TRY(aux.before_write(dz_kj));
  GP_TRY(gp_ew_gate_bwd(ctx, T2, s.z_kj, s.gate, dz_kj, dgate, EH));                         // dz_kj, dgate
  GP_TRY(gp_gemm_tn(ctx, basis->rbf, dgate, E, R, H, sc.dWrbf, nullptr, sc.part, sc.part_bytes));
  if (grad_rbf) {   // dL/drbf = dgate W_rbf^T
    gp_epilogue e; e.out = grad_rbf;
    if (accumulate_basis_grads) e.add_post = grad_rbf;
    GP_TRY(gp_gemm_nt(ctx, dgate, s.Wrbf, E, R, H, e));
  }
  {
    gp_epilogue e; e.out = gw->W_rbf1;
    GP_TRY(gp_gemm_nt(ctx, sc.dWrbf, w->W_rbf2, R, B, H, e));
  }
  GP_TRY(gp_gemm_tn(ctx, w->W_rbf1, sc.dWrbf, R, B, H, gw->W_rbf2, nullptr, sc.part, sc.part_bytes));
  GP_TRY(aux.on_aux([&] { return gp_gemm_tn(ctx, m_in, dz_kj, E, H, H, gw->W_kj, gw->b_kj, sc.part_aux, sc.part_bytes); }, {dz_kj}));
  {
    GP_TRY(aux.before_write(dm_ji));   // the side stream's input gradient of the ji path
    gp_epilogue e; e.add_pre = dm_ji; e.add_post = keep; e.out = grad_m_in;
    GP_TRY(gp_gemm_nt(ctx, dz_kj, w->W_kj, E, H, H, e));                                     // dm = kj path + ji path + skip
  }
  return aux.join();
}

}  // namespace

extern "C" {

int gp_block_backward_D(gp_ctx* ctx, const gp_dims* dims, const gp_weights_D* w, const gp_graph* graph,
                        const gp_basis* basis, const float* m_in, const void* saved, size_t saved_bytes,
                        const float* grad_m_out, float* grad_m_in, gp_weights_D* gw, void* scratch,
                        size_t scratch_bytes) {
  return backward_D(ctx, dims, w, graph, basis, m_in, saved, saved_bytes, grad_m_out, grad_m_in, gw, nullptr, nullptr, nullptr, 0,
                    scratch, scratch_bytes);
}

int gp_block_backward_D_basis(gp_ctx* ctx, const gp_dims* dims, const gp_weights_D* w, const gp_graph* graph,
                              const gp_basis* basis, const float* m_in, const void* saved, size_t saved_bytes,
                              const float* grad_m_out, float* grad_m_in, gp_weights_D* gw, float* grad_rbf, float* grad_rad,
                              float* grad_cos_kj, int32_t accumulate_basis_grads, void* scratch, size_t scratch_bytes) {
  return backward_D(ctx, dims, w, graph, basis, m_in, saved, saved_bytes, grad_m_out, grad_m_in, gw, grad_rbf, grad_rad,
                    grad_cos_kj, accumulate_basis_grads, scratch, scratch_bytes);
}

}  // extern "C"
