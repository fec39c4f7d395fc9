// Output block (paper Sec. 3.3: the updated messages are summed per target atom, EdgeAggr, and
// the sum is transformed by an MLP, NodeUpdate), forward and backward.
//
//   t_e = m_e * (rbf_e W_rbf)                       [E, emb]   radial weighting fused into the GEMM epilogue
//   h_i = sum_{e: dst[e] = i} t_e                   [N, emb]   in-edges of an atom are contiguous rows
//   u   = h W_up;  u = act(u W_k + b_k), k < L      [N, out]
//   P_i = u_i . w_final;  energy[g] (+)= sum_{i in g} P_i
//
// Backward of sum_g grad_energy[g] energy[g]: the node MLP in reverse (N rows: small GEMMs), then
// per edge  dt_e = dh[dst[e]],  grad_m_e (+)= dt_e * (rbf_e W_rbf)  (the gate is recomputed by the
// same GEMM, not stored),  grad_W_rbf = rbf^T (dt * m).  No atomics: every sum follows sorted order.
#include <stdarg.h>

#include <algorithm>

#include "gemm.h"

namespace {

constexpr int WPB = 4;

inline unsigned nblk(int64_t n) { return (unsigned)((n + 255) / 256); }
inline unsigned wblk(int64_t n) { return (unsigned)((n + WPB - 1) / WPB); }

// h[i, f] = sum over the in-edge rows of atom i of t[e, f]; one wavefront per (atom, 64 features)
__global__ void __launch_bounds__(256)
out_atom_sum_kernel(const float* __restrict__ t, const int32_t* __restrict__ row_ptr, int64_t n_atoms, int H,
                    float* __restrict__ h) {
  const int chunks = (H + 63) / 64;
  const int64_t w = (int64_t)blockIdx.x * WPB + (threadIdx.x >> 6);
  const int64_t i = w / chunks;
  if (i >= n_atoms) return;
  const int f = (int)(w % chunks) * 64 + (threadIdx.x & 63);
  if (f >= H) return;
  const int e0 = row_ptr[i], e1 = row_ptr[i + 1];
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  int e = e0;
  for (; e + 3 < e1; e += 4) {
    s0 += t[(int64_t)e * H + f];
    s1 += t[(int64_t)(e + 1) * H + f];
    s2 += t[(int64_t)(e + 2) * H + f];
    s3 += t[(int64_t)(e + 3) * H + f];
  }
  for (; e < e1; ++e) s0 += t[(int64_t)e * H + f];
  h[i * H + f] = (s0 + s1) + (s2 + s3);
}

// p[i] = u[i, :] . w; one wavefront per atom
__global__ void __launch_bounds__(256)
out_atom_dot_kernel(const float* __restrict__ u, const float* __restrict__ w, int64_t n_atoms, int K,
                    float* __restrict__ p) {
  const int64_t i = (int64_t)blockIdx.x * WPB + (threadIdx.x >> 6);
  if (i >= n_atoms) return;
  float s = 0.f;
  for (int k = threadIdx.x & 63; k < K; k += 64) s += u[i * K + k] * w[k];
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) p[i] = s;
}

// energy[g] (+)= sum of p over the atoms of structure g (fixed order); one wavefront per structure
__global__ void __launch_bounds__(256)
out_graph_sum_kernel(const float* __restrict__ p, const int32_t* __restrict__ graph_ptr, int n_graphs, int accumulate,
                     float* __restrict__ energy) {
  const int g = blockIdx.x * WPB + (threadIdx.x >> 6);
  if (g >= n_graphs) return;
  float s = 0.f;
  for (int i = graph_ptr[g] + (threadIdx.x & 63); i < graph_ptr[g + 1]; i += 64) s += p[i];
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) energy[g] = accumulate ? energy[g] + s : s;
}

// ga[i] = grad_energy[structure of atom i];  du[i, k] = ga[i] w[k]; one wavefront per structure walks its atoms
__global__ void __launch_bounds__(256)
out_seed_kernel(const float* __restrict__ grad_energy, const int32_t* __restrict__ graph_ptr, int n_graphs,
                const float* __restrict__ w, int K, float* __restrict__ ga, float* __restrict__ du) {
  const int g = blockIdx.x * WPB + (threadIdx.x >> 6);
  if (g >= n_graphs) return;
  const float ge = grad_energy[g];
  for (int i = graph_ptr[g]; i < graph_ptr[g + 1]; ++i) {
    if ((threadIdx.x & 63) == 0) ga[i] = ge;
    for (int k = threadIdx.x & 63; k < K; k += 64) du[(int64_t)i * K + k] = ge * w[k];
  }
}

// dt[e, :] = dh[dst[e], :]
__global__ void out_gather_rows_kernel(const float* __restrict__ dh, const int32_t* __restrict__ dst, int64_t n_edges,
                                       int H, float* __restrict__ dt) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_edges * H) return;
  dt[i] = dh[(int64_t)dst[i / H] * H + (i % H)];
}

// a[i] *= b[i]
__global__ void out_mul_inplace_kernel(float* __restrict__ a, const float* __restrict__ b, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) a[i] *= b[i];
}

__global__ void out_zero_kernel(float* __restrict__ a, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) a[i] = 0.f;
}

struct out_saved {
  float *h, *u0;
  float *z[GP_MAX_OUT_LAYERS], *u[GP_MAX_OUT_LAYERS];
};
size_t carve_out_saved(void* p, int64_t N, int H, int D, int L, out_saved* s) {
  gp_carver c(p);
  s->h = c.take<float>(N * H);
  s->u0 = c.take<float>(N * D);
  for (int k = 0; k < L; ++k) {
    s->z[k] = c.take<float>(N * D);
    s->u[k] = c.take<float>(N * D);
  }
  return c.off;
}
struct out_scratch {
  float *tE;          // [E, H]: t in the forward pass, dt (then dt * m) in the backward pass
  float *p, *ga;      // [N]
  float *du[2];       // [N, D]
  float *dh;          // [N, H]
  float* part;
  size_t part_bytes;
};
size_t carve_out_scratch(void* p, int64_t N, int64_t E, int H, int D, int R, out_scratch* s) {
  gp_carver c(p);
  s->tE = c.take<float>(E * H);
  s->p = c.take<float>(N);
  s->ga = c.take<float>(N);
  s->du[0] = c.take<float>(N * D);
  s->du[1] = c.take<float>(N * D);
  s->dh = c.take<float>(N * H);
  size_t m = gp_gemm_tn_scratch(E, R, H);
  m = std::max(m, gp_gemm_tn_scratch(N, H, D));
  m = std::max(m, gp_gemm_tn_scratch(N, D, D));
  m = std::max(m, gp_gemm_tn_scratch(N, D, 1));
  s->part_bytes = m;
  s->part = (float*)c.take<char>(m);
  return c.off;
}

int check_out_dims(gp_ctx* ctx, int H, int D, int R, int L) {
  if (H < 1 || H > 4096 || D < 1 || D > 4096 || R < 1 || R > 1024 || L < 0 || L > GP_MAX_OUT_LAYERS)
    return gp_fail(ctx, GP_UNSUPPORTED_DIMS, "output block: emb=%d out_emb=%d num_radial=%d layers=%d unsupported", H, D, R, L);
  return GP_OK;
}
int check_out_weights(gp_ctx* ctx, const gp_weights_out* w, int L, const char* what) {
  GP_REQUIRE(ctx, w && w->W_rbf && w->W_up && w->w_final, "%s has a NULL member", what);
  for (int k = 0; k < L; ++k) GP_REQUIRE(ctx, w->W[k] && w->b[k], "%s: layer %d missing", what, k);
  return GP_OK;
}

}  // namespace

extern "C" {

int gp_output_workspace(int32_t emb, int32_t out_emb, int32_t num_radial, int32_t n_layers, int64_t n_atoms,
                        int64_t n_edges, size_t* saved_bytes, size_t* scratch_bytes) {
  if (!saved_bytes || !scratch_bytes || n_atoms < 0 || n_edges < 0 || emb < 1 || out_emb < 1 || num_radial < 1 ||
      n_layers < 0 || n_layers > GP_MAX_OUT_LAYERS)
    return GP_BAD_ARG;
  out_saved s;
  out_scratch sc;
  *saved_bytes = carve_out_saved(nullptr, n_atoms, emb, out_emb, n_layers, &s);
  *scratch_bytes = carve_out_scratch(nullptr, n_atoms, n_edges, emb, out_emb, num_radial, &sc);
  return GP_OK;
}

int gp_output_forward(gp_ctx* ctx, int32_t emb, int32_t out_emb, int32_t num_radial, int32_t n_layers,
                      const gp_weights_out* w, const float* m, const float* rbf, const int32_t* row_ptr,
                      const int32_t* graph_ptr, int64_t n_atoms, int64_t n_edges, int32_t n_graphs, int32_t accumulate,
                      float* energy, void* saved, size_t saved_bytes, void* scratch, size_t scratch_bytes) {
  if (!ctx) return GP_BAD_ARG;
  const int H = emb, D = out_emb, R = num_radial, L = n_layers;
  GP_TRY(check_out_dims(ctx, H, D, R, L));
  GP_TRY(check_out_weights(ctx, w, L, "weights"));
  GP_REQUIRE(ctx, n_atoms >= 0 && n_edges >= 0 && n_graphs >= 0, "gp_output_forward: negative size");
  if (n_atoms == 0 || n_graphs == 0) return GP_OK;
  GP_REQUIRE(ctx, row_ptr && graph_ptr && energy && saved && scratch && (n_edges == 0 || (m && rbf)), "gp_output_forward: NULL pointer");
  out_saved s;
  out_scratch sc;
  if (saved_bytes < carve_out_saved(saved, n_atoms, H, D, L, &s)) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "gp_output_forward: saved buffer too small");
  if (scratch_bytes < carve_out_scratch(scratch, n_atoms, n_edges, H, D, R, &sc)) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "gp_output_forward: scratch too small");
  GP_HIP(ctx, hipSetDevice(ctx->device));
  hipStream_t st = ctx->stream;
  gp_epilogue e;
  if (n_edges > 0) {
    e = gp_epilogue(); e.mul = m; e.out = sc.tE;
    GP_TRY(gp_gemm_nn(ctx, rbf, w->W_rbf, n_edges, H, R, e));                         // t = (rbf W_rbf) * m
  }
  {
    gp_prof_scope prof(ctx, "out_atom_sum", (double)n_edges * H, 4.0 * ((double)n_edges * H + (double)n_atoms * H));
    out_atom_sum_kernel<<<wblk(n_atoms * ((H + 63) / 64)), 256, 0, st>>>(sc.tE, row_ptr, n_atoms, H, s.h);
    GP_LAUNCH_CHECK(ctx, "out_atom_sum_kernel");
  }
  e = gp_epilogue(); e.out = s.u0;
  GP_TRY(gp_gemm_nn(ctx, s.h, w->W_up, n_atoms, D, H, e));
  const float* u = s.u0;
  for (int k = 0; k < L; ++k) {
    e = gp_epilogue(); e.bias = w->b[k]; e.save_pre = s.z[k]; e.act = 1; e.out = s.u[k];
    GP_TRY(gp_gemm_nn(ctx, u, w->W[k], n_atoms, D, D, e));
    u = s.u[k];
  }
  out_atom_dot_kernel<<<wblk(n_atoms), 256, 0, st>>>(u, w->w_final, n_atoms, D, sc.p);
  out_graph_sum_kernel<<<wblk(n_graphs), 256, 0, st>>>(sc.p, graph_ptr, n_graphs, accumulate, energy);
  GP_LAUNCH_CHECK(ctx, "output block reductions");
  return GP_OK;
}

int gp_output_backward(gp_ctx* ctx, int32_t emb, int32_t out_emb, int32_t num_radial, int32_t n_layers,
                       const gp_weights_out* w, const float* m, const float* rbf, const int32_t* dst,
                       const int32_t* graph_ptr, int64_t n_atoms, int64_t n_edges, int32_t n_graphs,
                       const float* grad_energy, const void* saved, size_t saved_bytes, int32_t accumulate_grad_m,
                       float* grad_m, gp_weights_out* grad_w, void* scratch, size_t scratch_bytes) {
  if (!ctx) return GP_BAD_ARG;
  const int H = emb, D = out_emb, R = num_radial, L = n_layers;
  GP_TRY(check_out_dims(ctx, H, D, R, L));
  GP_TRY(check_out_weights(ctx, w, L, "weights"));
  if (grad_w) GP_TRY(check_out_weights(ctx, grad_w, L, "grad_w"));
  GP_REQUIRE(ctx, n_atoms >= 0 && n_edges >= 0 && n_graphs >= 0, "gp_output_backward: negative size");
  if (n_atoms == 0 || n_graphs == 0) return GP_OK;
  GP_REQUIRE(ctx, graph_ptr && grad_energy && saved && scratch && (n_edges == 0 || (m && rbf && dst && grad_m)),
             "gp_output_backward: NULL pointer");
  out_saved s;
  out_scratch sc;
  if (saved_bytes < carve_out_saved(const_cast<void*>(saved), n_atoms, H, D, L, &s)) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "gp_output_backward: saved buffer too small");
  if (scratch_bytes < carve_out_scratch(scratch, n_atoms, n_edges, H, D, R, &sc)) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "gp_output_backward: scratch too small");
  GP_HIP(ctx, hipSetDevice(ctx->device));
  hipStream_t st = ctx->stream;
  gp_epilogue e;
  float* du = sc.du[0];
  float* other = sc.du[1];
  out_seed_kernel<<<wblk(n_graphs), 256, 0, st>>>(grad_energy, graph_ptr, n_graphs, w->w_final, D, sc.ga, du);
  GP_LAUNCH_CHECK(ctx, "out_seed_kernel");
  const float* u_last = L > 0 ? s.u[L - 1] : s.u0;
  if (grad_w) GP_TRY(gp_gemm_tn(ctx, u_last, sc.ga, n_atoms, D, 1, grad_w->w_final, nullptr, sc.part, sc.part_bytes));
  for (int k = L - 1; k >= 0; --k) {
    GP_TRY(gp_ew_dsilu_mul(ctx, du, s.z[k], du, n_atoms * D));                          // dz_k (in place)
    const float* u_in = k > 0 ? s.u[k - 1] : s.u0;
    if (grad_w) GP_TRY(gp_gemm_tn(ctx, u_in, du, n_atoms, D, D, grad_w->W[k], grad_w->b[k], sc.part, sc.part_bytes));
    e = gp_epilogue(); e.out = other;
    GP_TRY(gp_gemm_nt(ctx, du, w->W[k], n_atoms, D, D, e));                             // du_{k-1}
    std::swap(du, other);
  }
  if (grad_w) GP_TRY(gp_gemm_tn(ctx, s.h, du, n_atoms, H, D, grad_w->W_up, nullptr, sc.part, sc.part_bytes));
  e = gp_epilogue(); e.out = sc.dh;
  GP_TRY(gp_gemm_nt(ctx, du, w->W_up, n_atoms, H, D, e));                               // dh
  if (n_edges > 0) {
    {
      gp_prof_scope prof(ctx, "out_gather_rows", 0.0, 4.0 * ((double)n_edges * H + (double)n_atoms * H));
      out_gather_rows_kernel<<<nblk(n_edges * H), 256, 0, st>>>(sc.dh, dst, n_edges, H, sc.tE);   // dt
      GP_LAUNCH_CHECK(ctx, "out_gather_rows_kernel");
    }
    e = gp_epilogue(); e.mul = sc.tE; e.out = grad_m;
    if (accumulate_grad_m) e.add_post = grad_m;
    GP_TRY(gp_gemm_nn(ctx, rbf, w->W_rbf, n_edges, H, R, e));                           // grad_m (+)= dt * gate
    if (grad_w) {
      out_mul_inplace_kernel<<<nblk(n_edges * H), 256, 0, st>>>(sc.tE, m, n_edges * H);  // dgate = dt * m
      GP_LAUNCH_CHECK(ctx, "out_mul_inplace_kernel");
      GP_TRY(gp_gemm_tn(ctx, rbf, sc.tE, n_edges, R, H, grad_w->W_rbf, nullptr, sc.part, sc.part_bytes));
    }
  } else if (grad_w) {
    out_zero_kernel<<<nblk((int64_t)R * H), 256, 0, st>>>(grad_w->W_rbf, (int64_t)R * H);
    GP_LAUNCH_CHECK(ctx, "out_zero_kernel");
  }
  return GP_OK;
}

}  // extern "C"
