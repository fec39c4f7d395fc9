// C ABI of the TripletUpdate + TripletAggr kernels on their own, in every form the interaction blocks run them
// (paper Sec. 3.3: Hadamard product with the projected basis; Sec. 3.4: bilinear layer), so that each can be
// called, checked and timed without the edge MLPs around it.
#include <algorithm>

#include "triplet.h"

namespace {
int need_lists(gp_ctx* ctx, const gp_graph* g, const char* who) {
  GP_REQUIRE(ctx, g->n_atoms > 0 && g->row_ptr && g->out_ptr && g->out_list,
             "%s: the per-centre-atom forms need the lists by centre atom of gp_graph", who);
  return GP_OK;
}
}  // namespace

extern "C" {

int gp_triplet_workspace(const gp_graph* graph, int32_t width, size_t* bytes) {
  if (!graph || !bytes || width < 1 || graph->n_edges < 0 || graph->n_triplets < 0) return GP_BAD_ARG;
  size_t b = gp_tripG_mfma_scratch(graph->n_edges, graph->n_triplets);
  if (graph->n_atoms > 0) {
    b = std::max(b, gp_tripG_fused_scratch(graph->n_atoms, graph->n_edges, width));
    b = std::max(b, gp_tripG_H_fused_scratch(graph->n_atoms, graph->n_edges, width));
    b = std::max(b, gp_tripD_mfma_bwd_scratch(graph, width));
    b = std::max(b, gp_tripG_dcos_fused_scratch(graph->n_atoms, graph->n_edges, width, 1));
  }
  *bytes = b;
  return GP_OK;
}

int gp_triplet_hadamard_fwd(gp_ctx* ctx, const gp_graph* graph, int32_t form, int32_t num_spherical, int32_t basis_emb,
                            int32_t width, const float* cos_alpha, const float* x, const float* Qt, const float* W_sbf2,
                            float* a, float* Bacc) {
  if (!ctx) return GP_BAD_ARG;
  GP_REQUIRE(ctx, graph && x && Qt && W_sbf2 && a, "gp_triplet_hadamard_fwd: NULL pointer");
  GP_HIP(ctx, hipSetDevice(ctx->device));
  if (form == GP_TRIPLET_PER_EDGE) {
    GP_REQUIRE(ctx, Bacc, "gp_triplet_hadamard_fwd: the per-edge form writes its accumulator Bacc[E, basis_emb, width]");
    return gp_tripD_forward(ctx, graph, cos_alpha, x, Qt, W_sbf2, width, num_spherical, basis_emb, a, Bacc);
  }
  if (form == GP_TRIPLET_PER_ATOM) {
    GP_TRY(need_lists(ctx, graph, "gp_triplet_hadamard_fwd"));
    if (!gp_tripD_mfma_usable(graph, width, num_spherical, basis_emb))
      return gp_fail(ctx, GP_UNSUPPORTED_DIMS, "gp_triplet_hadamard_fwd: the per-centre-atom form needs basis_emb 8, width 32..128 in "
                     "steps of 32, at least one triplet and max_in_degree * (width + 64) * 4 bytes within 64 KiB of LDS "
                     "(got basis_emb %d, width %d, max_in_degree %d)", basis_emb, width, graph->max_in_degree);
    GP_TRY(gp_take_deferred(ctx, "gp_triplet_hadamard_fwd"));
    GP_TRY(gp_check_degrees(ctx, graph));
    return gp_tripD_forward_mfma(ctx, graph, cos_alpha, x, Qt, W_sbf2, width, num_spherical, basis_emb, a, Bacc);
  }
  return gp_fail(ctx, GP_BAD_ARG, "gp_triplet_hadamard_fwd: form %d (use gp_triplet_aggregate_fwd for the streaming form)", form);
}

int gp_triplet_hadamard_bwd(gp_ctx* ctx, const gp_graph* graph, int32_t form, int32_t num_spherical, int32_t basis_emb,
                            int32_t width, const float* cos_alpha_kj, const float* x, const float* Qt, const float* W_sbf2,
                            const float* grad_a, float* grad_x, float* grad_Q, float* grad_W_sbf2, void* ws, size_t ws_bytes) {
  if (!ctx) return GP_BAD_ARG;
  GP_REQUIRE(ctx, graph && x && Qt && W_sbf2 && grad_a && grad_x && grad_Q, "gp_triplet_hadamard_bwd: NULL pointer");
  GP_HIP(ctx, hipSetDevice(ctx->device));
  if (form == GP_TRIPLET_PER_EDGE) {
    GP_REQUIRE(ctx, !grad_W_sbf2, "gp_triplet_hadamard_bwd: the per-edge form does not produce grad_W_sbf2 (it is sum_e grad_a * Bacc)");
    return gp_tripD_backward(ctx, graph, cos_alpha_kj, x, Qt, W_sbf2, grad_a, nullptr, width, num_spherical, basis_emb, grad_x, grad_Q);
  }
  if (form == GP_TRIPLET_PER_ATOM) {
    GP_TRY(need_lists(ctx, graph, "gp_triplet_hadamard_bwd"));
    GP_REQUIRE(ctx, grad_W_sbf2 && ws, "gp_triplet_hadamard_bwd: the per-centre-atom form also writes grad_W_sbf2 and needs a workspace");
    if (!gp_tripD_mfma_bwd_usable(graph, width, num_spherical, basis_emb))
      return gp_fail(ctx, GP_UNSUPPORTED_DIMS, "gp_triplet_hadamard_bwd: the per-centre-atom form needs basis_emb 8, width 32..128 in "
                     "steps of 32, the kj-major view, at least one triplet and the out-edges of an atom to fit 64 KiB of LDS "
                     "(got basis_emb %d, width %d, max_out_degree %d)", basis_emb, width, graph->max_out_degree);
    GP_TRY(gp_take_deferred(ctx, "gp_triplet_hadamard_bwd"));
    GP_TRY(gp_check_degrees(ctx, graph));
    return gp_tripD_backward_mfma(ctx, graph, cos_alpha_kj, x, Qt, W_sbf2, grad_a, nullptr, width, num_spherical, basis_emb,
                                  grad_x, grad_Q, grad_W_sbf2, static_cast<float*>(ws), ws_bytes);
  }
  return gp_fail(ctx, GP_BAD_ARG, "gp_triplet_hadamard_bwd: form %d (use gp_triplet_aggregate_bwd for the streaming form)", form);
}

int gp_triplet_bilinear_fwd(gp_ctx* ctx, const gp_graph* graph, int32_t form, int32_t num_spherical, int32_t emb_cbf,
                            int32_t width, const float* cos_alpha, const float* x, const float* Radt, float* A,
                            void* ws, size_t ws_bytes) {
  if (!ctx) return GP_BAD_ARG;
  GP_REQUIRE(ctx, graph && x && Radt && A, "gp_triplet_bilinear_fwd: NULL pointer");
  GP_HIP(ctx, hipSetDevice(ctx->device));
  if (form == GP_TRIPLET_PER_EDGE)
    return gp_tripD_forward(ctx, graph, cos_alpha, x, Radt, nullptr, width, num_spherical, emb_cbf, nullptr, A);
  if (form == GP_TRIPLET_PER_ATOM || form == GP_TRIPLET_PER_ATOM_TWO_KERNELS) {
    GP_TRY(need_lists(ctx, graph, "gp_triplet_bilinear_fwd"));
    GP_REQUIRE(ctx, ws, "gp_triplet_bilinear_fwd: the per-centre-atom forms need a workspace (gp_triplet_workspace)");
    const bool fused = form == GP_TRIPLET_PER_ATOM;
    if (fused ? !gp_tripG_fused_usable(graph, width, num_spherical, emb_cbf) : !gp_tripG_mfma_usable(graph, width, num_spherical, emb_cbf))
      return gp_fail(ctx, GP_UNSUPPORTED_DIMS, "gp_triplet_bilinear_fwd: form %d needs emb_cbf <= 16, width %s and at least one "
                     "triplet (got %d, %d)", form, fused ? "32, 64 or 128" : "32..128 in steps of 32", emb_cbf, width);
    GP_TRY(gp_take_deferred(ctx, "gp_triplet_bilinear_fwd"));
    GP_TRY(gp_check_degrees(ctx, graph));
    if (fused) return gp_tripG_forward_fused(ctx, graph, cos_alpha, x, Radt, width, num_spherical, emb_cbf, A, ws, ws_bytes, 0);
    return gp_tripG_forward_mfma(ctx, graph, cos_alpha, x, Radt, width, num_spherical, emb_cbf, A, ws, ws_bytes, 0);
  }
  return gp_fail(ctx, GP_BAD_ARG, "gp_triplet_bilinear_fwd: unknown form %d", form);
}

int gp_triplet_bilinear_bwd_H(gp_ctx* ctx, const gp_graph* graph, int32_t form, int32_t num_spherical, int32_t width,
                              const float* cos_alpha_kj, const float* dz, float* H, void* ws, size_t ws_bytes) {
  if (!ctx) return GP_BAD_ARG;
  GP_REQUIRE(ctx, graph && dz && H, "gp_triplet_bilinear_bwd_H: NULL pointer");
  GP_HIP(ctx, hipSetDevice(ctx->device));
  if (form == GP_TRIPLET_PER_EDGE)
    return gp_tripD_backward(ctx, graph, cos_alpha_kj, nullptr, nullptr, nullptr, dz, nullptr, width, num_spherical, 1, H, nullptr);
  if (form == GP_TRIPLET_PER_ATOM) {
    GP_TRY(need_lists(ctx, graph, "gp_triplet_bilinear_bwd_H"));
    if (!gp_tripG_mfma_H_usable(graph, width, num_spherical))
      return gp_fail(ctx, GP_UNSUPPORTED_DIMS, "gp_triplet_bilinear_bwd_H: the per-centre-atom form needs width 32..128 in steps of 32, "
                     "the kj-major view and at least one triplet (got %d)", width);
    GP_TRY(gp_take_deferred(ctx, "gp_triplet_bilinear_bwd_H"));
    GP_TRY(gp_check_degrees(ctx, graph));
    // the one-pass kernel where its widths allow and a workspace is given, else the kernel that keeps all of an atom's
    // out-edges in LDS
    if (ws && gp_tripG_H_fused_usable(graph, width, num_spherical) &&
        ws_bytes >= gp_tripG_H_fused_scratch(graph->n_atoms, graph->n_edges, width))
      return gp_tripG_backward_H_fused(ctx, graph, cos_alpha_kj, dz, width, num_spherical, H, ws, ws_bytes);
    return gp_tripG_backward_H_mfma(ctx, graph, cos_alpha_kj, dz, width, num_spherical, H);
  }
  return gp_fail(ctx, GP_BAD_ARG, "gp_triplet_bilinear_bwd_H: unknown form %d", form);
}

int gp_triplet_bilinear_grad_cos(gp_ctx* ctx, const gp_graph* graph, int32_t form, int32_t num_spherical, int32_t width,
                                 const float* cos_alpha_kj, const float* U, const float* dz, int32_t accumulate,
                                 float* grad_cos_kj, void* ws, size_t ws_bytes) {
  if (!ctx) return GP_BAD_ARG;
  GP_REQUIRE(ctx, graph && U && dz && (graph->n_triplets == 0 || (cos_alpha_kj && grad_cos_kj)), "gp_triplet_bilinear_grad_cos: NULL pointer");
  GP_HIP(ctx, hipSetDevice(ctx->device));
  if (form == GP_TRIPLET_PER_EDGE)
    return gp_tripG_grad_cos(ctx, graph, cos_alpha_kj, U, dz, width, num_spherical, accumulate, grad_cos_kj);
  if (form == GP_TRIPLET_PER_ATOM) {
    GP_TRY(need_lists(ctx, graph, "gp_triplet_bilinear_grad_cos"));
    if (!gp_tripG_mfma_bwd_usable(graph, width, num_spherical))
      return gp_fail(ctx, GP_UNSUPPORTED_DIMS, "gp_triplet_bilinear_grad_cos: the per-centre-atom form needs width 32..128 in steps of "
                     "32, the kj-major view and at least one triplet (got %d)", width);
    GP_TRY(gp_take_deferred(ctx, "gp_triplet_bilinear_grad_cos"));
    GP_TRY(gp_check_degrees(ctx, graph));
    // the one-pass kernel where its widths allow and a workspace is given, else the kernel that keeps all of an atom's
    // out-edges in LDS
    if (ws && gp_tripG_H_fused_usable(graph, width, num_spherical) &&
        ws_bytes >= gp_tripG_dcos_fused_scratch(graph->n_atoms, graph->n_edges, width, 1))
      return gp_tripG_grad_cos_fused(ctx, graph, cos_alpha_kj, U, 0, dz, width, num_spherical, accumulate, grad_cos_kj, ws, ws_bytes);
    return gp_tripG_grad_cos_mfma(ctx, graph, cos_alpha_kj, U, dz, width, num_spherical, accumulate, grad_cos_kj);
  }
  return gp_fail(ctx, GP_BAD_ARG, "gp_triplet_bilinear_grad_cos: unknown form %d", form);
}

}  // extern "C"
