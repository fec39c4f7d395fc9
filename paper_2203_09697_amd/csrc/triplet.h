// TripletUpdate + TripletAggr kernels, fused-basis forms used inside the interaction block
// (internal, not part of the C ABI).
#pragma once
#include "common.h"

// Variant D.  With Q[e',l,b] = sum_n rad[e',l,n] W_sbf1[l*R+n,b] (per edge) and
// p_t[b] = sum_l Y_l0(cos alpha_t) Q[kj(t),l,b], the projected basis of a triplet is
// s_t[f] = sum_b p_t[b] W_sbf2[b,f]; this is the two-step projection of the materialised
// spherical basis, re-associated so that nothing of size T x S*R is ever stored.

// Q from rad[E, S*R] and W_sbf1[S*R, B], stored transposed: Qt[(l*B+b)*E + e]
int gp_tripD_project_radial(gp_ctx* ctx, const float* rad, const float* W1, int64_t E, int S, int R, int B, float* Q);

// a[e,f] = sum_{t in seg_ji(e)} x[kj(t),f] s_t[f];  Bacc[e,b,f] = sum_t p_t[b] x[kj(t),f]
int gp_tripD_forward(gp_ctx* ctx, const gp_graph* g, const float* cos_alpha, const float* x, const float* Q,
                     const float* W2, int F, int S, int B, float* a, float* Bacc);

// From grad_a[E,F]:
//   grad_x[e',f] = sum_{t: kj(t)=e'} grad_a[ji(t),f] s_t[f], multiplied by silu'(z[e',f]) if z != NULL
//   grad_Q[e',l,b] = sum_{t: kj(t)=e'} Y_l(t) sum_f W2[b,f] grad_a[ji(t),f] x[e',f]
// The same result on the fp32 matrix cores, grouped by centre atom (needs the centre-atom lists of gp_graph,
// basis_emb 8, int_emb 32..128 in steps of 32, and the atom with the most in-edges to fit LDS).
bool gp_tripD_mfma_usable(const gp_graph* g, int F, int S, int B);
int gp_tripD_forward_mfma(gp_ctx* ctx, const gp_graph* g, const float* cos_alpha, const float* x, const float* Qt,
                          const float* W2, int F, int S, int B, float* a, float* Bacc);
int gp_tripD_backward(gp_ctx* ctx, const gp_graph* g, const float* cos_alpha_kj, const float* x, const float* Q,
                      const float* W2, const float* grad_a, const float* z, int F, int S, int B,
                      float* grad_x, float* grad_Q);
// Backward on the fp32 matrix cores, per centre atom: grad_x, grad_Q as gp_tripD_backward, and grad_W2 from the
// same pass (no Bacc needed).  part: gp_tripD_mfma_bwd_scratch bytes.
bool gp_tripD_mfma_bwd_usable(const gp_graph* g, int F, int S, int B);
size_t gp_tripD_mfma_bwd_scratch(const gp_graph* g, int F);
int gp_tripD_backward_mfma(gp_ctx* ctx, const gp_graph* g, const float* cos_alpha_kj, const float* x, const float* Qt,
                           const float* W2, const float* grad_a, const float* z, int F, int S, int B, float* grad_x,
                           float* grad_Q, float* grad_W2, float* part, size_t part_bytes);

// grad_W2[b,f] = sum_e grad_a[e,f] Bacc[e,b,f];  grad_W1[l*R+n,b] = sum_e rad[e,l*R+n] grad_Q[e,l*B+b]
size_t gp_tripD_wgrad_scratch(int64_t E, int F, int S, int R, int B);
int gp_tripD_weight_grads(gp_ctx* ctx, const float* grad_a, const float* Bacc, const float* rad, const float* grad_Q,
                          int64_t E, int F, int S, int R, int B, float* grad_W2, float* grad_W1,
                          float* part, size_t part_bytes);

// workspace sizes of the variant-G block (block_G.hip)
size_t gp_block_G_saved_bytes(const gp_dims* d, int64_t E);
size_t gp_block_G_scratch_bytes(const gp_dims* d, int64_t N, int64_t E, int64_t T);   // N: atoms of the graph's centre-atom lists, or 0

// ---- variant G (bilinear interaction, Sec. 3.4) ---------------------------------------------
// The forward accumulator A[e,c,f] = sum_t y_t[c] x[kj(t),f], y_t[c] = sum_l Y_l(t) Rad[kj(t),l,c],
// is gp_tripD_forward with W2 = NULL, B = emb_cbf and Q = the transposed radial table
// Radt[(l*C+c)*E + e].  The backward pass needs only H[e',l,o] = sum_{t: kj(t)=e'} Y_l(t) dz[ji(t),o],
// which is gp_tripD_backward with Q = NULL (grad_x receives H[E,S,O]); everything else per
// source edge follows from H by the two small per-edge products below.

// Gout[e, c*O + o] = sum_l Radt[(l*C+c)*E + e] * H[e, l, o]
// (out_half: Gout addresses bf16 elements; h_half: so does H, taken only together with out_half at widths 32, 64, 128)
int gp_tripG_edge_G(gp_ctx* ctx, const float* Radt, const float* H, int64_t E, int S, int C, int O, float* Gout,
                    int out_half = 0, int h_half = 0);
// whether the two per-edge products read a bf16 H at these widths (16-byte aligned H, V, G)
bool gp_tripG_edge_takes_half_H(int C, int O);
// dRad[e, l*C + c] = sum_o V[e, c*O + o] * H[e, l, o]
// v_half: V addresses bf16 elements; h_half: so does H (emb_cbf <= 16 and widths 32, 64, 128 only)
int gp_tripG_edge_dRad(gp_ctx* ctx, const float* V, const float* H, int64_t E, int S, int C, int O, float* dRad, int v_half = 0,
                       int h_half = 0);
// dst[a,b,c] = src element whose index along source dimension p0 is a, along p1 is b, along p2 is c
// (src has dimensions n0 x n1 x n2; dst has n[p0] x n[p1] x n[p2]); for small weight tensors
int gp_permute3(gp_ctx* ctx, const float* src, int n0, int n1, int n2, int p0, int p1, int p2, float* dst);
// d1 = g * s * silu'(z1), d2 = g * s * silu'(z2)
int gp_ew_dsilu2(gp_ctx* ctx, const float* g, float s, const float* z1, const float* z2, float* d1, float* d2, int64_t n);
// U[e, l, o] = sum_c Radt[(l*C+c)*E + e] * V[e, c*O + o]
// out16: U is written as bf16 [E][8][O] (rows l >= S zero) instead of fp32 [E][S][O]
int gp_tripG_edge_U(gp_ctx* ctx, const float* Radt, const float* V, int64_t E, int S, int C, int O, float* U, int v_half = 0,
                    int out16 = 0);
// grad_cos_kj[q] (+)= sum_l Y_l0'(cos_alpha_kj[q]) sum_o dz[ji(q), o] U[kj(q), l, o]   (kj-major order)
int gp_tripG_grad_cos(gp_ctx* ctx, const gp_graph* g, const float* cos_alpha_kj, const float* U, const float* dz,
                      int O, int S, int accumulate, float* grad_cos_kj);
// Matrix-core form of the forward accumulator A (triplet_g_mfma.hip), bf16 operands: usable when
// the graph carries its lists by centre atom and the widths fit (F a multiple of 32 up to 128,
// C <= 16, one atom's rows of x fit in LDS); ybuf is scratch of gp_tripG_mfma_scratch bytes.
bool gp_tripG_mfma_usable(const gp_graph* g, int F, int S, int C);
size_t gp_tripG_mfma_scratch(int64_t E, int64_t T);
int gp_tripG_forward_mfma(gp_ctx* ctx, const gp_graph* g, const float* cos_alpha, const float* x, const float* Radt,
                          int F, int S, int C, float* A, void* ybuf, size_t ybytes, int out_half = 0,   // out_half: A is bf16
                          const int32_t* row_list = nullptr, int rad_by_pos = 0);
// The same accumulator in one pass, without the per-triplet y buffer (triplet_g_fused.hip): y is evaluated in
// registers inside the contraction kernel from a per-row coefficient table that a pre-pass lays out per centre
// atom.  F = 32, 64 or 128.  ws: gp_tripG_fused_scratch bytes.  With a row_list (see below) the columns of Radt must
// already be in row_list order.
bool gp_tripG_fused_usable(const gp_graph* g, int F, int S, int C);
size_t gp_tripG_fused_scratch(int64_t N, int64_t E, int F);
int gp_tripG_forward_fused(gp_ctx* ctx, const gp_graph* g, const float* cos_alpha, const float* x, const float* Radt,
                           int F, int S, int C, float* A, void* ws, size_t ws_bytes, int out_half,
                           const int32_t* row_list = nullptr);
// H[e',l,o] in the same one-pass style (triplet_g_fused_bwd.hip): O = 32, 64 or 128.
bool gp_tripG_H_fused_usable(const gp_graph* g, int O, int S);
size_t gp_tripG_H_fused_scratch(int64_t N, int64_t E, int O);
int gp_tripG_backward_H_fused(gp_ctx* ctx, const gp_graph* g, const float* cos_alpha_kj, const float* dz, int O, int S, float* H,
                              void* ws, size_t ws_bytes, const int32_t* row_list = nullptr, int out_half = 0);   // out_half: H is bf16
// grad_cos_kj in the same per-(atom, 32 rows) decomposition, wavefronts working alone without LDS.  U: bf16 [E][8][O]
// (u_is_bf16_padded, as gp_tripG_edge_U writes it with out16) or fp32 [E][S][O] (converted into the workspace first).
size_t gp_tripG_dcos_fused_scratch(int64_t N, int64_t E, int O, int with_u16);
int gp_tripG_grad_cos_fused(gp_ctx* ctx, const gp_graph* g, const float* cos_alpha_kj, const void* U, int u_is_bf16_padded,
                            const float* dz, int O, int S, int accumulate, float* grad_cos_kj, void* ws, size_t ws_bytes);
// rad_by_pos: Radt's columns are in row_list order already (gathered by the caller)
// row_list: edge ids of the atoms' rows where these are not consecutive (the mirrored views of a block with the
// radial factor at the target edge: g->row_ptr then indexes row_list, and g->out_list holds consecutive ids)
// Matrix-core forms of H[e',l,o] and of grad_cos (kj-major), same conditions on the graph; O a multiple of 32 up to 128
bool gp_tripG_mfma_bwd_usable(const gp_graph* g, int O, int S);
bool gp_tripG_mfma_H_usable(const gp_graph* g, int O, int S);   // the H kernel alone (less LDS than grad_cos)
int gp_tripG_backward_H_mfma(gp_ctx* ctx, const gp_graph* g, const float* cos_alpha_kj, const float* dz, int O, int S,
                             float* H, const int32_t* row_list = nullptr);
int gp_tripG_grad_cos_mfma(gp_ctx* ctx, const gp_graph* g, const float* cos_alpha_kj, const float* U, const float* dz,
                           int O, int S, int accumulate, float* grad_cos_kj);
// 16-byte vectorised streaming kernels (triplet_stream.hip); return 1 if they handled the call
int gp_stream_fwd_fast(gp_ctx* ctx, const gp_graph* g, int F, const float* x, const float* s, float* a);
int gp_stream_bwd_fast(gp_ctx* ctx, const gp_graph* g, const int32_t* perm_kj, int F, const float* x, const float* s,
                       const float* ga, float* gx, float* gs);
