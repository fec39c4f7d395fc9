/*
 * gpgnn -- single-GPU (gfx950) triplet interaction block for DimeNet++ / GemNet-T
 * style atomic graph networks: the per-GPU work of graph-parallel training
 * (paper Sec. 2.2), i.e. radius-graph construction, triplet enumeration,
 * TripletUpdate + TripletAggr and the edge MLPs around them (Sec. 2.1, 3.3, 3.4),
 * forward and backward.
 *
 * Conventions
 *   - Every function returns GP_OK (0) or a negative gp_status; it never throws
 *     or aborts.  gp_last_error(ctx) gives a human-readable message for the last
 *     failure on that context.
 *   - Unless marked "host", every array pointer is a DEVICE pointer owned by the
 *     caller; the library allocates no user-visible memory.  Temporary storage is
 *     a caller-provided workspace whose size is queried first.
 *   - All work is enqueued on the hipStream_t given to gp_create; only the
 *     *_count calls synchronise (they return a host scalar).
 *   - Arrays are row-major and contiguous.  Indices are int32, counts int64.
 *     A weight matrix is W[in, out]; a layer computes x @ W + b.
 *   - Edge e runs from source src[e] to target dst[e] (message m_st of Sec. 3.1).
 *     A triplet t = (k -> j -> i) is the pair of edges (idx_kj[t], idx_ji[t]).
 */
#ifndef GPGNN_H
#define GPGNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  GP_OK = 0,
  GP_BAD_ARG = -1,           /* null pointer, negative size, inconsistent sizes   */
  GP_BUFFER_TOO_SMALL = -2,  /* workspace smaller than the *_workspace query      */
  GP_INT32_OVERFLOW = -3,    /* edge or triplet count does not fit int32 indices  */
  GP_HIP_ERROR = -4,         /* a HIP runtime call or kernel launch failed        */
  GP_UNSUPPORTED_DIMS = -5   /* layer widths outside what the kernels implement   */
} gp_status;

typedef struct gp_ctx gp_ctx;

/* Context: binds a device and a stream.  hip_stream may be NULL (default stream). */
int gp_create(gp_ctx** out /*host*/, int device_id, void* hip_stream);
void gp_destroy(gp_ctx* ctx);
const char* gp_last_error(const gp_ctx* ctx);
const char* gp_version(void);

/* The block calls issue work that their main chain does not wait for at once on a second, library-owned
 * stream and join it before returning, so callers see single-stream semantics: the weight-gradient GEMMs of
 * the backward passes next to the input-gradient chain; in the variant-D block also the branch through the
 * target-edge projection and, from 2048 edges on, one half of the rows of the layers after the triplet sum
 * (the same arithmetic per row: the forward result does not depend on the setting).
 * gp_set_side_stream(ctx, 0) keeps everything on the context's stream, e.g. to time kernels one
 * at a time; the environment variable GP_NO_AUX_STREAM=1 has the same effect at gp_create. */
int gp_set_side_stream(gp_ctx* ctx, int on);

/* Triplet sums of the bilinear block (Sec. 3.4) with bf16 GEMM operands selected: when gp_graph
 * carries its lists by centre atom they can run as dense products per centre atom on the matrix
 * cores.  mode 1: whenever the widths allow; 0: never (one wavefront per edge on the vector
 * units); -1 (default): only for graphs with at least 96 triplets per edge on average, where the
 * dense form pays; 2: as 1, but the forward sum in its two-kernel form (a kernel writes the per-triplet
 * basis projection y in bf16, a second one contracts it) instead of the one-pass kernel (kept for comparison);
 * 3: as 1, but the one-pass forward kernel evaluates y on the vector units (Horner's rule per value) instead of
 * forming it with a first matrix-core product (kept for comparison).  GP_TRIPLET_MFMA=0..3 in the environment
 * sets the mode at gp_create. */
int gp_set_triplet_mfma(gp_ctx* ctx, int mode);

/* GEMMs with fp32 operands and results (the fp32 blocks, Sec. 3.3; the energy head).  split = 1 (default): on the bf16
 * matrix cores, every operand element entering as three bf16 numbers whose sum is the fp32 value (24 significant
 * bits) and six of the nine plane products accumulated in fp32, the dropped ones below 2^-24 of the product: results
 * agree with fp32 arithmetic to its rounding error, at 2.7 times the fp32-operand matrix-core rate of this chip.
 * split = 0: the fp32-operand matrix-core instruction.  GP_F32_GEMM=0/1 in the environment sets it at gp_create. */
int gp_set_f32_gemm(gp_ctx* ctx, int split);

/* Errors that only a kernel can detect are deferred: a block call given gp_graph.max_in_degree / max_out_degree
 * below the true maxima skips the atoms above them (it never reads out of bounds) and leaves a mark that makes
 * the NEXT block call on the context, or this call, return GP_BAD_ARG with a message.  gp_deferred_status
 * synchronises the context's stream first, so it also reports what the calls still in flight find. */
int gp_deferred_status(gp_ctx* ctx);

/* Measurement aid (not a step of the method): while enabled, every kernel launch the library
 * issues on this context is bracketed by two HIP events on the context's stream.
 * gp_profile_get(i) synchronises on launch i and returns its kernel name (static string),
 * duration in ms, and the algorithmic flops and bytes of that launch.  gp_profile_reset
 * forgets the recorded launches (events are recycled). */
int gp_profile_enable(gp_ctx* ctx, int on);
int gp_profile_reset(gp_ctx* ctx);
int gp_profile_count(gp_ctx* ctx, int64_t* n /*host*/);
int gp_profile_get(gp_ctx* ctx, int64_t i, const char** name /*host*/, float* ms /*host*/,
                   double* flops /*host*/, double* bytes /*host*/);

/* Measurement aid: rates this GPU reaches with the simplest kernels that can reach them, for
 * quoting roofline fractions against measured as well as published peaks: a 16-byte copy of half
 * the workspace into the other half (GB/s, bytes read + written) and register-resident chains
 * of fp32 32x32x2 and bf16 32x32x16 matrix-core instructions (TFLOP/s).  ws: device scratch of at
 * least 64 MiB (contents destroyed).  Synchronises; the three results are host variables. */
int gp_measure_peaks(gp_ctx* ctx, void* ws, size_t ws_bytes, double* copy_gbps /*host*/,
                     double* mfma_f32_tflops /*host*/, double* mfma_bf16_tflops /*host*/);

/* ------------------------------------------------------------------------------------------
 * Graph construction (Sec. 3.1): target atom t gets an edge from every source atom s of the
 * same structure with |x_t - x_s| < cutoff.  The test is the fp32 expression
 *   d2 = ((dx*dx + dy*dy) + dz*dz), dx = x_t - x_s, each operation rounded once (no FMA),
 * compared with cutoff*cutoff in fp32.  If max_neighbors > 0, each target keeps the
 * max_neighbors sources with the smallest key (bits(d2), s).  Open boundaries.
 *
 * Two phases: gp_edges_count computes per-atom in-degrees and row_ptr into the workspace and
 * returns E on the host; the caller allocates; gp_edges_fill (same arguments, same workspace)
 * writes the edge list sorted by (dst, src).
 *   pos[n_atoms,3] f32; graph_ptr[n_graphs+1] i32 (atoms of structure g are
 *   graph_ptr[g]..graph_ptr[g+1]-1); outputs src[E], dst[E], row_ptr[n_atoms+1] (in-edges of
 *   atom i are row_ptr[i]..row_ptr[i+1]-1), dist[E] = |x_dst - x_src| (f32),
 *   unit[E,3] = (x_dst - x_src)/dist.  dist and unit may be NULL.
 * Errors: GP_BAD_ARG, GP_BUFFER_TOO_SMALL, GP_INT32_OVERFLOW, GP_HIP_ERROR.
 */
int gp_edges_workspace(int64_t n_atoms, size_t* bytes /*host*/);
int gp_edges_count(gp_ctx* ctx, const float* pos, const int32_t* graph_ptr, int64_t n_atoms,
                   int32_t n_graphs, float cutoff, int32_t max_neighbors,
                   void* ws, size_t ws_bytes, int64_t* n_edges /*host*/);
int gp_edges_fill(gp_ctx* ctx, const float* pos, const int32_t* graph_ptr, int64_t n_atoms,
                  int32_t n_graphs, float cutoff, int32_t max_neighbors,
                  const void* ws, size_t ws_bytes, int64_t n_edges,
                  int32_t* src, int32_t* dst, int32_t* row_ptr, float* dist, float* unit);

/* ------------------------------------------------------------------------------------------
 * Triplet enumeration (Sec. 3.1; the sum over k in N_j \ {i} in the update equation of
 * Sec. 3.3): for every edge e = (j->i), every edge e' = (k->j) with k != i.
 * Input: an edge list sorted by (dst, src) with its row_ptr (as produced above).
 * Output, "ji-major" order (idx_ji ascending, then idx_kj ascending):
 *   idx_kj[T], idx_ji[T], seg_ptr_ji[E+1] (triplets of target edge e are
 *   seg_ptr_ji[e]..seg_ptr_ji[e+1]-1).
 * Optional "kj-major" view used by the backward pass (all three NULL or all three given):
 *   perm_kj[T]     triplet ids sorted by (idx_kj, idx_ji),
 *   idx_ji_kj[T]   idx_ji[perm_kj[q]],
 *   seg_ptr_kj[E+1] slots of source edge e' are seg_ptr_kj[e']..seg_ptr_kj[e'+1]-1.
 * Errors as above; T > INT32_MAX gives GP_INT32_OVERFLOW.
 */
int gp_triplets_workspace(int64_t n_atoms, int64_t n_edges, size_t* bytes /*host*/);
int gp_triplets_count(gp_ctx* ctx, const int32_t* src, const int32_t* dst, const int32_t* row_ptr,
                      int64_t n_atoms, int64_t n_edges, void* ws, size_t ws_bytes,
                      int64_t* n_triplets /*host*/);
int gp_triplets_fill(gp_ctx* ctx, const int32_t* src, const int32_t* dst, const int32_t* row_ptr,
                     int64_t n_atoms, int64_t n_edges, void* ws, size_t ws_bytes,
                     int64_t n_triplets, int32_t* idx_kj, int32_t* idx_ji, int32_t* seg_ptr_ji,
                     int32_t* perm_kj, int32_t* idx_ji_kj, int32_t* seg_ptr_kj);

/* Opposite edges (Sec. 3.4, symmetric message passing couples m_ji and m_ij): for an edge list
 * sorted by (dst, src) with its row_ptr, id_swap[e] = id of the edge dst[e] -> src[e], or -1 if
 * the list has none (a neighbour cap can keep one direction only).  Exact (integer) result. */
int gp_reverse_edges(gp_ctx* ctx, const int32_t* src, const int32_t* dst,
                     const int32_t* offset /*[E,3] cell offsets of a periodic edge list, or NULL*/,
                     const int32_t* row_ptr, int64_t n_atoms, int64_t n_edges, int32_t* id_swap);

/* ------------------------------------------------------------------------------------------
 * Periodic structures.  cell[G,3,3] (device) holds the lattice vectors of every structure as
 * rows.  The source of an edge may be a periodic image of an atom, x_src + n0 a0 + n1 a1 + n2 a2;
 * the integer triple n is the edge's cell offset (offset[E,3]).  Every image with
 * |n_a| <= rep_a is tested (the caller chooses rep so that rep_a times the cell's height along
 * axis a covers the cutoff; 0..16) with the same fp32 predicate as gp_edges_count on the shifted
 * source position, shift component = fl(fl(fl(n0 a0) + fl(n1 a1)) + fl(n2 a2)), products and sums
 * rounded once each.  The atom itself (n = 0) is not its own neighbour, its images are.
 * Order: (dst, src, n0, n1, n2); cap key: (bits(d2), src, n0, n1, n2).  dist and unit refer to the
 * shifted source.  Triplets k->j->i of a periodic edge list leave out only the image of k that
 * coincides with atom i (same atom, offset_kj = -offset_ji); everything else is as in the
 * open-boundary calls, whose outputs these reproduce when no image is within the cutoff.
 */
int gp_edges_count_pbc(gp_ctx* ctx, const float* pos, const int32_t* graph_ptr, const float* cell,
                       int64_t n_atoms, int32_t n_graphs, float cutoff, int32_t max_neighbors,
                       int32_t rep0, int32_t rep1, int32_t rep2,
                       void* ws, size_t ws_bytes, int64_t* n_edges /*host*/);
int gp_edges_fill_pbc(gp_ctx* ctx, const float* pos, const int32_t* graph_ptr, const float* cell,
                      int64_t n_atoms, int32_t n_graphs, float cutoff, int32_t max_neighbors,
                      int32_t rep0, int32_t rep1, int32_t rep2,
                      const void* ws, size_t ws_bytes, int64_t n_edges,
                      int32_t* src, int32_t* dst, int32_t* offset, int32_t* row_ptr, float* dist, float* unit);
int gp_triplets_count_pbc(gp_ctx* ctx, const int32_t* src, const int32_t* dst, const int32_t* offset,
                          const int32_t* row_ptr, int64_t n_atoms, int64_t n_edges,
                          void* ws, size_t ws_bytes, int64_t* n_triplets /*host*/);
int gp_triplets_fill_pbc(gp_ctx* ctx, const int32_t* src, const int32_t* dst, const int32_t* offset,
                         const int32_t* row_ptr, int64_t n_atoms, int64_t n_edges,
                         void* ws, size_t ws_bytes, int64_t n_triplets,
                         int32_t* idx_kj, int32_t* idx_ji, int32_t* seg_ptr_ji,
                         int32_t* perm_kj, int32_t* idx_ji_kj, int32_t* seg_ptr_kj);

/* Largest row length ptr[i+1] - ptr[i], i < n, of a device-resident offsets array with n+1
 * entries (e.g. the largest in-degree, for gp_graph.max_in_degree).  ws: device scratch of at
 * least 4 bytes.  Synchronises the context's stream; *max_degree is a host variable. */
int gp_csr_max_degree(gp_ctx* ctx, const int32_t* ptr, int64_t n, void* ws, size_t ws_bytes,
                      int32_t* max_degree /*host*/);

/* ------------------------------------------------------------------------------------------
 * Layer widths of one interaction block.
 */
enum { GP_VARIANT_D = 0, GP_VARIANT_G = 1 };   /* Hadamard (Sec. 3.3) / bilinear (Sec. 3.4) */
enum { GP_F32 = 0, GP_BF16_F32ACC = 1 };       /* GEMM operand type; accumulation is fp32   */
#define GP_MAX_RES 4

typedef struct {
  int32_t variant, dtype;
  int32_t emb;            /* edge embedding width                                  */
  int32_t int_emb;        /* triplet width (down-projected); emb_trip in variant G */
  int32_t basis_emb;      /* D: width of the two-step basis projections            */
  int32_t emb_rbf, emb_cbf, emb_bil;   /* G                                        */
  int32_t num_radial, num_spherical, envelope_p;
  int32_t n_res_before, n_res_after;   /* D: residual layers around the skip       */
  int32_t symmetric;                   /* G: 1 = couple the two messages on a bond (Sec. 3.4, symmetric message
                                          passing): needs gp_graph.id_swap and gp_weights_G.W_up_ac */
  int32_t radial_at_target;            /* G: 0 = radial factor of the triplet basis taken at the source
                                          edge k->j; 1 = at the target edge j->i, where it leaves the sum
                                          over k (Sec. 3.4, order of operations of the bilinear layer) */
  float cutoff;
} gp_dims;

/* ------------------------------------------------------------------------------------------
 * Basis functions (Sec. 3.3 names a radial basis of the edge length and a spherical basis of
 * (d_kj, alpha_(kj,ji)); the paper prints no formulas, these are the ones this library computes).
 * With c = cutoff, x = d/c, p = envelope_p, R = num_radial, S = num_spherical:
 *   envelope   u(x) = 1 - (p+1)(p+2)/2 x^p + p(p+2) x^(p+1) - p(p+1)/2 x^(p+2)   (u(1) = u'(1) = u''(1) = 0)
 *   Bessel radial basis (variant D)    rbf_n(d) = u(x) sqrt(2/c) sin(n pi x) / d,          n = 1..R
 *   Gaussian radial basis (variant G)  rbf_n(d) = u(x) exp(-((x - mu_n)/Delta)^2 / 2),     mu_n = n/(R-1), Delta = 1/(R-1), n = 0..R-1
 *   spherical basis (variant D)        sbf_ln(d, alpha) = u(x) N_ln j_l(z_ln x) Y_l0(alpha), l = 0..S-1, n = 1..R,
 *       j_l the spherical Bessel function of the first kind, z_ln its n-th positive zero,
 *       N_ln = sqrt(2 / (c^3 j_(l+1)(z_ln)^2)), Y_l0(alpha) = sqrt((2l+1)/(4 pi)) P_l(cos alpha), P_l the Legendre
 *       polynomial; evaluated in fp64 and rounded once
 *   angular part (variant G)           Y_l0(alpha), l = 0..S-1
 * Arrays:
 *   rbf[E, R]        the radial basis of the variant selected by dims
 *   rad[E, S*R]      D only (else NULL): the radial part u(x) N_ln j_l(z_ln x) of sbf, flat index l*R + (n-1)
 *   cos_alpha[T]     cos of the angle at j between bonds j-i and j-k = -unit[ji].unit[kj]
 *   cos_alpha_kj[T]  the same values in kj-major order (needs perm_kj; may be NULL with it)
 *   sbf[T, S*R]      optional materialised spherical basis rad[idx_kj[t]] * Y_l0(cos_alpha[t])
 * The interaction kernels consume the factored form (rad per edge, cos_alpha per triplet).
 */
int gp_basis_forward(gp_ctx* ctx, const gp_dims* dims, const float* dist, const float* unit,
                     const int32_t* idx_kj, const int32_t* idx_ji, const int32_t* perm_kj,
                     int64_t n_edges, int64_t n_triplets,
                     float* rbf, float* rad, float* cos_alpha, float* cos_alpha_kj, float* sbf);

/* ------------------------------------------------------------------------------------------
 * Interaction block (Sec. 3.3 update equation; EdgeUpdate around TripletUpdate/TripletAggr).
 */
typedef struct {
  int64_t n_edges, n_triplets;
  const int32_t* idx_kj;       /* [T] ji-major */
  const int32_t* seg_ptr_ji;   /* [E+1]        */
  const int32_t* idx_ji_kj;    /* [T] kj-major */
  const int32_t* seg_ptr_kj;   /* [E+1]        */
  /* Optional lists by centre atom (the atom j shared by both edges of a triplet k->j->i); give
   * all of them or leave n_atoms = 0.  With them, and bf16 GEMM operands selected in gp_dims,
   * the bilinear block runs its triplet sums on the matrix cores.  They require what
   * gp_edges_fill / gp_triplets_fill produce: edges sorted by target atom, and idx_kj of the
   * segment of edge j->i equal to the in-edge rows of j in ascending order with at most the
   * row coming from atom i left out.  max_in_degree / max_out_degree must not be below the true
   * maxima: atoms above them are skipped (no access leaves its array) and the block call that notices leaves
   * a deferred GP_BAD_ARG, see gp_deferred_status. */
  int64_t n_atoms;
  int32_t max_in_degree;       /* max over atoms of row_ptr[j+1] - row_ptr[j] */
  int32_t max_out_degree;      /* max over atoms of out_ptr[j+1] - out_ptr[j] */
  const int32_t* row_ptr;      /* [N+1] in-edges of atom j are edge rows row_ptr[j] .. row_ptr[j+1]-1 */
  const int32_t* out_ptr;      /* [N+1] */
  const int32_t* out_list;     /* [E] out_list[out_ptr[j] .. out_ptr[j+1]-1] = ids of the edges whose source is j */
  const int32_t* perm_kj;      /* [T] optional: ji-major id of the triplet in kj-major slot q; needed only by
                                  gp_block_backward_G with radial_at_target = 1 and grad_cos_kj requested */
  const int32_t* id_swap;      /* [E] optional: id of the edge opposite to edge e, -1 if absent (gp_reverse_edges);
                                  needed only by blocks with gp_dims.symmetric = 1 */
} gp_graph;

typedef struct {
  const float* rbf;            /* [E, R]                 */
  const float* rad;            /* [E, S*R]   (D)         */
  const float* cos_alpha;      /* [T] ji-major           */
  const float* cos_alpha_kj;   /* [T] kj-major           */
} gp_basis;

/* Variant D weights, fp32, W[in,out].  The same struct (non-const use) receives gradients. */
typedef struct {
  float *W_ji, *b_ji, *W_kj, *b_kj;            /* [emb,emb],[emb]              */
  float *W_rbf1, *W_rbf2;                      /* [R,basis_emb],[basis_emb,emb] */
  float *W_down;                               /* [emb,int_emb]                */
  float *W_sbf1, *W_sbf2;                      /* [S*R,basis_emb],[basis_emb,int_emb] */
  float *W_up;                                 /* [int_emb,emb]                */
  float *res_before[GP_MAX_RES][4];            /* W1,b1,W2,b2 per residual layer */
  float *W_lin, *b_lin;
  float *res_after[GP_MAX_RES][4];
} gp_weights_D;

/* Bytes of the activation buffer kept from forward to backward, and of scratch space.  n_atoms: gp_graph.n_atoms
 * of the graph the block will run on (0 if it carries no lists by centre atom); a scratch buffer sized with 0 is
 * accepted for any graph, the one-pass matrix-core triplet kernel of the bilinear block then stays unused. */
int gp_block_workspace(const gp_dims* dims, int64_t n_atoms, int64_t n_edges, int64_t n_triplets,
                       size_t* saved_bytes /*host*/, size_t* scratch_bytes /*host*/);

/* m_out[E,emb] = Block(m_in[E,emb]).  `saved` is written for the backward pass. */
int gp_block_forward_D(gp_ctx* ctx, const gp_dims* dims, const gp_weights_D* w,
                       const gp_graph* graph, const gp_basis* basis,
                       const float* m_in, float* m_out,
                       void* saved, size_t saved_bytes, void* scratch, size_t scratch_bytes);

/* grad_m_in[E,emb] and all weight gradients (overwritten, not accumulated) from
 * grad_m_out[E,emb]; `saved` is the buffer the matching forward call filled. */
int gp_block_backward_D(gp_ctx* ctx, const gp_dims* dims, const gp_weights_D* w,
                        const gp_graph* graph, const gp_basis* basis,
                        const float* m_in, const void* saved, size_t saved_bytes,
                        const float* grad_m_out, float* grad_m_in, gp_weights_D* grad_w,
                        void* scratch, size_t scratch_bytes);
/* The same, and the gradient with respect to the basis (forces of the energy-centric model, Sec. 3.2, 3.3):
 * grad_rbf[E, num_radial] = dL/d(radial basis), grad_rad[E, num_spherical, num_radial] = dL/d(radial part of the
 * spherical basis, basis->rad), grad_cos_kj[T] = dL/dcos(alpha) in kj-major order; any of them may be NULL.  With
 * accumulate_basis_grads != 0 they are added to (several blocks share one basis), else overwritten. */
int gp_block_backward_D_basis(gp_ctx* ctx, const gp_dims* dims, const gp_weights_D* w,
                              const gp_graph* graph, const gp_basis* basis,
                              const float* m_in, const void* saved, size_t saved_bytes,
                              const float* grad_m_out, float* grad_m_in, gp_weights_D* grad_w,
                              float* grad_rbf, float* grad_rad, float* grad_cos_kj, int32_t accumulate_basis_grads,
                              void* scratch, size_t scratch_bytes);

/* ------------------------------------------------------------------------------------------
 * Interaction block, variant G (Sec. 3.4: a bilinear layer replaces the Hadamard product; the
 * order of operations is chosen so that no tensor of size T x width is stored):
 *   x = act(m W_ba) * (g (W_rbfS W_rbfB));  x = act(x W_down)            [E, int_emb]
 *   Rad[e,l,c] = sum_n g[e,n] W_c[l,n,c];   y_t[c] = sum_l Y_l0(cos alpha_t) Rad[kj(t),l,c]
 *   A_e[c,f]   = sum_{t in seg_ji(e)} y_t[c] x[kj(t),f];   z_e[o] = sum_{c,f} A_e[c,f] W_bil[c,f,o]
 *   m' = (act(m W_skip) + act(z W_up)) / sqrt(2)
 * basis->rbf is the Gaussian radial basis g[E, num_radial]; basis->rad is unused.
 * Weights fp32, W[in,out]: W_ba[emb,emb], W_rbfS[R,emb_rbf], W_rbfB[emb_rbf,emb],
 * W_down[emb,int_emb], W_c[S,R,emb_cbf], W_bil[emb_cbf,int_emb,emb_bil], W_up[emb_bil,emb],
 * W_skip[emb,emb].  gp_block_workspace sizes `saved` and `scratch` for this variant too.
 * Backward overwrites grad_m_in and every member of grad_w.  For forces (Sec. 3.2) it can also
 * return the gradient with respect to the basis: grad_rbf[E, num_radial] = dL/dg and
 * grad_cos_kj[T] = dL/dcos(alpha) in kj-major order (either may be NULL); with
 * accumulate_basis_grads != 0 they are added to (several blocks share one basis), else overwritten.
 */
typedef struct {
  float *W_ba, *W_rbfS, *W_rbfB, *W_down, *W_c, *W_bil, *W_up, *W_skip;
  float *W_up_ac;   /* [emb_bil, emb]; symmetric = 1 only (else ignored, may be NULL):
                       m' = (act(m W_skip) + (act(z W_up) + act(z W_up_ac)[id_swap]) / sqrt(2)) / sqrt(2),
                       the gathered term being zero where id_swap < 0 */
} gp_weights_G;

int gp_block_forward_G(gp_ctx* ctx, const gp_dims* dims, const gp_weights_G* w,
                       const gp_graph* graph, const gp_basis* basis,
                       const float* m_in, float* m_out,
                       void* saved, size_t saved_bytes, void* scratch, size_t scratch_bytes);
int gp_block_backward_G(gp_ctx* ctx, const gp_dims* dims, const gp_weights_G* w,
                        const gp_graph* graph, const gp_basis* basis,
                        const float* m_in, const void* saved, size_t saved_bytes,
                        const float* grad_m_out, float* grad_m_in, gp_weights_G* grad_w,
                        float* grad_rbf, float* grad_cos_kj, int32_t accumulate_basis_grads,
                        void* scratch, size_t scratch_bytes);

/* The same two calls for a stack of bilinear blocks with bf16 GEMM operands (Sec. 3.4; Sec. 4.5 stacks several blocks).
 * Such a block reads its input messages only as bf16 GEMM operands, so the block below can hand them over in that
 * storage: with m_out_bf16 != 0, m_out receives [E, emb] bf16 values (the fp32 result rounded to nearest even, i.e.
 * exactly what the next block would round it to) instead of fp32; with m_in_bf16 != 0, m_in is such a matrix and the
 * rounding pass over it is skipped; the backward call of that block must be given the same m_in with the same flag.
 * Likewise for the gradients in the backward pass: grad_m_in_bf16 != 0 stores grad_m_in as bf16, grad_m_out_bf16 != 0
 * reads grad_m_out as bf16 (this rounds a gradient once more than the fp32 hand-over does; not available for
 * symmetric blocks, whose opposite-edge gather reads fp32).  All flags 0: identical to the calls above.
 * gp_block_G_stacks_bf16(dims) returns 1 when dims allow the flags (variant G, bf16 operands, emb a multiple of 8,
 * even int_emb and emb_bil), else 0; a flag given for other dims fails with GP_BAD_ARG.  Everything else (pointers on the
 * device, sizes, ownership, errors) as for gp_block_forward_G / gp_block_backward_G. */
int gp_block_G_stacks_bf16(const gp_dims* dims);
int gp_block_forward_G_stacked(gp_ctx* ctx, const gp_dims* dims, const gp_weights_G* w,
                               const gp_graph* graph, const gp_basis* basis,
                               const void* m_in, int32_t m_in_bf16, void* m_out, int32_t m_out_bf16,
                               void* saved, size_t saved_bytes, void* scratch, size_t scratch_bytes);
int gp_block_backward_G_stacked(gp_ctx* ctx, const gp_dims* dims, const gp_weights_G* w,
                                const gp_graph* graph, const gp_basis* basis,
                                const void* m_in, int32_t m_in_bf16, const void* saved, size_t saved_bytes,
                                const void* grad_m_out, int32_t grad_m_out_bf16, void* grad_m_in, int32_t grad_m_in_bf16,
                                gp_weights_G* grad_w, float* grad_rbf, float* grad_cos_kj,
                                int32_t accumulate_basis_grads, void* scratch, size_t scratch_bytes);

/* ------------------------------------------------------------------------------------------
 * Energy head (Sec. 3.3 output step: messages summed per target atom, then an MLP) and forces
 * (Sec. 3.2, energy-centric: f = -dE/dx by back-propagation).
 *   h_i = sum_{e: dst[e]=i} m_e;  E_i = w2 . act(h_i W1 + b1) + b2;  energy[g] = sum_{i in g} E_i
 * W1[emb,hidden], b1[hidden], w2[hidden], b2[1]; energy[n_graphs] is a device array.
 * gp_energy_backward differentiates sum_g energy[g]: grad_m[E,emb] (overwritten) and, if
 * grad_w != NULL, the head's weight gradients.
 */
typedef struct {
  float *W1, *b1, *w2, *b2;
} gp_weights_head;

int gp_energy_workspace(int32_t emb, int32_t hidden, int64_t n_atoms,
                        size_t* saved_bytes /*host*/, size_t* scratch_bytes /*host*/);
int gp_energy_forward(gp_ctx* ctx, int32_t emb, int32_t hidden, const gp_weights_head* w,
                      const float* m, const int32_t* row_ptr, const int32_t* graph_ptr,
                      int64_t n_atoms, int32_t n_graphs, float* energy,
                      void* saved, size_t saved_bytes);
int gp_energy_backward(gp_ctx* ctx, int32_t emb, int32_t hidden, const gp_weights_head* w,
                       const int32_t* dst, int64_t n_atoms, int64_t n_edges,
                       const void* saved, size_t saved_bytes, float* grad_m,
                       gp_weights_head* grad_w, void* scratch, size_t scratch_bytes);

/* ------------------------------------------------------------------------------------------
 * Output block (Sec. 3.3: the updated messages are fed to an output block that sums them per
 * atom, EdgeAggr, and transforms the sum by an MLP, NodeUpdate), one per interaction block:
 *   t_e = m_e * (rbf_e W_rbf);  h_i = sum_{e: dst[e]=i} t_e;  u = h W_up;
 *   u = act(u W[k] + b[k]), k < n_layers;  P_i = u_i . w_final;  energy[g] (+)= sum_{i in g} P_i
 * W_rbf[num_radial, emb], W_up[emb, out_emb], W[k][out_emb, out_emb], b[k][out_emb],
 * w_final[out_emb]; energy[n_graphs] is a device array, overwritten unless accumulate != 0 (the
 * model's energy is the sum over its output blocks).  m[E, emb] are the block's output
 * messages, rbf[E, num_radial] the radial basis, row_ptr/dst/graph_ptr as produced by
 * gp_edges_fill.  gp_output_backward differentiates sum_g grad_energy[g] * energy[g]:
 * grad_m[E, emb] is overwritten, or added to if accumulate_grad_m != 0 (the gradient arriving
 * from the next interaction block), and grad_w (may be NULL) receives the weight gradients.
 * saved is written by the forward call and read by the backward call; scratch is free between
 * calls.  Errors: GP_UNSUPPORTED_DIMS for widths above 4096 or more than GP_MAX_OUT_LAYERS
 * layers, GP_BUFFER_TOO_SMALL, GP_BAD_ARG for NULL pointers.
 */
#define GP_MAX_OUT_LAYERS 4
typedef struct {
  float *W_rbf, *W_up;
  float *W[GP_MAX_OUT_LAYERS], *b[GP_MAX_OUT_LAYERS];
  float *w_final;
} gp_weights_out;

int gp_output_workspace(int32_t emb, int32_t out_emb, int32_t num_radial, int32_t n_layers,
                        int64_t n_atoms, int64_t n_edges,
                        size_t* saved_bytes /*host*/, size_t* scratch_bytes /*host*/);
int gp_output_forward(gp_ctx* ctx, int32_t emb, int32_t out_emb, int32_t num_radial, int32_t n_layers,
                      const gp_weights_out* w, const float* m, const float* rbf,
                      const int32_t* row_ptr, const int32_t* graph_ptr,
                      int64_t n_atoms, int64_t n_edges, int32_t n_graphs, int32_t accumulate,
                      float* energy, void* saved, size_t saved_bytes, void* scratch, size_t scratch_bytes);
int gp_output_backward(gp_ctx* ctx, int32_t emb, int32_t out_emb, int32_t num_radial, int32_t n_layers,
                       const gp_weights_out* w, const float* m, const float* rbf,
                       const int32_t* dst, const int32_t* graph_ptr,
                       int64_t n_atoms, int64_t n_edges, int32_t n_graphs, const float* grad_energy,
                       const void* saved, size_t saved_bytes, int32_t accumulate_grad_m, float* grad_m,
                       gp_weights_out* grad_w, void* scratch, size_t scratch_bytes);

/* Out-edge lists: out_list[out_ptr[j]..out_ptr[j+1]-1] are the ids of the edges whose source is
 * atom j, ascending.  (The edge list itself is sorted by target.) */
int gp_edges_by_source_workspace(int64_t n_atoms, int64_t n_edges, size_t* bytes /*host*/);
int gp_edges_by_source(gp_ctx* ctx, const int32_t* src, int64_t n_atoms, int64_t n_edges,
                       void* ws, size_t ws_bytes, int32_t* out_ptr, int32_t* out_list);

/* The same lists for callers that cannot allocate device memory or hand over a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the counters and the unsorted list live in a
 * static device array inside the library (about 8.5 MiB per GPU, held until the process ends), so the call takes
 * only inputs and outputs, allocates nothing and records no memset node (it clears its counters with a kernel).
 * Limits: n_atoms <= 65536 and n_edges <= 2097152, beyond which it returns GP_UNSUPPORTED_DIMS; results are
 * identical to gp_edges_by_source.  All calls on one GPU share that array: calls that overlap on one GPU (different
 * streams or contexts) race and must be serialised by the caller.  GP_HIP_ERROR if the array's address could not
 * be obtained on the context's device. */
int gp_edges_by_source_static(gp_ctx* ctx, const int32_t* src, int64_t n_atoms, int64_t n_edges,
                              int32_t* out_ptr, int32_t* out_list);

/* forces[N,3] = -dL/dx given dL/dg (grad_rbf[E,R], Gaussian radial basis of variant G) and
 * dL/dcos(alpha) (grad_cos_kj[T], kj-major), with the graph held fixed:
 *   d d_e/dx_dst = u_e, d d_e/dx_src = -u_e;  cos(alpha_t) = -u_ji . u_kj, u_e = (x_dst-x_src)/d_e.
 * No atomics: per-edge vector gradients are sorted-segment sums over the two triplet views,
 * per-atom sums run over the in-edge rows and the out-edge lists. */
int gp_forces_workspace(int64_t n_edges, int64_t n_triplets, size_t* bytes /*host*/);
int gp_forces_from_basis_grad(gp_ctx* ctx, const gp_dims* dims, const gp_graph* graph,
                              const int32_t* perm_kj, const int32_t* row_ptr,
                              const int32_t* out_ptr, const int32_t* out_list, int64_t n_atoms,
                              const float* dist, const float* unit, const float* grad_rbf,
                              const float* grad_cos_kj, float* forces, void* ws, size_t ws_bytes);
/* The same for variant D (Sec. 3.2, 3.3: forces of the energy-centric Hadamard model): grad_rbf[E,R] is the gradient
 * with respect to the Bessel radial basis, grad_rad[E,S,R] with respect to the radial part of the spherical basis
 * (basis->rad), both as gp_block_backward_D_basis returns them; same workspace. */
int gp_forces_from_basis_grad_D(gp_ctx* ctx, const gp_dims* dims, const gp_graph* graph,
                                const int32_t* perm_kj, const int32_t* row_ptr,
                                const int32_t* out_ptr, const int32_t* out_list, int64_t n_atoms,
                                const float* dist, const float* unit, const float* grad_rbf, const float* grad_rad,
                                const float* grad_cos_kj, float* forces, void* ws, size_t ws_bytes);

/* ------------------------------------------------------------------------------------------
 * The core TripletUpdate + TripletAggr kernels on their own (Sec. 3.3: Hadamard product of the
 * gathered message with the projected basis, summed over k into edge j->i).
 *   Streaming form (GP_TRIPLET_STREAM): s[T,F] is a materialised per-triplet basis projection (ji-major),
 *     a[e,f] = sum_{t in seg_ji(e)} x[idx_kj[t], f] * s[t, f].
 *   Backward: grad_x[e',f] = sum_{t: kj(t)=e'} grad_a[ji(t),f] * s[t,f]   (kj-major walk)
 *             grad_s[t,f]  = grad_a[ji(t),f] * x[kj(t),f].
 */
int gp_triplet_aggregate_fwd(gp_ctx* ctx, const gp_graph* graph, int32_t width,
                             const float* x, const float* s, float* a);
int gp_triplet_aggregate_bwd(gp_ctx* ctx, const gp_graph* graph, const int32_t* perm_kj,
                             int32_t width, const float* x, const float* s, const float* grad_a,
                             float* grad_x, float* grad_s);

/* The same two steps in the forms the interaction blocks run, which never materialise a per-triplet tensor: the
 * basis projection of a triplet is recomputed from cos_alpha (4 bytes per triplet) and a per-edge table.
 *   form GP_TRIPLET_PER_EDGE   one wavefront per target edge (forward) or source edge (backward), fp32 vector units
 *   form GP_TRIPLET_PER_ATOM   the sums regrouped by centre atom j (all out-edges of j sum over the same in-edge rows)
 *                              into dense products on the matrix cores; needs the lists by centre atom of gp_graph
 *   form GP_TRIPLET_PER_ATOM_TWO_KERNELS   bilinear forward only: the earlier two-kernel form with a per-triplet
 *                              buffer of the projection in bf16 (kept for comparison)
 * Tables are stored transposed, one line per (l, b): Qt[(l*basis_emb + b)*E + e], Radt[(l*emb_cbf + c)*E + e].
 * Y_l0 are the spherical harmonics of the basis comment above.  ws: gp_triplet_workspace(graph, width) bytes
 * (may be NULL for the per-edge forms).  Errors: GP_BAD_ARG, GP_UNSUPPORTED_DIMS (widths a form does not
 * implement, stated in the message), GP_BUFFER_TOO_SMALL.
 *
 * Hadamard form (Sec. 3.3), fp32:  p_t[b] = sum_l Y_l0(cos alpha_t) Q[kj(t), l, b];  s_t[f] = sum_b p_t[b] W_sbf2[b, f]
 *   forward   a[e, f] = sum_{t in seg_ji(e)} x[kj(t), f] s_t[f];   Bacc[e, b, f] = sum_t p_t[b] x[kj(t), f]
 *             (Bacc may be NULL in the per-atom form, which needs basis_emb = 8 and width 32, 64, 96 or 128)
 *   backward  grad_x[e', f] = sum_{t: kj(t)=e'} grad_a[ji(t), f] s_t[f]
 *             grad_Q[e', l, b] (stored [E, S, basis_emb]) = sum_{t: kj(t)=e'} Y_l0(t) sum_f W_sbf2[b, f] grad_a[ji(t), f] x[e', f]
 *             grad_W_sbf2[b, f] = sum_e grad_a[e, f] Bacc[e, b, f]    (per-atom form only; NULL in the per-edge form)
 * Bilinear form (Sec. 3.4):  y_t[c] = sum_l Y_l0(cos alpha_t) Rad[kj(t), l, c]
 *   forward   A[e, c, f] = sum_{t in seg_ji(e)} y_t[c] x[kj(t), f]   (fp32 result; the per-atom forms round x and y to
 *             bf16 on their way into the matrix cores and need emb_cbf <= 16, width 32, 64 or 128)
 *   backward  H[e', l, o] = sum_{t: kj(t)=e'} Y_l0(cos alpha_t) dz[ji(t), o]   (dz[E, width]: gradient of the block's
 *             bilinear result; everything else of the block's backward pass follows from H per edge)
 *             grad_cos_kj[q] (+)= sum_l Y_l0'(cos alpha_q) sum_o dz[ji(q), o] U[kj(q), l, o]   (U[E, S, width]; kj-major) */
enum { GP_TRIPLET_STREAM = 0, GP_TRIPLET_PER_EDGE = 1, GP_TRIPLET_PER_ATOM = 2, GP_TRIPLET_PER_ATOM_TWO_KERNELS = 3 };
int gp_triplet_workspace(const gp_graph* graph, int32_t width, size_t* bytes /*host*/);
int gp_triplet_hadamard_fwd(gp_ctx* ctx, const gp_graph* graph, int32_t form, int32_t num_spherical, int32_t basis_emb,
                            int32_t width, const float* cos_alpha, const float* x, const float* Qt, const float* W_sbf2,
                            float* a, float* Bacc);
int gp_triplet_hadamard_bwd(gp_ctx* ctx, const gp_graph* graph, int32_t form, int32_t num_spherical, int32_t basis_emb,
                            int32_t width, const float* cos_alpha_kj, const float* x, const float* Qt, const float* W_sbf2,
                            const float* grad_a, float* grad_x, float* grad_Q, float* grad_W_sbf2, void* ws, size_t ws_bytes);
int gp_triplet_bilinear_fwd(gp_ctx* ctx, const gp_graph* graph, int32_t form, int32_t num_spherical, int32_t emb_cbf,
                            int32_t width, const float* cos_alpha, const float* x, const float* Radt, float* A,
                            void* ws, size_t ws_bytes);
int gp_triplet_bilinear_bwd_H(gp_ctx* ctx, const gp_graph* graph, int32_t form, int32_t num_spherical, int32_t width,
                              const float* cos_alpha_kj, const float* dz, float* H, void* ws, size_t ws_bytes);
int gp_triplet_bilinear_grad_cos(gp_ctx* ctx, const gp_graph* graph, int32_t form, int32_t num_spherical, int32_t width,
                                 const float* cos_alpha_kj, const float* U, const float* dz, int32_t accumulate,
                                 float* grad_cos_kj, void* ws, size_t ws_bytes);

/* Dense layer on its own: out = act(x @ W + b), fp32 MFMA.  act: 0 none, 1 SiLU.
 * x[rows,k], W[k,n], b[n] or NULL, out[rows,n]. */
int gp_linear_forward(gp_ctx* ctx, const float* x, const float* W, const float* b,
                      int64_t rows, int32_t k, int32_t n, int32_t act, float* out);
/* The same layer with x and W rounded to bf16 on load (bf16 MFMA, fp32 accumulate and output),
 * the operand type the bilinear block uses when gp_dims.dtype == GP_BF16_F32ACC. */
int gp_linear_forward_bf16(gp_ctx* ctx, const float* x, const float* W, const float* b,
                           int64_t rows, int32_t k, int32_t n, int32_t act, float* out);

#ifdef __cplusplus
}
#endif
#endif /* GPGNN_H */
