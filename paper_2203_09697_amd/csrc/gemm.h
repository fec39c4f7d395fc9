// Dense fp32 building blocks used by the interaction block (internal, not part of the C ABI).
#pragma once
#include "common.h"

// What happens to an accumulator value v at (row, col) before it is stored.  Steps run in
// this order; null pointers / zero flags skip a step.  All matrices are [rows, n] row-major.
struct gp_epilogue {
  const float* bias = nullptr;      // v += bias[col]
  const float* add_pre = nullptr;   // v += add_pre[row,col]
  float* save_pre = nullptr;        // save_pre[row,col] = v            (pre-activation)
  int act = 0;                      // 1: v = silu(v); 2: v *= silu'(zsrc[row,col])
  const float* zsrc = nullptr;
  const float* mul = nullptr;       // v *= mul[row,col]
  const float* add_post = nullptr;  // v += add_post[row,col]
  // v *= sum_{k < lr_k} lr_a[row, k] lr_b[k, col]: a factor of rank lr_k <= 16 evaluated in the epilogue (lr_a to 16
  // bits as two bf16 terms, lr_b rounded to bf16, fp32 sum, two matrix-core instructions per 32x32 block) instead of
  // read from an [rows, n] matrix.
  // Takes the place of `mul` in the order of steps; only where gp_gemm_nt_takes_lowrank says so.
  const float* lr_a = nullptr;      // fp32 [rows, lr_k]
  const float* lr_b = nullptr;      // fp32 [lr_k, n]
  int lr_k = 0;
  float scale = 1.0f;               // v *= scale
  float* out = nullptr;             // out[row,col] = v
  float* out2 = nullptr;            // out2[row,col] = v * silu'(z2src[row,col])
  const float* z2src = nullptr;
  // Storage type of the [rows, n] matrices above: a set bit means the pointer addresses bf16
  // elements (2 bytes, round-to-nearest-even on store) instead of fp32; bias is always fp32.
  // Only the bf16-operand GEMM kernels accept a non-zero mask.
  unsigned bf16 = 0;
};
enum : unsigned {
  EPI_BF_ADD_PRE = 1u, EPI_BF_SAVE_PRE = 2u, EPI_BF_ZSRC = 4u, EPI_BF_MUL = 8u, EPI_BF_ADD_POST = 16u,
  EPI_BF_OUT = 32u, EPI_BF_OUT2 = 64u, EPI_BF_Z2SRC = 128u
};

// C = A[M,K] @ B[K,N]
// a_bf16 (bf16-operand kernels only): A addresses bf16 elements instead of fp32
int gp_gemm_nn(gp_ctx* ctx, const float* A, const float* B, int64_t M, int N, int K, const gp_epilogue& epi, int a_bf16 = 0,
               int b_bf16 = 0);
// C = A[M,K] @ Bt[N,K]^T
int gp_gemm_nt(gp_ctx* ctx, const float* A, const float* Bt, int64_t M, int N, int K, const gp_epilogue& epi, int a_bf16 = 0,
               int b_bf16 = 0);
// whether gp_gemm_nt with these shapes and bf16 operands runs in the kernel whose epilogue evaluates lr_a, lr_b
bool gp_gemm_nt_takes_lowrank(const gp_ctx* ctx, int64_t M, int N, int K);
// out = A[M,K] @ Bt[N,K]^T + A2[M,K] @ B2t[N,K]^T (fp32 result, no other epilogue step).  With tall bf16 operands this is
// ONE launch of the global->LDS kernel whose contraction runs over both pairs, so the result is written once instead
// of written, read back and written again; otherwise two launches, the second adding to the first's result.
// out_bf16: the result is stored as bf16 (bf16-operand kernels only).
int gp_gemm_nt2(gp_ctx* ctx, const float* A, const float* Bt, const float* A2, const float* B2t, int64_t M, int N, int K,
                float* out, int a_bf16 = 0, int b_bf16 = 0, int out_bf16 = 0);
// out[M,N] = A[rows,M]^T @ B[rows,N]; deterministic two-stage reduction through `part`.
// If colsum_out != NULL it also receives colsum_out[n] = sum_r B[r,n] (the bias gradient).
size_t gp_gemm_tn_scratch(int64_t rows, int M, int N);
int gp_gemm_tn(gp_ctx* ctx, const float* A, const float* B, int64_t rows, int M, int N, float* out,
               float* colsum_out, float* part, size_t part_bytes, int a_bf16 = 0, int b_bf16 = 0);
// out[n] = sum_r X[r,n]
size_t gp_colsum_scratch(int64_t rows, int N);
int gp_colsum(gp_ctx* ctx, const float* X, int64_t rows, int N, float* out, float* part, size_t part_bytes);

// elementwise helpers, n elements
int gp_ew_dsilu_mul(gp_ctx* ctx, const float* g, const float* z, float* out, int64_t n);   // out = g * silu'(z)
int gp_ew_gate_bwd(gp_ctx* ctx, const float* dxg, const float* z, const float* gate, float* dz, float* dgate,
                   int64_t n);   // dz = dxg*gate*silu'(z), dgate = dxg*silu(z)
int gp_ew_add3(gp_ctx* ctx, const float* a, const float* b, const float* c, float* out, int64_t n);  // c may be NULL
// bf16-operand kernels (gemm_bf16.hip); mode 0 NN, 1 NT, 2 TN; args is the fp32 path's argument block
int gp_gemm_bf16_launch(gp_ctx* ctx, int mode, void* args, int splits);
// fp32 operands and result on the bf16 matrix cores, each operand as three bf16 planes (gemm_bf16.hip)
int gp_gemm_split_launch(gp_ctx* ctx, int mode, void* args, int splits);
bool gp_gemm_split_tn_ok(int64_t M, int N, int vecA, int vecB);   // whether A^T B of this shape runs in that form
// A^T B with both operands bf16 through global->LDS loads and LDS transpose reads: number of splits of its plan (0: the
// shape is not taken), whether the filled argument block qualifies, launch
int gp_gemm_bf16_tn_dl_splits(int64_t rows, int M, int N);
bool gp_gemm_bf16_tn_dl_ok(const void* args);
int gp_gemm_bf16_tn_dl(gp_ctx* ctx, void* args, int splits);
// While alive, GEMMs issued on the context round their operands to bf16 if `on`.
struct gp_bf16_scope {
  gp_ctx* c;
  bool prev;
  gp_bf16_scope(gp_ctx* ctx, bool on) : c(ctx), prev(ctx->gemm_bf16) { c->gemm_bf16 = on; }
  ~gp_bf16_scope() { c->gemm_bf16 = prev; }
};
// out[i] = sum_z part[z*n + i], z < splits
int gp_reduce_parts(gp_ctx* ctx, const float* part, int splits, int64_t n, float* out);
