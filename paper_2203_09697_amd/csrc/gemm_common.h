// Pieces shared by the fp32 and bf16 GEMM kernels (internal): argument block, fused epilogue,
// workgroup-id renumbering.  Everything lives in an anonymous namespace per translation unit.
#pragma once
#include "gemm.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int THREADS = 256;
constexpr int EPI_LD = 36;             // row stride of a wavefront's 32x32 staging block (floats)
enum { MODE_NN = 0, MODE_NT = 1, MODE_TN = 2 };

struct gemm_args {
  const float* A;
  const float* B;
  int64_t M;   // rows of C
  int N, K;    // cols of C, contraction length (TN: total rows to reduce)
  int64_t lda, ldb;
  int vecA, vecB;          // 16-byte vector loads are legal for this operand
  int vecC;                // 16-byte accesses are legal for every matrix the epilogue touches
  int64_t k_per_split;     // TN only
  float* part;             // TN only: [splits, M, N]
  float* colsum_part;      // TN only, optional: [splits * tiles_m, N] partial column sums of B
  gp_epilogue epi;
};

__device__ __forceinline__ void epilogue_store(const gp_epilogue& e, int64_t row, int col, int n, float v) {
  const int64_t o = row * n + col;
  if (e.bias) v += e.bias[col];
  if (e.add_pre) v += e.add_pre[o];
  if (e.save_pre) e.save_pre[o] = v;
  if (e.act == 1) v = silu_f(v);
  else if (e.act == 2) v *= dsilu_f(e.zsrc[o]);
  if (e.mul) v *= e.mul[o];
  if (e.add_post) v += e.add_post[o];
  v *= e.scale;
  if (e.out) e.out[o] = v;
  if (e.out2) e.out2[o] = v * dsilu_f(e.z2src[o]);
}

__device__ __forceinline__ f32x4 ld4(const float* p) { return *reinterpret_cast<const f32x4*>(p); }
__device__ __forceinline__ void st4(float* p, f32x4 v) { *reinterpret_cast<f32x4*>(p) = v; }

// Same steps on 4 consecutive columns (col % 4 == 0, all pointers 16-byte aligned, n % 4 == 0).
__device__ __forceinline__ void epilogue_store4(const gp_epilogue& e, int64_t row, int col, int n, f32x4 v) {
  const int64_t o = row * n + col;
  if (e.bias) v += ld4(e.bias + col);
  if (e.add_pre) v += ld4(e.add_pre + o);
  if (e.save_pre) st4(e.save_pre + o, v);
  if (e.act == 1) {
#pragma unroll
    for (int c = 0; c < 4; ++c) v[c] = silu_f(v[c]);
  } else if (e.act == 2) {
    const f32x4 z = ld4(e.zsrc + o);
#pragma unroll
    for (int c = 0; c < 4; ++c) v[c] *= dsilu_f(z[c]);
  }
  if (e.mul) v *= ld4(e.mul + o);
  if (e.add_post) v += ld4(e.add_post + o);
  v *= e.scale;
  if (e.out) st4(e.out + o, v);
  if (e.out2) {
    const f32x4 z = ld4(e.z2src + o);
#pragma unroll
    for (int c = 0; c < 4; ++c) v[c] *= dsilu_f(z[c]);
    st4(e.out2 + o, v);
  }
}

// wavefront-local ordering of LDS traffic (no other wavefront touches this wave's slice)
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Workgroup ids are dealt round-robin to the 8 XCDs; renumber them so that each XCD works on
// a contiguous range of tiles and neighbouring tiles (same A rows) share that XCD's L2.
__device__ __forceinline__ int xcd_remap(int bid, int n) {
  const int q = n >> 3, r = n & 7;
  const int x = bid & 7, i = bid >> 3;
  return x * q + (x < r ? x : r) + i;
}

}  // namespace
