// Pieces shared by the fp32 and bf16 GEMM kernels (internal): argument block, fused epilogue,
// workgroup-id renumbering.  Everything lives in an anonymous namespace per translation unit.
#pragma once
#include "gemm.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int THREADS = 256;
constexpr int EPI_LD = 36;             // row stride of a wavefront's 32x32 staging block (floats)
constexpr int EPI_LD2 = 68;            // ... of a 32x64 staging block (two blocks side by side)
enum { MODE_NN = 0, MODE_NT = 1, MODE_TN = 2 };

struct gemm_args {
  const float* A;
  const float* B;
  int64_t M;   // rows of C
  int N, K;    // cols of C, contraction length (TN: total rows to reduce)
  int64_t lda, ldb;
  int vecA, vecB;          // 16-byte vector loads are legal for this operand
  int vecC;                // 16-byte accesses are legal for every matrix the epilogue touches
  int a_bf16, b_bf16;      // operand storage is bf16 (bf16-operand kernels only)
  int64_t k_per_split;     // TN only
  float* part;             // TN only: [splits, M, N]
  float* colsum_part;      // TN only, optional: [splits * tiles_m, N] partial column sums of B
  // NT only, optional second operand pair: C = A B^T + A2 B2^T, each contraction K / 2 long (same leading dimensions);
  // taken by the global->LDS kernel, which walks the second pair's slabs after the first's
  const float* A2 = nullptr;
  const float* B2 = nullptr;
  gp_epilogue epi;
  int epi_kind = 0;        // EK_*: which fixed sequence of epilogue steps `epi` amounts to (set by gp_epilogue_kind on the host)
  unsigned epi_mask = 0;   // EM_*: the steps present when every matrix is fp32 (0: take the general loop); fp32 kernels
};

// fp32 kernels: the steps present as a bit mask; the kernel switches once per tile over the masks listed in
// GP_EM_LIST (those of the variant-D block) to a loop compiled for that mask
enum : unsigned { EM_BIAS = 1, EM_ADD_PRE = 2, EM_SAVE_PRE = 4, EM_ACT1 = 8, EM_ACT2 = 16, EM_MUL = 32, EM_ADD_POST = 64, EM_SCALE = 128,
                  EM_OUT = 256, EM_OUT2 = 512 };
#define GP_EM_LIST(X) X(256) X(269) X(333) X(272) X(320) X(832) X(301) X(268) X(332) X(768) X(322)
inline unsigned gp_epilogue_mask(const gp_epilogue& e, int vecC) {
  if (!vecC || e.bf16 || e.lr_a) return 0;
  return (e.bias ? EM_BIAS : 0u) | (e.add_pre ? EM_ADD_PRE : 0u) | (e.save_pre ? EM_SAVE_PRE : 0u) | (e.act == 1 ? EM_ACT1 : 0u) |
         (e.act == 2 ? EM_ACT2 : 0u) | (e.mul ? EM_MUL : 0u) | (e.add_post ? EM_ADD_POST : 0u) | (e.scale != 1.0f ? EM_SCALE : 0u) |
         (e.out ? EM_OUT : 0u) | (e.out2 ? EM_OUT2 : 0u);
}

// The epilogue is a list of optional steps; tested inside the store loop, the options cost some forty branches per 4
// values and made the epilogue as long as a third of a 1024-deep main loop.  The combinations the blocks use are
// therefore recognised on the host and the tile epilogue switches ONCE per tile to a loop compiled for that combination;
// anything else takes the general loop.
enum {
  EK_GENERIC = 0,
  EK_OUT_F32,                 // out (fp32)
  EK_OUT_BF16,                // out (bf16)
  EK_PRE_SILU_BF16,           // save_pre (bf16), SiLU, out (bf16)
  EK_PRE_SILU_LR_BF16,        // save_pre (bf16), SiLU, times the low-rank factor, out (bf16)
  EK_PRE_SILU_ADD_F32,        // save_pre (bf16), SiLU, + add_post (bf16), times scale, out (fp32)
  EK_DSILU_BF16,              // times SiLU'(zsrc) (fp32), out (bf16)
  EK_PRE_SILU_F32,            // save_pre (fp32), SiLU, out (fp32)
  EK_PRE_SILU_ADD_BF16,       // save_pre (bf16), SiLU, + add_post (bf16), times scale, out (bf16)
};
inline int gp_epilogue_kind(const gp_epilogue& e, int vecC) {
  if (!vecC || e.bias || e.add_pre || e.out2 || e.mul || !e.out) return EK_GENERIC;
  const unsigned b = e.bf16;
  if (e.act == 2)
    return (!e.save_pre && !e.lr_a && !e.add_post && e.scale == 1.0f && e.zsrc && !(b & EPI_BF_ZSRC) && (b & EPI_BF_OUT)) ? EK_DSILU_BF16
                                                                                                                        : EK_GENERIC;
  if (!e.save_pre && e.act == 0 && !e.lr_a && !e.add_post && e.scale == 1.0f)
    return (b & EPI_BF_OUT) ? EK_OUT_BF16 : EK_OUT_F32;
  if (e.save_pre && b == 0u && e.act == 1 && !e.add_post && !e.lr_a && e.scale == 1.0f) return EK_PRE_SILU_F32;
  if (e.save_pre && (b & EPI_BF_SAVE_PRE) && e.act == 1) {
    if (!e.add_post && e.scale == 1.0f && (b & EPI_BF_OUT)) return e.lr_a ? EK_PRE_SILU_LR_BF16 : EK_PRE_SILU_BF16;
    if (e.add_post && (b & EPI_BF_ADD_POST) && !e.lr_a) return (b & EPI_BF_OUT) ? EK_PRE_SILU_ADD_BF16 : EK_PRE_SILU_ADD_F32;
  }
  return EK_GENERIC;
}

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x4 ld4(const float* p) { return *reinterpret_cast<const f32x4*>(p); }
// Epilogue outputs are streamed: [E, N] matrices far larger than the caches, read next by another kernel.  Non-temporal
// stores measured 1-3 % faster on the store-bound layers and nowhere slower.
__device__ __forceinline__ void st4(float* p, f32x4 v) { __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(p)); }

// element o of a matrix stored as fp32 or (bf) bf16
__device__ __forceinline__ float ldx(const float* p, int64_t o, unsigned bf) {
  return bf ? (float)reinterpret_cast<const __bf16*>(p)[o] : p[o];
}
__device__ __forceinline__ void stx(float* p, int64_t o, unsigned bf, float v) {
  if (bf) reinterpret_cast<__bf16*>(p)[o] = (__bf16)v;
  else p[o] = v;
}
// 4 consecutive elements from o (o % 4 == 0, base 16-byte aligned)
__device__ __forceinline__ f32x4 ldx4(const float* p, int64_t o, unsigned bf) {
  if (!bf) return ld4(p + o);
  const bf16x4 h = *reinterpret_cast<const bf16x4*>(reinterpret_cast<const __bf16*>(p) + o);
  f32x4 v;
#pragma unroll
  for (int c = 0; c < 4; ++c) v[c] = (float)h[c];
  return v;
}
__device__ __forceinline__ void stx4(float* p, int64_t o, unsigned bf, f32x4 v) {
  if (!bf) {
    st4(p + o, v);
    return;
  }
  bf16x4 h;
#pragma unroll
  for (int c = 0; c < 4; ++c) h[c] = (__bf16)v[c];
  __builtin_nontemporal_store(h, reinterpret_cast<bf16x4*>(reinterpret_cast<__bf16*>(p) + o));
}

__device__ __forceinline__ void epilogue_store(const gp_epilogue& e, int64_t row, int col, int n, float v) {
  const int64_t o = row * n + col;
  const unsigned b = e.bf16;
  if (e.bias) v += e.bias[col];
  if (e.add_pre) v += ldx(e.add_pre, o, b & EPI_BF_ADD_PRE);
  if (e.save_pre) stx(e.save_pre, o, b & EPI_BF_SAVE_PRE, v);
  if (e.act == 1) v = silu_f(v);
  else if (e.act == 2) v *= dsilu_f(ldx(e.zsrc, o, b & EPI_BF_ZSRC));
  if (e.mul) v *= ldx(e.mul, o, b & EPI_BF_MUL);
  if (e.add_post) v += ldx(e.add_post, o, b & EPI_BF_ADD_POST);
  v *= e.scale;
  if (e.out) stx(e.out, o, b & EPI_BF_OUT, v);
  if (e.out2) stx(e.out2, o, b & EPI_BF_OUT2, v * dsilu_f(ldx(e.z2src, o, b & EPI_BF_Z2SRC)));
}

// Same steps on 4 consecutive columns (col % 4 == 0, all pointers 16-byte aligned, n % 4 == 0).
// mulv: the low-rank factor's four values, where the kernel evaluates one
__device__ __forceinline__ void epilogue_store4(const gp_epilogue& e, int64_t row, int col, int n, f32x4 v, const f32x4* mulv = nullptr) {
  const int64_t o = row * n + col;
  const unsigned b = e.bf16;
  if (e.bias) v += ld4(e.bias + col);
  if (e.add_pre) v += ldx4(e.add_pre, o, b & EPI_BF_ADD_PRE);
  if (e.save_pre) stx4(e.save_pre, o, b & EPI_BF_SAVE_PRE, v);
  if (e.act == 1) {
#pragma unroll
    for (int c = 0; c < 4; ++c) v[c] = silu_f(v[c]);
  } else if (e.act == 2) {
    const f32x4 z = ldx4(e.zsrc, o, b & EPI_BF_ZSRC);
#pragma unroll
    for (int c = 0; c < 4; ++c) v[c] *= dsilu_f(z[c]);
  }
  if (e.mul) v *= ldx4(e.mul, o, b & EPI_BF_MUL);
  if (mulv) v *= *mulv;
  if (e.add_post) v += ldx4(e.add_post, o, b & EPI_BF_ADD_POST);
  v *= e.scale;
  if (e.out) stx4(e.out, o, b & EPI_BF_OUT, v);
  if (e.out2) {
    const f32x4 z = ldx4(e.z2src, o, b & EPI_BF_Z2SRC);
#pragma unroll
    for (int c = 0; c < 4; ++c) v[c] *= dsilu_f(z[c]);
    stx4(e.out2, o, b & EPI_BF_OUT2, v);
  }
}

__device__ __forceinline__ void st4h(float* p, int64_t o, f32x4 v) {
  bf16x4 h;
#pragma unroll
  for (int c = 0; c < 4; ++c) h[c] = (__bf16)v[c];
  __builtin_nontemporal_store(h, reinterpret_cast<bf16x4*>(reinterpret_cast<__bf16*>(p) + o));
}
// The steps of one of the fixed combinations on 4 consecutive columns; no option is tested here.
template <int KIND>
__device__ __forceinline__ void epilogue_store4_kind(const gp_epilogue& e, int64_t o, f32x4 v, f32x4 lr,
                                                     const bf16x4* add_loaded = nullptr) {
  static_assert(KIND != EK_GENERIC, "the general loop calls epilogue_store4");
  if constexpr (KIND == EK_OUT_F32) st4(e.out + o, v);
  else if constexpr (KIND == EK_OUT_BF16) st4h(e.out, o, v);
  else if constexpr (KIND == EK_PRE_SILU_F32) {
    st4(e.save_pre + o, v);
#pragma unroll
    for (int c = 0; c < 4; ++c) v[c] = silu_f(v[c]);
    st4(e.out + o, v);
  } else if constexpr (KIND == EK_DSILU_BF16) {
    const f32x4 z = ld4(e.zsrc + o);
#pragma unroll
    for (int c = 0; c < 4; ++c) v[c] *= dsilu_f(z[c]);
    st4h(e.out, o, v);
  } else {
    st4h(e.save_pre, o, v);
#pragma unroll
    for (int c = 0; c < 4; ++c) v[c] = silu_f(v[c]);
    if constexpr (KIND == EK_PRE_SILU_LR_BF16) v *= lr;
    if constexpr (KIND == EK_PRE_SILU_ADD_F32 || KIND == EK_PRE_SILU_ADD_BF16) {
      if (add_loaded) {   // the caller has fetched the addend's 4 values already
#pragma unroll
        for (int c = 0; c < 4; ++c) v[c] += (float)(*add_loaded)[c];
      } else v += ldx4(e.add_post, o, 1u);
      v *= e.scale;
      if constexpr (KIND == EK_PRE_SILU_ADD_BF16) st4h(e.out, o, v);
      else st4(e.out + o, v);
    } else st4h(e.out, o, v);
  }
}

// The steps named by the mask M on 4 consecutive columns of fp32 matrices, in the order of epilogue_store4; no option is tested.
template <unsigned M>
__device__ __forceinline__ void epilogue_store4_mask(const gp_epilogue& e, int64_t o, int col, f32x4 v) {
  if constexpr ((M & EM_BIAS) != 0) v += ld4(e.bias + col);
  if constexpr ((M & EM_ADD_PRE) != 0) v += ld4(e.add_pre + o);
  if constexpr ((M & EM_SAVE_PRE) != 0) st4(e.save_pre + o, v);
  if constexpr ((M & EM_ACT1) != 0) {
#pragma unroll
    for (int c = 0; c < 4; ++c) v[c] = silu_f(v[c]);
  }
  if constexpr ((M & EM_ACT2) != 0) {
    const f32x4 z = ld4(e.zsrc + o);
#pragma unroll
    for (int c = 0; c < 4; ++c) v[c] *= dsilu_f(z[c]);
  }
  if constexpr ((M & EM_MUL) != 0) v *= ld4(e.mul + o);
  if constexpr ((M & EM_ADD_POST) != 0) v += ld4(e.add_post + o);
  if constexpr ((M & EM_SCALE) != 0) v *= e.scale;
  if constexpr ((M & EM_OUT) != 0) st4(e.out + o, v);
  if constexpr ((M & EM_OUT2) != 0) {
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

// Epilogue of one workgroup tile whose matrices are all fp32 (the fp32-result kernels).  The 32x32 MFMA block keeps, in
// register v of lane l, row 8*(v/4) + 4*(l/32) + v%4 and column l%32.  Each wavefront transposes one block at a time
// through its own LDS slice (32 x EPI_LD floats at smem + wave * 32 * EPI_LD; the caller has synchronised the workgroup)
// so that a lane ends up with 4 consecutive columns: loads and stores become 16-byte accesses, eight 128-byte row
// segments per instruction.  Blocks inside the matrix take a loop compiled for exactly the steps g.epi_mask names, the
// others the general one (options tested per 4 values); MODE_TN writes the partial sums of split `split`.
template <int MB, int NB, int MODE, unsigned EMASK>
__device__ __forceinline__ void tile_epilogue_f32_blocks(const gemm_args& g, f32x16 (&acc)[MB][NB], float* smem, int64_t m0, int n0,
                                                         int wm0, int wn0, int split) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int kh = lane >> 5, l32 = lane & 31;
  float* stage = smem + wave * (32 * EPI_LD);
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j) {
#pragma unroll
      for (int v = 0; v < 16; ++v) stage[((v >> 2) * 8 + kh * 4 + (v & 3)) * EPI_LD + l32] = acc[i][j][v];
      wave_lds_sync();
      const bool inside = m0 + wm0 + i * 32 + 32 <= g.M && n0 + wn0 + j * 32 + 32 <= g.N;
      if (EMASK != 0 && MODE != MODE_TN && inside) {
        if constexpr (EMASK != 0) {
          const int c4 = (lane & 7) * 4, col = n0 + wn0 + j * 32 + c4;
          const int64_t o0 = (m0 + wm0 + i * 32 + (lane >> 3)) * g.N + col;
#pragma unroll
          for (int it = 0; it < 4; ++it) {
            const f32x4 v4 = *reinterpret_cast<const f32x4*>(&stage[(it * 8 + (lane >> 3)) * EPI_LD + c4]);
            epilogue_store4_mask<EMASK>(g.epi, o0 + (int64_t)it * 8 * g.N, col, v4);
          }
        }
      } else {
#pragma unroll 1
        for (int it = 0; it < 4; ++it) {
          const int r = it * 8 + (lane >> 3), c4 = (lane & 7) * 4;
          const f32x4 v4 = *reinterpret_cast<const f32x4*>(&stage[r * EPI_LD + c4]);
          const int64_t row = m0 + wm0 + i * 32 + r;
          const int col = n0 + wn0 + j * 32 + c4;
          if (row >= g.M || col >= g.N) continue;
          if (MODE == MODE_TN) {
            float* dst = g.part + ((int64_t)split * g.M + row) * g.N + col;
            if (g.vecC) *reinterpret_cast<f32x4*>(dst) = v4;
            else
              for (int c = 0; c < 4; ++c)
                if (col + c < g.N) dst[c] = v4[c];
          } else {
            if (g.vecC) epilogue_store4(g.epi, row, col, g.N, v4);
            else
              for (int c = 0; c < 4; ++c)
                if (col + c < g.N) epilogue_store(g.epi, row, col + c, g.N, v4[c]);
          }
        }
      }
      wave_lds_sync();
    }
}
template <int MB, int NB, int MODE>
__device__ __forceinline__ void tile_epilogue_f32(const gemm_args& g, f32x16 (&acc)[MB][NB], float* smem, int64_t m0, int n0,
                                                  int wm0, int wn0, int split) {
  if constexpr (MODE == MODE_TN) tile_epilogue_f32_blocks<MB, NB, MODE, 0u>(g, acc, smem, m0, n0, wm0, wn0, split);
  else {
    switch (g.epi_mask) {   // uniform
#define GP_EM_CASE(M) case M: tile_epilogue_f32_blocks<MB, NB, MODE, M>(g, acc, smem, m0, n0, wm0, wn0, split); break;
      GP_EM_LIST(GP_EM_CASE)
#undef GP_EM_CASE
      default: tile_epilogue_f32_blocks<MB, NB, MODE, 0u>(g, acc, smem, m0, n0, wm0, wn0, split); break;
    }
  }
}

// Workgroup ids are dealt round-robin to the 8 XCDs; renumber them so that each XCD works on
// a contiguous range of tiles and neighbouring tiles (same A rows) share that XCD's L2.
__device__ __forceinline__ int xcd_remap(int bid, int n) {
  const int q = n >> 3, r = n & 7;
  const int x = bid & 7, i = bid >> 3;
  return x * q + (x < r ? x : r) + i;
}

}  // namespace
