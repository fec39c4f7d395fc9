// GEMM with bf16 operands and fp32 accumulation on the matrix cores (v_mfma_f32_32x32x16_bf16), for the wide
// edge layers of the bilinear block (paper Sec. 3.4; Table 4 widths).  An operand is either an fp32 matrix that
// is rounded to bf16 (round-to-nearest-even) on its way into LDS, or a matrix already stored as bf16 by a
// producer's epilogue; outputs and the matrices the fused epilogue reads are fp32 or bf16 per a mask.
//
// Three kernels:
//  * gemm_bf16_kernel: any mix of operand storage, any shape.  LDS tiles As[m][k], Bs[n][k] with k contiguous
//    (rows padded to 80 bytes), so the 8 consecutive k one lane feeds to an MFMA are a single 16-byte read.  A
//    256-thread workgroup owns a BM x BN tile, each wavefront 32x32 blocks of it; K advances 32 per slab, the
//    global loads of the next slab are issued before the current one is multiplied.
//  * gemm_hh_kernel: both operands bf16.  Two slabs of loads in flight in registers, two LDS buffers and one
//    barrier per slab, operand fragments of the next MFMA group requested before the current group is issued.
//  * gemm_dl_kernel: C = A B^T, both operands bf16 and k-contiguous, tall A: tiles go from global memory
//    straight into LDS (see the comment at the kernel).
//
// One MFMA of this shape does 32768 flop in 32 cycles, so the loop around it has to stay within a few vector
// instructions per MFMA.  The loaders therefore keep a uniform base pointer that moves with the slab plus one
// 32-bit byte offset per item computed once, and full slabs take a path with no bounds arithmetic at all:
// rows/columns past the edge of the matrix are read from a clamped (valid) address and only influence outputs
// that are never stored.  Only the last, partial slab of the contraction masks its operands to zero.
#include <stdarg.h>

#include <type_traits>

#include "gemm_common.h"


namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int BKH = 32;        // k per slab
constexpr int LDK = BKH + 8;   // bf16 per LDS row: 80 bytes, 16-byte reads of 8 lanes cover all banks
constexpr int K8 = BKH / 8;    // 16-byte groups per row
constexpr int64_t MAX_LD = 1 << 21;   // keeps every per-thread byte offset below 2^32

__device__ __forceinline__ f32x4 ldg4(const float* base, uint32_t byte_off) {
  return *reinterpret_cast<const f32x4*>(reinterpret_cast<const char*>(base) + byte_off);
}
__device__ __forceinline__ float ldg1(const float* base, uint32_t byte_off) {
  return *reinterpret_cast<const float*>(reinterpret_cast<const char*>(base) + byte_off);
}

__device__ __forceinline__ bf16x8 to_bf16x8(const float* v) {
  bf16x8 r;
#pragma unroll
  for (int c = 0; c < 8; ++c) r[c] = (__bf16)v[c];
  return r;
}
__device__ __forceinline__ bf16x8 to_bf16x8_masked(const float* v, uint32_t bits) {
  bf16x8 r;
#pragma unroll
  for (int c = 0; c < 8; ++c) r[c] = (__bf16)(((bits >> c) & 1u) ? v[c] : 0.f);
  return r;
}

// 8 fp32 values as PL bf16 planes, `plane` elements apart: plane 0 holds the values rounded to bf16, plane p what is left
// after planes 0..p-1 rounded again.  Three planes carry 24 significant bits, i.e. the fp32 value itself.
template <int PL>
__device__ __forceinline__ void split_store8(__bf16* dst, int plane, const float* v) {
  float r[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) r[c] = v[c];
#pragma unroll
  for (int p = 0; p < PL; ++p) {
    const bf16x8 h = to_bf16x8(r);
    *reinterpret_cast<bf16x8*>(dst + p * plane) = h;
    if (p + 1 < PL) {
#pragma unroll
      for (int c = 0; c < 8; ++c) r[c] -= (float)h[c];
    }
  }
}

// Source rows = tile rows, contraction index contiguous; item = (row, group of 8 k).
template <int X, bool VEC>
struct bl_kcontig {
  static constexpr int ITEMS = X * K8;
  static constexpr int NV = (ITEMS + THREADS - 1) / THREADS;
  static constexpr bool ALL = ITEMS % THREADS == 0;
  const float* base;   // first row of the tile (uniform)
  uint32_t off[NV];    // bytes from base to the item's first element at k0 = 0
  float r[NV][8];
  uint32_t mask;       // partial slab only: bit 8*it+c set when that k lies inside the contraction

  __device__ __forceinline__ void init(const float* __restrict__ src, int64_t ld, int64_t row0, int64_t n_rows) {
    base = src + row0 * ld;
    const int last = (int)(n_rows - 1 - row0 < X - 1 ? n_rows - 1 - row0 : X - 1);
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      const int row = idx / K8, kq = (idx % K8) * 8;
      off[it] = (uint32_t)(((int64_t)(row < last ? row : last) * ld + kq) * 4);
    }
  }
  __device__ __forceinline__ void fetch_full(int64_t k0) {
    const float* p = base + k0;
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      if (!ALL && (int)threadIdx.x + it * THREADS >= ITEMS) continue;
      if (VEC) {
        const f32x4 v0 = ldg4(p, off[it]), v1 = ldg4(p, off[it] + 16);
#pragma unroll
        for (int c = 0; c < 4; ++c) r[it][c] = v0[c], r[it][4 + c] = v1[c];
      } else {
#pragma unroll
        for (int c = 0; c < 8; ++c) r[it][c] = ldg1(p, off[it] + 4 * c);
      }
    }
  }
  __device__ __forceinline__ void fetch_tail(int64_t k0, int64_t k_end) {
    mask = 0;
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      if (!ALL && idx >= ITEMS) continue;
      const int kq = (idx % K8) * 8;
      const float* prow = reinterpret_cast<const float*>(reinterpret_cast<const char*>(base) + (off[it] - 4u * kq));
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const int64_t k = k0 + kq + c;
        r[it][c] = prow[k < k_end ? k : k_end - 1];
        mask |= (k < k_end ? 1u : 0u) << (8 * it + c);
      }
    }
  }
  __device__ __forceinline__ void store(__bf16* __restrict__ S, bool tail) const {
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      if (!ALL && idx >= ITEMS) continue;
      const int row = idx / K8, kq = (idx % K8) * 8;
      *reinterpret_cast<bf16x8*>(&S[row * LDK + kq]) =
          tail ? to_bf16x8_masked(r[it], (mask >> (8 * it)) & 0xFFu) : to_bf16x8(r[it]);
    }
  }
  template <int PL>
  __device__ __forceinline__ void store_planes(__bf16* __restrict__ S, int plane, bool tail) const {
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      if (!ALL && idx >= ITEMS) continue;
      const int row = idx / K8, kq = (idx % K8) * 8;
      float v[8];
#pragma unroll
      for (int c = 0; c < 8; ++c) v[c] = (!tail || ((mask >> (8 * it + c)) & 1u)) ? r[it][c] : 0.f;
      split_store8<PL>(&S[row * LDK + kq], plane, v);
    }
  }
};

// Source has the tile's m/n index (x) contiguous and the contraction index strided.  A thread
// owns a group of 4 consecutive x by 8 consecutive k: eight 16-byte loads (one per k row),
// regrouped in registers into four 8-k items.  Lanes take consecutive k-groups first, then
// consecutive x-groups, so the LDS writes of 8 lanes cover all banks.  Without VEC (extent not
// a multiple of 4, or unaligned) the same group is read by 32 scalar loads.
template <int X, bool VEC>
struct bl_xcontig {
  static constexpr int GROUPS = (X / 4) * K8;
  static constexpr int NV = (GROUPS + THREADS - 1) / THREADS;
  static constexpr bool ALL = GROUPS % THREADS == 0;
  static constexpr int NX = VEC ? 1 : 4;
  const float* base;       // first x of the tile at k = 0 (uniform)
  int64_t ld;
  uint32_t off[NV][NX];    // bytes from the slab's first k row to (first k of the group, clamped x)
  float r[NV][8][4];       // [k][x]
  uint32_t kmask[NV];      // partial slab only

  __device__ __forceinline__ void init(const float* __restrict__ src, int64_t ld_, int64_t x0, int64_t n_x) {
    base = src + x0;
    ld = ld_;
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      const int kq = (idx % K8) * 8, xq = (idx / K8) * 4;
#pragma unroll
      for (int c = 0; c < NX; ++c) {
        const int64_t lim = n_x - x0 - (VEC ? 4 : 1);     // last legal start inside the matrix
        const int64_t x = xq + c < lim ? xq + c : lim;
        off[it][c] = (uint32_t)((kq * ld + x) * 4);
      }
    }
  }
  __device__ __forceinline__ void fetch_full(int64_t k0) {
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const float* p = base + (k0 + kk) * ld;
#pragma unroll
      for (int it = 0; it < NV; ++it) {
        if (!ALL && (int)threadIdx.x + it * THREADS >= GROUPS) continue;
        if (VEC) {
          const f32x4 v = ldg4(p, off[it][0]);
#pragma unroll
          for (int c = 0; c < 4; ++c) r[it][kk][c] = v[c];
        } else {
#pragma unroll
          for (int c = 0; c < 4; ++c) r[it][kk][c] = ldg1(p, off[it][c]);
        }
      }
    }
  }
  __device__ __forceinline__ void fetch_tail(int64_t k0, int64_t k_end) {
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      kmask[it] = 0;
      if (!ALL && idx >= GROUPS) continue;
      const int kq = (idx % K8) * 8;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        const int64_t k = k0 + kq + kk;
        kmask[it] |= (k < k_end ? 1u : 0u) << kk;
        // row k (clamped), then the group's x offset without its k part
        const float* p = base + (k < k_end ? k : k_end - 1) * ld - (int64_t)kq * ld;
        if (VEC) {
          const f32x4 v = ldg4(p, off[it][0]);
#pragma unroll
          for (int c = 0; c < 4; ++c) r[it][kk][c] = v[c];
        } else {
#pragma unroll
          for (int c = 0; c < 4; ++c) r[it][kk][c] = ldg1(p, off[it][c]);
        }
      }
    }
  }
  __device__ __forceinline__ void store(__bf16* __restrict__ S, bool tail) const {
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      if (!ALL && idx >= GROUPS) continue;
      const int kq = (idx % K8) * 8, xq = (idx / K8) * 4;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        float col[8];
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) col[kk] = r[it][kk][c];
        *reinterpret_cast<bf16x8*>(&S[(xq + c) * LDK + kq]) = tail ? to_bf16x8_masked(col, kmask[it]) : to_bf16x8(col);
      }
    }
  }
  template <int PL>
  __device__ __forceinline__ void store_planes(__bf16* __restrict__ S, int plane, bool tail) const {
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      if (!ALL && idx >= GROUPS) continue;
      const int kq = (idx % K8) * 8, xq = (idx / K8) * 4;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        float col[8];
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) col[kk] = (!tail || ((kmask[it] >> kk) & 1u)) ? r[it][kk][c] : 0.f;
        split_store8<PL>(&S[(xq + c) * LDK + kq], plane, col);
      }
    }
  }
};

// ---- operands already stored as bf16 (activations written by a producer's epilogue): no conversion,
// half the bytes; 16-byte / 4-byte aligned rows are required (leading dimension a multiple of 8 / 2).

// rows = tile rows, k contiguous: one 16-byte load is one LDS item
template <int X>
struct bl_kcontig_bf {
  static constexpr int ITEMS = X * K8;
  static constexpr int NV = (ITEMS + THREADS - 1) / THREADS;
  static constexpr bool ALL = ITEMS % THREADS == 0;
  const __bf16* base;
  uint32_t off[NV];   // bytes
  bf16x8 r[NV];

  __device__ __forceinline__ void init(const float* __restrict__ src, int64_t ld, int64_t row0, int64_t n_rows) {
    base = reinterpret_cast<const __bf16*>(src) + row0 * ld;
    const int last = (int)(n_rows - 1 - row0 < X - 1 ? n_rows - 1 - row0 : X - 1);
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      const int row = idx / K8, kq = (idx % K8) * 8;
      off[it] = (uint32_t)(((int64_t)(row < last ? row : last) * ld + kq) * 2);
    }
  }
  __device__ __forceinline__ void fetch_full(int64_t k0) {
    const char* p = reinterpret_cast<const char*>(base + k0);
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      if (!ALL && (int)threadIdx.x + it * THREADS >= ITEMS) continue;
      r[it] = *reinterpret_cast<const bf16x8*>(p + off[it]);
    }
  }
  __device__ __forceinline__ void fetch_tail(int64_t k0, int64_t k_end) {
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      if (!ALL && idx >= ITEMS) continue;
      const int kq = (idx % K8) * 8;
      const __bf16* prow = reinterpret_cast<const __bf16*>(reinterpret_cast<const char*>(base) + (off[it] - 2u * kq));
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const int64_t k = k0 + kq + c;
        const __bf16 v = prow[k < k_end ? k : k_end - 1];
        r[it][c] = k < k_end ? v : (__bf16)0.f;
      }
    }
  }
  __device__ __forceinline__ void store(__bf16* __restrict__ S, bool) const {
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      if (!ALL && idx >= ITEMS) continue;
      const int row = idx / K8, kq = (idx % K8) * 8;
      *reinterpret_cast<bf16x8*>(&S[row * LDK + kq]) = r[it];
    }
  }
};

// x contiguous, k strided: a thread owns 2 consecutive x by 8 consecutive k; eight 4-byte loads, repacked
// into two 8-k items.  Lanes take consecutive x pairs (256 contiguous bytes per k row and wavefront; the
// two 16-byte LDS writes of neighbouring lanes are 160 bytes apart and cover all banks).
template <int X>
struct bl_xcontig_bf {
  static constexpr int ITEMS = (X / 2) * K8;
  static constexpr int NV = (ITEMS + THREADS - 1) / THREADS;
  static constexpr bool ALL = ITEMS % THREADS == 0;
  const __bf16* base;
  int64_t ld;
  uint32_t off[NV];       // bytes from the slab's first k row
  uint32_t r[NV][8];      // [k] = (x, x+1)
  uint32_t kmask[NV];

  __device__ __forceinline__ void init(const float* __restrict__ src, int64_t ld_, int64_t x0, int64_t n_x) {
    base = reinterpret_cast<const __bf16*>(src) + x0;
    ld = ld_;
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      const int xq = (idx % (X / 2)) * 2, kq = (idx / (X / 2)) * 8;
      const int64_t lim = n_x - x0 - 2;
      off[it] = (uint32_t)((kq * ld + (xq < lim ? xq : lim)) * 2);
      kmask[it] = 0xFFu;
    }
  }
  __device__ __forceinline__ void fetch_full(int64_t k0) {
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const char* p = reinterpret_cast<const char*>(base + (k0 + kk) * ld);
#pragma unroll
      for (int it = 0; it < NV; ++it) {
        if (!ALL && (int)threadIdx.x + it * THREADS >= ITEMS) continue;
        r[it][kk] = *reinterpret_cast<const uint32_t*>(p + off[it]);
      }
    }
  }
  __device__ __forceinline__ void fetch_tail(int64_t k0, int64_t k_end) {
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      kmask[it] = 0;
      if (!ALL && idx >= ITEMS) continue;
      const int kq = (idx / (X / 2)) * 8;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        const int64_t k = k0 + kq + kk;
        kmask[it] |= (k < k_end ? 1u : 0u) << kk;
        const char* p = reinterpret_cast<const char*>(base + ((k < k_end ? k : k_end - 1) - kq) * ld);
        r[it][kk] = *reinterpret_cast<const uint32_t*>(p + off[it]);
      }
    }
  }
  __device__ __forceinline__ void store(__bf16* __restrict__ S, bool tail) const {
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = threadIdx.x + it * THREADS;
      if (!ALL && idx >= ITEMS) continue;
      const int xq = (idx % (X / 2)) * 2, kq = (idx / (X / 2)) * 8;
      uint32_t d[8];
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) d[kk] = (!tail || ((kmask[it] >> kk) & 1u)) ? r[it][kk] : 0u;
      uint32_t lo[4], hi[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        lo[j] = (d[2 * j] & 0xFFFFu) | (d[2 * j + 1] << 16);
        hi[j] = (d[2 * j] >> 16) | (d[2 * j + 1] & 0xFFFF0000u);
      }
      uint32_t* s0 = reinterpret_cast<uint32_t*>(&S[xq * LDK + kq]);
      uint32_t* s1 = reinterpret_cast<uint32_t*>(&S[(xq + 1) * LDK + kq]);
      typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
      *reinterpret_cast<u32x4*>(s0) = u32x4{lo[0], lo[1], lo[2], lo[3]};
      *reinterpret_cast<u32x4*>(s1) = u32x4{hi[0], hi[1], hi[2], hi[3]};
    }
  }
};

// Epilogue of one workgroup tile: accumulators have the register layout of the 32x32 MFMA and are transposed
// through a per-wavefront LDS slice so that loads and stores are 16-byte accesses.
// LR_WAVES > 0 (the number of wavefronts of the workgroup): the kernel can evaluate the epilogue's low-rank factor; its
// 32x32 blocks go through a second staging slice per wavefront, behind the first ones.
// The paired path for one combination of epilogue steps (KIND; EK_GENERIC tests the options per value).
template <int MB, int NB, int LR_WAVES, int KIND>
__device__ __forceinline__ void tile_epilogue_pairs(const gemm_args& g, f32x16 (&acc)[MB][NB], float* smem, int64_t m0, int n0,
                                                    int wm0, int wn0) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int kh = lane >> 5, l32 = lane & 31;
  // Two blocks side by side (32 rows x 64 columns): 16 lanes cover 64 consecutive columns of a row, so a store
  // instruction writes whole 128-byte lines of a bf16 matrix (two per row of an fp32 one) instead of halves.
  float* stage = smem + wave * (32 * EPI_LD2);
  // Low-rank factor: operand fragments of the wavefront's rows and columns (k = 8 kh + c, zero from lr_k on), two
  // MFMAs per block, in the accumulators' own register layout.  The row factor (an activation) enters as the sum of
  // two bf16 numbers, i.e. to 16 bits: rounded to 8 bits, a model's energy turned out too rough a function of the
  // positions for a finite difference of it to match its forces; the column factor is a weight like any other.
  constexpr bool LR_POSSIBLE = LR_WAVES > 0 && (KIND == EK_GENERIC || KIND == EK_PRE_SILU_LR_BF16);
  const bool lr = LR_POSSIBLE && g.epi.lr_a != nullptr;
  float* stage_lr = smem + (LR_WAVES + wave) * (32 * EPI_LD2);
  bf16x8 ga[LR_POSSIBLE ? MB : 1], ga_lo[LR_POSSIBLE ? MB : 1], gb[LR_POSSIBLE ? NB : 1];
  if constexpr (LR_POSSIBLE) {
    if (lr) {
      const int kk = g.epi.lr_k;
#pragma unroll
      for (int i = 0; i < MB; ++i) {
        const int64_t row = m0 + wm0 + i * 32 + l32 < g.M ? m0 + wm0 + i * 32 + l32 : g.M - 1;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
          const int k = 8 * kh + c;
          const float a0 = g.epi.lr_a[row * kk + (k < kk ? k : kk - 1)];  // clamped: the load stays unconditional
          const float a = k < kk ? a0 : 0.f;
          ga[i][c] = (__bf16)a;
          ga_lo[i][c] = (__bf16)(a - (float)ga[i][c]);
        }
      }
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const int col = n0 + wn0 + j * 32 + l32 < g.N ? n0 + wn0 + j * 32 + l32 : g.N - 1;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
          const int k = 8 * kh + c;
          const float b = g.epi.lr_b[(int64_t)(k < kk ? k : kk - 1) * g.N + col];
          gb[j][c] = (__bf16)(k < kk ? b : 0.f);
        }
      }
    }
  }
  // The addend of a small tile that lies inside the matrix is fetched for all of the wavefront's blocks at once, before
  // the first block is staged: fetched block by block in the loop below, each block waited for its own loads (a narrow
  // contraction leaves nothing else to hide them behind).
  constexpr bool PRELOAD = (KIND == EK_PRE_SILU_ADD_F32 || KIND == EK_PRE_SILU_ADD_BF16) && MB * NB <= 4;
  bf16x4 addp[PRELOAD ? MB : 1][PRELOAD ? NB / 2 : 1][PRELOAD ? 8 : 1];
  bool preloaded = false;
  if constexpr (PRELOAD) {
    preloaded = m0 + wm0 + MB * 32 <= g.M && n0 + wn0 + NB * 32 <= g.N;
    if (preloaded) {
      const __bf16* ap = reinterpret_cast<const __bf16*>(g.epi.add_post) + (m0 + wm0 + (lane >> 4)) * g.N + (n0 + wn0 + (lane & 15) * 4);
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; j += 2)
#pragma unroll
          for (int it = 0; it < 8; ++it)
            addp[i][j / 2][it] = *reinterpret_cast<const bf16x4*>(ap + (int64_t)(i * 32 + it * 4) * g.N + j * 32);
    }
  }
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; j += 2) {
#pragma unroll
      for (int jj = 0; jj < 2; ++jj)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          stage[((v >> 2) * 8 + kh * 4 + (v & 3)) * EPI_LD2 + jj * 32 + l32] = acc[i][j + jj][v];
      if constexpr (LR_POSSIBLE) {
        if (lr) {
#pragma unroll
          for (int jj = 0; jj < 2; ++jj) {
            f32x16 z;
#pragma unroll
            for (int v = 0; v < 16; ++v) z[v] = 0.f;
            f32x16 f = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ga_lo[i], gb[j + jj], z, 0, 0, 0);
            f = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ga[i], gb[j + jj], f, 0, 0, 0);
#pragma unroll
            for (int v = 0; v < 16; ++v) stage_lr[((v >> 2) * 8 + kh * 4 + (v & 3)) * EPI_LD2 + jj * 32 + l32] = f[v];
          }
        }
      }
      wave_lds_sync();
      // a block pair that lies inside the matrix takes the loop without bounds or option tests
      const bool inside = m0 + wm0 + i * 32 + 32 <= g.M && n0 + wn0 + j * 32 + 64 <= g.N;
      if (KIND != EK_GENERIC && inside) {
        if constexpr (KIND != EK_GENERIC) {
          const int c4 = (lane & 15) * 4;
          const int64_t o0 = (m0 + wm0 + i * 32 + (lane >> 4)) * g.N + (n0 + wn0 + j * 32 + c4);
          if constexpr (PRELOAD) {
            if (preloaded) {
#pragma unroll
              for (int it = 0; it < 8; ++it) {
                const f32x4 v4 = *reinterpret_cast<const f32x4*>(&stage[(it * 4 + (lane >> 4)) * EPI_LD2 + c4]);
                epilogue_store4_kind<KIND>(g.epi, o0 + (int64_t)it * 4 * g.N, v4, f32x4{1.f, 1.f, 1.f, 1.f}, &addp[i][j / 2][it]);
              }
              wave_lds_sync();
              continue;
            }
          }
#pragma unroll 4
          for (int it = 0; it < 8; ++it) {
            const int r = it * 4 + (lane >> 4);
            const f32x4 v4 = *reinterpret_cast<const f32x4*>(&stage[r * EPI_LD2 + c4]);
            f32x4 f4 = {1.f, 1.f, 1.f, 1.f};
            if constexpr (KIND == EK_PRE_SILU_LR_BF16) f4 = *reinterpret_cast<const f32x4*>(&stage_lr[r * EPI_LD2 + c4]);
            epilogue_store4_kind<KIND>(g.epi, o0 + (int64_t)it * 4 * g.N, v4, f4);
          }
        }
      } else {
#pragma unroll 1
        for (int it = 0; it < 8; ++it) {
          const int r = it * 4 + (lane >> 4), c4 = (lane & 15) * 4;
          const f32x4 v4 = *reinterpret_cast<const f32x4*>(&stage[r * EPI_LD2 + c4]);
          const int64_t row = m0 + wm0 + i * 32 + r;
          const int col = n0 + wn0 + j * 32 + c4;
          if (row >= g.M || col >= g.N) continue;
          if constexpr (LR_POSSIBLE) {
            if (lr) {   // dispatch has checked vecC
              const f32x4 f4 = *reinterpret_cast<const f32x4*>(&stage_lr[r * EPI_LD2 + c4]);
              epilogue_store4(g.epi, row, col, g.N, v4, &f4);
              continue;
            }
          }
          if (g.vecC) epilogue_store4(g.epi, row, col, g.N, v4);
          else
            for (int c = 0; c < 4; ++c)
              if (col + c < g.N) epilogue_store(g.epi, row, col + c, g.N, v4[c]);
        }
      }
      wave_lds_sync();
    }
}

template <int MB, int NB, int MODE, int LR_WAVES = 0>
__device__ __forceinline__ void tile_epilogue(const gemm_args& g, f32x16 (&acc)[MB][NB], float* smem, int64_t m0, int n0,
                                              int wm0, int wn0, int split) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int kh = lane >> 5, l32 = lane & 31;
  if constexpr (MODE != MODE_TN && NB % 2 == 0) {
    switch (g.epi_kind) {   // uniform
      case EK_OUT_F32: tile_epilogue_pairs<MB, NB, LR_WAVES, EK_OUT_F32>(g, acc, smem, m0, n0, wm0, wn0); break;
      case EK_OUT_BF16: tile_epilogue_pairs<MB, NB, LR_WAVES, EK_OUT_BF16>(g, acc, smem, m0, n0, wm0, wn0); break;
      case EK_PRE_SILU_BF16: tile_epilogue_pairs<MB, NB, LR_WAVES, EK_PRE_SILU_BF16>(g, acc, smem, m0, n0, wm0, wn0); break;
      case EK_DSILU_BF16: tile_epilogue_pairs<MB, NB, LR_WAVES, EK_DSILU_BF16>(g, acc, smem, m0, n0, wm0, wn0); break;
      case EK_PRE_SILU_F32: tile_epilogue_pairs<MB, NB, LR_WAVES, EK_PRE_SILU_F32>(g, acc, smem, m0, n0, wm0, wn0); break;
      case EK_PRE_SILU_LR_BF16:
        if constexpr (LR_WAVES > 0) { tile_epilogue_pairs<MB, NB, LR_WAVES, EK_PRE_SILU_LR_BF16>(g, acc, smem, m0, n0, wm0, wn0); break; }
        [[fallthrough]];
      case EK_PRE_SILU_ADD_F32:
        if (g.epi_kind == EK_PRE_SILU_ADD_F32) { tile_epilogue_pairs<MB, NB, LR_WAVES, EK_PRE_SILU_ADD_F32>(g, acc, smem, m0, n0, wm0, wn0); break; }
        [[fallthrough]];
      case EK_PRE_SILU_ADD_BF16:
        if (g.epi_kind == EK_PRE_SILU_ADD_BF16) { tile_epilogue_pairs<MB, NB, LR_WAVES, EK_PRE_SILU_ADD_BF16>(g, acc, smem, m0, n0, wm0, wn0); break; }
        [[fallthrough]];
      default: tile_epilogue_pairs<MB, NB, LR_WAVES, EK_GENERIC>(g, acc, smem, m0, n0, wm0, wn0); break;
    }
    return;
  }
  float* stage = smem + wave * (32 * EPI_LD);
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j) {
#pragma unroll
      for (int v = 0; v < 16; ++v) stage[((v >> 2) * 8 + kh * 4 + (v & 3)) * EPI_LD + l32] = acc[i][j][v];
      wave_lds_sync();
#pragma unroll 1   // the typed epilogue is long; unrolled 4 x MB x NB times it would not fit the register file
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
      wave_lds_sync();
    }
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int MODE, bool VEC, bool ABF, bool BBF>
__global__ void __launch_bounds__(THREADS, 2)   // two wavefronts per SIMD: 256 registers each
gemm_bf16_kernel(const gemm_args g) {
  static_assert(WAVES_M * WAVES_N == 4, "four wavefronts per workgroup");
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int MB = WM / 32, NB = WN / 32;
  using loadA32 = typename std::conditional<MODE != MODE_TN, bl_kcontig<BM, VEC>, bl_xcontig<BM, VEC>>::type;
  using loadA16 = typename std::conditional<MODE != MODE_TN, bl_kcontig_bf<BM>, bl_xcontig_bf<BM>>::type;
  using loadB32 = typename std::conditional<MODE == MODE_NT, bl_kcontig<BN, VEC>, bl_xcontig<BN, VEC>>::type;
  using loadA = typename std::conditional<ABF, loadA16, loadA32>::type;
  using loadB16 = typename std::conditional<MODE == MODE_NT, bl_kcontig_bf<BN>, bl_xcontig_bf<BN>>::type;
  using loadB = typename std::conditional<BBF, loadB16, loadB32>::type;
  extern __shared__ __attribute__((aligned(16))) float smem[];
  __bf16* As = reinterpret_cast<__bf16*>(smem);
  __bf16* Bs = As + BM * LDK;

  const int tiles_n = (g.N + BN - 1) / BN;
  const int tiles_m = (int)((g.M + BM - 1) / BM);
  const int tile = xcd_remap(blockIdx.x, tiles_m * tiles_n);
  const int64_t m0 = (int64_t)(tile / tiles_n) * BM;
  const int n0 = (tile % tiles_n) * BN;

  int64_t k_begin = 0, k_end = g.K;
  if (MODE == MODE_TN) {
    k_begin = (int64_t)blockIdx.y * g.k_per_split;
    k_end = k_begin + g.k_per_split < (int64_t)g.K ? k_begin + g.k_per_split : (int64_t)g.K;
  }

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
  const int kh = lane >> 5, l32 = lane & 31;

  f32x16 acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  if (k_begin < k_end) {
    loadA la;
    loadB lb;
    la.init(g.A, g.lda, m0, g.M);
    lb.init(g.B, g.ldb, n0, g.N);
    auto multiply = [&]() {
#pragma unroll
      for (int kk = 0; kk < BKH; kk += 16) {
        bf16x8 a[MB], b[NB];
#pragma unroll
        for (int i = 0; i < MB; ++i) a[i] = *reinterpret_cast<const bf16x8*>(&As[(wm0 + i * 32 + l32) * LDK + kk + kh * 8]);
#pragma unroll
        for (int j = 0; j < NB; ++j) b[j] = *reinterpret_cast<const bf16x8*>(&Bs[(wn0 + j * 32 + l32) * LDK + kk + kh * 8]);
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
          for (int j = 0; j < NB; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
      }
    };
    // complete slabs, software-pipelined: the loads of slab s+1 are in flight while slab s is multiplied
    const int64_t n_full = (k_end - k_begin) / BKH;
    if (n_full > 0) {
      la.fetch_full(k_begin);
      lb.fetch_full(k_begin);
      la.store(As, false);
      lb.store(Bs, false);
      __syncthreads();
      for (int64_t s = 1; s < n_full; ++s) {
        la.fetch_full(k_begin + s * BKH);
        lb.fetch_full(k_begin + s * BKH);
        multiply();
        __syncthreads();
        la.store(As, false);
        lb.store(Bs, false);
        __syncthreads();
      }
      multiply();
      __syncthreads();
    }
    // the partial slab at the end of the contraction, operands masked to zero past k_end
    const int64_t k_tail = k_begin + n_full * BKH;
    if (k_tail < k_end) {
      la.fetch_tail(k_tail, k_end);
      lb.fetch_tail(k_tail, k_end);
      la.store(As, true);
      lb.store(Bs, true);
      __syncthreads();
      multiply();
      __syncthreads();
    }
  }

  tile_epilogue<MB, NB, MODE>(g, acc, smem, m0, n0, wm0, wn0, blockIdx.y);
}

// fp32 operands, fp32 result, on the bf16 matrix cores: each operand element goes into LDS as three bf16 numbers whose
// sum is the fp32 value (hi + mid + lo, 24 significant bits), and a k-step multiplies the six plane pairs whose
// product is not below 2^-24 of the full one (hi.hi, hi.mid, mid.hi, hi.lo, mid.mid, lo.hi), smallest first, into the
// fp32 accumulator: the error of a product is that of one fp32 rounding.  Six bf16 MFMAs (32 cycles each for 16 k)
// replace eight fp32 ones (64 cycles each for 2 k): the fp32-operand MFMA rate of this chip is a sixteenth of the
// bf16 one.  Same tiles, loaders and pipeline as gemm_bf16_kernel, the fp32 kernel's epilogue (all matrices fp32).
// A B and A B^T; A^T B has a kernel of its own (gemm_split_tn_kernel).
template <int BM, int BN, int WAVES_M, int WAVES_N, int MODE, bool VEC>
__global__ void __launch_bounds__(THREADS, 2)
gemm_split_kernel(const gemm_args g) {
  static_assert(WAVES_M * WAVES_N == 4, "four wavefronts per workgroup");
  static_assert(MODE != MODE_TN, "the reduction over rows runs in gemm_split_tn_kernel");
  constexpr int PL = 3;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int MB = WM / 32, NB = WN / 32;
  using loadA = bl_kcontig<BM, VEC>;
  using loadB = typename std::conditional<MODE == MODE_NT, bl_kcontig<BN, VEC>, bl_xcontig<BN, VEC>>::type;
  extern __shared__ __attribute__((aligned(16))) float smem[];
  constexpr int PA = BM * LDK, PB = BN * LDK;   // plane strides (bf16 elements)
  __bf16* As = reinterpret_cast<__bf16*>(smem);
  __bf16* Bs = As + PL * PA;

  const int tiles_n = (g.N + BN - 1) / BN;
  const int tiles_m = (int)((g.M + BM - 1) / BM);
  const int tile = xcd_remap(blockIdx.x, tiles_m * tiles_n);
  const int64_t m0 = (int64_t)(tile / tiles_n) * BM;
  const int n0 = (tile % tiles_n) * BN;
  const int64_t k_begin = 0, k_end = g.K;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
  const int kh = lane >> 5, l32 = lane & 31;

  f32x16 acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  if (k_begin < k_end) {
    loadA la;
    loadB lb;
    la.init(g.A, g.lda, m0, g.M);
    lb.init(g.B, g.ldb, n0, g.N);
    auto multiply = [&]() {
#pragma unroll
      for (int kk = 0; kk < BKH; kk += 16) {
        bf16x8 a[PL][MB], b[PL][NB];
#pragma unroll
        for (int p = 0; p < PL; ++p) {
#pragma unroll
          for (int i = 0; i < MB; ++i) a[p][i] = *reinterpret_cast<const bf16x8*>(&As[p * PA + (wm0 + i * 32 + l32) * LDK + kk + kh * 8]);
#pragma unroll
          for (int j = 0; j < NB; ++j) b[p][j] = *reinterpret_cast<const bf16x8*>(&Bs[p * PB + (wn0 + j * 32 + l32) * LDK + kk + kh * 8]);
        }
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
          for (int j = 0; j < NB; ++j) {
            f32x16 c = acc[i][j];
            c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2][i], b[0][j], c, 0, 0, 0);
            c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0][i], b[2][j], c, 0, 0, 0);
            c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1][i], b[1][j], c, 0, 0, 0);
            c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1][i], b[0][j], c, 0, 0, 0);
            c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0][i], b[1][j], c, 0, 0, 0);
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0][i], b[0][j], c, 0, 0, 0);
          }
      }
    };
    auto store = [&](int64_t, bool tail) {   // the slab held in the loaders' registers goes to LDS
      la.template store_planes<PL>(As, PA, tail);
      lb.template store_planes<PL>(Bs, PB, tail);
    };
    const int64_t n_full = (k_end - k_begin) / BKH;
    if (n_full > 0) {
      la.fetch_full(k_begin);
      lb.fetch_full(k_begin);
      store(0, false);
      __syncthreads();
      for (int64_t s = 1; s < n_full; ++s) {
        la.fetch_full(k_begin + s * BKH);
        lb.fetch_full(k_begin + s * BKH);
        multiply();
        __syncthreads();
        store(s, false);
        __syncthreads();
      }
      multiply();
      __syncthreads();
    }
    const int64_t k_tail = k_begin + n_full * BKH;
    if (k_tail < k_end) {
      la.fetch_tail(k_tail, k_end);
      lb.fetch_tail(k_tail, k_end);
      store(n_full, true);
      __syncthreads();
      multiply();
      __syncthreads();
    }
  }

  tile_epilogue_f32<MB, NB, MODE>(g, acc, smem, m0, n0, wm0, wn0, 0);
}

// Both operands stored as bf16.  A slab is then only 6 sixteen-byte loads per thread, so NS slabs are kept in
// flight in registers (memory latency under load is several slab times), LDS holds two slabs so that one
// barrier per slab suffices: while slab t is multiplied out of one buffer, slab t+1 is written to the other.
// Register sets and buffers rotate statically (the loop is unrolled over one full rotation); loads past the
// last full slab re-read that slab (in bounds, never used).
template <int BM, int BN, int WAVES_M, int WAVES_N, int MODE>
__global__ void __launch_bounds__(THREADS, 2)
gemm_hh_kernel(const gemm_args g) {
  static_assert(WAVES_M * WAVES_N == 4, "four wavefronts per workgroup");
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int MB = WM / 32, NB = WN / 32;
  using loadA = typename std::conditional<MODE != MODE_TN, bl_kcontig_bf<BM>, bl_xcontig_bf<BM>>::type;
  using loadB = typename std::conditional<MODE == MODE_NT, bl_kcontig_bf<BN>, bl_xcontig_bf<BN>>::type;
  constexpr int STAGE = (BM + BN) * LDK;           // bf16 elements per LDS buffer
  extern __shared__ __attribute__((aligned(16))) float smem[];
  __bf16* S = reinterpret_cast<__bf16*>(smem);

  const int tiles_n = (g.N + BN - 1) / BN;
  const int tiles_m = (int)((g.M + BM - 1) / BM);
  // one-dimensional grid over (split, tile), split-major: each XCD gets a contiguous range, so the tiles of one
  // split (which all read the same rows of both operands) run side by side on one XCD and share its L2
  const int work = xcd_remap(blockIdx.x, gridDim.x);
  const int split = work / (tiles_m * tiles_n);
  const int tile = work % (tiles_m * tiles_n);
  const int64_t m0 = (int64_t)(tile / tiles_n) * BM;
  const int n0 = (tile % tiles_n) * BN;
  int64_t k_begin = 0, k_end = g.K;
  if (MODE == MODE_TN) {
    k_begin = (int64_t)split * g.k_per_split;
    k_end = k_begin + g.k_per_split < (int64_t)g.K ? k_begin + g.k_per_split : (int64_t)g.K;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
  const int kh = lane >> 5, l32 = lane & 31;

  f32x16 acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  if (k_begin < k_end) {
    static_assert(BKH == 32, "the schedule below is written for two MFMA steps per slab");
    loadA la[2];
    loadB lb[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      la[u].init(g.A, g.lda, m0, g.M);
      lb[u].init(g.B, g.ldb, n0, g.N);
    }
    bf16x8 fa[2][MB], fb[2][NB];   // operand fragments of the two MFMA steps
    auto read_frags = [&](const __bf16* __restrict__ As, int kk, int q) __attribute__((always_inline)) {
      const __bf16* Bs = As + BM * LDK;
#pragma unroll
      for (int i = 0; i < MB; ++i) fa[q][i] = *reinterpret_cast<const bf16x8*>(&As[(wm0 + i * 32 + l32) * LDK + kk + kh * 8]);
#pragma unroll
      for (int j = 0; j < NB; ++j) fb[q][j] = *reinterpret_cast<const bf16x8*>(&Bs[(wn0 + j * 32 + l32) * LDK + kk + kh * 8]);
    };
    auto mfma_group = [&](int q) __attribute__((always_inline)) {
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[q][i], fb[q][j], acc[i][j], 0, 0, 0);
    };
    const int64_t n_full = (k_end - k_begin) / BKH;
    if (n_full > 0) {
      auto at = [&](int64_t s) { return k_begin + (s < n_full ? s : n_full - 1) * BKH; };
      la[0].fetch_full(at(0));
      lb[0].fetch_full(at(0));
      la[1].fetch_full(at(1));
      lb[1].fetch_full(at(1));
      __builtin_amdgcn_sched_barrier(0);   // keep the issue order of the loads the same as in the loop
      la[0].store(S, false);
      lb[0].store(S + BM * LDK, false);
      la[0].fetch_full(at(2));
      lb[0].fetch_full(at(2));
      __builtin_amdgcn_sched_barrier(0);
      __syncthreads();
      read_frags(S, 0, 0);
      // Slab t is multiplied in two MFMA groups.  While the first runs, the fragments of the second are already
      // on their way from LDS, slab t+1 moves from registers to the other LDS buffer and the loads of slab t+3
      // are issued into the registers it leaves; after the barrier the first fragments of slab t+1 are requested
      // and the second group runs.  Every LDS or global access thus has one MFMA group (256 cycles) to complete.
      auto slab = [&](const int u, int64_t t) __attribute__((always_inline)) {
        const __bf16* cur = S + u * STAGE;
        __bf16* nxt = S + (1 - u) * STAGE;
        read_frags(cur, 16, 1);
        __builtin_amdgcn_sched_barrier(0);
        mfma_group(0);
        la[1 - u].store(nxt, false);                 // slab t+1
        lb[1 - u].store(nxt + BM * LDK, false);
        la[1 - u].fetch_full(at(t + 3));
        lb[1 - u].fetch_full(at(t + 3));
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        read_frags(nxt, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        mfma_group(1);
      };
      int64_t t = 0;
      for (; t + 1 < n_full; t += 2) {   // no exit between the two halves: the wait counts stay exact
        slab(0, t);
        slab(1, t + 1);
      }
      if (t < n_full) slab(0, t);
      __syncthreads();   // the fragments requested last are not used; nobody reads LDS past this point
    }
    // the partial slab at the end of the contraction, operands masked to zero past k_end
    const int64_t k_tail = k_begin + n_full * BKH;
    if (k_tail < k_end) {
      la[0].fetch_tail(k_tail, k_end);
      lb[0].fetch_tail(k_tail, k_end);
      la[0].store(S, true);
      lb[0].store(S + BM * LDK, true);
      __syncthreads();
      read_frags(S, 0, 0);
      read_frags(S, 16, 1);
      mfma_group(0);
      mfma_group(1);
      __syncthreads();
    }
  }
  tile_epilogue<MB, NB, MODE>(g, acc, smem, m0, n0, wm0, wn0, split);
}

template <int BM, int BN, int WMS, int WNS, int MODE>
int launch_hh(gp_ctx* ctx, gemm_args& g, int splits) {
  const int64_t tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
  if (tiles > INT32_MAX) return gp_fail(ctx, GP_BAD_ARG, "gemm: too many tiles");
  if (g.lda >= MAX_LD || g.ldb >= MAX_LD) return gp_fail(ctx, GP_BAD_ARG, "gemm (bf16): leading dimension above %lld", (long long)MAX_LD);
  if (tiles * splits > INT32_MAX) return gp_fail(ctx, GP_BAD_ARG, "gemm: too many tiles");
  dim3 grid((unsigned)(tiles * splits), 1, 1);
  static char name[48];
  if (!name[0]) snprintf(name, sizeof(name), "gemm_bf16_hh_%s_%dx%d", MODE == MODE_NN ? "nn" : MODE == MODE_NT ? "nt" : "tn", BM, BN);
  const double mnk = (double)g.M * g.N * g.K;
  gp_prof_scope prof(ctx, name, 2.0 * mnk,
                     2.0 * (double)g.M * g.K + 2.0 * (double)g.K * g.N + 4.0 * (double)g.M * g.N * (MODE == MODE_TN ? splits : 1));
  constexpr size_t lds_main = sizeof(__bf16) * 2 * (size_t)(BM + BN) * LDK;
  constexpr size_t lds_epi = sizeof(float) * 4 * 32 * EPI_LD2;
  constexpr size_t lds = lds_main > lds_epi ? lds_main : lds_epi;
  static_assert(lds <= 64 * 1024, "two slabs fit the default dynamic LDS limit");
  gemm_hh_kernel<BM, BN, WMS, WNS, MODE><<<grid, THREADS, lds, ctx->stream>>>(g);
  GP_LAUNCH_CHECK(ctx, "gemm_hh_kernel");
  return GP_OK;
}

// ---- C = A B^T with both operands stored as bf16 and k contiguous (activations times a weight matrix held as
// [N, K]), K a multiple of the slab depth BK: the tiles go from global memory straight into LDS (16-byte
// global->LDS loads: no registers, no LDS write instructions in the wavefronts' instruction streams) through a
// ring of STAGES LDS buffers.
//
// What bounds these GEMMs on this chip is the path from L2 into the compute unit, not the matrix cores: a
// 256x128 tile needs 47 bytes per clock and compute unit at full MFMA rate, and loads whose 64 lanes fetch
// 64-byte pieces of 16 different rows deliver about a quarter of that.  Hence 256x256 tiles (32 bytes per
// clock) and slabs of 64 k, so that every row contributes a whole 128-byte line to each load instruction
// (measured: twice the throughput of half lines).  Eight wavefronts share the tile; each owns 128x64.
//
// LDS tile layout: row r (an m or n index) occupies BK*2 bytes = BK/8 groups of 8 consecutive k; group c is
// stored at position c ^ swz(r) with swz(r) = (r >> 2) & 3 for 64-byte rows and (r >> 1) & 7 for 128-byte
// rows.  A global->LDS load writes the 64 lanes' 16 bytes to consecutive LDS addresses, so lane l of the load
// that covers groups [64 j, 64 j + 64) fetches the group that belongs there; the swizzle makes the fragment
// reads (32 rows x one group per half-wavefront) touch every bank equally.
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(1))) void* global_void_ptr;

// s_waitcnt with vmcnt = N, lgkmcnt = 0 (gfx9 encoding: vmcnt in bits [3:0] and [15:14], expcnt [6:4] = 7: no
// wait, lgkmcnt [11:8])
template <int N>
__device__ __forceinline__ void wait_vmcnt_lgkmcnt0() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | ((N >> 4) << 14));
}

// REFILL = false: the contraction is at most STAGES slabs long, the prologue has requested all of it and the loop requests
// nothing more (with refills, a 128-long contraction re-read its last slab twice: twice the load traffic).
template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int STAGES, bool REFILL = true>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N, WAVES_M * WAVES_N == 8 ? 1 : 2)
gemm_dl_kernel(const gemm_args g) {
  constexpr int NW = WAVES_M * WAVES_N;
  static_assert(NW == 4 || NW == 8, "one or two wavefronts per SIMD and workgroup");
  static_assert(BK == 32 || BK == 64, "slab depth");
  static_assert(STAGES == 2 || STAGES == 3, "ring depth");
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int MB = WM / 32, NB = WN / 32;
  constexpr int ROWB = BK * 2;                        // bytes per LDS row
  constexpr int CH = BK / 8;                          // 16-byte groups per row
  constexpr int KS = BK / 16;                         // MFMA steps per slab
  constexpr int STAGE_B = (BM + BN) * ROWB;           // bytes per stage
  constexpr int LOADS = (BM + BN) * CH / 64;          // wavefront-wide 16-byte loads per slab
  constexpr int PER = LOADS / NW;                     // per wavefront
  constexpr int A_LOADS = BM * CH / 64;
  static_assert(LOADS % NW == 0 && PER * (STAGES - 1) < 64, "the loads of a slab are dealt evenly to the wavefronts");
  extern __shared__ __attribute__((aligned(16))) float smem[];
  char* lds = reinterpret_cast<char*>(smem);

  const int tiles_n = (g.N + BN - 1) / BN;
  const int tiles_m = (int)((g.M + BM - 1) / BM);
  const int tile = xcd_remap(blockIdx.x, tiles_m * tiles_n);
  const int64_t m0 = (int64_t)(tile / tiles_n) * BM;
  const int n0 = (tile % tiles_n) * BN;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
  const int kh = lane >> 5, l32 = lane & 31;
  auto swz = [](int r) { return BK == 32 ? (r >> 2) & 3 : (r >> 1) & 7; };

  // this lane's source address for each of the wavefront's loads (slab 0); rows past the matrix are clamped
  const char* src[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int j = wave * PER + i;                     // load index within the slab (uniform)
    const bool is_a = j < A_LOADS;
    const int q = (is_a ? j : j - A_LOADS) * 64 + lane;
    const int row = q / CH, c = (q % CH) ^ swz(row);
    if (is_a) {
      const int64_t r = m0 + row < g.M ? m0 + row : g.M - 1;
      src[i] = reinterpret_cast<const char*>(g.A) + (r * g.lda + c * 8) * 2;
    } else {
      const int64_t r = n0 + row < g.N ? n0 + row : g.N - 1;
      src[i] = reinterpret_cast<const char*>(g.B) + (r * g.ldb + c * 8) * 2;
    }
  }
  const int n_slabs = g.K / BK;
  // a second operand pair continues the contraction: its slabs follow the first pair's, at the same offsets from
  // its own base addresses
  const int n1 = g.A2 ? n_slabs / 2 : n_slabs;
  const int64_t dA = g.A2 ? reinterpret_cast<const char*>(g.A2) - reinterpret_cast<const char*>(g.A) : 0;
  const int64_t dB = g.A2 ? reinterpret_cast<const char*>(g.B2) - reinterpret_cast<const char*>(g.B) : 0;
  auto issue = [&](int slab, int stage) __attribute__((always_inline)) {
    const int sl = slab < n_slabs ? slab : n_slabs - 1;   // past the end: re-read the last slab
    const bool second = sl >= n1;
    const int64_t kb = (int64_t)(second ? sl - n1 : sl) * ROWB;
    char* dst = lds + stage * STAGE_B + wave * PER * 1024;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int64_t d2 = second ? (wave * PER + i < A_LOADS ? dA : dB) : 0;   // uniform
      __builtin_amdgcn_global_load_lds((global_void_ptr)(src[i] + kb + d2), (lds_void_ptr)(dst + i * 1024), 16, 0, 0);
    }
  };

  f32x16 acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // fragment addresses inside a stage: row base plus, per MFMA step, the swizzled position of the lane's group
  const int sw = swz(l32);   // rows of a fragment differ from l32 by multiples of 32, which the swizzle ignores
  const int a_row = (wm0 + l32) * ROWB, b_row = BM * ROWB + (wn0 + l32) * ROWB;
  int koff[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) koff[ks] = ((2 * ks + kh) ^ sw) << 4;
  bf16x8 fa[2][MB], fb[2][NB];
  auto read_frags = [&](int stage, int ks) __attribute__((always_inline)) {
    const char* sa = lds + stage * STAGE_B + a_row + koff[ks];
    const char* sb = lds + stage * STAGE_B + b_row + koff[ks];
#pragma unroll
    for (int i = 0; i < MB; ++i) fa[ks & 1][i] = *reinterpret_cast<const bf16x8*>(sa + i * 32 * ROWB);
#pragma unroll
    for (int j = 0; j < NB; ++j) fb[ks & 1][j] = *reinterpret_cast<const bf16x8*>(sb + j * 32 * ROWB);
  };
  auto mfma_group = [&](int ks) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks & 1][i], fb[ks & 1][j], acc[i][j], 0, 0, 0);
  };

#pragma unroll
  for (int s = 0; s < STAGES; ++s) issue(s, s);
  wait_vmcnt_lgkmcnt0<(STAGES - 1) * PER>();   // slab 0 has landed (this wavefront's part)
  __syncthreads();                             // ... and everybody else's
  read_frags(0, 0);
  int st = 0;                                  // stage of slab t
  for (int t = 0; t < n_slabs; ++t) {
    const int st1 = st == STAGES - 1 ? 0 : st + 1;
    // While one MFMA group runs, the fragments of the next are on their way from LDS.  Before the last group
    // the wavefront holds all it needs from stage st in registers: after the barrier that stage is refilled
    // with slab t+STAGES, and the first fragments of slab t+1 (landed: each wavefront waited for its own loads
    // before the barrier) are requested.
#pragma unroll
    for (int ks = 0; ks + 1 < KS; ++ks) {
      read_frags(st, ks + 1);
      __builtin_amdgcn_sched_barrier(0);
      mfma_group(ks);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (REFILL) wait_vmcnt_lgkmcnt0<(STAGES - 2) * PER>();
    else wait_vmcnt_lgkmcnt0<0>();   // nothing is requested in the loop: every slab's loads were issued in the prologue
    __syncthreads();
    read_frags(st1, 0);
    __builtin_amdgcn_sched_barrier(0);
    {
      // The refill of the stage just freed goes out one load behind each MFMA of the slab's last group: issued in a
      // block right after the barrier, the loads held every wavefront's first MFMA back by their own issue time.
      const int slab = t + STAGES;
      const int sl = slab < n_slabs ? slab : n_slabs - 1;   // past the end: re-read the last slab
      const bool second = sl >= n1;
      const int64_t kb = (int64_t)(second ? sl - n1 : sl) * ROWB;
      char* dst = lds + st * STAGE_B + wave * PER * 1024;
      constexpr int LPM = (PER + MB * NB - 1) / (MB * NB);   // loads behind each MFMA (1 for the 256x256 tile)
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[(KS - 1) & 1][i], fb[(KS - 1) & 1][j], acc[i][j], 0, 0, 0);
#pragma unroll
          for (int u = 0; u < LPM; ++u) {
            const int q = (i * NB + j) * LPM + u;
            if (REFILL && q < PER) {
              const int64_t d2 = second ? (wave * PER + q < A_LOADS ? dA : dB) : 0;   // uniform
              __builtin_amdgcn_global_load_lds((global_void_ptr)(src[q] + kb + d2), (lds_void_ptr)(dst + q * 1024), 16, 0, 0);
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
    }
    st = st1;
  }
  wait_vmcnt_lgkmcnt0<0>();                    // the loads issued past the end must not land in the epilogue's staging area
  __syncthreads();
  tile_epilogue<MB, NB, MODE_NT, NW>(g, acc, smem, m0, n0, wm0, wn0, 0);
}

template <int BM, int BN, int WMS, int WNS, int BK, int STAGES, bool REFILL = true>
int launch_dl(gp_ctx* ctx, gemm_args& g) {
  const int64_t tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
  if (tiles > INT32_MAX) return gp_fail(ctx, GP_BAD_ARG, "gemm: too many tiles");
  static char name[48];
  if (!name[0]) snprintf(name, sizeof(name), "gemm_bf16_dl_nt_%dx%d%s", BM, BN, REFILL ? "" : "_shortk");
  const double mnk = (double)g.M * g.N * g.K;
  gp_prof_scope prof(ctx, name, 2.0 * mnk,
                     2.0 * (double)g.M * g.K + 2.0 * (double)g.K * g.N + ((g.epi.bf16 & EPI_BF_OUT) ? 2.0 : 4.0) * (double)g.M * g.N);
  constexpr int NW = WMS * WNS;
  constexpr size_t lds_main = (size_t)STAGES * (BM + BN) * BK * 2;
  constexpr size_t lds_epi = sizeof(float) * 2 * NW * 32 * EPI_LD2;   // accumulator blocks and low-rank factor blocks
  constexpr size_t lds = lds_main > lds_epi ? lds_main : lds_epi;
  static_assert((NW == 8 ? 1 : 2) * lds <= 160 * 1024, "fits the compute unit's LDS");
  if (g.epi.lr_a && (!g.vecC || !g.epi.lr_b || g.epi.lr_k < 1 || g.epi.lr_k > 16))
    return gp_fail(ctx, GP_BAD_ARG, "gemm: low-rank epilogue factor needs rank 1..16 and 16-byte aligned epilogue matrices");
  static bool raised = false;
  if (!raised && lds > 64 * 1024) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_dl_kernel<BM, BN, WMS, WNS, BK, STAGES, REFILL>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return gp_fail(ctx, GP_HIP_ERROR, "gemm: cannot raise the dynamic LDS limit to %zu bytes", lds);
    raised = true;
  }
  if (!REFILL && g.K > BK * STAGES) return gp_fail(ctx, GP_BAD_ARG, "gemm: contraction longer than the ring of the no-refill kernel");
  gemm_dl_kernel<BM, BN, WMS, WNS, BK, STAGES, REFILL><<<dim3((unsigned)tiles), 64 * NW, lds, ctx->stream>>>(g);
  GP_LAUNCH_CHECK(ctx, "gemm_dl_kernel");
  return GP_OK;
}

// ---- C = A^T B with both operands stored as bf16, [rows, M] and [rows, N], the contraction running over the rows (the
// weight gradients of the wide layers: rows = edges).  Both operands have the contraction index as their slow one, so
// a global->LDS load brings whole 512-byte row pieces [k][x] and the MFMA operand fragments (8 consecutive k for one
// x per lane) are read with the LDS transpose loads of this target: within 16 lanes, lane i of ds_read_b64_tr_b16
// receives element i % 4 of the 8 bytes addressed by lanes i / 4, 4 + i / 4, 8 + i / 4, 12 + i / 4 (checked on the
// device).  With lane i addressing k-row i / 4, x-columns 4 (i % 4) .. + 3 of a 4 x 16 block, it receives 4 consecutive k
// of column i.  No register staging, no repacking: the kernel that converts column pairs in registers spends as
// many vector instructions on that as on the products.
//
// 256x256 tiles, 8 wavefronts of 128x64 as in gemm_dl_kernel; a slab is BK rows of both operands (BK KB), ring of
// STAGES (64 rows, two stages).  LDS: [k][32 chunks of 16 bytes], chunk c of row k at position c ^ 2 (k % 4): the four rows a transpose load
// touches (32 bytes each) fall into four different quarters of the 128 bytes of banks.
// Workgroup = (tile, split): the splits cut the rows into runs of whole slabs; partial sums go to part[split].
typedef short v4s __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v4s* lds_v4s_ptr;

template <int BK, int STAGES>
__global__ void __launch_bounds__(512, 1)
gemm_tn_dl_kernel(const gemm_args g, int slabs_per_split) {
  constexpr int BM = 256, BN = 256, NW = 8, WAVES_N = 4, WM = 128, WN = 64, MB = 4, NB = 2;
  constexpr int PART_B = BK * 512;                    // bytes of one operand's slab
  constexpr int STAGE_B = 2 * PART_B;
  constexpr int PER = STAGE_B / 1024 / NW;            // 16-byte loads per wavefront and slab (two rows each)
  constexpr int KS = BK / 16;
  static_assert(BK % 16 == 0 && PER >= 1 && PER <= MB * NB && PER * (STAGES - 1) < 64, "slab shape");
  extern __shared__ __attribute__((aligned(16))) float smem[];
  char* lds = reinterpret_cast<char*>(smem);

  const int tiles_n = g.N / BN, tiles = (int)(g.M / BM) * tiles_n;
  const int wg = xcd_remap(blockIdx.x, gridDim.x);    // the tiles of a split (same rows of both operands) share an XCD's L2
  const int tile = wg % tiles, split = wg / tiles;
  const int64_t m0 = (int64_t)(tile / tiles_n) * BM;
  const int n0 = (tile % tiles_n) * BN;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
  const int64_t rows = g.K;
  const int64_t k_begin = (int64_t)split * slabs_per_split * BK;
  int64_t k_end = k_begin + (int64_t)slabs_per_split * BK;
  if (k_end > rows) k_end = rows;
  const int n_slabs = (int)((k_end - k_begin + BK - 1) / BK);   // >= 1: the host makes no empty split
  const int rem = (int)(k_end - k_begin) - (n_slabs - 1) * BK;  // rows of the last slab

  // this lane's source for each of the wavefront's loads (slab 0): wavefronts 0-3 bring A, 4-7 bring B
  const bool is_a = wave < NW / 2;
  const int64_t ld2 = (is_a ? g.lda : g.ldb) * 2;     // bytes per row
  const char* src[PER];   // the lane's 16 bytes in slab 0
  const char* lim[PER];   // the same columns in the matrix's last row: rows past it read that one (and are zeroed in LDS)
#pragma unroll
  for (int q = 0; q < PER; ++q) {
    const int j = (wave & 3) * PER + q;               // pair of rows within the operand's slab
    const int row = 2 * j + (lane >> 5), pos = lane & 31;
    const int c = pos ^ (2 * (row & 3));
    const char* col = is_a ? reinterpret_cast<const char*>(g.A) + (m0 + c * 8) * 2 : reinterpret_cast<const char*>(g.B) + ((int64_t)n0 + c * 8) * 2;
    src[q] = col + (k_begin + row) * ld2;
    lim[q] = col + (rows - 1) * ld2;
  }
  const int64_t slab_b = BK * ld2;
  auto issue_one = [&](int slab, int stage, int q) __attribute__((always_inline)) {
    const int sl = slab < n_slabs ? slab : n_slabs - 1;           // past the end: re-read the last slab
    const char* p = src[q] + sl * slab_b;
    p = p < lim[q] ? p : lim[q];
    char* dst = lds + stage * STAGE_B + (is_a ? 0 : PART_B) + ((wave & 3) * PER + q) * 1024;
    __builtin_amdgcn_global_load_lds((global_void_ptr)p, (lds_void_ptr)dst, 16, 0, 0);
  };
  // the last slab of the last split may be short: its missing rows are zeroed in LDS once it has landed
  auto zero_tail = [&](int stage) __attribute__((always_inline)) {
    typedef float f32x4_t __attribute__((ext_vector_type(4)));
    for (int part = 0; part < 2; ++part) {
      char* base = lds + stage * STAGE_B + part * PART_B + rem * 512;
      for (int i = threadIdx.x; i < (BK - rem) * 32; i += 512) *reinterpret_cast<f32x4_t*>(base + i * 16) = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }
    __syncthreads();
  };

  f32x16 acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // transpose-load addresses: 16-lane block b = lane / 16 holds k-half kh = b / 2 and x-half b % 2 of a 32-wide MFMA
  // block; its lane i addresses row 8 kh + 4 h + i / 4 (h = 0, 1: the two loads of a fragment), 8 bytes at x = 16 (b % 2) + 4 (i % 4)
  const int b16 = lane >> 4, i16 = lane & 15;
  const int kh = b16 >> 1;
  const int krow = 8 * kh + (i16 >> 2);               // + 4 h + 16 ks
  const int sw = 2 * (i16 >> 2);                      // 2 (row % 4): 4 h, 8 kh and 16 ks are multiples of 4
  int a_off[MB], b_off[NB];                           // byte offset of the lane's 8 bytes within a row, swizzled
#pragma unroll
  for (int i = 0; i < MB; ++i) {
    const int c = (wm0 + 32 * i) / 8 + 2 * (b16 & 1) + ((i16 & 3) >> 1);
    a_off[i] = ((c ^ sw) << 4) + ((i16 & 1) << 3);
  }
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    const int c = (wn0 + 32 * j) / 8 + 2 * (b16 & 1) + ((i16 & 3) >> 1);
    b_off[j] = PART_B + ((c ^ sw) << 4) + ((i16 & 1) << 3);
  }
  bf16x8 fa[2][MB], fb[2][NB];
  auto read_frags = [&](int stage, int ks) __attribute__((always_inline)) {
    const char* sb = lds + stage * STAGE_B + (16 * ks + krow) * 512;
#pragma unroll
    for (int i = 0; i < MB; ++i) {
      const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(sb + a_off[i]));
      const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(sb + 4 * 512 + a_off[i]));
      typedef short v8s __attribute__((ext_vector_type(8)));
      const v8s both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      fa[ks & 1][i] = __builtin_bit_cast(bf16x8, both);
    }
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(sb + b_off[j]));
      const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(sb + 4 * 512 + b_off[j]));
      typedef short v8s __attribute__((ext_vector_type(8)));
      const v8s both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      fb[ks & 1][j] = __builtin_bit_cast(bf16x8, both);
    }
  };
  auto mfma_group = [&](int ks) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks & 1][i], fb[ks & 1][j], acc[i][j], 0, 0, 0);
  };

#pragma unroll
  for (int s = 0; s < STAGES; ++s)
#pragma unroll
    for (int q = 0; q < PER; ++q) issue_one(s, s, q);
  wait_vmcnt_lgkmcnt0<(STAGES - 1) * PER>();   // slab 0 has landed (this wavefront's part)
  __syncthreads();                             // ... and everybody else's
  if (n_slabs == 1 && rem < BK) zero_tail(0);
  read_frags(0, 0);
  int st = 0;
  for (int t = 0; t < n_slabs; ++t) {
    const int st1 = st == STAGES - 1 ? 0 : st + 1;
#pragma unroll
    for (int ks = 0; ks + 1 < KS; ++ks) {
      read_frags(st, ks + 1);
      __builtin_amdgcn_sched_barrier(0);
      mfma_group(ks);
      __builtin_amdgcn_sched_barrier(0);
    }
    wait_vmcnt_lgkmcnt0<(STAGES - 2) * PER>();
    __syncthreads();
    if (t + 2 == n_slabs && rem < BK) zero_tail(st1);   // slab t + 1 is the short one (uniform)
    read_frags(st1, 0);
    __builtin_amdgcn_sched_barrier(0);
    {
      // the refill of the stage just freed, one load behind each MFMA of the slab's last group
      int q = 0;
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[(KS - 1) & 1][i], fb[(KS - 1) & 1][j], acc[i][j], 0, 0, 0);
          if (q < PER) issue_one(t + STAGES, st, q);
          ++q;
          __builtin_amdgcn_sched_barrier(0);
        }
    }
    st = st1;
  }
  wait_vmcnt_lgkmcnt0<0>();                    // the loads issued past the end must not land in the epilogue's staging area
  __syncthreads();
  tile_epilogue<MB, NB, MODE_TN>(g, acc, smem, m0, n0, wm0, wn0, split);
}

constexpr int TN_DL_BK = 64;   // rows per slab

// shapes the transposed global->LDS kernel takes: both operands bf16, widths multiples of 256, many rows
bool tn_dl_shape(const gemm_args& g) {
  return g.a_bf16 && g.b_bf16 && g.M % 256 == 0 && g.N % 256 == 0 && g.M <= 4096 && g.N <= 4096 && g.K >= 8192 && g.lda % 8 == 0 &&
         g.ldb % 8 == 0 && (reinterpret_cast<uintptr_t>(g.A) & 15) == 0 && (reinterpret_cast<uintptr_t>(g.B) & 15) == 0 && g.vecC;
}

int launch_tn_dl(gp_ctx* ctx, gemm_args& g, int splits) {
  constexpr int BK = TN_DL_BK, STAGES = 2;   // 32-row slabs with a ring of 3, 4 or 5: 10 % slower (twice the barriers per MFMA)
  const int tiles = (int)(g.M / 256) * (g.N / 256);
  const int64_t slabs = ((int64_t)g.K + BK - 1) / BK;
  const int per = (int)((slabs + splits - 1) / splits);
  if ((int64_t)(splits - 1) * per >= slabs) return gp_fail(ctx, GP_BAD_ARG, "gemm_tn: empty split in the plan");
  gp_prof_scope prof(ctx, "gemm_bf16_dl_tn_256x256", 2.0 * (double)g.M * g.N * g.K,
                     2.0 * (double)g.K * (g.M + g.N) + 4.0 * (double)g.M * g.N * splits);
  constexpr size_t lds_main = (size_t)STAGES * BK * 1024;
  constexpr size_t lds_epi = sizeof(float) * 8 * 32 * EPI_LD;
  constexpr size_t lds = lds_main > lds_epi ? lds_main : lds_epi;
  static_assert(lds <= 160 * 1024, "fits the compute unit's LDS");
  static bool raised = false;
  if (!raised) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_tn_dl_kernel<BK, STAGES>), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds) != hipSuccess)
      return gp_fail(ctx, GP_HIP_ERROR, "gemm: cannot raise the dynamic LDS limit to %zu bytes", lds);
    raised = true;
  }
  gemm_tn_dl_kernel<BK, STAGES><<<dim3((unsigned)(tiles * splits)), 512, lds, ctx->stream>>>(g, per);
  GP_LAUNCH_CHECK(ctx, "gemm_tn_dl_kernel");
  return GP_OK;
}

template <int BM, int BN, int WMS, int WNS, int MODE, bool VEC, bool ABF = false, bool BBF = false>
int launch_v(gp_ctx* ctx, gemm_args& g, int splits) {
  const int64_t tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
  if (tiles > INT32_MAX) return gp_fail(ctx, GP_BAD_ARG, "gemm: too many tiles");
  if (g.lda >= MAX_LD || g.ldb >= MAX_LD) return gp_fail(ctx, GP_BAD_ARG, "gemm (bf16): leading dimension above %lld", (long long)MAX_LD);
  dim3 grid((unsigned)tiles, (unsigned)splits, 1);
  static char name[48];
  if (!name[0])
    snprintf(name, sizeof(name), "gemm_bf16%s_%s_%dx%d", (ABF || BBF) ? (ABF && BBF ? "_hh" : ABF ? "_hf" : "_fh") : "",
             MODE == MODE_NN ? "nn" : MODE == MODE_NT ? "nt" : "tn", BM, BN);
  const double mnk = (double)g.M * g.N * g.K;
  gp_prof_scope prof(ctx, name, 2.0 * mnk,
                     (ABF ? 2.0 : 4.0) * (double)g.M * g.K + (BBF ? 2.0 : 4.0) * (double)g.K * g.N +
                         4.0 * (double)g.M * g.N * (MODE == MODE_TN ? splits : 1));
  constexpr size_t lds_main = sizeof(__bf16) * (size_t)(BM + BN) * LDK;
  constexpr size_t lds_epi = sizeof(float) * 4 * 32 * EPI_LD2;
  constexpr size_t lds = lds_main > lds_epi ? lds_main : lds_epi;
  static_assert(lds <= 64 * 1024, "tile fits the default dynamic LDS limit");
  gemm_bf16_kernel<BM, BN, WMS, WNS, MODE, VEC, ABF, BBF><<<grid, THREADS, lds, ctx->stream>>>(g);
  GP_LAUNCH_CHECK(ctx, "gemm_bf16_kernel");
  return GP_OK;
}

// both operands bf16: the register-pipelined kernel needs at least 64 columns per tile
template <int BM, int BN, int WMS, int WNS, int MODE>
int launch_both_bf16(gp_ctx* ctx, gemm_args& g, int splits) {
  if constexpr (BN >= 64) return launch_hh<BM, BN, WMS, WNS, MODE>(ctx, g, splits);
  else return launch_v<BM, BN, WMS, WNS, MODE, true, true, true>(ctx, g, splits);
}

template <int MODE>
int dispatch(gp_ctx* ctx, gemm_args& g, int splits) {
  // an operand stored as bf16 must satisfy its loader's alignment (vecA / vecB say so); VEC then only
  // describes the remaining fp32 operand
  if ((g.a_bf16 && !g.vecA) || (g.b_bf16 && !g.vecB))
    return gp_fail(ctx, GP_BAD_ARG, "gemm (bf16 storage): operand not aligned / extent not a multiple of 8");
#define GP_BF16_LAUNCH(BM, BN, WMS, WNS)                                                                            \
  do {                                                                                                              \
    if (g.a_bf16 && g.b_bf16) return launch_both_bf16<BM, BN, WMS, WNS, MODE>(ctx, g, splits);                      \
    if (g.a_bf16) {                                                                                                 \
      if (g.vecB) return launch_v<BM, BN, WMS, WNS, MODE, true, true, false>(ctx, g, splits);                       \
      return launch_v<BM, BN, WMS, WNS, MODE, false, true, false>(ctx, g, splits);                                  \
    }                                                                                                               \
    if (g.b_bf16) {                                                                                                 \
      if (g.vecA) return launch_v<BM, BN, WMS, WNS, MODE, true, false, true>(ctx, g, splits);                       \
      return launch_v<BM, BN, WMS, WNS, MODE, false, false, true>(ctx, g, splits);                                  \
    }                                                                                                               \
    if (g.vecA && g.vecB) return launch_v<BM, BN, WMS, WNS, MODE, true>(ctx, g, splits);                            \
    return launch_v<BM, BN, WMS, WNS, MODE, false>(ctx, g, splits);                                                 \
  } while (0)
  // tall activations times a wide weight matrix, both bf16 and k-contiguous: global->LDS loads, 256x256 tiles
  if (MODE == MODE_NT && g.a_bf16 && g.b_bf16 && g.M >= 8192 && g.N > 128 && g.K % 64 == 0 && g.K >= 128 &&
      g.lda % 8 == 0 && g.ldb % 8 == 0 && (!g.A2 || g.K % 128 == 0))
    return g.K <= 128 ? launch_dl<256, 256, 2, 4, 64, 2, false>(ctx, g) : launch_dl<256, 256, 2, 4, 64, 2>(ctx, g);
  // ... times a narrow one (a long contraction into 33..128 columns): the same kernel streams the activations, which is all
  // that bounds these products, through a deeper ring; 8 wavefronts of 64x64 or 32x64
  if (MODE == MODE_NT && g.a_bf16 && g.b_bf16 && g.M >= 8192 && g.N > 32 && g.N <= 128 && g.K % 64 == 0 && g.K >= 256 &&
      g.lda % 8 == 0 && g.ldb % 8 == 0 && !g.A2 && !g.epi.lr_a) {
    if (g.N > 64) return launch_dl<256, 128, 4, 2, 64, 3>(ctx, g);
    return launch_dl<256, 64, 8, 1, 64, 3>(ctx, g);
  }
  if (g.A2) return gp_fail(ctx, GP_BAD_ARG, "gemm: a second operand pair is only taken by the global->LDS kernel");
  if (g.epi.lr_a) return gp_fail(ctx, GP_BAD_ARG, "gemm: a low-rank epilogue factor is only taken by the global->LDS kernel");
  // the reduction over rows (TN) keeps the 128-row tiles its split plan was made for
  // short contractions are all prologue and epilogue: smaller tiles, more workgroups per CU to overlap them
  if (MODE != MODE_TN && g.K <= 128 && g.N > 64) GP_BF16_LAUNCH(128, 128, 2, 2);
  if (MODE != MODE_TN && g.M >= 8192 && g.N > 64) GP_BF16_LAUNCH(256, 128, 2, 2);
  if (g.N > 64) GP_BF16_LAUNCH(128, 128, 2, 2);
  if (g.N > 32) GP_BF16_LAUNCH(128, 64, 2, 2);
  GP_BF16_LAUNCH(128, 32, 4, 1);
#undef GP_BF16_LAUNCH
}

}  // namespace

// ---- C = A^T B with fp32 operands [rows, M], [rows, N] as three bf16 planes each (see gemm_split_kernel): the weight
// gradients of the fp32 blocks.  The contraction index is the slow one of both operands, so a slab (32 rows x 128
// columns per operand) is split where it is loaded, 4 consecutive columns per thread, and stored as it lies in memory,
// [plane][k][x] in bf16; the MFMA operand fragments (8 consecutive k of one x per lane) come from the LDS transpose loads
// as in gemm_tn_dl_kernel (chunk c of row k at c ^ 2 (k % 4)), so nothing is transposed in registers.  128x128 tiles, four
// wavefronts of 64x64, grid (tiles, splits) and partial sums as the fp32 kernel's plan (tn_plan) lays them out; the
// column sums of B (bias gradients) are taken from the loaded fp32 values.  Needs 16-byte aligned rows (the caller
// falls back to the fp32-operand kernel otherwise).
__global__ void __launch_bounds__(THREADS, 2)
gemm_split_tn_kernel(const gemm_args g) {
  constexpr int PL = 3, BM = 128, BN = 128, BK = 32, MB = 2, NB = 2;
  constexpr int ROW_B = 256;                          // bytes of a slab row of one operand and plane (128 bf16)
  constexpr int PLANE_B = BK * ROW_B, OPER_B = PL * PLANE_B;
  extern __shared__ __attribute__((aligned(16))) float smem[];
  char* lds = reinterpret_cast<char*>(smem);

  const int tiles_n = (g.N + BN - 1) / BN;
  const int tiles_m = (int)((g.M + BM - 1) / BM);
  const int tile = xcd_remap(blockIdx.x, tiles_m * tiles_n);
  const int tile_m = tile / tiles_n;
  const int m0 = tile_m * BM, n0 = (tile % tiles_n) * BN;
  const int64_t k_begin = (int64_t)blockIdx.y * g.k_per_split;
  const int64_t k_end = k_begin + g.k_per_split < (int64_t)g.K ? k_begin + g.k_per_split : (int64_t)g.K;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm0 = (wave >> 1) * 64, wn0 = (wave & 1) * 64;

  // loader: thread t holds, per operand, the 4 columns 4 (t % 32) .. + 3 of the rows t / 32 + 8 i (i = 0..3) of the slab;
  // columns past the matrix are read from its last 4 (their products are never stored)
  const int lx = (threadIdx.x & 31) * 4, lr = threadIdx.x >> 5;
  const int ax = m0 + lx + 4 <= (int)g.M ? m0 + lx : (int)g.M - 4;
  const int bx = n0 + lx + 4 <= g.N ? n0 + lx : g.N - 4;
  f32x4 ra[4], rb[4];
  auto fetch = [&](int64_t k0) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t k = k0 + lr + 8 * i;
      const int64_t kc = k < k_end ? k : k_end - 1;   // rows past the end: a valid row, zeroed below
      ra[i] = *reinterpret_cast<const f32x4*>(g.A + kc * g.lda + ax);
      rb[i] = *reinterpret_cast<const f32x4*>(g.B + kc * g.ldb + bx);
    }
  };
  f32x4 cs = {0.f, 0.f, 0.f, 0.f};                   // column sums of B over this thread's rows
  const bool want_cs = g.colsum_part != nullptr;
  auto split4 = [&](char* dst, f32x4 v) __attribute__((always_inline)) {
#pragma unroll
    for (int p = 0; p < PL; ++p) {
      bf16x4 h;
#pragma unroll
      for (int c = 0; c < 4; ++c) h[c] = (__bf16)v[c];
      *reinterpret_cast<bf16x4*>(dst + p * PLANE_B) = h;
      if (p + 1 < PL) {
#pragma unroll
        for (int c = 0; c < 4; ++c) v[c] -= (float)h[c];
      }
    }
  };
  auto store = [&](int64_t k0, int slab) __attribute__((always_inline)) {
    const bool mine = want_cs && (slab % tiles_m) == tile_m;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = lr + 8 * i;
      const float keep = k0 + row < k_end ? 1.f : 0.f;
      const int off = row * ROW_B + ((((lx >> 3) ^ (2 * (row & 3)))) << 4) + ((lx & 4) << 1);
      split4(lds + off, ra[i] * keep);
      split4(lds + OPER_B + off, rb[i] * keep);
      if (mine) cs += rb[i] * keep;
    }
  };

  f32x16 acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // transpose-load addresses (see gemm_tn_dl_kernel): 16-lane block b holds k-half b / 2 and x-half b % 2 of a 32-wide block
  const int b16 = lane >> 4, i16 = lane & 15;
  const int krow = 8 * (b16 >> 1) + (i16 >> 2);       // + 4 h + 16 ks
  const int sw = 2 * (i16 >> 2);
  int a_off[MB], b_off[NB];
#pragma unroll
  for (int i = 0; i < MB; ++i) a_off[i] = ((((wm0 + 32 * i) / 8 + 2 * (b16 & 1) + ((i16 & 3) >> 1)) ^ sw) << 4) + ((i16 & 1) << 3);
#pragma unroll
  for (int j = 0; j < NB; ++j) b_off[j] = OPER_B + ((((wn0 + 32 * j) / 8 + 2 * (b16 & 1) + ((i16 & 3) >> 1)) ^ sw) << 4) + ((i16 & 1) << 3);
  auto frag = [&](const char* p) __attribute__((always_inline)) {
    const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)p);
    const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(p + 4 * ROW_B));
    typedef short v8s __attribute__((ext_vector_type(8)));
    const v8s both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, both);
  };
  auto multiply = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      const char* sb = lds + (16 * ks + krow) * ROW_B;
      bf16x8 a[PL][MB], b[PL][NB];
#pragma unroll
      for (int p = 0; p < PL; ++p) {
#pragma unroll
        for (int i = 0; i < MB; ++i) a[p][i] = frag(sb + p * PLANE_B + a_off[i]);
#pragma unroll
        for (int j = 0; j < NB; ++j) b[p][j] = frag(sb + p * PLANE_B + b_off[j]);
      }
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) {
          f32x16 c = acc[i][j];
          c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2][i], b[0][j], c, 0, 0, 0);
          c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0][i], b[2][j], c, 0, 0, 0);
          c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1][i], b[1][j], c, 0, 0, 0);
          c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1][i], b[0][j], c, 0, 0, 0);
          c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0][i], b[1][j], c, 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0][i], b[0][j], c, 0, 0, 0);
        }
    }
  };

  if (k_begin < k_end) {
    const int n_slabs = (int)((k_end - k_begin + BK - 1) / BK);
    fetch(k_begin);
    store(k_begin, 0);
    __syncthreads();
    for (int s = 1; s < n_slabs; ++s) {
      fetch(k_begin + (int64_t)s * BK);
      multiply();
      __syncthreads();
      store(k_begin + (int64_t)s * BK, s);
      __syncthreads();
    }
    multiply();
  }
  __syncthreads();   // all wavefronts are done with the operand planes; LDS is reused below
  if (want_cs) {
    // the 8 threads that share 4 columns (one per row group) sit in different wavefronts: through LDS, fixed order
    float* red = smem;
    *reinterpret_cast<f32x4*>(red + lr * BN + lx) = cs;
    __syncthreads();
    if (threadIdx.x < BN) {
      float t = 0.f;
#pragma unroll
      for (int r = 0; r < 8; ++r) t += red[r * BN + threadIdx.x];
      // a thread whose columns were clamped into the matrix holds sums of other columns: only true columns are written
      if (n0 + (int)threadIdx.x < g.N) g.colsum_part[((int64_t)blockIdx.y * tiles_m + tile_m) * g.N + n0 + threadIdx.x] = t;
    }
    __syncthreads();
  }
  tile_epilogue_f32<MB, NB, MODE_TN>(g, acc, smem, m0, n0, wm0, wn0, blockIdx.y);
}

template <int BM, int BN, int WMS, int WNS, int MODE>
int launch_split(gp_ctx* ctx, gemm_args& g, int splits) {
  const int64_t tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
  if (tiles > INT32_MAX) return gp_fail(ctx, GP_BAD_ARG, "gemm: too many tiles");
  if (g.lda >= MAX_LD || g.ldb >= MAX_LD) return gp_fail(ctx, GP_BAD_ARG, "gemm (split fp32): leading dimension above %lld", (long long)MAX_LD);
  dim3 grid((unsigned)tiles, (unsigned)splits, 1);
  static char name[48];
  if (!name[0]) snprintf(name, sizeof(name), "gemm_f32x3_%s_%dx%d", MODE == MODE_NN ? "nn" : MODE == MODE_NT ? "nt" : "tn", BM, BN);
  const double mnk = (double)g.M * g.N * g.K;
  gp_prof_scope prof(ctx, name, 2.0 * mnk,
                     4.0 * ((double)g.M * g.K + (double)g.K * g.N + (double)g.M * g.N * (MODE == MODE_TN ? splits : 1)));
  constexpr size_t lds_main = sizeof(__bf16) * 3 * (size_t)(BM + BN) * LDK;
  constexpr size_t lds_epi = sizeof(float) * 4 * 32 * EPI_LD;
  constexpr size_t lds = lds_main > lds_epi ? lds_main : lds_epi;
  static_assert(lds <= 64 * 1024, "tile fits the default dynamic LDS limit");
  if (g.vecA && g.vecB) gemm_split_kernel<BM, BN, WMS, WNS, MODE, true><<<grid, THREADS, lds, ctx->stream>>>(g);
  else gemm_split_kernel<BM, BN, WMS, WNS, MODE, false><<<grid, THREADS, lds, ctx->stream>>>(g);
  GP_LAUNCH_CHECK(ctx, "gemm_split_kernel");
  return GP_OK;
}

int launch_split_tn(gp_ctx* ctx, gemm_args& g, int splits) {
  const int64_t tiles = ((g.M + 127) / 128) * ((g.N + 127) / 128);
  if (tiles > INT32_MAX) return gp_fail(ctx, GP_BAD_ARG, "gemm: too many tiles");
  if (!gp_gemm_split_tn_ok(g.M, g.N, g.vecA, g.vecB)) return gp_fail(ctx, GP_BAD_ARG, "gemm (split fp32, A^T B): shape or alignment not taken");
  gp_prof_scope prof(ctx, "gemm_f32x3_tn_128x128", 2.0 * (double)g.M * g.N * g.K,
                     4.0 * ((double)g.M * g.K + (double)g.K * g.N + (double)g.M * g.N * splits));
  constexpr size_t lds = 2 * 3 * 32 * 256;   // both operands, three planes, 32 rows of 128 bf16 (above the epilogue's staging)
  static_assert(lds >= sizeof(float) * 4 * 32 * EPI_LD && lds >= sizeof(float) * 8 * 128 && lds <= 64 * 1024, "LDS uses of the kernel");
  gemm_split_tn_kernel<<<dim3((unsigned)tiles, (unsigned)splits, 1), THREADS, lds, ctx->stream>>>(g);
  GP_LAUNCH_CHECK(ctx, "gemm_split_tn_kernel");
  return GP_OK;
}

template <int MODE>
int dispatch_split(gp_ctx* ctx, gemm_args& g, int splits) {
  if constexpr (MODE == MODE_TN) return launch_split_tn(ctx, g, splits);
  else {
  // wide results with work for every compute unit several times over: twice the MFMAs per operand fragment read
  if (g.N > 64 && ((g.M + 127) / 128) * ((g.N + 127) / 128) >= 2048) return launch_split<128, 128, 2, 2, MODE>(ctx, g, splits);
  if (g.N > 64) return launch_split<128, 64, 2, 2, MODE>(ctx, g, splits);
  return launch_split<128, 32, 4, 1, MODE>(ctx, g, splits);
  }
}

// The transposed global->LDS kernel: whether it takes the shape, how it splits the rows (about one workgroup per compute
// unit: tiles x splits), and its launch.  gp_gemm_tn sizes its partial sums with the same plan.
int gp_gemm_bf16_tn_dl_splits(int64_t rows, int M, int N) {
  if (M % 256 || N % 256 || M > 4096 || N > 4096 || rows < 8192) return 0;
  const int tiles = (M / 256) * (N / 256);
  const int64_t slabs = (rows + TN_DL_BK - 1) / TN_DL_BK;
  int64_t s = tiles >= 256 ? 1 : 256 / tiles;
  if (s > slabs) s = slabs;
  const int64_t per = (slabs + s - 1) / s;
  return (int)((slabs + per - 1) / per);
}
bool gp_gemm_bf16_tn_dl_ok(const void* args) { return tn_dl_shape(*static_cast<const gemm_args*>(args)); }
int gp_gemm_bf16_tn_dl(gp_ctx* ctx, void* args, int splits) { return launch_tn_dl(ctx, *static_cast<gemm_args*>(args), splits); }

// Called by gp_gemm_nn / gp_gemm_nt / gp_gemm_tn when the context asks for bf16 operands; `g` has
// been filled exactly as for the fp32 kernels (same tile geometry, same split-K plan).
int gp_gemm_bf16_launch(gp_ctx* ctx, int mode, void* args, int splits) {
  gemm_args& g = *static_cast<gemm_args*>(args);
  if (mode == MODE_NN) return dispatch<MODE_NN>(ctx, g, splits);
  if (mode == MODE_NT) return dispatch<MODE_NT>(ctx, g, splits);
  return dispatch<MODE_TN>(ctx, g, splits);
}

// fp32 operands and result through three bf16 planes per operand (gemm_split_kernel); `g` filled as for the fp32 kernels
int gp_gemm_split_launch(gp_ctx* ctx, int mode, void* args, int splits) {
  gemm_args& g = *static_cast<gemm_args*>(args);
  if (mode == MODE_NN) return dispatch_split<MODE_NN>(ctx, g, splits);
  if (mode == MODE_NT) return dispatch_split<MODE_NT>(ctx, g, splits);
  return dispatch_split<MODE_TN>(ctx, g, splits);
}

// A^T B in the three-plane form: 128-wide tiles of its plan (N > 64), rows of both operands in 16-byte pieces
bool gp_gemm_split_tn_ok(int64_t M, int N, int vecA, int vecB) { return N > 64 && M >= 4 && vecA && vecB; }
