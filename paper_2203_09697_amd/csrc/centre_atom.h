// Helpers shared by the kernels that regroup the triplet sums by centre atom (the atom j shared by the two edges
// of a triplet k->j->i): workgroup numbering over (atom, part) pairs, the share of one workgroup, the search for
// the one row a segment leaves out, and the Legendre tables.  Internal, not part of the C ABI.
#pragma once
#include "common.h"

namespace {


typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int ST = 8;        // max num_spherical
constexpr int CP = 16;       // rows per edge in an MFMA tile = max emb_cbf
constexpr int PARTS = 8;     // at most this many workgroups share one centre atom
#ifndef GP_PARTS_IN
#define GP_PARTS_IN 12
#endif
constexpr int PARTS_IN = GP_PARTS_IN;   // ... for the backward kernels, whose shares are in-edge rows (configuration 4: H kernel 1.19 ms
                                        // with 8, 1.04 with 12 or 16; the forward kernels get 1 % slower above 8)
constexpr int EPP = 64;      // target edges per workgroup
constexpr int YT = 256;      // most threads of the y kernel (one per position of the longest row, rounded to 64)
constexpr int MT = 512;      // most threads of the contraction kernel
constexpr int KU = 4;        // k-steps of A fragments loaded ahead
constexpr size_t LDS_MAX = 160 * 1024;

__device__ __constant__ float Y_NORM_M[ST] = {
    0.28209479177387814f, 0.4886025119029199f, 0.6307831305050401f, 0.7463526651802308f,
    0.8462843753216345f, 0.9356025796273888f, 1.0171072362820548f, 1.0925484305920792f};  // sqrt((2l+1)/(4 pi))


// wavefront-local ordering of LDS traffic (no other wavefront touches the slice concerned)
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Workgroup ids are dealt round-robin to the 8 XCDs.  Numbering the (atom, part) pairs atom-major and giving
// each XCD a contiguous range of them keeps every XCD equally busy (with part = id % 8 the XCDs that get the
// high part numbers, which most atoms do not have, would idle) and runs the parts of one atom, which read the
// same in-edge rows, side by side on one L2.
__device__ __forceinline__ void atom_and_part(int parts, int& j, int& part) {
  const int n = (int)gridDim.x, q = n >> 3, r = n & 7;
  const int x = (int)blockIdx.x & 7, i = (int)blockIdx.x >> 3;
  const int w = x * q + (x < r ? x : r) + i;
  j = w / parts;
  part = w % parts;
}

// Edge id of row position pos: the rows of an atom are consecutive edge ids (edges are sorted by target atom) unless
// a list is given (the mirrored use: rows are the atom's out-edges, listed in out_list order).
__device__ __forceinline__ int row_edge(const int32_t* __restrict__ row_list, int pos) { return row_list ? row_list[pos] : pos; }

// First slot of a segment whose entry differs from the expected one, given that entries match up to some slot and
// differ from it on (the segment is the expected list with at most one element left out); cnt if none differs.
// (An 8-way search with its 8 probes loaded together, 3 memory round trips instead of 9 for 512 slots, measured
// slower than this binary search: 0.117 vs 0.106 ms for the variant-D forward kernel at configuration 2.)
template <class Expected>
__device__ __forceinline__ int first_mismatch(const int32_t* __restrict__ seg_list, int cnt, Expected expected) {
  int lo = 0, hi = cnt;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (seg_list[mid] == expected(mid)) lo = mid + 1;
    else hi = mid;
  }
  return lo;
}

// The share of one workgroup: centre atom j, its in-edge rows r0 .. r0+d-1
// (Kp = d rounded up to 16) and the slice [eb, ee) of its out-edge list.
struct part_t {
  int r0, d, Kp, o0, eb, ee;
};

// false (for every thread of the workgroup alike) if this workgroup has nothing to do
__device__ __forceinline__ bool centre_part(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ out_ptr,
                                            int kp_cap, int parts, part_t& P) {
  int j, part;
  atom_and_part(parts, j, part);
  P.r0 = row_ptr[j];
  P.d = row_ptr[j + 1] - P.r0;
  P.Kp = (P.d + 15) & ~15;
  P.o0 = out_ptr[j];
  const int dout = out_ptr[j + 1] - P.o0;
  if (dout <= 0 || P.Kp > kp_cap) return false;
  int nparts = (dout + EPP - 1) / EPP;
  nparts = nparts < parts ? nparts : parts;
  if (part >= nparts) return false;
  const int len = (((dout + nparts - 1) / nparts) + 3) & ~3;
  P.eb = part * len;
  P.ee = P.eb + len < dout ? P.eb + len : dout;
  return P.eb < P.ee;
}


// coefficient of x^k in the Legendre polynomial P_l, l <= 7
__host__ __device__ constexpr float leg_mono(int l, int k) {
  constexpr float T[8][8] = {{1.f},
                             {0.f, 1.f},
                             {-0.5f, 0.f, 1.5f},
                             {0.f, -1.5f, 0.f, 2.5f},
                             {0.375f, 0.f, -3.75f, 0.f, 4.375f},
                             {0.f, 1.875f, 0.f, -8.75f, 0.f, 7.875f},
                             {-0.3125f, 0.f, 6.5625f, 0.f, -19.6875f, 0.f, 14.4375f},
                             {0.f, -2.1875f, 0.f, 19.6875f, 0.f, -43.3125f, 0.f, 26.8125f}};
  return T[l][k];
}
// ---- shared by the one-pass kernels that stage per-atom operand tables through an LDS ring (triplet_g_fused*.hip)
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(1))) void* global_void_ptr;

constexpr int ROWPAD = 64;      // every atom's rows are padded to a multiple of this in the packed tables
constexpr int PADJ = 72;        // padded row space per atom: base_j = roundup8(row_ptr[j]) + PADJ j leaves room for
                                // rounding every atom's rows up to a multiple of 64 (d + 63) on an 8-aligned base (+ 7)
__host__ __device__ inline int64_t padded_base(int r0, int64_t j) { return (((int64_t)r0 + 7) & ~(int64_t)7) + PADJ * j; }
inline int64_t padded_rows(int64_t E, int64_t N) { return ((E + 7) & ~(int64_t)7) + PADJ * N + ROWPAD; }

// Row r of a 16-row tile t of the matrix-core product stands for feature NT * rowperm(r) + t.  With rowperm the
// transposition of r = 4 g + i to 4 i + g, the 4 accumulator registers i of lane (g, c) hold, over the NT tiles,
// features NT (4 i + g) .. + NT - 1: for every i the lanes g = 0..3 of a column c together own 4 NT consecutive
// features, so a store instruction writes whole 64-byte runs (NT = 8, bf16).  In LDS a slab's X^T is ordered
// [p-block][t][r], so the 16 lanes of a fragment read 256 consecutive bytes.
__device__ __forceinline__ int rowperm(int r) { return ((r & 3) << 2) | (r >> 2); }

// s_waitcnt vmcnt(N) only (gfx9 encoding: vmcnt in bits [3:0] and [15:14], expcnt [6:4] = 7 and lgkmcnt [11:8] = 15: no wait)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}
__device__ __forceinline__ void wait_vm0() { wait_vmcnt<0>(); }
constexpr int STAGES = 3;       // LDS ring: the loads of two slabs are under way while a third is worked on


}  // namespace
