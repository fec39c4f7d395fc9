// Radius-graph construction and triplet enumeration (paper Sec. 3.1; the index set
// N_j \ {i} of the update equation in Sec. 3.3).  Integer outputs are bit-exact and
// deterministic: positions are compared with an uncontracted fp32 expression, output
// slots come from wavefront ballots and prefix counts, never from atomics' arrival order.
#include <stdarg.h>

#include "common.h"

namespace {

// ------------------------------------------------------------------ exclusive scan
// One workgroup walks the array in chunks of its own size, carrying the running total.
// in[n] (int32) -> out[n+1] (int32, exclusive prefix, out[n] = total); total64 gets the
// untruncated sum so the host can detect int32 overflow.
constexpr int SCAN_THREADS = 1024;
__global__ void __launch_bounds__(SCAN_THREADS)
scan_exclusive_kernel(const int32_t* __restrict__ in, int32_t* __restrict__ out, int64_t n,
                      int64_t* __restrict__ total64) {
  __shared__ int64_t wave_tot[SCAN_THREADS / WAVE];
  __shared__ int64_t carry_s;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  if (tid == 0) carry_s = 0;
  __syncthreads();
  for (int64_t base = 0; base < n; base += SCAN_THREADS) {
    int64_t i = base + tid;
    int64_t v = (i < n) ? (int64_t)in[i] : 0;
    int64_t incl = v;
#pragma unroll
    for (int o = 1; o < WAVE; o <<= 1) {
      int64_t u = __shfl_up(incl, o, WAVE);
      if (lane >= o) incl += u;
    }
    if (lane == WAVE - 1) wave_tot[w] = incl;
    __syncthreads();
    int64_t before = carry_s;
    for (int k = 0; k < w; ++k) before += wave_tot[k];
    if (i < n) out[i] = (int32_t)(before + incl - v);
    __syncthreads();
    if (tid == SCAN_THREADS - 1) carry_s = before + incl;
    __syncthreads();
  }
  if (tid == 0) {
    out[n] = (int32_t)carry_s;
    *total64 = carry_s;
  }
}

// The same scan for long arrays as three launches: every workgroup sums its chunk of SCAN_CHUNK elements, one
// workgroup scans the chunk sums, every workgroup scans its chunk again from its offset.  (The single-workgroup
// kernel above took 0.2-0.4 ms for the 3e5 edges of the largest workload.)
constexpr int SCAN_CHUNK = 4 * SCAN_THREADS;
__device__ __forceinline__ int64_t block_sum_i64(int64_t v, int64_t* wave_tot) {
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  if (lane == 0) wave_tot[w] = v;
  __syncthreads();
  int64_t s = 0;
  for (int k = 0; k < SCAN_THREADS / WAVE; ++k) s += wave_tot[k];
  return s;
}
__global__ void __launch_bounds__(SCAN_THREADS)
scan_chunk_sums_kernel(const int32_t* __restrict__ in, int64_t n, int64_t* __restrict__ sums) {
  __shared__ int64_t wave_tot[SCAN_THREADS / WAVE];
  const int64_t base = (int64_t)blockIdx.x * SCAN_CHUNK + 4 * (int64_t)threadIdx.x;
  int64_t v = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) v += base + i < n ? (int64_t)in[base + i] : 0;
  const int64_t s = block_sum_i64(v, wave_tot);
  if (threadIdx.x == 0) sums[blockIdx.x] = s;
}
// one workgroup: sums[nb] -> exclusive offsets in place, total64 = the grand total
__global__ void __launch_bounds__(SCAN_THREADS)
scan_sums_kernel(int64_t* __restrict__ sums, int64_t nb, int64_t* __restrict__ total64) {
  __shared__ int64_t wave_tot[SCAN_THREADS / WAVE];
  __shared__ int64_t carry_s;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  if (tid == 0) carry_s = 0;
  __syncthreads();
  for (int64_t base = 0; base < nb; base += SCAN_THREADS) {
    const int64_t i = base + tid;
    const int64_t v = i < nb ? sums[i] : 0;
    int64_t incl = v;
#pragma unroll
    for (int o = 1; o < WAVE; o <<= 1) {
      const int64_t u = __shfl_up(incl, o, WAVE);
      if (lane >= o) incl += u;
    }
    if (lane == WAVE - 1) wave_tot[w] = incl;
    __syncthreads();
    int64_t before = carry_s;
    for (int k = 0; k < w; ++k) before += wave_tot[k];
    if (i < nb) sums[i] = before + incl - v;
    __syncthreads();
    if (tid == SCAN_THREADS - 1) carry_s = before + incl;
    __syncthreads();
  }
  if (tid == 0) *total64 = carry_s;
}
__global__ void __launch_bounds__(SCAN_THREADS)
scan_chunk_apply_kernel(const int32_t* __restrict__ in, const int64_t* __restrict__ offs, const int64_t* __restrict__ total64,
                        int64_t n, int32_t* __restrict__ out) {
  __shared__ int64_t wave_tot[SCAN_THREADS / WAVE];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int64_t base = (int64_t)blockIdx.x * SCAN_CHUNK + 4 * (int64_t)tid;
  int64_t v[4], mine = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    v[i] = base + i < n ? (int64_t)in[base + i] : 0;
    mine += v[i];
  }
  int64_t incl = mine;
#pragma unroll
  for (int o = 1; o < WAVE; o <<= 1) {
    const int64_t u = __shfl_up(incl, o, WAVE);
    if (lane >= o) incl += u;
  }
  if (lane == WAVE - 1) wave_tot[w] = incl;
  __syncthreads();
  int64_t run = offs[blockIdx.x] + incl - mine;
  for (int k = 0; k < w; ++k) run += wave_tot[k];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (base + i < n) out[base + i] = (int32_t)run;
    run += v[i];
  }
  if (blockIdx.x == 0 && tid == 0) out[n] = (int32_t)*total64;
}
inline int64_t scan_chunks(int64_t n) { return (n + SCAN_CHUNK - 1) / SCAN_CHUNK; }

// ------------------------------------------------------------------ edges
// The distance predicate: every operation rounded once to fp32, no fused multiply-add.
__device__ __forceinline__ float dist2_f32(float xi, float yi, float zi, float xj, float yj, float zj) {
#pragma clang fp contract(off)
  float dx = __fsub_rn(xi, xj), dy = __fsub_rn(yi, yj), dz = __fsub_rn(zi, zj);
  return __fadd_rn(__fadd_rn(__fmul_rn(dx, dx), __fmul_rn(dy, dy)), __fmul_rn(dz, dz));
}

// Periodic images tested per source atom: n_a = -rep[a] .. rep[a]; image index img counts them in
// lexicographic order of (n0, n1, n2).  Without a cell there is the one image n = 0.
struct images_t {
  const float* cell;   // [G, 3, 3] rows = lattice vectors, or NULL
  int r0, r1, r2;
  __host__ __device__ int count() const { return cell ? (2 * r0 + 1) * (2 * r1 + 1) * (2 * r2 + 1) : 1; }
};

// shift of image (n0, n1, n2) of structure g: n0 a0 + n1 a1 + n2 a2, every product and sum rounded once
__device__ __forceinline__ void image_of(const images_t& im, int g, int img, int& n0, int& n1, int& n2, float& sx,
                                         float& sy, float& sz) {
#pragma clang fp contract(off)
  if (!im.cell) {
    n0 = n1 = n2 = 0;
    sx = sy = sz = 0.f;
    return;
  }
  const int w2 = 2 * im.r2 + 1, w1 = 2 * im.r1 + 1;
  n2 = img % w2 - im.r2;
  n1 = (img / w2) % w1 - im.r1;
  n0 = img / (w2 * w1) - im.r0;
  const float* c = im.cell + 9 * (int64_t)g;
  const float f0 = (float)n0, f1 = (float)n1, f2 = (float)n2;
  sx = __fadd_rn(__fadd_rn(__fmul_rn(f0, c[0]), __fmul_rn(f1, c[3])), __fmul_rn(f2, c[6]));
  sy = __fadd_rn(__fadd_rn(__fmul_rn(f0, c[1]), __fmul_rn(f1, c[4])), __fmul_rn(f2, c[7]));
  sz = __fadd_rn(__fadd_rn(__fmul_rn(f0, c[2]), __fmul_rn(f1, c[5])), __fmul_rn(f2, c[8]));
}

// One wavefront per target atom i; candidates are (source atom j, image) pairs in the order
// (j, image index), the atom itself (j = i, n = 0) left out.  FILL = false: deg[i] = number of kept
// candidates.  FILL = true: write them in that order at row_ptr[i].
template <bool FILL>
__global__ void __launch_bounds__(256)
edges_kernel(const float* __restrict__ pos, const int32_t* __restrict__ graph_ptr, int n_atoms,
             int n_graphs, float c2, int max_nb, images_t im, int32_t* __restrict__ deg,
             const int32_t* __restrict__ row_ptr, int32_t* __restrict__ src, int32_t* __restrict__ dst,
             int32_t* __restrict__ offset, float* __restrict__ dist, float* __restrict__ unit) {
  const int i = blockIdx.x * (blockDim.x / WAVE) + (threadIdx.x >> 6);
  if (i >= n_atoms) return;
  const int lane = lane_id();
  // structure containing atom i: largest g with graph_ptr[g] <= i
  int lo_g = 0, hi_g = n_graphs;
  while (hi_g - lo_g > 1) {
    int mid = (lo_g + hi_g) >> 1;
    if (graph_ptr[mid] <= i) lo_g = mid; else hi_g = mid;
  }
  const int lo = graph_ptr[lo_g], hi = graph_ptr[lo_g + 1];
  const float xi = pos[3 * i], yi = pos[3 * i + 1], zi = pos[3 * i + 2];
  const int NI = im.count();
  const int centre = im.cell ? ((im.r0 * (2 * im.r1 + 1) + im.r1) * (2 * im.r2 + 1) + im.r2) : 0;
  const int n_cand = (hi - lo) * NI;

  // squared distance from atom i to candidate q (and where that candidate sits)
  auto cand_d2 = [&](int q, int& j, int& n0, int& n1, int& n2, float& xs, float& ys, float& zs) -> float {
    j = lo + q / NI;
    float sx, sy, sz;
    image_of(im, lo_g, q % NI, n0, n1, n2, sx, sy, sz);
    xs = __fadd_rn(pos[3 * j], sx);
    ys = __fadd_rn(pos[3 * j + 1], sy);
    zs = __fadd_rn(pos[3 * j + 2], sz);
    return dist2_f32(xi, yi, zi, xs, ys, zs);
  };
  const int self_q = (i - lo) * NI + centre;

  bool capped = false;
  if (max_nb > 0) {
    int cand = 0;
    for (int base = 0; base < n_cand; base += WAVE) {
      const int q = base + lane;
      bool in = false;
      if (q < n_cand && q != self_q) {
        int j, n0, n1, n2;
        float xs, ys, zs;
        in = cand_d2(q, j, n0, n1, n2, xs, ys, zs) < c2;
      }
      cand += __popcll(__ballot(in));
    }
    capped = cand > max_nb;
  }

  int total = 0;
  for (int base = 0; base < n_cand; base += WAVE) {
    const int q = base + lane;
    float d2 = 0.f, xs = 0.f, ys = 0.f, zs = 0.f;
    int j = 0, n0 = 0, n1 = 0, n2 = 0;
    bool keep = false;
    if (q < n_cand && q != self_q) {
      d2 = cand_d2(q, j, n0, n1, n2, xs, ys, zs);
      keep = d2 < c2;
    }
    if (capped) {
      // rank of this candidate among all in-range candidates by key (d2, candidate order); keep the first max_nb
      int rank = 0;
      for (int p = 0; p < n_cand; ++p) {
        int jp, a0, a1, a2;
        float xp, yp, zp;
        const float dq = cand_d2(p, jp, a0, a1, a2, xp, yp, zp);
        const bool in_q = (p != self_q) && (dq < c2);
        rank += (in_q && (dq < d2 || (dq == d2 && p < q))) ? 1 : 0;
      }
      keep = keep && (rank < max_nb);
    }
    const uint64_t mask = __ballot(keep);
    if (FILL && keep) {
      const int slot = row_ptr[i] + total + mbcnt(mask);
      src[slot] = j;
      dst[slot] = i;
      if (offset) {
        offset[3 * slot + 0] = n0;
        offset[3 * slot + 1] = n1;
        offset[3 * slot + 2] = n2;
      }
      if (dist || unit) {
        float d = sqrtf(d2);
        if (dist) dist[slot] = d;
        if (unit) {
          float inv = 1.0f / d;
          unit[3 * slot + 0] = (xi - xs) * inv;
          unit[3 * slot + 1] = (yi - ys) * inv;
          unit[3 * slot + 2] = (zi - zs) * inv;
        }
      }
    }
    total += __popcll(mask);
  }
  if (!FILL && lane == 0) deg[i] = total;
}

// ------------------------------------------------------------------ triplets
// Position, inside rows b .. b+n of an edge list sorted by (source, cell offset), of the edge with
// source v and offset (t0, t1, t2); -1 if there is none.  off == NULL: open boundaries, all offsets zero.
__device__ __forceinline__ int find_edge(const int32_t* __restrict__ src, const int32_t* __restrict__ off, int b, int n,
                                         int v, int t0, int t1, int t2) {
  int lo = 0, hi = n;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1, e = b + mid;
    bool less = src[e] < v;
    if (off && src[e] == v) {
      const int o0 = off[3 * e], o1 = off[3 * e + 1], o2 = off[3 * e + 2];
      less = o0 < t0 || (o0 == t0 && (o1 < t1 || (o1 == t1 && o2 < t2)));
    }
    if (less) lo = mid + 1; else hi = mid;
  }
  if (lo >= n || src[b + lo] != v) return -1;
  if (off && (off[3 * (b + lo)] != t0 || off[3 * (b + lo) + 1] != t1 || off[3 * (b + lo) + 2] != t2)) return -1;
  return lo;
}

// Per edge e = (j->i): cnt[e] = indeg(j) - [the opposite edge exists]; skip[e] = position of the opposite
// edge (source i, negated offset: the image of k that is atom i itself) inside the in-list of j, or -1.
// Also histograms out-degrees.
__global__ void triplet_count_kernel(const int32_t* __restrict__ src, const int32_t* __restrict__ dst,
                                     const int32_t* __restrict__ off, const int32_t* __restrict__ row_ptr, int n_edges,
                                     int32_t* __restrict__ cnt, int32_t* __restrict__ skip,
                                     int32_t* __restrict__ out_deg) {
  int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= n_edges) return;
  int j = src[e], i = dst[e];
  int b = row_ptr[j], n = row_ptr[j + 1] - b;
  int p = off ? find_edge(src, off, b, n, i, -off[3 * e], -off[3 * e + 1], -off[3 * e + 2])
              : find_edge(src, nullptr, b, n, i, 0, 0, 0);
  skip[e] = p;
  cnt[e] = n - (p >= 0 ? 1 : 0);
  if (out_deg) atomicAdd(&out_deg[j], 1);
}

// One wavefront per target edge: its triplets are the in-edges of j minus the one from i.
__global__ void __launch_bounds__(256)
triplet_fill_ji_kernel(const int32_t* __restrict__ src, const int32_t* __restrict__ row_ptr,
                       const int32_t* __restrict__ seg, const int32_t* __restrict__ skip, int n_edges,
                       int32_t* __restrict__ idx_kj, int32_t* __restrict__ idx_ji) {
  const int e = blockIdx.x * (blockDim.x / WAVE) + (threadIdx.x >> 6);
  if (e >= n_edges) return;
  const int j = src[e];
  const int b = row_ptr[j], n = row_ptr[j + 1] - b;
  const int sk = skip[e], out = seg[e];
  for (int r = lane_id(); r < n; r += WAVE) {
    if (r == sk) continue;
    int slot = out + r - ((sk >= 0 && r > sk) ? 1 : 0);
    idx_kj[slot] = b + r;
    idx_ji[slot] = e;
  }
}

// Out-edge lists: first in arrival order (atomic cursor), then ordered by edge id by counting.
__global__ void out_scatter_kernel(const int32_t* __restrict__ src, int n_edges,
                                   const int32_t* __restrict__ out_ptr, int32_t* __restrict__ cursor,
                                   int32_t* __restrict__ out_tmp) {
  int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= n_edges) return;
  int j = src[e];
  out_tmp[out_ptr[j] + atomicAdd(&cursor[j], 1)] = e;
}

__global__ void __launch_bounds__(256)
out_sort_kernel(const int32_t* __restrict__ out_ptr, const int32_t* __restrict__ out_tmp, int n_atoms,
                int32_t* __restrict__ out_list) {
  __shared__ int32_t lds[SORT_LDS];
  const int j = blockIdx.x;   // one workgroup per atom
  const int b = out_ptr[j], n = out_ptr[j + 1] - b;
  sort_list_block(out_tmp + b, n, out_list + b, lds);
}

// Per source edge e' = (k->j): number of out-edges of j that do not end in k.
__global__ void triplet_count_kj_kernel(const int32_t* __restrict__ src, const int32_t* __restrict__ dst,
                                        const int32_t* __restrict__ off, const int32_t* __restrict__ row_ptr,
                                        const int32_t* __restrict__ out_ptr, int n_edges,
                                        int32_t* __restrict__ cnt_kj) {
  int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= n_edges) return;
  int k = src[e], j = dst[e];
  int b = row_ptr[k], n = row_ptr[k + 1] - b;           // in-list of k: does it contain the opposite edge ?
  int p = off ? find_edge(src, off, b, n, j, -off[3 * e], -off[3 * e + 1], -off[3 * e + 2])
              : find_edge(src, nullptr, b, n, j, 0, 0, 0);
  cnt_kj[e] = out_ptr[j + 1] - out_ptr[j] - (p >= 0 ? 1 : 0);
}

// Slots of source edge e' = (k->j) in the kj-major view: the out-edges e = (j->i) of j in ascending edge id, i == k
// dropped, each with the ji-major triplet id of (e', e).
// The same lists per centre atom j: all in-edges e' = (k->j) walk the same out-edges of j, so a workgroup stages
// what it needs of them (edge id, target atom, first ji-major triplet, skipped position; the cell offset of periodic
// edges) in LDS once, 256 out-edges at a time, for the up to 32 in-edge rows it owns, instead of gathering three
// values per triplet from memory (0.96 -> 0.3 ms for the 1e8 triplets of the largest workload).
// Work items (atom, group of 32 in-edge rows): item[w] = {atom, first row of the group}; n_items[0] = their number.
constexpr int KJ_ROWS = 32, KJ_CHUNK = 256;
__global__ void __launch_bounds__(1024)
kj_items_kernel(const int32_t* __restrict__ row_ptr, int n_atoms, int32_t* __restrict__ n_items, int32_t* __restrict__ item) {
  __shared__ int32_t wave_tot[16];
  __shared__ int32_t carry;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  if (tid == 0) carry = 0;
  __syncthreads();
  for (int base = 0; base < n_atoms; base += 1024) {
    const int j = base + tid;
    const int d = j < n_atoms ? row_ptr[j + 1] - row_ptr[j] : 0;
    const int v = (d + KJ_ROWS - 1) / KJ_ROWS;
    int incl = v;
    for (int o = 1; o < 64; o <<= 1) {
      const int u = __shfl_up(incl, o, 64);
      if (lane >= o) incl += u;
    }
    if (lane == 63) wave_tot[w] = incl;
    __syncthreads();
    int before = carry;
    for (int k = 0; k < w; ++k) before += wave_tot[k];
    for (int k = 0; k < v; ++k) {
      item[2 * (int64_t)(before + incl - v + k)] = j;
      item[2 * (int64_t)(before + incl - v + k) + 1] = KJ_ROWS * k;
    }
    __syncthreads();
    if (tid == 1023) carry = before + incl;
    __syncthreads();
  }
  if (tid == 0) n_items[0] = carry;
}

template <bool PBC>
__global__ void __launch_bounds__(256)
triplet_fill_kj_atom_kernel(const int32_t* __restrict__ src, const int32_t* __restrict__ dst, const int32_t* __restrict__ off,
                            const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ out_ptr,
                            const int32_t* __restrict__ out_list, const int32_t* __restrict__ seg_ji,
                            const int32_t* __restrict__ skip, const int32_t* __restrict__ seg_kj,
                            const int32_t* __restrict__ n_items, const int32_t* __restrict__ item,
                            int32_t* __restrict__ perm_kj, int32_t* __restrict__ idx_ji_kj) {
  if ((int)blockIdx.x >= n_items[0]) return;
  __shared__ int32_t t_e[KJ_CHUNK], t_dst[KJ_CHUNK], t_seg[KJ_CHUNK], t_skip[KJ_CHUNK], t_off[PBC ? 3 * KJ_CHUNK : 1];
  __shared__ int32_t tot[KJ_ROWS];
  const int j = item[2 * (int64_t)blockIdx.x], r_lo = item[2 * (int64_t)blockIdx.x + 1];
  const int r0 = row_ptr[j], d = row_ptr[j + 1] - r0;
  const int r_hi = r_lo + KJ_ROWS < d ? r_lo + KJ_ROWS : d;
  const int ob = out_ptr[j], on = out_ptr[j + 1] - ob;
  const int lane = lane_id(), wave = threadIdx.x >> 6;
  if (threadIdx.x < KJ_ROWS) tot[threadIdx.x] = 0;
  for (int c0 = 0; c0 < on; c0 += KJ_CHUNK) {
    __syncthreads();   // the previous chunk has been consumed (and tot is initialised)
    const int n = on - c0 < KJ_CHUNK ? on - c0 : KJ_CHUNK;
    if ((int)threadIdx.x < n) {
      const int e = out_list[ob + c0 + threadIdx.x];
      t_e[threadIdx.x] = e;
      t_dst[threadIdx.x] = dst[e];
      t_seg[threadIdx.x] = seg_ji[e];
      t_skip[threadIdx.x] = skip[e];
      if (PBC) {
        t_off[3 * threadIdx.x] = off[3 * (int64_t)e];
        t_off[3 * threadIdx.x + 1] = off[3 * (int64_t)e + 1];
        t_off[3 * threadIdx.x + 2] = off[3 * (int64_t)e + 2];
      }
    }
    __syncthreads();
    for (int r_in = r_lo + wave; r_in < r_hi; r_in += 4) {   // a row is handled by the same wavefront in every chunk
      const int ep = r0 + r_in, k = src[ep];
      int o0 = 0, o1 = 0, o2 = 0;
      if (PBC) o0 = -off[3 * (int64_t)ep], o1 = -off[3 * (int64_t)ep + 1], o2 = -off[3 * (int64_t)ep + 2];
      int total = tot[r_in - r_lo];
      const int seg = seg_kj[ep];
      for (int base = 0; base < n; base += WAVE) {
        const int q = base + lane;
        bool keep = false;
        if (q < n) {
          keep = t_dst[q] != k;
          if (PBC && !keep)   // ends in atom k: excluded only if it is the opposite edge (negated offset)
            keep = t_off[3 * q] != o0 || t_off[3 * q + 1] != o1 || t_off[3 * q + 2] != o2;
        }
        const uint64_t mask = __ballot(keep);
        if (keep) {
          const int slot = seg + total + mbcnt(mask);
          const int sk = t_skip[q];
          perm_kj[slot] = t_seg[q] + r_in - ((sk >= 0 && r_in > sk) ? 1 : 0);
          idx_ji_kj[slot] = t_e[q];
        }
        total += __popcll(mask);
      }
      if (lane == 0) tot[r_in - r_lo] = total;
    }
  }
}

struct edges_ws {
  int32_t* deg;      // [N]
  int32_t* row_ptr;  // [N+1]
  int64_t* total;    // [1]
};
inline size_t carve_edges(void* p, int64_t n_atoms, edges_ws* w) {
  gp_carver c(p);
  w->deg = c.take<int32_t>(n_atoms);
  w->row_ptr = c.take<int32_t>(n_atoms + 1);
  w->total = c.take<int64_t>(1);
  return c.off;
}

struct triplets_ws {
  int32_t *cnt, *skip, *seg_ji, *cnt_kj, *seg_kj, *out_tmp, *out_list;  // [E] / [E+1]
  int32_t *out_deg, *out_ptr, *cursor;                                   // [N] / [N+1]
  int64_t* totals;                                                       // [3]
  int64_t* scan_tmp;                                                     // chunk sums of the long scans
  int32_t *kj_n, *kj_item;                                               // work items of the per-atom kj fill
};
inline size_t carve_triplets(void* p, int64_t n_atoms, int64_t n_edges, triplets_ws* w) {
  gp_carver c(p);
  w->cnt = c.take<int32_t>(n_edges);
  w->skip = c.take<int32_t>(n_edges);
  w->seg_ji = c.take<int32_t>(n_edges + 1);
  w->cnt_kj = c.take<int32_t>(n_edges);
  w->seg_kj = c.take<int32_t>(n_edges + 1);
  w->out_tmp = c.take<int32_t>(n_edges);
  w->out_list = c.take<int32_t>(n_edges);
  w->out_deg = c.take<int32_t>(n_atoms);
  w->out_ptr = c.take<int32_t>(n_atoms + 1);
  w->cursor = c.take<int32_t>(n_atoms);
  w->totals = c.take<int64_t>(3);
  w->scan_tmp = c.take<int64_t>((size_t)scan_chunks(n_edges) + 1);
  w->kj_n = c.take<int32_t>(4);
  w->kj_item = c.take<int32_t>(2 * (size_t)(n_edges / KJ_ROWS + n_atoms + 1));
  return c.off;
}

// exclusive scan of in[n] into out[n+1] (out[n] = total, also written untruncated to total64) on the stream
int scan_exclusive(gp_ctx* ctx, const int32_t* in, int32_t* out, int64_t n, int64_t* total64, int64_t* tmp) {
  hipStream_t st = ctx->stream;
  if (n <= 4 * SCAN_CHUNK || !tmp) {
    scan_exclusive_kernel<<<1, SCAN_THREADS, 0, st>>>(in, out, n, total64);
  } else {
    const int64_t nb = scan_chunks(n);
    scan_chunk_sums_kernel<<<(unsigned)nb, SCAN_THREADS, 0, st>>>(in, n, tmp);
    scan_sums_kernel<<<1, SCAN_THREADS, 0, st>>>(tmp, nb, total64);
    scan_chunk_apply_kernel<<<(unsigned)nb, SCAN_THREADS, 0, st>>>(in, tmp, total64, n, out);
  }
  GP_LAUNCH_CHECK(ctx, "scan kernels");
  return GP_OK;
}

inline int blocks_for(int64_t n, int per_block) { return (int)((n + per_block - 1) / per_block); }

// id_swap[e] = the edge dst[e] -> src[e] with the negated cell offset, found in the row of target src[e]
__global__ void reverse_edges_kernel(const int32_t* __restrict__ src, const int32_t* __restrict__ dst,
                                     const int32_t* __restrict__ off, const int32_t* __restrict__ row_ptr,
                                     int64_t n_edges, int32_t* __restrict__ id_swap) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= n_edges) return;
  const int j = src[e], i = dst[e];
  const int b = row_ptr[j], n = row_ptr[j + 1] - b;
  const int p = off ? find_edge(src, off, b, n, i, -off[3 * e], -off[3 * e + 1], -off[3 * e + 2])
                    : find_edge(src, nullptr, b, n, i, 0, 0, 0);
  id_swap[e] = p >= 0 ? b + p : -1;
}

// largest ptr[i+1] - ptr[i]; one workgroup
__global__ void __launch_bounds__(1024)
max_degree_kernel(const int32_t* __restrict__ ptr, int64_t n, int32_t* __restrict__ out) {
  __shared__ int red[16];
  int m = 0;
  for (int64_t i = threadIdx.x; i < n; i += blockDim.x) {
    const int d = ptr[i + 1] - ptr[i];
    m = d > m ? d : m;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const int v = __shfl_xor(m, o, 64);
    m = v > m ? v : m;
  }
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < (int)(blockDim.x >> 6); ++w) m = red[w] > m ? red[w] : m;
    *out = m;
  }
}

}  // namespace

extern "C" {

int gp_reverse_edges(gp_ctx* ctx, const int32_t* src, const int32_t* dst, const int32_t* offset,
                     const int32_t* row_ptr, int64_t n_atoms, int64_t n_edges, int32_t* id_swap) {
  if (!ctx) return GP_BAD_ARG;
  GP_REQUIRE(ctx, n_atoms >= 0 && n_edges >= 0, "gp_reverse_edges: negative size");
  if (n_edges > INT32_MAX - 1 || n_atoms > INT32_MAX - 1) return gp_fail(ctx, GP_INT32_OVERFLOW, "gp_reverse_edges: sizes exceed int32");
  if (n_edges == 0) return GP_OK;
  GP_REQUIRE(ctx, src && dst && row_ptr && id_swap, "gp_reverse_edges: NULL pointer");
  GP_HIP(ctx, hipSetDevice(ctx->device));
  reverse_edges_kernel<<<blocks_for(n_edges, 256), 256, 0, ctx->stream>>>(src, dst, offset, row_ptr, n_edges, id_swap);
  GP_LAUNCH_CHECK(ctx, "reverse_edges_kernel");
  return GP_OK;
}

int gp_csr_max_degree(gp_ctx* ctx, const int32_t* ptr, int64_t n, void* ws, size_t ws_bytes, int32_t* max_degree) {
  if (!ctx) return GP_BAD_ARG;
  GP_REQUIRE(ctx, max_degree, "gp_csr_max_degree: max_degree is NULL");
  GP_REQUIRE(ctx, n >= 0, "gp_csr_max_degree: negative size");
  *max_degree = 0;
  if (n == 0) return GP_OK;
  GP_REQUIRE(ctx, ptr && ws, "gp_csr_max_degree: NULL pointer");
  if (ws_bytes < sizeof(int32_t)) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "gp_csr_max_degree: workspace below 4 bytes");
  GP_HIP(ctx, hipSetDevice(ctx->device));
  max_degree_kernel<<<1, 1024, 0, ctx->stream>>>(ptr, n, static_cast<int32_t*>(ws));
  GP_LAUNCH_CHECK(ctx, "max_degree_kernel");
  GP_HIP(ctx, hipMemcpyAsync(max_degree, ws, sizeof(int32_t), hipMemcpyDeviceToHost, ctx->stream));
  GP_HIP(ctx, hipStreamSynchronize(ctx->stream));
  return GP_OK;
}

int gp_edges_workspace(int64_t n_atoms, size_t* bytes) {
  if (!bytes || n_atoms < 0) return GP_BAD_ARG;
  edges_ws w;
  *bytes = carve_edges(nullptr, n_atoms, &w);
  return GP_OK;
}

}  // extern "C"

namespace {

int check_images(gp_ctx* ctx, const char* who, const float* cell, int r0, int r1, int r2, int64_t n_atoms, images_t* im) {
  GP_REQUIRE(ctx, cell, "%s: cell is NULL", who);
  GP_REQUIRE(ctx, r0 >= 0 && r1 >= 0 && r2 >= 0 && r0 <= 16 && r1 <= 16 && r2 <= 16, "%s: image range must be 0..16 per axis", who);
  *im = images_t{cell, r0, r1, r2};
  if ((int64_t)im->count() * n_atoms > INT32_MAX) return gp_fail(ctx, GP_INT32_OVERFLOW, "%s: atoms x images exceed int32", who);
  return GP_OK;
}

int edges_count_impl(gp_ctx* ctx, const char* who, const float* pos, const int32_t* graph_ptr, images_t im, int64_t n_atoms,
                     int32_t n_graphs, float cutoff, int32_t max_neighbors, void* ws, size_t ws_bytes, int64_t* n_edges) {
  GP_REQUIRE(ctx, n_edges, "%s: n_edges is NULL", who);
  GP_REQUIRE(ctx, n_atoms >= 0 && n_graphs >= 0 && max_neighbors >= 0, "%s: negative size", who);
  GP_REQUIRE(ctx, cutoff > 0.f && cutoff == cutoff, "%s: cutoff must be positive", who);
  if (n_atoms > INT32_MAX - 1) return gp_fail(ctx, GP_INT32_OVERFLOW, "%s: too many atoms", who);
  *n_edges = 0;
  if (n_atoms == 0 || n_graphs == 0) return GP_OK;
  GP_REQUIRE(ctx, pos && graph_ptr && ws, "%s: NULL pointer", who);
  edges_ws w;
  size_t need = carve_edges(ws, n_atoms, &w);
  if (ws_bytes < need) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "%s: workspace %zu < %zu", who, ws_bytes, need);
  GP_HIP(ctx, hipSetDevice(ctx->device));
  const float c2 = cutoff * cutoff;
  edges_kernel<false><<<blocks_for(n_atoms, 4), 256, 0, ctx->stream>>>(
      pos, graph_ptr, (int)n_atoms, n_graphs, c2, max_neighbors, im, w.deg, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
  GP_LAUNCH_CHECK(ctx, "edges_kernel<count>");
  scan_exclusive_kernel<<<1, SCAN_THREADS, 0, ctx->stream>>>(w.deg, w.row_ptr, n_atoms, w.total);
  GP_LAUNCH_CHECK(ctx, "scan_exclusive_kernel");
  int64_t total = 0;
  GP_HIP(ctx, hipMemcpyAsync(&total, w.total, sizeof(total), hipMemcpyDeviceToHost, ctx->stream));
  GP_HIP(ctx, hipStreamSynchronize(ctx->stream));
  *n_edges = total;
  if (total > INT32_MAX) return gp_fail(ctx, GP_INT32_OVERFLOW, "%s: %lld edges exceed int32", who, (long long)total);
  return GP_OK;
}

int edges_fill_impl(gp_ctx* ctx, const char* who, const float* pos, const int32_t* graph_ptr, images_t im, int64_t n_atoms,
                    int32_t n_graphs, float cutoff, int32_t max_neighbors, const void* ws, size_t ws_bytes, int64_t n_edges,
                    int32_t* src, int32_t* dst, int32_t* offset, int32_t* row_ptr, float* dist, float* unit) {
  GP_REQUIRE(ctx, n_atoms >= 0 && n_graphs >= 0 && max_neighbors >= 0 && n_edges >= 0, "%s: negative size", who);
  GP_REQUIRE(ctx, cutoff > 0.f && cutoff == cutoff, "%s: cutoff must be positive", who);
  GP_REQUIRE(ctx, row_ptr, "%s: row_ptr is NULL", who);
  if (n_atoms > INT32_MAX - 1 || n_edges > INT32_MAX) return gp_fail(ctx, GP_INT32_OVERFLOW, "%s: sizes exceed int32", who);
  GP_HIP(ctx, hipSetDevice(ctx->device));
  if (n_atoms == 0 || n_graphs == 0) {
    GP_HIP(ctx, (hipError_t)gp_zero_async(ctx->stream, row_ptr, sizeof(int32_t) * (n_atoms + 1)));
    return GP_OK;
  }
  GP_REQUIRE(ctx, pos && graph_ptr && ws, "%s: NULL pointer", who);
  GP_REQUIRE(ctx, n_edges == 0 || (src && dst), "%s: src/dst is NULL", who);
  edges_ws w;
  size_t need = carve_edges(const_cast<void*>(ws), n_atoms, &w);
  if (ws_bytes < need) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "%s: workspace %zu < %zu", who, ws_bytes, need);
  GP_HIP(ctx, hipMemcpyAsync(row_ptr, w.row_ptr, sizeof(int32_t) * (n_atoms + 1), hipMemcpyDeviceToDevice, ctx->stream));
  if (n_edges == 0) return GP_OK;
  const float c2 = cutoff * cutoff;
  edges_kernel<true><<<blocks_for(n_atoms, 4), 256, 0, ctx->stream>>>(
      pos, graph_ptr, (int)n_atoms, n_graphs, c2, max_neighbors, im, nullptr, w.row_ptr, src, dst, offset, dist, unit);
  GP_LAUNCH_CHECK(ctx, "edges_kernel<fill>");
  return GP_OK;
}

}  // namespace

extern "C" {

int gp_edges_count(gp_ctx* ctx, const float* pos, const int32_t* graph_ptr, int64_t n_atoms,
                   int32_t n_graphs, float cutoff, int32_t max_neighbors, void* ws, size_t ws_bytes,
                   int64_t* n_edges) {
  if (!ctx) return GP_BAD_ARG;
  return edges_count_impl(ctx, "gp_edges_count", pos, graph_ptr, images_t{nullptr, 0, 0, 0}, n_atoms, n_graphs, cutoff,
                          max_neighbors, ws, ws_bytes, n_edges);
}

int gp_edges_fill(gp_ctx* ctx, const float* pos, const int32_t* graph_ptr, int64_t n_atoms,
                  int32_t n_graphs, float cutoff, int32_t max_neighbors, const void* ws, size_t ws_bytes,
                  int64_t n_edges, int32_t* src, int32_t* dst, int32_t* row_ptr, float* dist, float* unit) {
  if (!ctx) return GP_BAD_ARG;
  return edges_fill_impl(ctx, "gp_edges_fill", pos, graph_ptr, images_t{nullptr, 0, 0, 0}, n_atoms, n_graphs, cutoff,
                         max_neighbors, ws, ws_bytes, n_edges, src, dst, nullptr, row_ptr, dist, unit);
}

int gp_edges_count_pbc(gp_ctx* ctx, const float* pos, const int32_t* graph_ptr, const float* cell, int64_t n_atoms,
                       int32_t n_graphs, float cutoff, int32_t max_neighbors, int32_t rep0, int32_t rep1, int32_t rep2,
                       void* ws, size_t ws_bytes, int64_t* n_edges) {
  if (!ctx) return GP_BAD_ARG;
  images_t im;
  GP_TRY(check_images(ctx, "gp_edges_count_pbc", cell, rep0, rep1, rep2, n_atoms, &im));
  return edges_count_impl(ctx, "gp_edges_count_pbc", pos, graph_ptr, im, n_atoms, n_graphs, cutoff, max_neighbors, ws,
                          ws_bytes, n_edges);
}

int gp_edges_fill_pbc(gp_ctx* ctx, const float* pos, const int32_t* graph_ptr, const float* cell, int64_t n_atoms,
                      int32_t n_graphs, float cutoff, int32_t max_neighbors, int32_t rep0, int32_t rep1, int32_t rep2,
                      const void* ws, size_t ws_bytes, int64_t n_edges, int32_t* src, int32_t* dst, int32_t* offset,
                      int32_t* row_ptr, float* dist, float* unit) {
  if (!ctx) return GP_BAD_ARG;
  images_t im;
  GP_TRY(check_images(ctx, "gp_edges_fill_pbc", cell, rep0, rep1, rep2, n_atoms, &im));
  GP_REQUIRE(ctx, n_edges == 0 || offset, "gp_edges_fill_pbc: offset is NULL");
  return edges_fill_impl(ctx, "gp_edges_fill_pbc", pos, graph_ptr, im, n_atoms, n_graphs, cutoff, max_neighbors, ws,
                         ws_bytes, n_edges, src, dst, offset, row_ptr, dist, unit);
}

int gp_triplets_workspace(int64_t n_atoms, int64_t n_edges, size_t* bytes) {
  if (!bytes || n_atoms < 0 || n_edges < 0) return GP_BAD_ARG;
  triplets_ws w;
  *bytes = carve_triplets(nullptr, n_atoms, n_edges, &w);
  return GP_OK;
}

}  // extern "C"

namespace {

int triplets_count_impl(gp_ctx* ctx, const int32_t* src, const int32_t* dst, const int32_t* offset, const int32_t* row_ptr,
                        int64_t n_atoms, int64_t n_edges, void* ws, size_t ws_bytes, int64_t* n_triplets) {
  GP_REQUIRE(ctx, n_triplets, "gp_triplets_count: n_triplets is NULL");
  GP_REQUIRE(ctx, n_atoms >= 0 && n_edges >= 0, "gp_triplets_count: negative size");
  if (n_atoms > INT32_MAX - 1 || n_edges > INT32_MAX - 1) return gp_fail(ctx, GP_INT32_OVERFLOW, "gp_triplets_count: sizes exceed int32");
  *n_triplets = 0;
  if (n_edges == 0 || n_atoms == 0) return GP_OK;
  GP_REQUIRE(ctx, src && dst && row_ptr && ws, "gp_triplets_count: NULL pointer");
  triplets_ws w;
  size_t need = carve_triplets(ws, n_atoms, n_edges, &w);
  if (ws_bytes < need) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "gp_triplets_count: workspace %zu < %zu", ws_bytes, need);
  GP_HIP(ctx, hipSetDevice(ctx->device));
  hipStream_t st = ctx->stream;
  GP_HIP(ctx, (hipError_t)gp_zero_async(st, w.out_deg, sizeof(int32_t) * n_atoms));
  GP_HIP(ctx, (hipError_t)gp_zero_async(st, w.cursor, sizeof(int32_t) * n_atoms));
  triplet_count_kernel<<<blocks_for(n_edges, 256), 256, 0, st>>>(src, dst, offset, row_ptr, (int)n_edges, w.cnt, w.skip, w.out_deg);
  GP_LAUNCH_CHECK(ctx, "triplet_count_kernel");
  GP_TRY(scan_exclusive(ctx, w.cnt, w.seg_ji, n_edges, w.totals + 0, w.scan_tmp));
  int64_t total = 0;
  GP_HIP(ctx, hipMemcpyAsync(&total, w.totals, sizeof(total), hipMemcpyDeviceToHost, st));
  GP_HIP(ctx, hipStreamSynchronize(st));
  *n_triplets = total;
  if (total > INT32_MAX) return gp_fail(ctx, GP_INT32_OVERFLOW, "gp_triplets_count: %lld triplets exceed int32", (long long)total);
  return GP_OK;
}

int triplets_fill_impl(gp_ctx* ctx, const int32_t* src, const int32_t* dst, const int32_t* offset, const int32_t* row_ptr,
                       int64_t n_atoms, int64_t n_edges, void* ws, size_t ws_bytes, int64_t n_triplets,
                       int32_t* idx_kj, int32_t* idx_ji, int32_t* seg_ptr_ji, int32_t* perm_kj,
                       int32_t* idx_ji_kj, int32_t* seg_ptr_kj) {
  GP_REQUIRE(ctx, n_atoms >= 0 && n_edges >= 0 && n_triplets >= 0, "gp_triplets_fill: negative size");
  if (n_atoms > INT32_MAX - 1 || n_edges > INT32_MAX - 1 || n_triplets > INT32_MAX)
    return gp_fail(ctx, GP_INT32_OVERFLOW, "gp_triplets_fill: sizes exceed int32");
  GP_REQUIRE(ctx, seg_ptr_ji, "gp_triplets_fill: seg_ptr_ji is NULL");
  const bool want_kj = perm_kj || idx_ji_kj || seg_ptr_kj;
  GP_REQUIRE(ctx, !want_kj || (seg_ptr_kj && (n_triplets == 0 || (perm_kj && idx_ji_kj))),
             "gp_triplets_fill: perm_kj, idx_ji_kj, seg_ptr_kj must be given together");
  GP_HIP(ctx, hipSetDevice(ctx->device));
  hipStream_t st = ctx->stream;
  if (n_edges == 0 || n_atoms == 0) {
    GP_HIP(ctx, (hipError_t)gp_zero_async(st, seg_ptr_ji, sizeof(int32_t) * (n_edges + 1)));
    if (seg_ptr_kj) GP_HIP(ctx, (hipError_t)gp_zero_async(st, seg_ptr_kj, sizeof(int32_t) * (n_edges + 1)));
    return GP_OK;
  }
  GP_REQUIRE(ctx, src && dst && row_ptr && ws, "gp_triplets_fill: NULL pointer");
  GP_REQUIRE(ctx, n_triplets == 0 || (idx_kj && idx_ji), "gp_triplets_fill: idx_kj/idx_ji is NULL");
  triplets_ws w;
  size_t need = carve_triplets(ws, n_atoms, n_edges, &w);
  if (ws_bytes < need) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "gp_triplets_fill: workspace %zu < %zu", ws_bytes, need);
  GP_HIP(ctx, hipMemcpyAsync(seg_ptr_ji, w.seg_ji, sizeof(int32_t) * (n_edges + 1), hipMemcpyDeviceToDevice, st));
  if (n_triplets > 0) {
    triplet_fill_ji_kernel<<<blocks_for(n_edges, 4), 256, 0, st>>>(src, row_ptr, w.seg_ji, w.skip, (int)n_edges, idx_kj, idx_ji);
    GP_LAUNCH_CHECK(ctx, "triplet_fill_ji_kernel");
  }
  if (!want_kj) return GP_OK;
  GP_TRY(scan_exclusive(ctx, w.out_deg, w.out_ptr, n_atoms, w.totals + 1, nullptr));
  GP_HIP(ctx, (hipError_t)gp_zero_async(st, w.cursor, sizeof(int32_t) * n_atoms));
  out_scatter_kernel<<<blocks_for(n_edges, 256), 256, 0, st>>>(src, (int)n_edges, w.out_ptr, w.cursor, w.out_tmp);
  GP_LAUNCH_CHECK(ctx, "out_scatter_kernel");
  out_sort_kernel<<<(unsigned)n_atoms, 256, 0, st>>>(w.out_ptr, w.out_tmp, (int)n_atoms, w.out_list);
  GP_LAUNCH_CHECK(ctx, "out_sort_kernel");
  triplet_count_kj_kernel<<<blocks_for(n_edges, 256), 256, 0, st>>>(src, dst, offset, row_ptr, w.out_ptr, (int)n_edges, w.cnt_kj);
  GP_LAUNCH_CHECK(ctx, "triplet_count_kj_kernel");
  GP_TRY(scan_exclusive(ctx, w.cnt_kj, w.seg_kj, n_edges, w.totals + 2, w.scan_tmp));
  GP_HIP(ctx, hipMemcpyAsync(seg_ptr_kj, w.seg_kj, sizeof(int32_t) * (n_edges + 1), hipMemcpyDeviceToDevice, st));
  if (n_triplets > 0) {
    kj_items_kernel<<<1, 1024, 0, st>>>(row_ptr, (int)n_atoms, w.kj_n, w.kj_item);
    const unsigned grid = (unsigned)(n_edges / KJ_ROWS + n_atoms);   // an upper bound of the number of work items
    if (offset)
      triplet_fill_kj_atom_kernel<true><<<grid, 256, 0, st>>>(src, dst, offset, row_ptr, w.out_ptr, w.out_list, w.seg_ji, w.skip,
                                                              w.seg_kj, w.kj_n, w.kj_item, perm_kj, idx_ji_kj);
    else
      triplet_fill_kj_atom_kernel<false><<<grid, 256, 0, st>>>(src, dst, offset, row_ptr, w.out_ptr, w.out_list, w.seg_ji, w.skip,
                                                               w.seg_kj, w.kj_n, w.kj_item, perm_kj, idx_ji_kj);
    GP_LAUNCH_CHECK(ctx, "triplet_fill_kj_atom_kernel");
  }
  return GP_OK;
}

}  // namespace

extern "C" {

int gp_triplets_count(gp_ctx* ctx, const int32_t* src, const int32_t* dst, const int32_t* row_ptr,
                      int64_t n_atoms, int64_t n_edges, void* ws, size_t ws_bytes, int64_t* n_triplets) {
  if (!ctx) return GP_BAD_ARG;
  return triplets_count_impl(ctx, src, dst, nullptr, row_ptr, n_atoms, n_edges, ws, ws_bytes, n_triplets);
}

int gp_triplets_fill(gp_ctx* ctx, const int32_t* src, const int32_t* dst, const int32_t* row_ptr,
                     int64_t n_atoms, int64_t n_edges, void* ws, size_t ws_bytes, int64_t n_triplets,
                     int32_t* idx_kj, int32_t* idx_ji, int32_t* seg_ptr_ji, int32_t* perm_kj,
                     int32_t* idx_ji_kj, int32_t* seg_ptr_kj) {
  if (!ctx) return GP_BAD_ARG;
  return triplets_fill_impl(ctx, src, dst, nullptr, row_ptr, n_atoms, n_edges, ws, ws_bytes, n_triplets, idx_kj, idx_ji,
                            seg_ptr_ji, perm_kj, idx_ji_kj, seg_ptr_kj);
}

int gp_triplets_count_pbc(gp_ctx* ctx, const int32_t* src, const int32_t* dst, const int32_t* offset,
                          const int32_t* row_ptr, int64_t n_atoms, int64_t n_edges, void* ws, size_t ws_bytes,
                          int64_t* n_triplets) {
  if (!ctx) return GP_BAD_ARG;
  GP_REQUIRE(ctx, n_edges == 0 || offset, "gp_triplets_count_pbc: offset is NULL");
  return triplets_count_impl(ctx, src, dst, offset, row_ptr, n_atoms, n_edges, ws, ws_bytes, n_triplets);
}

int gp_triplets_fill_pbc(gp_ctx* ctx, const int32_t* src, const int32_t* dst, const int32_t* offset,
                         const int32_t* row_ptr, int64_t n_atoms, int64_t n_edges, void* ws, size_t ws_bytes,
                         int64_t n_triplets, int32_t* idx_kj, int32_t* idx_ji, int32_t* seg_ptr_ji, int32_t* perm_kj,
                         int32_t* idx_ji_kj, int32_t* seg_ptr_kj) {
  if (!ctx) return GP_BAD_ARG;
  GP_REQUIRE(ctx, n_edges == 0 || offset, "gp_triplets_fill_pbc: offset is NULL");
  return triplets_fill_impl(ctx, src, dst, offset, row_ptr, n_atoms, n_edges, ws, ws_bytes, n_triplets, idx_kj, idx_ji,
                            seg_ptr_ji, perm_kj, idx_ji_kj, seg_ptr_kj);
}

}  // extern "C"
