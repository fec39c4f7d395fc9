// Energy head and forces (paper Sec. 3.3: per-atom sum of incoming messages followed by an MLP;
// Sec. 3.2, energy-centric paradigm: forces are the negative gradient of the energy with respect
// to the positions).  The position gradient is assembled without atomics: per-edge vector
// gradients come from sorted-segment sums over the ji-major and kj-major triplet views, per-atom
// sums from the in-edge rows and the out-edge lists.
#include <math.h>
#include <stdarg.h>

#include <algorithm>

#include "gemm.h"
#include "triplet.h"

#include <mutex>

namespace {

constexpr int WPB = 4;

// ------------------------------------------------------------------ scratch of the allocation-free entry point
// gp_edges_by_source_static keeps its counters and its unsorted list in this file-scope device array instead of a
// caller's workspace.  Every GPU the library runs on holds its own copy for the life of the process.  In host code
// the array's name is only a handle for hipGetSymbolAddress: the device address is looked up once per device
// (gp_static_scratch_init, called by gp_create with that device current) and only that address is ever handed to
// kernels.
constexpr int64_t STATIC_MAX_ATOMS = 65536;
constexpr int64_t STATIC_MAX_EDGES = 2097152;
constexpr size_t STATIC_CNT_BYTES = sizeof(int32_t) * STATIC_MAX_ATOMS;            // a multiple of 256
constexpr size_t STATIC_BYTES = 2 * STATIC_CNT_BYTES + sizeof(int32_t) * STATIC_MAX_EDGES;
static __device__ __align__(256) unsigned char scratch[STATIC_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_static_mutex;
void* g_static_ptr[MAX_DEVICES] = {nullptr};
hipError_t g_static_err[MAX_DEVICES] = {hipSuccess};

__global__ void fill_zero_kernel(int32_t* __restrict__ p, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

// ------------------------------------------------------------------ out-edge lists (by source)
__global__ void hist_kernel(const int32_t* __restrict__ key, int64_t n, int32_t* __restrict__ cnt) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) atomicAdd(&cnt[key[i]], 1);
}
// one workgroup: exclusive scan of cnt[n] -> ptr[n+1]
__global__ void __launch_bounds__(1024) scan_small_kernel(const int32_t* __restrict__ cnt, int64_t n, int32_t* __restrict__ ptr) {
  __shared__ int32_t wave_tot[16];
  __shared__ int32_t carry;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  if (tid == 0) carry = 0;
  __syncthreads();
  for (int64_t base = 0; base < n; base += 1024) {
    const int64_t i = base + tid;
    const int v = i < n ? cnt[i] : 0;
    int incl = v;
    for (int o = 1; o < 64; o <<= 1) {
      int u = __shfl_up(incl, o, 64);
      if (lane >= o) incl += u;
    }
    if (lane == 63) wave_tot[w] = incl;
    __syncthreads();
    int before = carry;
    for (int k = 0; k < w; ++k) before += wave_tot[k];
    if (i < n) ptr[i] = before + incl - v;
    __syncthreads();
    if (tid == 1023) carry = before + incl;
    __syncthreads();
  }
  if (tid == 0) ptr[n] = carry;
}
__global__ void scatter_by_key_kernel(const int32_t* __restrict__ key, int64_t n, const int32_t* __restrict__ ptr,
                                      int32_t* __restrict__ cursor, int32_t* __restrict__ tmp) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) tmp[ptr[key[i]] + atomicAdd(&cursor[key[i]], 1)] = (int32_t)i;
}
// order each list ascending by counting; one workgroup per atom
__global__ void __launch_bounds__(256)
sort_lists_kernel(const int32_t* __restrict__ ptr, const int32_t* __restrict__ tmp, int64_t n_atoms, int32_t* __restrict__ out) {
  __shared__ int32_t lds[SORT_LDS];
  const int64_t j = blockIdx.x;
  const int b = ptr[j], n = ptr[j + 1] - b;
  sort_list_block(tmp + b, n, out + b, lds);
}

// ------------------------------------------------------------------ energy head
// h[i, f] = sum over the in-edge row of atom i of m[e, f]; one wavefront per (atom, 64 features),
// four rows in flight, partial sums combined in a fixed order
__global__ void __launch_bounds__(256)
atom_sum_kernel(const float* __restrict__ m, const int32_t* __restrict__ row_ptr, int64_t n_atoms, int H,
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
    s0 += m[(int64_t)e * H + f];
    s1 += m[(int64_t)(e + 1) * H + f];
    s2 += m[(int64_t)(e + 2) * H + f];
    s3 += m[(int64_t)(e + 3) * H + f];
  }
  for (; e < e1; ++e) s0 += m[(int64_t)e * H + f];
  h[i * H + f] = (s0 + s1) + (s2 + s3);
}
// e_atom[i] = sum_k a1[i,k] w2[k] + b2; one wavefront per atom
__global__ void __launch_bounds__(256)
atom_energy_kernel(const float* __restrict__ a1, const float* __restrict__ w2, const float* __restrict__ b2,
                   int64_t n_atoms, int K, float* __restrict__ e_atom) {
  const int64_t i = (int64_t)blockIdx.x * WPB + (threadIdx.x >> 6);
  if (i >= n_atoms) return;
  float s = 0.f;
  for (int k = threadIdx.x & 63; k < K; k += 64) s += a1[i * K + k] * w2[k];
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) e_atom[i] = s + b2[0];
}
// energy[g] = sum of e_atom over the atoms of structure g (fixed order); one wavefront per structure
__global__ void __launch_bounds__(256)
graph_energy_kernel(const float* __restrict__ e_atom, const int32_t* __restrict__ graph_ptr, int n_graphs,
                    float* __restrict__ energy) {
  const int g = blockIdx.x * WPB + (threadIdx.x >> 6);
  if (g >= n_graphs) return;
  float s = 0.f;
  for (int i = graph_ptr[g] + (threadIdx.x & 63); i < graph_ptr[g + 1]; i += 64) s += e_atom[i];
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) energy[g] = s;
}
// dz1[i,k] = w2[k] * silu'(z1[i,k])
__global__ void head_dz_kernel(const float* __restrict__ z1, const float* __restrict__ w2, int64_t n, int K,
                               float* __restrict__ dz1) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dz1[i] = w2[i % K] * dsilu_f(z1[i]);
}
// grad_m[e, :] = dh[dst[e], :]
__global__ void gather_rows_kernel(const float* __restrict__ dh, const int32_t* __restrict__ dst, int64_t n_edges, int H,
                                   float* __restrict__ gm) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_edges * H) return;
  const int64_t e = i / H;
  gm[i] = dh[(int64_t)dst[e] * H + (i % H)];
}
// the same for H % 4 == 0: one wavefront per edge row, 16 bytes per lane and step (the source rows are few and stay cached;
// the [E, H] result is a pure write stream)
__global__ void __launch_bounds__(256)
gather_rows4_kernel(const float* __restrict__ dh, const int32_t* __restrict__ dst, int64_t n_edges, int H, float* __restrict__ gm) {
  typedef float f4 __attribute__((ext_vector_type(4)));
  const int64_t e = (int64_t)blockIdx.x * WPB + (threadIdx.x >> 6);
  if (e >= n_edges) return;
  const f4* src = reinterpret_cast<const f4*>(dh + (int64_t)dst[e] * H);
  f4* out = reinterpret_cast<f4*>(gm + e * H);
  for (int i = threadIdx.x & 63; i < H / 4; i += 64) __builtin_nontemporal_store(src[i], out + i);
}
__global__ void fill_kernel(float* p, int64_t n, float v) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// ------------------------------------------------------------------ forces
// grad_d[e] = sum_n grad_g[e,n] * d g_n / d d,  g_n(d) = u(d/c) exp(-((d/c - mu_n)/Delta)^2 / 2)
__global__ void __launch_bounds__(256)
grad_dist_gauss_kernel(const float* __restrict__ dist, const float* __restrict__ gg, int64_t n_edges, int R, int p,
                       double cutoff, float* __restrict__ gd) {
  const int64_t e = (int64_t)blockIdx.x * WPB + (threadIdx.x >> 6);
  if (e >= n_edges) return;
  const double x = (double)dist[e] / cutoff;
  double xp1 = 1.0;                       // x^(p-1)
  for (int k = 0; k < p - 1; ++k) xp1 *= x;
  const double a = -0.5 * (p + 1) * (p + 2), b = (double)p * (p + 2), c = -0.5 * p * (p + 1);
  const double u = 1.0 + xp1 * x * (a + x * (b + x * c));
  const double du = xp1 * (p * a + x * ((p + 1) * b + x * (p + 2) * c));
  const double inv_delta = (double)(R - 1);
  double s = 0.0;
  for (int n = threadIdx.x & 63; n < R; n += 64) {
    const double t = (x - (double)n / (double)(R - 1)) * inv_delta;
    const double ex = exp(-0.5 * t * t);
    s += (double)gg[e * R + n] * ex * (du - u * t * inv_delta);
  }
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
  if ((threadIdx.x & 63) == 0) gd[e] = (float)(s / cutoff);
}
// out[perm[q]] = in[q]
__global__ void unpermute_kernel(const float* __restrict__ in, const int32_t* __restrict__ perm, int64_t n,
                                 float* __restrict__ out) {
  int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (q < n) out[perm[q]] = in[q];
}
// gu[e, :] (+)= -sum_{t in seg(e)} gc[t] * unit[other[t], :]; one wavefront per edge
__global__ void __launch_bounds__(256)
edge_unit_grad_kernel(const int32_t* __restrict__ seg, const int32_t* __restrict__ other, const float* __restrict__ gc,
                      const float* __restrict__ unit, int64_t n_edges, int accumulate, float* __restrict__ gu) {
  const int64_t e = (int64_t)blockIdx.x * WPB + (threadIdx.x >> 6);
  if (e >= n_edges) return;
  float sx = 0.f, sy = 0.f, sz = 0.f;
  for (int t = seg[e] + (threadIdx.x & 63); t < seg[e + 1]; t += 64) {
    const float g = gc[t];
    const float* u = unit + 3 * (int64_t)other[t];
    sx -= g * u[0]; sy -= g * u[1]; sz -= g * u[2];
  }
  sx = wave_sum(sx); sy = wave_sum(sy); sz = wave_sum(sz);
  if ((threadIdx.x & 63) == 0) {
    float* o = gu + 3 * e;
    if (accumulate) { o[0] += sx; o[1] += sy; o[2] += sz; }
    else { o[0] = sx; o[1] = sy; o[2] = sz; }
  }
}
// The ji-major walk without reordering grad cos: for centre atom j the triplets (in-edge row p, out-list position n)
// form a d_in x d_out matrix stored by rows (kj-major) with one position left out per row; the sum over the triplets of
// out-edge e = out_list[n] is a column sum of it.  gap[e'] = the left-out position of row e' (the number of positions
// if none), one binary search per in-edge.
__global__ void __launch_bounds__(256)
row_gap_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ out_ptr, const int32_t* __restrict__ out_list,
               const int32_t* __restrict__ seg_kj, const int32_t* __restrict__ idx_ji_kj, int32_t* __restrict__ gap) {
  const int j = blockIdx.x;
  const int r0 = row_ptr[j], d = row_ptr[j + 1] - r0;
  const int32_t* outs = out_list + out_ptr[j];
  for (int p = threadIdx.x; p < d; p += 256) {
    const int seg = seg_kj[r0 + p], cnt = seg_kj[r0 + p + 1] - seg;
    int lo = 0, hi = cnt;   // first slot whose target edge is not the out-list entry of the same position
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (idx_ji_kj[seg + mid] == outs[mid]) lo = mid + 1;
      else hi = mid;
    }
    gap[r0 + p] = lo;
  }
}
// gu[e, :] = -sum_{rows p of j} gc_kj[(p, n)] unit[e'_p, :] for e = out_list[out_ptr[j] + n]; workgroup = (atom, 64 positions),
// lanes over positions (consecutive triplets of a row), the four wavefronts over rows
// Sum over the wavefront, valid in lane 63 only, with data-parallel-primitive moves (no LDS crossbar): an inclusive scan
// inside each row of 16 lanes (row_shr 1, 2, 4, 8; lanes without a source add 0), then lane 15 of rows 0 and 2 into rows 1
// and 3 (row_bcast:15), then lane 31 into rows 2 and 3 (row_bcast:31).
__device__ __forceinline__ float wave_sum_lane63(float v) {
  auto add = [](float x, int moved) { return x + __builtin_bit_cast(float, moved); };
  const auto bits = [](float x) { return __builtin_bit_cast(int, x); };
  v = add(v, __builtin_amdgcn_update_dpp(0, bits(v), 0x111, 0xf, 0xf, false));
  v = add(v, __builtin_amdgcn_update_dpp(0, bits(v), 0x112, 0xf, 0xf, false));
  v = add(v, __builtin_amdgcn_update_dpp(0, bits(v), 0x114, 0xf, 0xf, false));
  v = add(v, __builtin_amdgcn_update_dpp(0, bits(v), 0x118, 0xf, 0xf, false));
  v = add(v, __builtin_amdgcn_update_dpp(0, bits(v), 0x142, 0xa, 0xf, false));
  v = add(v, __builtin_amdgcn_update_dpp(0, bits(v), 0x143, 0xc, 0xf, false));
  return v;
}
// ROWS: the same pass also takes the kj-major walk, whose sum over the triplets of in-edge e' is a ROW sum of the same
// matrix: rpart[(e', chunk), :] = -sum over this workgroup's 64 positions of gc unit[out-edge]; the caller adds the chunks
// of a row up (every (row, chunk) pair below gridDim.y is written, zeros past the atom's last chunk), so grad cos is read
// once for both walks and the kj-major one needs no index per triplet.
template <bool ROWS>
__global__ void __launch_bounds__(256)
edge_unit_grad_cols_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ out_ptr,
                           const int32_t* __restrict__ out_list, const int32_t* __restrict__ seg_kj, const int32_t* __restrict__ gap,
                           const float* __restrict__ gc_kj, int64_t T, const float* __restrict__ unit, float* __restrict__ gu,
                           float* __restrict__ rpart) {
  const int j = blockIdx.x, lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int ob = out_ptr[j], dout = out_ptr[j + 1] - ob;
  const int n = 64 * (int)blockIdx.y + lane;
  const int r0 = row_ptr[j], d = row_ptr[j + 1] - r0;
  if (64 * (int)blockIdx.y >= dout) {
    if (ROWS)
      for (int i = threadIdx.x; i < 3 * d; i += 256) rpart[((int64_t)(r0 + i / 3) * gridDim.y + blockIdx.y) * 3 + i % 3] = 0.f;
    return;
  }
  float ox = 0.f, oy = 0.f, oz = 0.f;   // unit vector of this lane's out-edge
  if (ROWS && n < dout) {
    const float* u = unit + 3 * (int64_t)out_list[ob + n];
    ox = u[0]; oy = u[1]; oz = u[2];
  }
  float sx = 0.f, sy = 0.f, sz = 0.f;
  // the rows' segment starts and left-out positions first, 1024 rows at a time: read in the loop they made every row a
  // chain of two memory round trips (segment start, then the value), 75 rows per wavefront one after the other
  constexpr int RCH = 1024;
  __shared__ int32_t s_seg[RCH], s_gap[RCH];
  for (int pb = 0; pb < d; pb += RCH) {
    const int dn = d - pb < RCH ? d - pb : RCH;
    __syncthreads();
    for (int i = threadIdx.x; i < dn; i += 256) {
      s_seg[i] = seg_kj[r0 + pb + i];
      s_gap[i] = gap[r0 + pb + i];
    }
    __syncthreads();
    // batches of 8 rows per wavefront: all loads of a batch first, its stores last (loads and stores complete through one
    // counter: a store inside the loop would make the next row's load wait for it)
    for (int p0 = wv; p0 < dn; p0 += 32) {
      float g[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int p = p0 + 4 * q, pc = p < dn ? p : dn - 1;
        const int seg = s_seg[pc], gp = s_gap[pc];
        const bool valid = p < dn && n < dout && n != gp;
        int64_t at = valid ? seg + n - (n > gp ? 1 : 0) : seg;
        at = at < T ? at : T - 1;                                     // a row without triplets at the very end
        g[q] = gc_kj[at] * (valid ? 1.f : 0.f);                       // unconditional load
      }
      float rx[8], ry[8], rz[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int p = p0 + 4 * q, pc = p < dn ? p : dn - 1;
        const float* u = unit + 3 * (int64_t)(r0 + pb + pc);
        sx -= g[q] * u[0]; sy -= g[q] * u[1]; sz -= g[q] * u[2];      // g = 0 for rows past the end
        if (ROWS) { rx[q] = wave_sum_lane63(g[q] * ox); ry[q] = wave_sum_lane63(g[q] * oy); rz[q] = wave_sum_lane63(g[q] * oz); }
      }
      if (ROWS && lane == 63) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          const int p = p0 + 4 * q;
          if (p < dn) {
            float* o = rpart + ((int64_t)(r0 + pb + p) * gridDim.y + blockIdx.y) * 3;
            o[0] = -rx[q]; o[1] = -ry[q]; o[2] = -rz[q];
          }
        }
      }
    }
  }
  __shared__ float red[3][3][64];
  if (wv > 0) { red[wv - 1][0][lane] = sx; red[wv - 1][1][lane] = sy; red[wv - 1][2][lane] = sz; }
  __syncthreads();
  if (wv == 0 && n < dout) {
#pragma unroll
    for (int k = 0; k < 3; ++k) { sx += red[k][0][lane]; sy += red[k][1][lane]; sz += red[k][2][lane]; }
    float* o = gu + 3 * (int64_t)out_list[ob + n];
    o[0] = sx; o[1] = sy; o[2] = sz;
  }
}
// gu[e, :] += sum_c rpart[(e, c), :]
__global__ void add_row_parts_kernel(const float* __restrict__ rpart, int nc, int64_t n3, float* __restrict__ gu) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // (edge, component)
  if (i >= n3) return;
  const float* p = rpart + (i / 3) * nc * 3 + i % 3;
  float t = 0.f;
  for (int c = 0; c < nc; ++c) t += p[3 * c];
  gu[i] += t;
}
// dv[e,:] = (gu - (gu.u) u) / d + gd * u   (gradient w.r.t. the edge vector x_dst - x_src)
__global__ void edge_vec_grad_kernel(const float* __restrict__ gu, const float* __restrict__ gd,
                                     const float* __restrict__ unit, const float* __restrict__ dist, int64_t n_edges,
                                     float* __restrict__ dv) {
  int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= n_edges) return;
  const float ux = unit[3 * e], uy = unit[3 * e + 1], uz = unit[3 * e + 2];
  const float gx = gu[3 * e], gy = gu[3 * e + 1], gz = gu[3 * e + 2];
  const float dot = gx * ux + gy * uy + gz * uz, inv = 1.0f / dist[e], g = gd[e];
  dv[3 * e] = (gx - dot * ux) * inv + g * ux;
  dv[3 * e + 1] = (gy - dot * uy) * inv + g * uy;
  dv[3 * e + 2] = (gz - dot * uz) * inv + g * uz;
}
// forces[i] = -( sum_{e into i} dv[e] - sum_{e out of i} dv[e] ); one wavefront per atom
__global__ void __launch_bounds__(256)
atom_force_kernel(const float* __restrict__ dv, const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ out_ptr,
                  const int32_t* __restrict__ out_list, int64_t n_atoms, float* __restrict__ forces) {
  const int64_t i = (int64_t)blockIdx.x * WPB + (threadIdx.x >> 6);
  if (i >= n_atoms) return;
  float sx = 0.f, sy = 0.f, sz = 0.f;
  for (int e = row_ptr[i] + (threadIdx.x & 63); e < row_ptr[i + 1]; e += 64) {
    sx += dv[3 * (int64_t)e]; sy += dv[3 * (int64_t)e + 1]; sz += dv[3 * (int64_t)e + 2];
  }
  for (int r = out_ptr[i] + (threadIdx.x & 63); r < out_ptr[i + 1]; r += 64) {
    const int64_t e = out_list[r];
    sx -= dv[3 * e]; sy -= dv[3 * e + 1]; sz -= dv[3 * e + 2];
  }
  sx = wave_sum(sx); sy = wave_sum(sy); sz = wave_sum(sz);
  if ((threadIdx.x & 63) == 0) {
    forces[3 * i] = -sx; forces[3 * i + 1] = -sy; forces[3 * i + 2] = -sz;
  }
}

inline unsigned nblk(int64_t n) { return (unsigned)((n + 255) / 256); }
inline unsigned wblk(int64_t n) { return (unsigned)((n + WPB - 1) / WPB); }

struct head_saved {
  float *h, *z1, *a1, *e_atom;
};
size_t carve_head_saved(void* p, int64_t N, int H, int K, head_saved* s) {
  gp_carver c(p);
  s->h = c.take<float>(N * H);
  s->z1 = c.take<float>(N * K);
  s->a1 = c.take<float>(N * K);
  s->e_atom = c.take<float>(N);
  return c.off;
}
struct head_scratch {
  float *dz1, *dh, *part;
  size_t part_bytes;
};
size_t carve_head_scratch(void* p, int64_t N, int H, int K, head_scratch* s) {
  gp_carver c(p);
  s->dz1 = c.take<float>(N * K);
  s->dh = c.take<float>(N * H);
  s->part_bytes = std::max(gp_gemm_tn_scratch(N, H, K), gp_colsum_scratch(N, K));
  s->part = (float*)c.take<char>(s->part_bytes);
  return c.off;
}
struct forces_ws {
  float *gd, *gc_ji, *gu, *dv;
  int32_t* gap;
};
size_t carve_forces(void* p, int64_t E, int64_t T, forces_ws* w) {
  gp_carver c(p);
  w->gd = c.take<float>(E);
  w->gc_ji = c.take<float>(T);
  w->gap = c.take<int32_t>(E);
  w->gu = c.take<float>(3 * E);
  w->dv = c.take<float>(3 * E);
  return c.off;
}

}  // namespace

// Looks up this device's address of the static scratch array (once per device; the device must be current).
int gp_static_scratch_init(int device) {
  if (device < 0 || device >= MAX_DEVICES) return GP_BAD_ARG;
  std::lock_guard<std::mutex> lock(g_static_mutex);
  if (g_static_ptr[device]) return GP_OK;
  void* ptr = nullptr;
  hipError_t e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
  g_static_err[device] = e;
  if (e != hipSuccess || !ptr) return GP_HIP_ERROR;
  g_static_ptr[device] = ptr;
  return GP_OK;
}

extern "C" {

int gp_edges_by_source_static(gp_ctx* ctx, const int32_t* src, int64_t n_atoms, int64_t n_edges,
                              int32_t* out_ptr, int32_t* out_list) {
  if (!ctx) return GP_BAD_ARG;
  GP_REQUIRE(ctx, n_atoms >= 0 && n_edges >= 0 && out_ptr, "gp_edges_by_source_static: bad arguments");
  if (n_atoms > STATIC_MAX_ATOMS || n_edges > STATIC_MAX_EDGES)
    return gp_fail(ctx, GP_UNSUPPORTED_DIMS, "gp_edges_by_source_static: %lld atoms / %lld edges exceed the static scratch "
                   "(at most %lld atoms, %lld edges); use gp_edges_by_source with a workspace", (long long)n_atoms,
                   (long long)n_edges, (long long)STATIC_MAX_ATOMS, (long long)STATIC_MAX_EDGES);
  GP_HIP(ctx, hipSetDevice(ctx->device));
  void* base = nullptr;
  hipError_t init_err = hipSuccess;
  if (ctx->device < MAX_DEVICES) {
    std::lock_guard<std::mutex> lock(g_static_mutex);
    base = g_static_ptr[ctx->device];
    init_err = g_static_err[ctx->device];
  }
  if (!base)
    return gp_fail(ctx, GP_HIP_ERROR, "gp_edges_by_source_static: no address for the static scratch on device %d (%s)",
                   ctx->device, hipGetErrorString(init_err));
  hipStream_t st = ctx->stream;
  if (n_atoms == 0 || n_edges == 0) {
    fill_zero_kernel<<<nblk(n_atoms + 1), 256, 0, st>>>(out_ptr, n_atoms + 1);
    GP_LAUNCH_CHECK(ctx, "fill_zero_kernel");
    return GP_OK;
  }
  GP_REQUIRE(ctx, src && out_list, "gp_edges_by_source_static: NULL pointer");
  // the two counter arrays are adjacent: one fill clears both; the array keeps the previous call's contents
  int32_t* cnt = (int32_t*)base;
  int32_t* cursor = (int32_t*)((char*)base + STATIC_CNT_BYTES);
  int32_t* tmp = (int32_t*)((char*)base + 2 * STATIC_CNT_BYTES);
  fill_zero_kernel<<<nblk(2 * STATIC_MAX_ATOMS), 256, 0, st>>>(cnt, 2 * STATIC_MAX_ATOMS);
  hist_kernel<<<nblk(n_edges), 256, 0, st>>>(src, n_edges, cnt);
  scan_small_kernel<<<1, 1024, 0, st>>>(cnt, n_atoms, out_ptr);
  scatter_by_key_kernel<<<nblk(n_edges), 256, 0, st>>>(src, n_edges, out_ptr, cursor, tmp);
  sort_lists_kernel<<<(unsigned)n_atoms, 256, 0, st>>>(out_ptr, tmp, n_atoms, out_list);
  GP_LAUNCH_CHECK(ctx, "edges_by_source kernels");
  return GP_OK;
}

int gp_edges_by_source_workspace(int64_t n_atoms, int64_t n_edges, size_t* bytes) {
  if (!bytes || n_atoms < 0 || n_edges < 0) return GP_BAD_ARG;
  *bytes = gp_align(sizeof(int32_t) * n_atoms) * 2 + gp_align(sizeof(int32_t) * n_edges);
  return GP_OK;
}

int gp_edges_by_source(gp_ctx* ctx, const int32_t* src, int64_t n_atoms, int64_t n_edges, void* ws, size_t ws_bytes,
                       int32_t* out_ptr, int32_t* out_list) {
  if (!ctx) return GP_BAD_ARG;
  GP_REQUIRE(ctx, n_atoms >= 0 && n_edges >= 0 && out_ptr, "gp_edges_by_source: bad arguments");
  if (n_atoms > INT32_MAX - 1 || n_edges > INT32_MAX) return gp_fail(ctx, GP_INT32_OVERFLOW, "gp_edges_by_source: sizes exceed int32");
  GP_HIP(ctx, hipSetDevice(ctx->device));
  hipStream_t st = ctx->stream;
  if (n_atoms == 0 || n_edges == 0) {
    GP_HIP(ctx, (hipError_t)gp_zero_async(st, out_ptr, sizeof(int32_t) * (n_atoms + 1)));
    return GP_OK;
  }
  GP_REQUIRE(ctx, src && out_list && ws, "gp_edges_by_source: NULL pointer");
  size_t need;
  gp_edges_by_source_workspace(n_atoms, n_edges, &need);
  if (ws_bytes < need) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "gp_edges_by_source: workspace %zu < %zu", ws_bytes, need);
  gp_carver c(ws);
  int32_t* cnt = c.take<int32_t>(n_atoms);
  int32_t* cursor = c.take<int32_t>(n_atoms);
  int32_t* tmp = c.take<int32_t>(n_edges);
  GP_HIP(ctx, (hipError_t)gp_zero_async(st, cnt, sizeof(int32_t) * n_atoms));
  GP_HIP(ctx, (hipError_t)gp_zero_async(st, cursor, sizeof(int32_t) * n_atoms));
  hist_kernel<<<nblk(n_edges), 256, 0, st>>>(src, n_edges, cnt);
  scan_small_kernel<<<1, 1024, 0, st>>>(cnt, n_atoms, out_ptr);
  scatter_by_key_kernel<<<nblk(n_edges), 256, 0, st>>>(src, n_edges, out_ptr, cursor, tmp);
  sort_lists_kernel<<<(unsigned)n_atoms, 256, 0, st>>>(out_ptr, tmp, n_atoms, out_list);
  GP_LAUNCH_CHECK(ctx, "edges_by_source kernels");
  return GP_OK;
}

int gp_energy_workspace(int32_t emb, int32_t hidden, int64_t n_atoms, size_t* saved_bytes, size_t* scratch_bytes) {
  if (!saved_bytes || !scratch_bytes || emb < 1 || hidden < 1 || n_atoms < 0) return GP_BAD_ARG;
  head_saved s;
  head_scratch sc;
  *saved_bytes = carve_head_saved(nullptr, n_atoms, emb, hidden, &s);
  *scratch_bytes = carve_head_scratch(nullptr, n_atoms, emb, hidden, &sc);
  return GP_OK;
}

int gp_energy_forward(gp_ctx* ctx, int32_t emb, int32_t hidden, const gp_weights_head* w, const float* m,
                      const int32_t* row_ptr, const int32_t* graph_ptr, int64_t n_atoms, int32_t n_graphs,
                      float* energy, void* saved, size_t saved_bytes) {
  if (!ctx) return GP_BAD_ARG;
  GP_REQUIRE(ctx, emb >= 1 && hidden >= 1 && n_atoms >= 0 && n_graphs >= 0, "gp_energy_forward: bad sizes");
  GP_REQUIRE(ctx, w && w->W1 && w->b1 && w->w2 && w->b2, "gp_energy_forward: weights missing");
  if (n_atoms == 0 || n_graphs == 0) return GP_OK;
  GP_REQUIRE(ctx, m && row_ptr && graph_ptr && energy && saved, "gp_energy_forward: NULL pointer");
  head_saved s;
  if (saved_bytes < carve_head_saved(saved, n_atoms, emb, hidden, &s)) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "gp_energy_forward: saved buffer too small");
  GP_HIP(ctx, hipSetDevice(ctx->device));
  hipStream_t st = ctx->stream;
  {
    gp_prof_scope prof(ctx, "head_atom_sum", 0.0, 0.0);   // the number of edges is not known here: time only
    atom_sum_kernel<<<wblk(n_atoms * ((emb + 63) / 64)), 256, 0, st>>>(m, row_ptr, n_atoms, emb, s.h);
    GP_LAUNCH_CHECK(ctx, "atom_sum_kernel");
  }
  gp_epilogue e;
  e.bias = w->b1; e.save_pre = s.z1; e.act = 1; e.out = s.a1;
  GP_TRY(gp_gemm_nn(ctx, s.h, w->W1, n_atoms, hidden, emb, e));
  atom_energy_kernel<<<wblk(n_atoms), 256, 0, st>>>(s.a1, w->w2, w->b2, n_atoms, hidden, s.e_atom);
  graph_energy_kernel<<<wblk(n_graphs), 256, 0, st>>>(s.e_atom, graph_ptr, n_graphs, energy);
  GP_LAUNCH_CHECK(ctx, "energy kernels");
  return GP_OK;
}

int gp_energy_backward(gp_ctx* ctx, int32_t emb, int32_t hidden, const gp_weights_head* w, const int32_t* dst,
                       int64_t n_atoms, int64_t n_edges, const void* saved, size_t saved_bytes, float* grad_m,
                       gp_weights_head* grad_w, void* scratch, size_t scratch_bytes) {
  if (!ctx) return GP_BAD_ARG;
  GP_REQUIRE(ctx, emb >= 1 && hidden >= 1 && n_atoms > 0 && n_edges >= 0, "gp_energy_backward: bad sizes");
  GP_REQUIRE(ctx, w && w->W1 && w->w2 && saved && scratch && (n_edges == 0 || (dst && grad_m)), "gp_energy_backward: NULL pointer");
  head_saved s;
  head_scratch sc;
  if (saved_bytes < carve_head_saved(const_cast<void*>(saved), n_atoms, emb, hidden, &s)) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "gp_energy_backward: saved buffer too small");
  if (scratch_bytes < carve_head_scratch(scratch, n_atoms, emb, hidden, &sc)) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "gp_energy_backward: scratch too small");
  GP_HIP(ctx, hipSetDevice(ctx->device));
  hipStream_t st = ctx->stream;
  head_dz_kernel<<<nblk(n_atoms * hidden), 256, 0, st>>>(s.z1, w->w2, n_atoms * hidden, hidden, sc.dz1);
  GP_LAUNCH_CHECK(ctx, "head_dz_kernel");
  gp_epilogue e;
  e.out = sc.dh;
  GP_TRY(gp_gemm_nt(ctx, sc.dz1, w->W1, n_atoms, emb, hidden, e));
  if (n_edges > 0) {
    gp_prof_scope prof(ctx, "head_gather_rows", 0.0, 4.0 * (double)emb * ((double)n_edges + (double)n_atoms));
    if (emb % 4 == 0 && (reinterpret_cast<uintptr_t>(grad_m) & 15) == 0 && (reinterpret_cast<uintptr_t>(sc.dh) & 15) == 0)
      gather_rows4_kernel<<<wblk(n_edges), 256, 0, st>>>(sc.dh, dst, n_edges, emb, grad_m);
    else
      gather_rows_kernel<<<nblk(n_edges * emb), 256, 0, st>>>(sc.dh, dst, n_edges, emb, grad_m);
    GP_LAUNCH_CHECK(ctx, "gather_rows_kernel");
  }
  if (grad_w) {
    GP_REQUIRE(ctx, grad_w->W1 && grad_w->b1 && grad_w->w2 && grad_w->b2, "gp_energy_backward: grad_w has a NULL member");
    GP_TRY(gp_gemm_tn(ctx, s.h, sc.dz1, n_atoms, emb, hidden, grad_w->W1, grad_w->b1, sc.part, sc.part_bytes));
    GP_TRY(gp_colsum(ctx, s.a1, n_atoms, hidden, grad_w->w2, sc.part, sc.part_bytes));
    fill_kernel<<<1, 64, 0, st>>>(grad_w->b2, 1, (float)n_atoms);
    GP_LAUNCH_CHECK(ctx, "fill_kernel");
  }
  return GP_OK;
}

int gp_forces_workspace(int64_t n_edges, int64_t n_triplets, size_t* bytes) {
  if (!bytes || n_edges < 0 || n_triplets < 0) return GP_BAD_ARG;
  forces_ws w;
  *bytes = carve_forces(nullptr, n_edges, n_triplets, &w);
  return GP_OK;
}

}  // extern "C"

namespace {
// variant G: grad_rad is NULL and the radial basis is the Gaussian one; variant D: Bessel radial basis and the radial
// part of the spherical basis
int forces_from_basis_grad(gp_ctx* ctx, const gp_dims* dims, const gp_graph* graph, const int32_t* perm_kj,
                           const int32_t* row_ptr, const int32_t* out_ptr, const int32_t* out_list,
                           int64_t n_atoms, const float* dist, const float* unit, const float* grad_rbf, const float* grad_rad,
                           const float* grad_cos_kj, float* forces, void* ws, size_t ws_bytes) {
  if (!ctx) return GP_BAD_ARG;
  GP_REQUIRE(ctx, dims && graph, "gp_forces_from_basis_grad: dims/graph is NULL");
  const bool bessel = dims->variant == GP_VARIANT_D;
  if (!bessel && dims->variant != GP_VARIANT_G) return gp_fail(ctx, GP_BAD_ARG, "gp_forces_from_basis_grad: unknown variant %d", dims->variant);
  const int64_t E = graph->n_edges, T = graph->n_triplets;
  GP_REQUIRE(ctx, n_atoms >= 0 && E >= 0 && T >= 0, "gp_forces_from_basis_grad: negative size");
  if (n_atoms == 0) return GP_OK;
  GP_REQUIRE(ctx, forces && row_ptr && out_ptr, "gp_forces_from_basis_grad: NULL pointer");
  GP_HIP(ctx, hipSetDevice(ctx->device));
  hipStream_t st = ctx->stream;
  if (E == 0) {
    fill_kernel<<<nblk(3 * n_atoms), 256, 0, st>>>(forces, 3 * n_atoms, 0.f);
    GP_LAUNCH_CHECK(ctx, "fill_kernel");
    return GP_OK;
  }
  GP_REQUIRE(ctx, out_list && dist && unit && grad_rbf && ws && (!bessel || grad_rad), "gp_forces_from_basis_grad: NULL pointer");
  GP_REQUIRE(ctx, T == 0 || (grad_cos_kj && perm_kj && graph->idx_kj && graph->seg_ptr_ji && graph->idx_ji_kj && graph->seg_ptr_kj),
             "gp_forces_from_basis_grad: triplet arrays missing");
  forces_ws w;
  if (ws_bytes < carve_forces(ws, E, T, &w)) return gp_fail(ctx, GP_BUFFER_TOO_SMALL, "gp_forces_from_basis_grad: workspace too small");
  if (bessel) GP_TRY(gp_grad_dist_bessel(ctx, dims, dist, grad_rbf, grad_rad, E, w.gd));
  else
    grad_dist_gauss_kernel<<<wblk(E), 256, 0, st>>>(dist, grad_rbf, E, dims->num_radial, dims->envelope_p,
                                                    (double)dims->cutoff, w.gd);
  if (T > 0) {
    // cos = -unit[ji].unit[kj]: d/d unit[ji] = -unit[kj] (ji-major walk), d/d unit[kj] = -unit[ji] (kj-major walk)
    gp_prof_scope prof(ctx, "forces_edge_sums", 12.0 * (double)T, 12.0 * (double)T);
    const int nc = (graph->max_out_degree + 63) / 64;
    if (graph->max_out_degree > 0 && (int64_t)E * nc * 3 <= T) {
      // both walks as sums over the per-atom (in-edge, out-position) matrix in kj-major order, grad cos read once: columns
      // = the ji-major walk, rows = the kj-major one, per 64-position chunk; the chunks' row sums (E x nc x 3 floats)
      // borrow the buffer of the reordered copy that this path does not make
      row_gap_kernel<<<(unsigned)n_atoms, 256, 0, st>>>(row_ptr, out_ptr, out_list, graph->seg_ptr_kj, graph->idx_ji_kj, w.gap);
      edge_unit_grad_cols_kernel<true><<<dim3((unsigned)n_atoms, (unsigned)nc), 256, 0, st>>>(
          row_ptr, out_ptr, out_list, graph->seg_ptr_kj, w.gap, grad_cos_kj, T, unit, w.gu, w.gc_ji);
      add_row_parts_kernel<<<nblk(3 * E), 256, 0, st>>>(w.gc_ji, nc, 3 * E, w.gu);
    } else {
      if (graph->max_out_degree > 0) {
        // the ji-major walk as column sums over the kj-major order: no reordered copy of grad cos
        row_gap_kernel<<<(unsigned)n_atoms, 256, 0, st>>>(row_ptr, out_ptr, out_list, graph->seg_ptr_kj, graph->idx_ji_kj, w.gap);
        edge_unit_grad_cols_kernel<false><<<dim3((unsigned)n_atoms, (unsigned)nc), 256, 0, st>>>(
            row_ptr, out_ptr, out_list, graph->seg_ptr_kj, w.gap, grad_cos_kj, T, unit, w.gu, nullptr);
      } else {
        unpermute_kernel<<<nblk(T), 256, 0, st>>>(grad_cos_kj, perm_kj, T, w.gc_ji);
        edge_unit_grad_kernel<<<wblk(E), 256, 0, st>>>(graph->seg_ptr_ji, graph->idx_kj, w.gc_ji, unit, E, 0, w.gu);
      }
      edge_unit_grad_kernel<<<wblk(E), 256, 0, st>>>(graph->seg_ptr_kj, graph->idx_ji_kj, grad_cos_kj, unit, E, 1, w.gu);
    }
  } else {
    fill_kernel<<<nblk(3 * E), 256, 0, st>>>(w.gu, 3 * E, 0.f);
  }
  edge_vec_grad_kernel<<<nblk(E), 256, 0, st>>>(w.gu, w.gd, unit, dist, E, w.dv);
  atom_force_kernel<<<wblk(n_atoms), 256, 0, st>>>(w.dv, row_ptr, out_ptr, out_list, n_atoms, forces);
  GP_LAUNCH_CHECK(ctx, "force kernels");
  return GP_OK;
}
}  // namespace

extern "C" {

int gp_forces_from_basis_grad(gp_ctx* ctx, const gp_dims* dims, const gp_graph* graph, const int32_t* perm_kj,
                              const int32_t* row_ptr, const int32_t* out_ptr, const int32_t* out_list,
                              int64_t n_atoms, const float* dist, const float* unit, const float* grad_rbf,
                              const float* grad_cos_kj, float* forces, void* ws, size_t ws_bytes) {
  if (!ctx) return GP_BAD_ARG;
  if (dims && dims->variant != GP_VARIANT_G)
    return gp_fail(ctx, GP_UNSUPPORTED_DIMS, "gp_forces_from_basis_grad: the Gaussian radial basis (variant G); variant D has "
                   "gp_forces_from_basis_grad_D");
  return forces_from_basis_grad(ctx, dims, graph, perm_kj, row_ptr, out_ptr, out_list, n_atoms, dist, unit, grad_rbf, nullptr,
                                grad_cos_kj, forces, ws, ws_bytes);
}

int gp_forces_from_basis_grad_D(gp_ctx* ctx, const gp_dims* dims, const gp_graph* graph, const int32_t* perm_kj,
                                const int32_t* row_ptr, const int32_t* out_ptr, const int32_t* out_list,
                                int64_t n_atoms, const float* dist, const float* unit, const float* grad_rbf,
                                const float* grad_rad, const float* grad_cos_kj, float* forces, void* ws, size_t ws_bytes) {
  if (!ctx) return GP_BAD_ARG;
  if (dims && dims->variant != GP_VARIANT_D)
    return gp_fail(ctx, GP_UNSUPPORTED_DIMS, "gp_forces_from_basis_grad_D: the Bessel bases of variant D");
  return forces_from_basis_grad(ctx, dims, graph, perm_kj, row_ptr, out_ptr, out_list, n_atoms, dist, unit, grad_rbf, grad_rad,
                                grad_cos_kj, forces, ws, ws_bytes);
}

}  // extern "C"
