// Internal helpers shared by the library's translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include <unordered_map>
#include <vector>

#include "../../include/gpgnn.h"

// One bracketed kernel launch (only recorded while profiling is enabled).
struct gp_prof_entry {
  const char* name;   // static string naming the kernel instantiation
  hipEvent_t t0, t1;
  double flops, bytes;  // algorithmic work of this launch
};

struct gp_ctx {
  int device = 0;
  hipStream_t stream = nullptr;
  char err[512] = {0};
  bool prof_on = false;
  bool gemm_bf16 = false;   // set by a block call whose dims ask for bf16 GEMM operands
  bool f32_split = true;    // fp32 GEMMs on the bf16 matrix cores with three bf16 planes per operand (false: fp32 MFMA)
  hipStream_t aux_stream = nullptr;   // side stream for weight-gradient GEMMs (see aux_stream.h)
  bool use_aux = true;
  int trip_mfma = -1;       // matrix-core triplet kernels of the bilinear block: -1 by graph density, 0 never, 1 whenever usable,
                            // 2 as 1 but the forward pass in its two-kernel form (per-triplet y buffer) instead of the fused one
  std::vector<hipEvent_t> aux_event_pool;
  std::vector<gp_prof_entry> prof;
  std::vector<hipEvent_t> event_pool;
  // Storage decisions of a block's forward call that its backward call must repeat (which buffers were written and
  // in which element type), keyed by the `saved` buffer: the backward call compares instead of trusting the
  // context's settings to be unchanged.
  std::unordered_map<const void*, uint32_t> fwd_flags;
  // Deferred errors of kernels (one int in pinned host memory that the device writes): set when a graph's
  // max_in_degree / max_out_degree turn out to be below the true maxima; reported by the next block call or
  // gp_deferred_status.
  int* dflag = nullptr;       // host address
  int* dflag_dev = nullptr;   // the same word as the device sees it
};

// Launches the check of gp_graph.max_in_degree / max_out_degree against the lists (sets the deferred-error word).
int gp_check_degrees(gp_ctx* ctx, const gp_graph* g);
// Clears `bytes` (a multiple of 4) of device memory with a kernel on `st`.  The library records no memset nodes: a caller
// may capture its calls in a HIP graph, and memset nodes have given wrong results on replays on this target.
int gp_zero_async(hipStream_t st, void* p, size_t bytes);
// dL/dd per edge from the gradients with respect to the Bessel radial basis and the radial part of the spherical basis of
// the Hadamard variant (basis.hip; either gradient may be NULL)
int gp_grad_dist_bessel(gp_ctx* ctx, const gp_dims* dims, const float* dist, const float* grad_rbf, const float* grad_rad,
                        int64_t n_edges, float* gd);
// GP_BAD_ARG (and a message) if an earlier call on this context left a deferred error; clears it.
int gp_take_deferred(gp_ctx* ctx, const char* who);

// Brackets the launches issued during its lifetime with two HIP events on the context's
// stream when profiling is on; otherwise does nothing.
struct gp_prof_scope {
  gp_ctx* c;
  bool active;
  hipEvent_t t1;
  gp_prof_scope(gp_ctx* ctx, const char* name, double flops, double bytes) : c(ctx), active(false), t1(nullptr) {
    if (!c || !c->prof_on) return;
    hipEvent_t ev[2];
    for (int i = 0; i < 2; ++i) {
      if (!c->event_pool.empty()) {
        ev[i] = c->event_pool.back();
        c->event_pool.pop_back();
      } else if (hipEventCreate(&ev[i]) != hipSuccess) {
        return;
      }
    }
    c->prof.push_back({name, ev[0], ev[1], flops, bytes});
    t1 = ev[1];
    active = hipEventRecord(ev[0], c->stream) == hipSuccess;
  }
  ~gp_prof_scope() {
    if (active) (void)hipEventRecord(t1, c->stream);
  }
};

inline int gp_fail(gp_ctx* ctx, int code, const char* fmt, ...) __attribute__((format(printf, 3, 4)));
inline int gp_fail(gp_ctx* ctx, int code, const char* fmt, ...) {
  if (ctx) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
    va_end(ap);
  }
  return code;
}

#define GP_HIP(ctx, expr)                                                                  \
  do {                                                                                     \
    hipError_t _e = (expr);                                                                \
    if (_e != hipSuccess)                                                                  \
      return gp_fail((ctx), GP_HIP_ERROR, "%s failed: %s (%s:%d)", #expr,                  \
                     hipGetErrorString(_e), __FILE__, __LINE__);                           \
  } while (0)

#define GP_LAUNCH_CHECK(ctx, name)                                                         \
  do {                                                                                     \
    hipError_t _e = hipGetLastError();                                                     \
    if (_e != hipSuccess)                                                                  \
      return gp_fail((ctx), GP_HIP_ERROR, "launch of %s failed: %s", name,                 \
                     hipGetErrorString(_e));                                               \
  } while (0)

#define GP_REQUIRE(ctx, cond, ...)                                                         \
  do {                                                                                     \
    if (!(cond)) return gp_fail((ctx), GP_BAD_ARG, __VA_ARGS__);                           \
  } while (0)

#define GP_TRY(expr)                                                                       \
  do {                                                                                     \
    int _s = (expr);                                                                       \
    if (_s != GP_OK) return _s;                                                            \
  } while (0)

static inline size_t gp_align(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// Sequential carve-out of a caller-provided buffer.
struct gp_carver {
  char* base;
  size_t off;
  explicit gp_carver(void* p) : base((char*)p), off(0) {}
  template <class T>
  T* take(size_t n) {
    T* r = base ? (T*)(base + off) : nullptr;
    off += gp_align(n * sizeof(T));
    return r;
  }
};

constexpr int WAVE = 64;

__device__ __forceinline__ int lane_id() { return threadIdx.x & (WAVE - 1); }

// number of set bits of `mask` strictly below this lane
__device__ __forceinline__ int mbcnt(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}

// Orders the distinct values tmp[0..n) ascending into out[0..n) by rank counting, one workgroup per list: the list is
// parked in LDS (lists longer than SORT_LDS values are read from memory instead), every thread counts, for its
// elements, the smaller ones.  All threads of the workgroup must call it.
constexpr int SORT_LDS = 2048;
__device__ __forceinline__ void sort_list_block(const int32_t* __restrict__ tmp, int n, int32_t* __restrict__ out, int32_t* lds) {
  const bool staged = n <= SORT_LDS;
  if (staged) {
    for (int r = threadIdx.x; r < n; r += blockDim.x) lds[r] = tmp[r];
    __syncthreads();
  }
  const int32_t* list = staged ? lds : tmp;
  for (int r = threadIdx.x; r < n; r += blockDim.x) {
    const int v = list[r];
    int rank = 0;
    for (int q = 0; q < n; ++q) rank += list[q] < v ? 1 : 0;
    out[rank] = v;
  }
}

// The sigmoid through the hardware reciprocal (1 ulp, one instruction) instead of an IEEE division (a dozen): these
// functions sit in GEMM epilogues and streaming kernels, where the division was a visible share of the time.
__device__ __forceinline__ float sigmoid_f(float z) { return __builtin_amdgcn_rcpf(1.0f + __expf(-z)); }
__device__ __forceinline__ float silu_f(float z) { return z * sigmoid_f(z); }
// d/dz [ z * sigmoid(z) ]
__device__ __forceinline__ float dsilu_f(float z) {
  const float s = sigmoid_f(z);
  return s * (1.0f + z * (1.0f - s));
}
