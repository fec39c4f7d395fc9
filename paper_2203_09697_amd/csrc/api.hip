// Context management for the C ABI.
#include <stdarg.h>
#include <stdlib.h>

#include <new>

#include "common.h"

namespace {
__global__ void degree_check_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ out_ptr, int64_t n,
                                    int max_in, int max_out, int* __restrict__ flag) {
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= n) return;
  if (row_ptr[j + 1] - row_ptr[j] > max_in || out_ptr[j + 1] - out_ptr[j] > max_out) *flag = 1;
}
}  // namespace

int gp_check_degrees(gp_ctx* ctx, const gp_graph* g) {
  if (!ctx->dflag_dev || !g || g->n_atoms <= 0 || !g->row_ptr || !g->out_ptr) return GP_OK;
  degree_check_kernel<<<(unsigned)((g->n_atoms + 255) / 256), 256, 0, ctx->stream>>>(g->row_ptr, g->out_ptr, g->n_atoms,
                                                                                   g->max_in_degree, g->max_out_degree, ctx->dflag_dev);
  GP_LAUNCH_CHECK(ctx, "degree_check_kernel");
  return GP_OK;
}

int gp_take_deferred(gp_ctx* ctx, const char* who) {
  if (!ctx->dflag || !*(volatile int*)ctx->dflag) return GP_OK;
  *(volatile int*)ctx->dflag = 0;
  return gp_fail(ctx, GP_BAD_ARG, "%s: an earlier block call on this context was given gp_graph.max_in_degree / max_out_degree "
                 "below the true maxima; the atoms above them were skipped and that call's results are incomplete", who);
}

int gp_static_scratch_init(int device);   // energy.hip: address of the allocation-free entry point's scratch array

extern "C" {

const char* gp_version(void) { return "gpgnn 0.1 (gfx950)"; }

int gp_create(gp_ctx** out, int device_id, void* hip_stream) {
  if (!out) return GP_BAD_ARG;
  *out = nullptr;
  int n = 0;
  if (hipGetDeviceCount(&n) != hipSuccess || device_id < 0 || device_id >= n) return GP_HIP_ERROR;
  gp_ctx* c = new (std::nothrow) gp_ctx();
  if (!c) return GP_HIP_ERROR;
  c->device = device_id;
  c->stream = (hipStream_t)hip_stream;
  // side stream at the default priority; without it everything simply runs on the main stream
  if (hipSetDevice(device_id) != hipSuccess || hipStreamCreateWithFlags(&c->aux_stream, hipStreamNonBlocking) != hipSuccess)
    c->aux_stream = nullptr;
  // per-device address of the static scratch (the device is current here); a failure is reported by the entry point
  // that needs it, not here
  (void)gp_static_scratch_init(device_id);
  // one pinned, device-visible word for errors that only a kernel can detect
  if (hipHostMalloc((void**)&c->dflag, sizeof(int), hipHostMallocMapped) == hipSuccess) {
    *c->dflag = 0;
    if (hipHostGetDevicePointer((void**)&c->dflag_dev, c->dflag, 0) != hipSuccess) c->dflag_dev = nullptr;
  } else {
    c->dflag = nullptr;
  }
  const char* no_aux = getenv("GP_NO_AUX_STREAM");
  c->use_aux = !(no_aux && no_aux[0] == '1');
  const char* tm = getenv("GP_TRIPLET_MFMA");
  if (tm && tm[0] >= '0' && tm[0] <= '3') c->trip_mfma = tm[0] - '0';
  const char* fg = getenv("GP_F32_GEMM");
  if (fg && (fg[0] == '0' || fg[0] == '1')) c->f32_split = fg[0] == '1';
  *out = c;
  return GP_OK;
}

void gp_destroy(gp_ctx* ctx) {
  if (!ctx) return;
  for (auto& p : ctx->prof) {
    (void)hipEventDestroy(p.t0);
    (void)hipEventDestroy(p.t1);
  }
  for (auto e : ctx->event_pool) (void)hipEventDestroy(e);
  for (auto e : ctx->aux_event_pool) (void)hipEventDestroy(e);
  if (ctx->aux_stream) (void)hipStreamDestroy(ctx->aux_stream);
  if (ctx->dflag) (void)hipHostFree(ctx->dflag);
  delete ctx;
}

int gp_set_side_stream(gp_ctx* ctx, int on) {
  if (!ctx) return GP_BAD_ARG;
  ctx->use_aux = on != 0;
  return GP_OK;
}

int gp_set_triplet_mfma(gp_ctx* ctx, int mode) {
  if (!ctx || mode < -1 || mode > 3) return GP_BAD_ARG;
  ctx->trip_mfma = mode;
  return GP_OK;
}

int gp_set_f32_gemm(gp_ctx* ctx, int split) {
  if (!ctx || split < 0 || split > 1) return GP_BAD_ARG;
  ctx->f32_split = split != 0;
  return GP_OK;
}

int gp_profile_enable(gp_ctx* ctx, int on) {
  if (!ctx) return GP_BAD_ARG;
  ctx->prof_on = on != 0;
  return GP_OK;
}

int gp_profile_reset(gp_ctx* ctx) {
  if (!ctx) return GP_BAD_ARG;
  for (auto& p : ctx->prof) {
    ctx->event_pool.push_back(p.t0);
    ctx->event_pool.push_back(p.t1);
  }
  ctx->prof.clear();
  return GP_OK;
}

int gp_profile_count(gp_ctx* ctx, int64_t* n) {
  if (!ctx || !n) return GP_BAD_ARG;
  *n = (int64_t)ctx->prof.size();
  return GP_OK;
}

int gp_profile_get(gp_ctx* ctx, int64_t i, const char** name, float* ms, double* flops, double* bytes) {
  if (!ctx || !name || !ms || !flops || !bytes) return GP_BAD_ARG;
  GP_REQUIRE(ctx, i >= 0 && i < (int64_t)ctx->prof.size(), "gp_profile_get: index out of range");
  const gp_prof_entry& p = ctx->prof[(size_t)i];
  GP_HIP(ctx, hipEventSynchronize(p.t1));
  GP_HIP(ctx, hipEventElapsedTime(ms, p.t0, p.t1));
  *name = p.name;
  *flops = p.flops;
  *bytes = p.bytes;
  return GP_OK;
}

int gp_deferred_status(gp_ctx* ctx) {
  if (!ctx) return GP_BAD_ARG;
  GP_HIP(ctx, hipSetDevice(ctx->device));
  GP_HIP(ctx, hipStreamSynchronize(ctx->stream));
  return gp_take_deferred(ctx, "gp_deferred_status");
}

const char* gp_last_error(const gp_ctx* ctx) { return ctx ? ctx->err : "null context"; }

}  // extern "C"

namespace {
__global__ void zero_words_kernel(uint32_t* __restrict__ p, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}
}  // namespace

int gp_zero_async(hipStream_t st, void* p, size_t bytes) {
  const size_t n = bytes / 4;
  if (n == 0) return (int)hipSuccess;
  zero_words_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(static_cast<uint32_t*>(p), n);
  return (int)hipGetLastError();
}
