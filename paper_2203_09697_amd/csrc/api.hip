// Context management for the C ABI.
#include <stdarg.h>
#include <stdlib.h>

#include <new>

#include "common.h"

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
  const char* no_aux = getenv("GP_NO_AUX_STREAM");
  c->use_aux = !(no_aux && no_aux[0] == '1');
  const char* tm = getenv("GP_TRIPLET_MFMA");
  if (tm && tm[0] >= '0' && tm[0] <= '2') c->trip_mfma = tm[0] - '0';
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
  delete ctx;
}

int gp_set_side_stream(gp_ctx* ctx, int on) {
  if (!ctx) return GP_BAD_ARG;
  ctx->use_aux = on != 0;
  return GP_OK;
}

int gp_set_triplet_mfma(gp_ctx* ctx, int mode) {
  if (!ctx || mode < -1 || mode > 2) return GP_BAD_ARG;
  ctx->trip_mfma = mode;
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

const char* gp_last_error(const gp_ctx* ctx) { return ctx ? ctx->err : "null context"; }

}  // extern "C"
