// Context management for the C ABI.
#include <stdarg.h>
#include <stdlib.h>

#include "common.h"

extern "C" {

const char* gp_version(void) { return "gpgnn 0.1 (gfx950)"; }

int gp_create(gp_ctx** out, int device_id, void* hip_stream) {
  if (!out) return GP_BAD_ARG;
  *out = nullptr;
  int n = 0;
  if (hipGetDeviceCount(&n) != hipSuccess || device_id < 0 || device_id >= n) return GP_HIP_ERROR;
  gp_ctx* c = (gp_ctx*)calloc(1, sizeof(gp_ctx));
  if (!c) return GP_HIP_ERROR;
  c->device = device_id;
  c->stream = (hipStream_t)hip_stream;
  c->err[0] = 0;
  *out = c;
  return GP_OK;
}

void gp_destroy(gp_ctx* ctx) { free(ctx); }

const char* gp_last_error(const gp_ctx* ctx) { return ctx ? ctx->err : "null context"; }

}  // extern "C"
