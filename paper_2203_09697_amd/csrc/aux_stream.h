// Side stream for work that nothing on the main stream waits for until the end of a call
// (weight-gradient GEMMs of the backward pass).  Two kernels of that size do not fill the chip
// on their own (a few hundred workgroups each), so running the weight-gradient chain next to the
// input-gradient chain recovers the idle tail of both.
//
// Rules kept by this helper:
//   * work moved to the side stream starts after everything issued so far on the main stream;
//   * before the main stream overwrites a buffer the side stream may still be reading,
//     before_write(buffer) makes it wait for that reader;
//   * join() makes the main stream wait for all side work; it is called before the entry point
//     returns (the destructor does the same on an early error return), so callers see ordinary
//     single-stream semantics.
#pragma once
#include <initializer_list>

#include "common.h"

struct gp_aux {
  gp_ctx* c;
  hipStream_t main_s, aux_s;
  hipEvent_t last = nullptr;
  struct reader { const void* p; hipEvent_t ev; };
  reader readers[24];
  int nr = 0;
  std::vector<hipEvent_t> used;

  explicit gp_aux(gp_ctx* ctx) : c(ctx), main_s(ctx->stream), aux_s(ctx->use_aux ? ctx->aux_stream : nullptr) {}
  ~gp_aux() {
    // an entry point that returns early (an error between on_aux and join) still leaves the main stream ordered
    // behind the side work it started
    if (last) (void)hipStreamWaitEvent(main_s, last, 0);
    for (hipEvent_t e : used) c->aux_event_pool.push_back(e);
  }
  bool active() const { return aux_s != nullptr; }

  hipEvent_t get_event() {
    hipEvent_t e = nullptr;
    if (!c->aux_event_pool.empty()) {
      e = c->aux_event_pool.back();
      c->aux_event_pool.pop_back();
    } else if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) {
      return nullptr;
    }
    used.push_back(e);
    return e;
  }

  // fn() issues its launches on c->stream; `reads` are the buffers it reads that the main
  // stream will overwrite later in this call
  template <class F>
  int on_aux(F fn, std::initializer_list<const void*> reads) {
    if (!active()) return fn();
    hipEvent_t fork = get_event(), done = get_event();
    if (!fork || !done) return fn();
    if (hipEventRecord(fork, main_s) != hipSuccess || hipStreamWaitEvent(aux_s, fork, 0) != hipSuccess) return fn();
    c->stream = aux_s;
    const int rc = fn();
    c->stream = main_s;
    if (hipEventRecord(done, aux_s) != hipSuccess) return gp_fail(c, GP_HIP_ERROR, "hipEventRecord on the side stream failed");
    last = done;
    for (const void* p : reads) {
      int i = 0;
      while (i < nr && readers[i].p != p) ++i;
      if (i == nr && nr < 24) ++nr;
      if (i < 24) readers[i] = {p, done};
    }
    return rc;
  }

  int before_write(const void* p) {
    for (int i = 0; i < nr; ++i)
      if (readers[i].p == p) {
        if (hipStreamWaitEvent(main_s, readers[i].ev, 0) != hipSuccess)
          return gp_fail(c, GP_HIP_ERROR, "hipStreamWaitEvent failed");
        readers[i] = readers[--nr];
        break;
      }
    return GP_OK;
  }

  int join() {
    if (last && hipStreamWaitEvent(main_s, last, 0) != hipSuccess) return gp_fail(c, GP_HIP_ERROR, "hipStreamWaitEvent failed");
    last = nullptr;
    nr = 0;
    return GP_OK;
  }
};
