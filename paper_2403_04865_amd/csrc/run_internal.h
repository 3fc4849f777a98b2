// Launch bookkeeping shared by the context types of libslide: the first failing launch of a call stops the rest of
// its sequence, and the measurement hooks bracket launches of chosen kernel families with HIP events.
#pragma once
#include "../../include/slide_prof.h"
#include "slide_internal.h"
#include <vector>

namespace sl {

constexpr int PROF_FAMILIES = 24;   // upper bound on the kernel families of one context type

extern thread_local int g_last_hip;   // hipError_t of the most recent failing HIP call on this thread

struct Prof {
  bool active = false;
  int id = -1;                 // family being recorded, SLIDE_PROF_ALL = every family
  int count = 0;
  std::vector<hipEvent_t> ev;  // 2 per launch
  std::vector<int> fam;        // family of recorded launch i
  // per family, filled by launch() (flops, bytes, n) and prof_end (ms)
  double flops[PROF_FAMILIES] = {}, bytes[PROF_FAMILIES] = {}, ms[PROF_FAMILIES] = {};
  int n[PROF_FAMILIES] = {};
};

template <typename Ctx>
struct RunT {
  Ctx* c;
  hipStream_t s;
  hipError_t err = hipSuccess;
  bool ok() const { return err == hipSuccess; }
};

// Launch wrapper: skips work after the first failure and records profiling events.
template <typename Ctx, typename F>
void launch(RunT<Ctx>& r, int id, double flops, double bytes, F f) {
  if (!r.ok()) return;
  Prof& p = r.c->prof;
  bool rec = p.active && (p.id == id || p.id == SLIDE_PROF_ALL) && p.count < SLIDE_PROF_MAX;
  if (rec) {
    while ((int)p.ev.size() < 2 * (p.count + 1)) {
      hipEvent_t e;
      if (hipEventCreate(&e) != hipSuccess) { rec = false; break; }
      p.ev.push_back(e);
    }
  }
  if (rec) (void)hipEventRecord(p.ev[2 * p.count], r.s);
  hipError_t e = f();
  if (rec) {
    (void)hipEventRecord(p.ev[2 * p.count + 1], r.s);
    if ((int)p.fam.size() <= p.count) p.fam.resize(p.count + 1);
    p.fam[p.count] = id;
    p.count++;
    p.flops[id] += flops;
    p.bytes[id] += bytes;
    p.n[id]++;
  }
  if (e != hipSuccess) { r.err = e; g_last_hip = (int)e; }
}

template <typename Ctx>
int finish(RunT<Ctx>& r) { return r.ok() ? SLIDE_OK : SLIDE_EHIP; }

inline int prof_begin(Prof& p, int kernel_id, int families) {
  if (kernel_id < SLIDE_PROF_ALL || kernel_id >= families) return SLIDE_EINVAL;
  p.active = true; p.id = kernel_id; p.count = 0;
  for (int k = 0; k < PROF_FAMILIES; ++k) { p.flops[k] = p.bytes[k] = p.ms[k] = 0; p.n[k] = 0; }
  return SLIDE_OK;
}

inline int prof_end(Prof& p, double* total_ms, int* launches, double* flops, double* bytes) {
  int rc = SLIDE_OK;
  for (int i = 0; i < p.count; ++i) {
    float ms = 0.f;
    hipError_t e = hipEventSynchronize(p.ev[2 * i + 1]);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, p.ev[2 * i], p.ev[2 * i + 1]);
    if (e != hipSuccess) { g_last_hip = (int)e; rc = SLIDE_EHIP; break; }
    p.ms[p.fam[i]] += ms;
  }
  double tot = 0, fl = 0, by = 0;
  for (int k = 0; k < PROF_FAMILIES; ++k) { tot += p.ms[k]; fl += p.flops[k]; by += p.bytes[k]; }
  if (total_ms) *total_ms = tot;
  if (launches) *launches = p.count;
  if (flops) *flops = fl;
  if (bytes) *bytes = by;
  p.active = false;
  return rc;
}

inline int prof_family(const Prof& p, int kernel_id, int families, double* total_ms, int* launches, double* flops,
                       double* bytes) {
  if (kernel_id < 0 || kernel_id >= families) return SLIDE_EINVAL;
  if (total_ms) *total_ms = p.ms[kernel_id];
  if (launches) *launches = p.n[kernel_id];
  if (flops) *flops = p.flops[kernel_id];
  if (bytes) *bytes = p.bytes[kernel_id];
  return SLIDE_OK;
}

// aggregator-only context (slide_lib.hip); destroyed with slide_ctx_destroy
int pool_ctx_create(int D, int Mh, int C, int dt, slide_ctx** out);

inline void prof_destroy(Prof& p) {
  for (hipEvent_t e : p.ev) (void)hipEventDestroy(e);
  p.ev.clear();
}

}  // namespace sl
