// Optional per-launch timing of the matrix-product and attention kernels with HIP events recorded
// on the launch stream.  Off by default; when off the hooks cost one branch.
#include <hip/hip_runtime.h>

#include <mutex>
#include <vector>

#include "internal.h"

namespace sp {

namespace {
struct Rec { int cls; hipEvent_t a, b; double flops; };
bool g_on = false;
std::vector<Rec> g_recs;
std::vector<hipEvent_t> g_pool;
std::mutex g_mu;

hipEvent_t take_event() {
  if (!g_pool.empty()) {
    hipEvent_t e = g_pool.back();
    g_pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}
}  // namespace

int prof_start(int cls, hipStream_t s) {
  if (!g_on) return -1;
  std::lock_guard<std::mutex> lk(g_mu);
  Rec r{cls, take_event(), take_event(), 0.0};
  if (!r.a || !r.b) return -1;
  (void)hipEventRecord(r.a, s);
  g_recs.push_back(r);
  return (int)g_recs.size() - 1;
}

void prof_stop(int idx, hipStream_t s, double flops) {
  if (idx < 0) return;
  std::lock_guard<std::mutex> lk(g_mu);
  if (idx >= (int)g_recs.size()) return;
  g_recs[idx].flops = flops;
  (void)hipEventRecord(g_recs[idx].b, s);
}

}  // namespace sp

using namespace sp;

extern "C" {

int sp_prof_begin(void) {
  std::lock_guard<std::mutex> lk(g_mu);
  for (auto& r : g_recs) { g_pool.push_back(r.a); g_pool.push_back(r.b); }
  g_recs.clear();
  g_on = true;
  return SP_OK;
}

int sp_prof_end(int n_classes, double* ms, double* flops, int64_t* launches) {
  std::lock_guard<std::mutex> lk(g_mu);
  g_on = false;
  if (n_classes < 1 || !ms || !flops || !launches) return fail(SP_EINVAL, "prof_end: bad argument");
  for (int c = 0; c < n_classes; ++c) { ms[c] = 0; flops[c] = 0; launches[c] = 0; }
  int rc = SP_OK;
  for (auto& r : g_recs) {
    hipError_t e = hipEventSynchronize(r.b);
    float t = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&t, r.a, r.b);
    if (e != hipSuccess) rc = hip_fail((int)e, "profiling event");
    else if (r.cls >= 0 && r.cls < n_classes) { ms[r.cls] += t; flops[r.cls] += r.flops; launches[r.cls] += 1; }
    g_pool.push_back(r.a);
    g_pool.push_back(r.b);
  }
  g_recs.clear();
  return rc;
}

}  // extern "C"
