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

// Matrix cores alone: every wave keeps the 24 operand fragments of one 256 x 256 x 64 k-step of the product
// kernel in registers and repeats that step's 64 v_mfma_f32_16x16x32_bf16 `iters` times: no LDS, no global
// loads inside the loop.  The rate it sustains is what the chip's clock and power management leave of the
// published peak for a given operand content (zeros toggle nothing; random values draw full power).
typedef __attribute__((ext_vector_type(8))) __bf16 probe_bf16x8;
typedef __attribute__((ext_vector_type(4))) float probe_f32x4;

__global__ __launch_bounds__(512, 1) void k_mfma_probe(const uint4* __restrict__ src, int64_t n_quads, int iters,
                                                      float* __restrict__ sink) {
  const int lane_id = threadIdx.x + blockIdx.x * 512;
  probe_bf16x8 fa[2][8], fb[2][4];
#pragma unroll
  for (int k = 0; k < 2; ++k) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      uint4 q = src[((int64_t)lane_id * 24 + k * 12 + j) % n_quads];
      fa[k][j] = *reinterpret_cast<probe_bf16x8*>(&q);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      uint4 q = src[((int64_t)lane_id * 24 + k * 12 + 8 + i) % n_quads];
      fb[k][i] = *reinterpret_cast<probe_bf16x8*>(&q);
    }
  }
  probe_f32x4 acc[8][4];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[j][i] = probe_f32x4{0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int k = 0; k < 2; ++k)
#pragma unroll
      for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[j][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[k][j], fb[k][i], acc[j][i], 0, 0, 0);
  }
  probe_f32x4 t = probe_f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int i = 0; i < 4; ++i) t += acc[j][i];
  sink[lane_id] = t[0] + t[1] + t[2] + t[3];
}

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

int sp_probe_mfma_rate(void* hip_stream, const void* src, int64_t src_bytes, int n_blocks, int iters, float* sink,
                       double* flops) {
  if (!src || !sink || !flops || src_bytes < 16 || n_blocks < 1 || n_blocks > 65536 || iters < 1)
    return fail(SP_EINVAL, "probe_mfma_rate: bad argument");
  if (reinterpret_cast<uintptr_t>(src) % 16) return fail(SP_EINVAL, "probe_mfma_rate: src not 16-byte aligned");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  k_mfma_probe<<<dim3(n_blocks), dim3(512), 0, s>>>(static_cast<const uint4*>(src), src_bytes / 16, iters, sink);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail((int)e, "probe_mfma_rate launch");
  *flops = (double)n_blocks * 8 * (double)iters * 64 * (2.0 * 16 * 16 * 32);
  return SP_OK;
}

}  // extern "C"
