// The update that closes an iteration: one norm over all gradients, clipping, and an AdamW step.
//
// The paper fixes the learning rate (3e-4) and the clipping of gradient norms to 1.0 for its convergence
// runs (appendix "Test Configurations") and does not name the optimiser; AdamW is this library's reading.
//
//   pass 1  sum of squares of the gradients: kPartials workgroups, each a fixed strided share, double
//           accumulation, one partial per workgroup (a fixed order, so the norm is reproducible)
//   pass 2  one workgroup adds the partials in index order: norm, and the factor min(1, clip/(norm+1e-6))
//   pass 3  m, v, master parameter and its low-precision copy in one sweep: 4 floats per lane per access.
// HBM traffic per parameter: 4 (norm) + 16 read + 12 written + 2 (bf16 copy) = 34 bytes.
#include <mutex>

#include "devutil.h"
#include "internal.h"

namespace sp {

namespace {

constexpr int kBlock = 256;
constexpr int kPartials = 2048;

struct Scalars {   // lives at the start of the caller's workspace, after the partials
  float norm, coef;
};

__global__ __launch_bounds__(kBlock) void k_sumsq(const float* __restrict__ g, int64_t n, double* __restrict__ partial) {
  const int64_t n4 = n / 4;
  double acc = 0.0;
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n4; i += (int64_t)gridDim.x * kBlock) {
    const float4 x = reinterpret_cast<const float4*>(g)[i];
    acc += (double)x.x * x.x + (double)x.y * x.y + (double)x.z * x.z + (double)x.w * x.w;
  }
  if (blockIdx.x == 0)
    for (int64_t i = n4 * 4 + threadIdx.x; i < n; i += kBlock) acc += (double)g[i] * g[i];
  __shared__ double red[kBlock];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int o = kBlock / 2; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

__global__ __launch_bounds__(kBlock) void k_norm(const double* __restrict__ partial, int n_partial, float clip,
                                                 Scalars* __restrict__ out, float* __restrict__ norm_out) {
  __shared__ double red[kBlock];
  double acc = 0.0;
  for (int i = threadIdx.x; i < n_partial; i += kBlock) acc += partial[i];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int o = kBlock / 2; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double norm = sqrt(red[0]);
    out->norm = (float)norm;
    out->coef = clip > 0.f ? (float)fmin(1.0, (double)clip / (norm + 1e-6)) : 1.f;
    if (norm_out) *norm_out = (float)norm;
  }
}

struct Hyper {
  float lr, beta1, beta2, eps, decay_mul, inv_bc1, inv_bc2;
};

__device__ __forceinline__ float update_one(float p, float g, float& m, float& v, const Hyper& h) {
  m = h.beta1 * m + (1.f - h.beta1) * g;
  v = h.beta2 * v + (1.f - h.beta2) * g * g;
  return p * h.decay_mul - h.lr * (m * h.inv_bc1) / (sqrtf(v * h.inv_bc2) + h.eps);
}

__device__ __forceinline__ void store4(float* q, const float4& x) { *reinterpret_cast<float4*>(q) = x; }
__device__ __forceinline__ void store4(bf16* q, const float4& x) {
  *reinterpret_cast<uint2*>(q) = make_uint2(pack_bf16(x.x, x.y), pack_bf16(x.z, x.w));
}

__device__ __forceinline__ float4 load4_stream(const float* q) {
  typedef __attribute__((ext_vector_type(4))) float f4;
  const f4 v = __builtin_nontemporal_load(reinterpret_cast<const f4*>(q));
  return make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void store4_stream(float* q, const float4& x) {
  typedef __attribute__((ext_vector_type(4))) float f4;
  const f4 v = {x.x, x.y, x.z, x.w};
  __builtin_nontemporal_store(v, reinterpret_cast<f4*>(q));
}

// Every element is read once and written once: all accesses carry the streaming hint, and a thread keeps two
// quads (8 loads) in flight.
template <class LP>   // LP: float (a plain copy) or bf16
__global__ __launch_bounds__(kBlock) void k_adamw(float* __restrict__ p, const float* __restrict__ g, float* __restrict__ m,
                                                  float* __restrict__ v, LP* __restrict__ lp, int64_t n, Hyper h,
                                                  const Scalars* __restrict__ sc) {
  const float coef = sc->coef;
  const int64_t n4 = n / 4, stride = (int64_t)gridDim.x * kBlock;
  auto one = [&](int64_t i, float4 pp, float4 gg, float4 mm, float4 vv) {
    pp.x = update_one(pp.x, gg.x * coef, mm.x, vv.x, h);
    pp.y = update_one(pp.y, gg.y * coef, mm.y, vv.y, h);
    pp.z = update_one(pp.z, gg.z * coef, mm.z, vv.z, h);
    pp.w = update_one(pp.w, gg.w * coef, mm.w, vv.w, h);
    store4_stream(p + 4 * i, pp);
    store4_stream(m + 4 * i, mm);
    store4_stream(v + 4 * i, vv);
    if (lp) store4(lp + 4 * i, pp);   // one 8-byte (bf16) or 16-byte (float) store
  };
  int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  for (; i + stride < n4; i += 2 * stride) {
    const int64_t j = i + stride;
    const float4 p0 = load4_stream(p + 4 * i), g0 = load4_stream(g + 4 * i), m0 = load4_stream(m + 4 * i), v0 = load4_stream(v + 4 * i);
    const float4 p1 = load4_stream(p + 4 * j), g1 = load4_stream(g + 4 * j), m1 = load4_stream(m + 4 * j), v1 = load4_stream(v + 4 * j);
    one(i, p0, g0, m0, v0);
    one(j, p1, g1, m1, v1);
  }
  if (i < n4) one(i, load4_stream(p + 4 * i), load4_stream(g + 4 * i), load4_stream(m + 4 * i), load4_stream(v + 4 * i));
  if (blockIdx.x == 0)
    for (int64_t t = n4 * 4 + threadIdx.x; t < n; t += kBlock) {
      float mm = m[t], vv = v[t];
      const float pn = update_one(p[t], g[t] * coef, mm, vv, h);
      p[t] = pn; m[t] = mm; v[t] = vv;
      if (lp) lp[t] = from_float<LP>(pn);
    }
}

// out = scale * (g_0 + g_1 + ... + g_{n_rep-1}), added in index order
constexpr int kMaxReplicas = 64;
struct ReplicaPtrs { const float* g[kMaxReplicas]; };
__global__ __launch_bounds__(kBlock) void k_grad_sum(ReplicaPtrs rp, int n_rep, int64_t n, float scale, float* __restrict__ out) {
  const int64_t n4 = n / 4;
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n4; i += (int64_t)gridDim.x * kBlock) {
    float4 acc = reinterpret_cast<const float4*>(rp.g[0])[i];
    for (int r = 1; r < n_rep; ++r) {
      const float4 x = reinterpret_cast<const float4*>(rp.g[r])[i];
      acc.x += x.x; acc.y += x.y; acc.z += x.z; acc.w += x.w;
    }
    acc.x *= scale; acc.y *= scale; acc.z *= scale; acc.w *= scale;
    reinterpret_cast<float4*>(out)[i] = acc;
  }
  if (blockIdx.x == 0)
    for (int64_t i = n4 * 4 + threadIdx.x; i < n; i += kBlock) {
      float acc = rp.g[0][i];
      for (int r = 1; r < n_rep; ++r) acc += rp.g[r][i];
      out[i] = acc * scale;
    }
}

}  // namespace
}  // namespace sp

using namespace sp;

extern "C" int sp_grad_reduce(void* hip_stream, const float* const* replica_grads, int n_replicas, int64_t n, float scale,
                              float* out) {
  if (!replica_grads || !out || n_replicas < 1 || n_replicas > kMaxReplicas || n < 0)
    return fail(SP_EINVAL, "grad_reduce: null argument, or a replica count outside [1, 64]");
  ReplicaPtrs rp{};
  uintptr_t al = (uintptr_t)out;
  for (int r = 0; r < n_replicas; ++r) {
    if (!replica_grads[r]) return fail(SP_EINVAL, "grad_reduce: null replica buffer");
    rp.g[r] = replica_grads[r];
    al |= (uintptr_t)replica_grads[r];
  }
  if (al & 15) return fail(SP_EINVAL, "grad_reduce: buffers must be 16-byte aligned");
  if (n == 0) return SP_OK;
  const int grid = (int)std::max<int64_t>(1, std::min<int64_t>(8192, (n / 4 + kBlock - 1) / kBlock));
  hipLaunchKernelGGL(k_grad_sum, dim3(grid), dim3(kBlock), 0, (hipStream_t)hip_stream, rp, n_replicas, n, scale, out);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail((int)e, "grad_reduce");
  return SP_OK;
}

extern "C" int64_t sp_optim_workspace_bytes(void) { return (int64_t)kPartials * sizeof(double) + 256; }

static int optim_step_impl(void* hip_stream, const sp_adamw* hy, int64_t n, int step, float* master, const float* grads,
                           float* m, float* v, void* params_out, int out_dtype, void* workspace, float* grad_norm) {
  if (!hy || n < 0 || step < 1) return fail(SP_EINVAL, "optim_step: null hyper-parameters, negative size or step < 1");
  if (n == 0) return SP_OK;
  if (!master || !grads || !m || !v || !workspace) return fail(SP_EINVAL, "optim_step: null operand");
  if (params_out && out_dtype != SP_F32 && out_dtype != SP_BF16) return fail(SP_EINVAL, "optim_step: bad out_dtype");
  if (!(hy->lr >= 0.f) || !(hy->beta1 >= 0.f && hy->beta1 < 1.f) || !(hy->beta2 >= 0.f && hy->beta2 < 1.f) ||
      !(hy->eps >= 0.f) || !(hy->weight_decay >= 0.f) || !(hy->clip_norm >= 0.f))
    return fail(SP_EINVAL, "optim_step: hyper-parameter out of range");
  const uintptr_t al = (uintptr_t)master | (uintptr_t)grads | (uintptr_t)m | (uintptr_t)v | (uintptr_t)workspace;
  if (al & 15) return fail(SP_EINVAL, "optim_step: master, grads, m, v and workspace must be 16-byte aligned");
  if (params_out && ((uintptr_t)params_out & 15)) return fail(SP_EINVAL, "optim_step: params_out must be 16-byte aligned");
  hipStream_t s = (hipStream_t)hip_stream;
  double* partial = (double*)workspace;
  Scalars* sc = (Scalars*)((char*)workspace + (size_t)kPartials * sizeof(double));
  const int64_t n4 = n / 4;
  const int grid = (int)std::max<int64_t>(1, std::min<int64_t>(kPartials, (n4 + kBlock - 1) / kBlock));
  hipLaunchKernelGGL(k_sumsq, dim3(grid), dim3(kBlock), 0, s, grads, n, partial);
  hipLaunchKernelGGL(k_norm, dim3(1), dim3(kBlock), 0, s, partial, grid, hy->clip_norm, sc, grad_norm);
  Hyper h;
  h.lr = hy->lr; h.beta1 = hy->beta1; h.beta2 = hy->beta2; h.eps = hy->eps;
  h.decay_mul = 1.f - hy->lr * hy->weight_decay;
  h.inv_bc1 = (float)(1.0 / (1.0 - pow((double)hy->beta1, (double)step)));
  h.inv_bc2 = (float)(1.0 / (1.0 - pow((double)hy->beta2, (double)step)));
  const int ugrid = (int)std::max<int64_t>(1, std::min<int64_t>(16384, (n4 + kBlock - 1) / kBlock));
  if (params_out && out_dtype == SP_BF16)
    hipLaunchKernelGGL(k_adamw<bf16>, dim3(ugrid), dim3(kBlock), 0, s, master, grads, m, v, (bf16*)params_out, n, h, sc);
  else
    hipLaunchKernelGGL(k_adamw<float>, dim3(ugrid), dim3(kBlock), 0, s, master, grads, m, v, (float*)params_out, n, h, sc);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail((int)e, "optim_step");
  return SP_OK;
}

extern "C" int sp_optim_step(void* hip_stream, const sp_adamw* hy, int64_t n, int step, float* master, const float* grads,
                             float* m, float* v, void* params_out, int out_dtype, void* workspace, float* grad_norm) {
  return optim_step_impl(hip_stream, hy, n, step, master, grads, m, v, params_out, out_dtype, workspace, grad_norm);
}

// ---- the same update for callers that must not allocate: the norm partials and the two scalars live in a
// file-scope device array instead of a caller-provided workspace.  Each GPU the library runs on holds its own
// copy of the array (at its own address) from the moment the code object is loaded until the process ends.
namespace {
constexpr size_t kScratchBytes = (size_t)kPartials * sizeof(double) + 256;   // 16 640 bytes
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
void* g_scratch_addr[kMaxDevices];   // device address of `scratch` per device, looked up once
std::mutex g_scratch_mutex;
constexpr int64_t kNoAllocMaxN = (int64_t)1 << 32;
}  // namespace

extern "C" int sp_optim_step_noalloc(void* hip_stream, const sp_adamw* hy, int64_t n, int step, float* master,
                                     const float* grads, float* m, float* v, void* params_out, int out_dtype,
                                     float* grad_norm) {
  if (n > kNoAllocMaxN)
    return fail(SP_EINVAL, "optim_step_noalloc: n = " + std::to_string(n) + " exceeds the maximum of 2^32 elements per call");
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail((int)e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(SP_EINVAL, "optim_step_noalloc: device index outside [0, 64)");
  void* ptr = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_addr[dev]) {
      // in host code the array's name is only a handle: this is the address the kernels may use, on this device
      void* p = nullptr;
      e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !p) return hip_fail((int)e, "hipGetSymbolAddress(scratch)");
      g_scratch_addr[dev] = p;
    }
    ptr = g_scratch_addr[dev];
  }
  return optim_step_impl(hip_stream, hy, n, step, master, grads, m, v, params_out, out_dtype, ptr, grad_norm);
}
