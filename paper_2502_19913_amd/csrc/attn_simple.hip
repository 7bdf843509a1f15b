// Causal attention for any head dimension and element type, one wavefront per output row.
// Slow and plain: it carries the float mode and head sizes the MFMA kernels do not take.
//
// Layout: qkv rows of (H + 2*Hkv)*hd elements = query heads | key heads | value heads; rows are
// B sequences of T positions; o rows of H*hd; lse[b][a][i] = log sum_j exp(q_i.k_j/sqrt(hd)).
#include "devutil.h"
#include "internal.h"

namespace sp {

namespace {

constexpr int kMaxHd = 256;

// delta[b][a][i] = sum_c dO[i][a][c] * O[i][a][c]
template <class T>
__global__ __launch_bounds__(64) void k_attn_delta(const T* __restrict__ o, const T* __restrict__ dO, int T_, int H,
                                                   int hd, float* __restrict__ delta) {
  const int i = blockIdx.x, a = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
  const int64_t row = (int64_t)b * T_ + i;
  float s = 0.f;
  for (int c = lane; c < hd; c += 64)
    s += to_float(o[row * H * hd + a * hd + c]) * to_float(dO[row * H * hd + a * hd + c]);
  s = wave_sum(s);
  if (lane == 0) delta[((int64_t)b * H + a) * T_ + i] = s;
}

template <class T>
__global__ __launch_bounds__(64) void k_attn_fwd(const T* __restrict__ qkv, int T_, int H, int Hkv, int hd,
                                                 T* __restrict__ o, float* __restrict__ lse) {
  __shared__ float s_q[kMaxHd];
  __shared__ float s_p[64];
  const int i = blockIdx.x, a = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
  const int nq = (H + 2 * Hkv) * hd, kvh = a / (H / Hkv);
  const float scale = 1.0f / sqrtf((float)hd);
  const T* base = qkv + (int64_t)b * T_ * nq;
  const T* kp = base + H * hd + kvh * hd;
  const T* vp = base + (H + Hkv) * hd + kvh * hd;
  for (int c = lane; c < hd; c += 64) s_q[c] = to_float(base[(int64_t)i * nq + a * hd + c]);
  __syncthreads();
  float m = -INFINITY, l = 0.f;
  float acc[kMaxHd / 64] = {};
  for (int j0 = 0; j0 <= i; j0 += 64) {
    const int j = j0 + lane;
    float s = -INFINITY;
    if (j <= i) {
      float d = 0.f;
      for (int c = 0; c < hd; ++c) d += s_q[c] * to_float(kp[(int64_t)j * nq + c]);
      s = d * scale;
    }
    const float mn = fmaxf(m, wave_max(s));
    const float p = j <= i ? expf(s - mn) : 0.f;
    const float corr = expf(m - mn);  // first block: exp(-inf) = 0
    l = l * corr + wave_sum(p);
    m = mn;
    __syncthreads();
    s_p[lane] = p;
    __syncthreads();
    const int cnt = min(64, i - j0 + 1);
#pragma unroll
    for (int u = 0; u < kMaxHd / 64; ++u) {
      const int c = lane + 64 * u;
      if (c < hd) {
        float t = acc[u] * corr;
        for (int jj = 0; jj < cnt; ++jj) t += s_p[jj] * to_float(vp[(int64_t)(j0 + jj) * nq + c]);
        acc[u] = t;
      }
    }
  }
  const int64_t row = (int64_t)b * T_ + i;
#pragma unroll
  for (int u = 0; u < kMaxHd / 64; ++u) {
    const int c = lane + 64 * u;
    if (c < hd) o[row * H * hd + a * hd + c] = from_float<T>(acc[u] / l);
  }
  if (lane == 0) lse[((int64_t)b * H + a) * T_ + i] = m + logf(l);
}

// dq_i = sum_{j<=i} ds_ij k_j,  ds_ij = p_ij (dO_i.v_j - delta_i) / sqrt(hd),  p_ij = exp(s_ij - lse_i)
template <class T>
__global__ __launch_bounds__(64) void k_attn_bwd_dq(const T* __restrict__ qkv, const float* __restrict__ lse,
                                                    const float* __restrict__ delta, const T* __restrict__ dO, int T_,
                                                    int H, int Hkv, int hd, T* __restrict__ dqkv) {
  __shared__ float s_q[kMaxHd], s_do[kMaxHd];
  __shared__ float s_ds[64];
  const int i = blockIdx.x, a = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
  const int nq = (H + 2 * Hkv) * hd, kvh = a / (H / Hkv);
  const float scale = 1.0f / sqrtf((float)hd);
  const T* base = qkv + (int64_t)b * T_ * nq;
  const T* kp = base + H * hd + kvh * hd;
  const T* vp = base + (H + Hkv) * hd + kvh * hd;
  const int64_t row = (int64_t)b * T_ + i;
  for (int c = lane; c < hd; c += 64) {
    s_q[c] = to_float(base[(int64_t)i * nq + a * hd + c]);
    s_do[c] = to_float(dO[row * H * hd + a * hd + c]);
  }
  __syncthreads();
  const float L = lse[((int64_t)b * H + a) * T_ + i], D = delta[((int64_t)b * H + a) * T_ + i];
  float acc[kMaxHd / 64] = {};
  for (int j0 = 0; j0 <= i; j0 += 64) {
    const int j = j0 + lane;
    float ds = 0.f;
    if (j <= i) {
      float s = 0.f, dp = 0.f;
      for (int c = 0; c < hd; ++c) {
        s += s_q[c] * to_float(kp[(int64_t)j * nq + c]);
        dp += s_do[c] * to_float(vp[(int64_t)j * nq + c]);
      }
      ds = expf(s * scale - L) * (dp - D) * scale;
    }
    __syncthreads();
    s_ds[lane] = ds;
    __syncthreads();
    const int cnt = min(64, i - j0 + 1);
#pragma unroll
    for (int u = 0; u < kMaxHd / 64; ++u) {
      const int c = lane + 64 * u;
      if (c < hd) {
        float t = acc[u];
        for (int jj = 0; jj < cnt; ++jj) t += s_ds[jj] * to_float(kp[(int64_t)(j0 + jj) * nq + c]);
        acc[u] = t;
      }
    }
  }
#pragma unroll
  for (int u = 0; u < kMaxHd / 64; ++u) {
    const int c = lane + 64 * u;
    if (c < hd) dqkv[row * nq + a * hd + c] = from_float<T>(acc[u]);
  }
}

// dk_j = sum_a sum_{i>=j} ds_ij q_i ; dv_j = sum_a sum_{i>=j} p_ij dO_i   (a over the q heads of this kv head)
template <class T>
__global__ __launch_bounds__(64) void k_attn_bwd_dkv(const T* __restrict__ qkv, const float* __restrict__ lse,
                                                     const float* __restrict__ delta, const T* __restrict__ dO, int T_,
                                                     int H, int Hkv, int hd, T* __restrict__ dqkv) {
  __shared__ float s_k[kMaxHd], s_v[kMaxHd];
  __shared__ float s_p[64], s_ds[64];
  const int j = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
  const int nq = (H + 2 * Hkv) * hd, rep = H / Hkv;
  const float scale = 1.0f / sqrtf((float)hd);
  const T* base = qkv + (int64_t)b * T_ * nq;
  for (int c = lane; c < hd; c += 64) {
    s_k[c] = to_float(base[(int64_t)j * nq + H * hd + kvh * hd + c]);
    s_v[c] = to_float(base[(int64_t)j * nq + (H + Hkv) * hd + kvh * hd + c]);
  }
  __syncthreads();
  float dk[kMaxHd / 64] = {}, dv[kMaxHd / 64] = {};
  for (int a = kvh * rep; a < (kvh + 1) * rep; ++a) {
    const T* qp = base + a * hd;
    const T* dop = dO + (int64_t)b * T_ * H * hd + a * hd;
    for (int i0 = j; i0 < T_; i0 += 64) {
      const int i = i0 + lane;
      float p = 0.f, ds = 0.f;
      if (i < T_) {
        float s = 0.f, dp = 0.f;
        for (int c = 0; c < hd; ++c) {
          s += to_float(qp[(int64_t)i * nq + c]) * s_k[c];
          dp += to_float(dop[(int64_t)i * H * hd + c]) * s_v[c];
        }
        p = expf(s * scale - lse[((int64_t)b * H + a) * T_ + i]);
        ds = p * (dp - delta[((int64_t)b * H + a) * T_ + i]) * scale;
      }
      __syncthreads();
      s_p[lane] = p; s_ds[lane] = ds;
      __syncthreads();
      const int cnt = min(64, T_ - i0);
#pragma unroll
      for (int u = 0; u < kMaxHd / 64; ++u) {
        const int c = lane + 64 * u;
        if (c < hd) {
          float tk = dk[u], tv = dv[u];
          for (int ii = 0; ii < cnt; ++ii) {
            tk += s_ds[ii] * to_float(qp[(int64_t)(i0 + ii) * nq + c]);
            tv += s_p[ii] * to_float(dop[(int64_t)(i0 + ii) * H * hd + c]);
          }
          dk[u] = tk; dv[u] = tv;
        }
      }
    }
  }
  const int64_t row = (int64_t)b * T_ + j;
#pragma unroll
  for (int u = 0; u < kMaxHd / 64; ++u) {
    const int c = lane + 64 * u;
    if (c < hd) {
      dqkv[row * nq + H * hd + kvh * hd + c] = from_float<T>(dk[u]);
      dqkv[row * nq + (H + Hkv) * hd + kvh * hd + c] = from_float<T>(dv[u]);
    }
  }
}

template <class T>
void fwd_t(hipStream_t s, int B, int T_, int H, int Hkv, int hd, const void* qkv, void* o, float* lse) {
  hipLaunchKernelGGL(k_attn_fwd<T>, dim3(T_, H, B), dim3(64), 0, s, (const T*)qkv, T_, H, Hkv, hd, (T*)o, lse);
}

template <class T>
void bwd_t(hipStream_t s, int B, int T_, int H, int Hkv, int hd, const void* qkv, const void* o, const float* lse,
           const void* dO, void* dqkv, float* delta) {
  hipLaunchKernelGGL(k_attn_delta<T>, dim3(T_, H, B), dim3(64), 0, s, (const T*)o, (const T*)dO, T_, H, hd, delta);
  hipLaunchKernelGGL(k_attn_bwd_dq<T>, dim3(T_, H, B), dim3(64), 0, s, (const T*)qkv, lse, delta, (const T*)dO, T_, H,
                     Hkv, hd, (T*)dqkv);
  hipLaunchKernelGGL(k_attn_bwd_dkv<T>, dim3(T_, Hkv, B), dim3(64), 0, s, (const T*)qkv, lse, delta, (const T*)dO, T_,
                     H, Hkv, hd, (T*)dqkv);
}

}  // namespace

void attention_simple_fwd(hipStream_t s, int dtype, int B, int T, int H, int Hkv, int hd, const void* qkv, void* o,
                          float* lse) {
  if (dtype == SP_BF16) fwd_t<bf16>(s, B, T, H, Hkv, hd, qkv, o, lse);
  else fwd_t<float>(s, B, T, H, Hkv, hd, qkv, o, lse);
}

void attention_simple_bwd(hipStream_t s, int dtype, int B, int T, int H, int Hkv, int hd, const void* qkv,
                          const void* o, const float* lse, const void* do_, void* dqkv, float* delta) {
  if (dtype == SP_BF16) bwd_t<bf16>(s, B, T, H, Hkv, hd, qkv, o, lse, do_, dqkv, delta);
  else bwd_t<float>(s, B, T, H, Hkv, hd, qkv, o, lse, do_, dqkv, delta);
}

static int check_attn(int B, int T, int H, int Hkv, int hd) {
  if (B <= 0 || T <= 0 || H <= 0 || Hkv <= 0 || hd <= 0 || H % Hkv) return fail(SP_EINVAL, "attention: bad shape");
  if (hd > kMaxHd) return fail(SP_EINVAL, "attention: head dimension above 256");
  if (B > 65535 || H > 65535) return fail(SP_EINVAL, "attention: batch or head count above 65535");
  return SP_OK;
}

int attention_fwd(hipStream_t s, int dtype, int B, int T, int H, int Hkv, int hd, const void* qkv, void* o, float* lse) {
  int rc = check_attn(B, T, H, Hkv, hd);
  if (rc) return rc;
  if (!qkv || !o || !lse) return fail(SP_EINVAL, "attention: null operand");
  const bool fast = dtype == SP_BF16 && attention_flash_supported(B, T, H, Hkv, hd);
  const int pi = prof_start(fast ? PROF_ATTN_FWD : PROF_ATTN_PLAIN, s);
  if (fast) attention_flash_fwd(s, B, T, H, Hkv, hd, qkv, o, lse);
  else attention_simple_fwd(s, dtype, B, T, H, Hkv, hd, qkv, o, lse);
  prof_stop(pi, s, 2.0 * (double)B * H * (double)T * (T + 1) * hd);   // QK^T and PV over the causal half
  return SP_OK;
}

int attention_bwd(hipStream_t s, int dtype, int B, int T, int H, int Hkv, int hd, const void* qkv, const void* o,
                  const float* lse, const void* do_, void* dqkv, float* delta, const float* rope_tab, float rope_theta) {
  int rc = check_attn(B, T, H, Hkv, hd);
  if (rc) return rc;
  if (!qkv || !o || !lse || !do_ || !dqkv || !delta) return fail(SP_EINVAL, "attention: null operand");
  if (dtype == SP_BF16 && attention_flash_supported(B, T, H, Hkv, hd)) {
    attention_flash_bwd(s, B, T, H, Hkv, hd, qkv, o, lse, do_, dqkv, delta, rope_tab);   // rotates dq, dk on the way out
  } else {
    const int pi = prof_start(PROF_ATTN_PLAIN, s);
    attention_simple_bwd(s, dtype, B, T, H, Hkv, hd, qkv, o, lse, do_, dqkv, delta);
    prof_stop(pi, s, 4.0 * (double)B * H * (double)T * (T + 1) * hd);
    if (rope_tab) rope(s, dtype, dqkv, (int64_t)B * T, T, H + Hkv, hd, (H + 2 * Hkv) * hd, rope_theta, -1);
  }
  return SP_OK;
}

}  // namespace sp
