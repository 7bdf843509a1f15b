// Plain LDS-tiled matrix product with float accumulation for any shape, stride and element type.
// It carries the float mode and every shape the MFMA kernels do not take; it is not the fast path.
#include "devutil.h"
#include "internal.h"

namespace sp {

namespace {

constexpr int TM = 64, TN = 64, TK = 16;

// C(m,n) = sum_k A(m,k) * B(k,n), A(m,k) = A[m*sam + k*sak], B(k,n) = B[k*sbk + n*sbn].
// ACC: C is float and is added to.  Otherwise C is T and R (same shape, may be null) is added.
template <class T, bool ACC>
__global__ __launch_bounds__(256) void k_gemm_simple(const T* __restrict__ A, const T* __restrict__ B, void* Cv,
                                                     const T* __restrict__ Rr, int64_t M, int64_t N, int64_t K,
                                                     int64_t sam, int64_t sak, int64_t sbk, int64_t sbn) {
  __shared__ float As[TK][TM + 1];
  __shared__ float Bs[TK][TN + 1];
  const int tid = threadIdx.x;
  const int64_t m0 = (int64_t)blockIdx.y * TM, n0 = (int64_t)blockIdx.x * TN;
  const int tx = tid % 16, ty = tid / 16;  // 4x4 outputs per thread: rows ty*4.., cols tx*4..
  float acc[4][4] = {};
  for (int64_t k0 = 0; k0 < K; k0 += TK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int e = tid + i * 256;
      // fastest-varying index follows the contiguous dimension of each operand
      int ka, ma, kb, nb;
      if (sak == 1) { ka = e % TK; ma = e / TK; } else { ma = e % TM; ka = e / TM; }
      if (sbk == 1) { kb = e % TK; nb = e / TK; } else { nb = e % TN; kb = e / TN; }
      int64_t gm = m0 + ma, gk = k0 + ka;
      As[ka][ma] = (gm < M && gk < K) ? to_float(A[gm * sam + gk * sak]) : 0.f;
      int64_t gn = n0 + nb, gk2 = k0 + kb;
      Bs[kb][nb] = (gn < N && gk2 < K) ? to_float(B[gk2 * sbk + gn * sbn]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < TK; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[k][ty * 4 + i]; b[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int64_t m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m < M && n < N) {
        if (ACC) {
          float* C = (float*)Cv;
          C[m * N + n] += acc[i][j];
        } else {
          T* C = (T*)Cv;
          float v = acc[i][j];
          if (Rr) v += to_float(Rr[m * N + n]);
          C[m * N + n] = from_float<T>(v);
        }
      }
    }
}

template <class T>
void launch(hipStream_t s, int op, int64_t M, int64_t N, int64_t K, const void* A, const void* B, void* C,
            const void* R) {
  dim3 grid((unsigned)((N + TN - 1) / TN), (unsigned)((M + TM - 1) / TM));
  if (op == 0)
    hipLaunchKernelGGL((k_gemm_simple<T, false>), grid, dim3(256), 0, s, (const T*)A, (const T*)B, C, (const T*)R, M,
                       N, K, K, (int64_t)1, (int64_t)1, K);
  else if (op == 1)
    hipLaunchKernelGGL((k_gemm_simple<T, false>), grid, dim3(256), 0, s, (const T*)A, (const T*)B, C, (const T*)nullptr,
                       M, N, K, K, (int64_t)1, N, (int64_t)1);
  else
    hipLaunchKernelGGL((k_gemm_simple<T, true>), grid, dim3(256), 0, s, (const T*)A, (const T*)B, C, (const T*)nullptr,
                       M, N, K, (int64_t)1, M, N, (int64_t)1);
}

}  // namespace

void gemm_simple(hipStream_t s, int dtype, int op, int64_t M, int64_t N, int64_t K, const void* A, const void* B,
                 void* C, const void* R) {
  if (M <= 0 || N <= 0) return;
  if (dtype == SP_BF16) launch<bf16>(s, op, M, N, K, A, B, C, R);
  else launch<float>(s, op, M, N, K, A, B, C, R);
}

int gemm(hipStream_t s, int dtype, int op, int64_t M, int64_t N, int64_t K, const void* A, const void* B, void* C,
         const void* R) {
  if (op < 0 || op > 2 || M < 0 || N < 0 || K < 0) return fail(SP_EINVAL, "gemm: bad op or shape");
  if ((M > 0 && N > 0) && (!C || (K > 0 && (!A || !B)))) return fail(SP_EINVAL, "gemm: null operand");
  if (M == 0 || N == 0) return SP_OK;
  const bool fast = dtype == SP_BF16 && gemm_mfma_supported(op, M, N, K, A, B, C, R);
  const int pi = prof_start(fast ? op : PROF_GEMM_PLAIN, s);
  if (fast) gemm_mfma(s, op, M, N, K, A, B, C, R);
  else gemm_simple(s, dtype, op, M, N, K, A, B, C, R);
  prof_stop(pi, s, 2.0 * (double)M * (double)N * (double)K);
  return SP_OK;
}

int gemm_rope(hipStream_t s, int dtype, int64_t M, int64_t N, int64_t K, const void* A, const void* B, void* C,
              const RopeArgs& ra, float rope_theta) {
  if (M < 0 || N < 0 || K < 0 || ra.hd < 2 || ra.hd % 2 || ra.rot_cols % ra.hd || ra.rot_cols > N || ra.T < 1)
    return fail(SP_EINVAL, "gemm_rope: bad shape");
  if ((M > 0 && N > 0) && (!C || (K > 0 && (!A || !B)))) return fail(SP_EINVAL, "gemm_rope: null operand");
  if (M == 0 || N == 0) return SP_OK;
  // fused when the matrix-core path takes the product and a 16-byte output chunk never straddles a head
  const bool fast = dtype == SP_BF16 && ra.table && ra.hd % 8 == 0 && gemm_mfma_supported(0, M, N, K, A, B, C, nullptr);
  if (!fast) {
    int rc = gemm(s, dtype, 0, M, N, K, A, B, C, nullptr);
    if (rc) return rc;
    rope(s, dtype, C, M, ra.T, ra.rot_cols / ra.hd, ra.hd, (int)N, rope_theta, +1);
    return SP_OK;
  }
  const int pi = prof_start(0, s);
  gemm_mfma(s, 0, M, N, K, A, B, C, nullptr, &ra);
  prof_stop(pi, s, 2.0 * (double)M * (double)N * (double)K);
  return SP_OK;
}

int ffn_up_fwd(hipStream_t s, int dtype, int64_t R, int64_t h, int64_t d, const void* hn, const void* wgu, void* gu, void* act) {
  if (R < 0 || h < 1 || d < 1) return fail(SP_EINVAL, "ffn_up_fwd: bad shape");
  if (R == 0) return SP_OK;
  if (!hn || !wgu || !gu || !act) return fail(SP_EINVAL, "ffn_up_fwd: null operand");
  if (dtype == SP_BF16 && gemm_swiglu_supported(false, R, h, d, hn, wgu, gu, act)) {
    const int pi = prof_start(0, s);
    gemm_mfma_swiglu_fwd(s, R, h, d, hn, wgu, gu, act);
    prof_stop(pi, s, 4.0 * (double)R * (double)h * (double)d);
    return SP_OK;
  }
  int rc = gemm(s, dtype, 0, R, 2 * h, d, hn, wgu, gu, nullptr);
  if (rc) return rc;
  swiglu_fwd(s, dtype, gu, R, (int)h, act);
  return SP_OK;
}

int ffn_down_bwd(hipStream_t s, int dtype, int64_t R, int64_t h, int64_t d, const void* dy, const void* wd, const void* gu,
                 void* dgu, void* da_tmp) {
  if (R < 0 || h < 1 || d < 1) return fail(SP_EINVAL, "ffn_down_bwd: bad shape");
  if (R == 0) return SP_OK;
  if (!dy || !wd || !gu || !dgu || !da_tmp) return fail(SP_EINVAL, "ffn_down_bwd: null operand");
  if (dtype == SP_BF16 && gemm_swiglu_supported(true, R, h, d, dy, wd, gu, dgu)) {
    const int pi = prof_start(1, s);
    gemm_mfma_swiglu_bwd(s, R, h, d, dy, wd, gu, dgu);
    prof_stop(pi, s, 2.0 * (double)R * (double)h * (double)d);
    return SP_OK;
  }
  int rc = gemm(s, dtype, 1, R, h, d, dy, wd, da_tmp, nullptr);
  if (rc) return rc;
  swiglu_bwd(s, dtype, da_tmp, gu, R, (int)h, dgu);
  return SP_OK;
}

}  // namespace sp
