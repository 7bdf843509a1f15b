// Causal attention on the CDNA4 matrix cores for bf16, head dimension 64 or 128.
//
// Forward and both backward kernels tile the score matrix and never write it to memory: a block
// of query rows meets the key/value rows in tiles staged through LDS, scores are recomputed in
// the backward pass from the saved log-sum-exp.
//
// All products are issued in the transposed form  D^T = B^T A^T  of v_mfma_f32_32x32x16_bf16 so
// that the index a lane keeps fixed (the MFMA column, lane % 32) is the one its row statistics
// belong to: a query in the forward and dQ kernels (running max / sum, log-sum-exp, delta are
// per-lane scalars), a key in the dK/dV kernel (the gradients a wavefront owns).  The
// accumulator of one MFMA then serves directly as the k-operand of the next (P for P V, dS for
// dS K, ...) after rounding to bf16, with the 16 k-slots of the instruction assigned to rows in
// the accumulator's own order; the LDS-side operand is gathered in the matching order by the LDS
// transpose read, so every tile sits in LDS exactly as it sits in memory.
//
// Layout: qkv rows of (H + 2*Hkv)*hd = queries | keys | values; o rows of H*hd; lse, delta [B][H][T].
#include "devutil.h"
#include "internal.h"

namespace sp {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;   // one staged 16-byte chunk (a native vector: stays in registers)

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int r = 0; r < 16; ++r) z[r] = 0.f;
  return z;
}

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// accumulator registers [8u, 8u+8) of a 32x32 tile -> one bf16 k-operand.
// k-slot e of lane half hh then stands for tile row 16u + (e/4)*8 + hh*4 + e%4.
__device__ __forceinline__ bf16x8 pack8(const f32x16& v, int u) {
  bf16x8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = (bf16)v[8 * u + e];
  return o;
}

// LDS operand that pairs with pack8, gathered from a row-major [row][col] tile (row stride RS bytes)
// with the LDS transpose read: MFMA row (lane % 32) = tile column col_base + lane % 32, and the 8
// k-slots of lane half hh = tile rows row_base + hh*4 + {0..3} and row_base + 8 + hh*4 + {0..3}.
// (ds_read_b64_tr_b16: within 16 lanes, lane i receives element i%4 of the 8-byte pieces addressed by
// lanes i/4, i/4+4, i/4+8, i/4+12; here piece s of a group is row s/4, columns 4*(s%4)..+3.)
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
__device__ __forceinline__ bf16x8 read_tr(const char* tile, int RS, int col_base, int row_base, int lane) {
  const int g16 = (lane >> 4) & 1, hh = lane >> 5, sl = lane & 15;
  const char* p = tile + (row_base + hh * 4 + (sl >> 2)) * RS + (col_base + g16 * 16 + (sl & 3) * 4) * 2;
  typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 8 * RS));
  const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, v);
}

// ---- staging of a [ROWS x HD] block of a row-major matrix (row stride ld elements): 16-byte chunks,
// consecutive lanes take consecutive chunks of a row.  NCH chunks per thread (256 threads).
template <int HD, int ROWS>
struct Stage {
  static constexpr int kChunksPerRow = HD / 8;
  static constexpr int kChunks = ROWS * kChunksPerRow;
  static constexpr int NCH = (kChunks + 255) / 256;
  __device__ __forceinline__ static void load(u32x4 (&reg)[NCH], const bf16* __restrict__ X, int64_t ld, int row0, int row_max, int tid) {
#pragma unroll
    for (int n = 0; n < NCH; ++n) {
      const int c = tid + 256 * n;
      if (kChunks % 256 == 0 || c < kChunks) {
        const int r = min(row0 + c / kChunksPerRow, row_max);
        reg[n] = *reinterpret_cast<const u32x4*>(X + (int64_t)r * ld + (c % kChunksPerRow) * 8);
      }
    }
  }
  __device__ __forceinline__ static void store(const u32x4 (&reg)[NCH], char* tile, int stride, int tid) {
#pragma unroll
    for (int n = 0; n < NCH; ++n) {
      const int c = tid + 256 * n;
      if (kChunks % 256 == 0 || c < kChunks)
        *reinterpret_cast<u32x4*>(tile + (c / kChunksPerRow) * stride + (c % kChunksPerRow) * 16) = reg[n];
    }
  }
};

// ================================================================================ forward
// Workgroup: 128 queries of one (sequence, head), 4 wavefronts x 32 queries; key/value tiles of 64.
// Per tile and wavefront: S^T[key][query] = K Q^T, online softmax down each lane's query,
// O^T[col][query] += V^T P^T.
template <int HD>
__global__ __launch_bounds__(256, 2) void k_flash_fwd(const bf16* __restrict__ qkv, bf16* __restrict__ o,
                                                      float* __restrict__ lse, int T, int H, int Hkv, float scale_log2) {
  constexpr int BQ = 128, BKV = 64;
  constexpr int KS = HD * 2 + 16;   // K tile row stride (bytes): [key][hd]
  constexpr int VS = HD * 2 + 64;   // V tile row stride (bytes): [key][hd], read through the transpose read
  constexpr int kKTile = BKV * KS, kVTile = BKV * VS;
  __shared__ __attribute__((aligned(16))) char smem[2 * (kKTile + kVTile)];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lq = lane & 31, hh = lane >> 5;
  const int qb = gridDim.x - 1 - blockIdx.x, a = blockIdx.y, b = blockIdx.z;
  const int kvh = a / (H / Hkv);
  const int64_t ld = (int64_t)(H + 2 * Hkv) * HD;
  const bf16* Q = qkv + (int64_t)b * T * ld + a * HD;
  const bf16* Kp = qkv + (int64_t)b * T * ld + (H + kvh) * HD;
  const bf16* Vp = qkv + (int64_t)b * T * ld + (H + Hkv + kvh) * HD;
  const int q0 = qb * BQ, qw0 = q0 + wave * 32, q = qw0 + lq;

  bf16x8 qf[HD / 16];
  {
    const bf16* qr = Q + (int64_t)min(q, T - 1) * ld + hh * 8;
#pragma unroll
    for (int kk = 0; kk < HD / 16; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qr + kk * 16);
  }
  f32x16 oacc[HD / 32];
#pragma unroll
  for (int c = 0; c < HD / 32; ++c) oacc[c] = zero16();
  float m_i = -INFINITY, l_i = 0.f;

  const int kv_end = min(T, q0 + BQ);
  const int ntiles = (kv_end + BKV - 1) / BKV;
  typedef Stage<HD, BKV> ST;
  u32x4 rk[ST::NCH], rv[ST::NCH];
  ST::load(rk, Kp, ld, 0, T - 1, tid);
  ST::load(rv, Vp, ld, 0, T - 1, tid);
  ST::store(rk, smem, KS, tid);
  ST::store(rv, smem + kKTile, VS, tid);
  __syncthreads();
  for (int kt = 0; kt < ntiles; ++kt) {
    const int k0 = kt * BKV;
    // The loop body is one straight block (no wave-dependent branch around the arithmetic): the loads of
    // the next tile are issued here and must stay here, a whole tile of work ahead of their use.  After
    // the last tile they re-read it, and a wavefront whose queries see no key of a tile computes zeros.
    const int kn = min(k0 + BKV, (ntiles - 1) * BKV);
    ST::load(rk, Kp, ld, kn, T - 1, tid);
    const char* ks = smem + (kt & 1) * (kKTile + kVTile);
    const char* vs = ks + kKTile;
    {
      // S^T = K Q^T on two independent accumulators (32 keys each); the K fragments of the next two
      // k-steps are fetched while the MFMAs of the current two run
      f32x16 st[2] = {zero16(), zero16()};
      bf16x8 fb[2][4];
      const char* kr = ks + lq * KS + hh * 16;
      auto ldk = [&](int g, bf16x8 (&f)[4]) {
        f[0] = *reinterpret_cast<const bf16x8*>(kr + (2 * g) * 32);
        f[1] = *reinterpret_cast<const bf16x8*>(kr + 32 * KS + (2 * g) * 32);
        f[2] = *reinterpret_cast<const bf16x8*>(kr + (2 * g + 1) * 32);
        f[3] = *reinterpret_cast<const bf16x8*>(kr + 32 * KS + (2 * g + 1) * 32);
      };
      auto ldv = [&](int tu, bf16x8 (&f)[4]) {
#pragma unroll
        for (int c = 0; c < HD / 32; ++c) f[c] = read_tr(vs, VS, c * 32, (tu >> 1) * 32 + 16 * (tu & 1), lane);
      };
      ldk(0, fb[0]);
#pragma unroll
      for (int g = 0; g < HD / 32; ++g) {
        if (g + 1 < HD / 32) ldk(g + 1, fb[(g + 1) & 1]);
        __builtin_amdgcn_sched_barrier(0);
        st[0] = mfma(fb[g & 1][0], qf[2 * g], st[0]);
        st[1] = mfma(fb[g & 1][1], qf[2 * g], st[1]);
        st[0] = mfma(fb[g & 1][2], qf[2 * g + 1], st[0]);
        st[1] = mfma(fb[g & 1][3], qf[2 * g + 1], st[1]);
        __builtin_amdgcn_sched_barrier(0);
      }
      ST::load(rv, Vp, ld, kn, T - 1, tid);   // next V tile: in flight during softmax and P V
      ldv(0, fb[0]);  // first V fragments: their latency hides behind the softmax arithmetic
      __builtin_amdgcn_sched_barrier(0);
      const bool mask = k0 + BKV - 1 > qw0;
      float mx = -INFINITY;
      if (mask) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = k0 + t * 32 + (r >> 2) * 8 + hh * 4 + (r & 3);
            if (key > q) st[t][r] = -INFINITY;
          }
      }
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, st[t][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32)) * scale_log2;
      // the running maximum only moves when it is exceeded by more than 2^8: probabilities stay below 256,
      // exact after the final division, and the accumulator is rescaled rarely
      const float m_new = mx > m_i + 8.0f ? mx : m_i;   // first tile: m_i = -inf, so m_new = mx (finite: key 0)
      const float alpha = __builtin_amdgcn_exp2f(m_i - m_new);
      float rs = 0.f;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(st[t][r], scale_log2, -m_new));
          st[t][r] = pv;
          rs += pv;
        }
      l_i = l_i * alpha + rs;
      m_i = m_new;
      if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
        for (int c = 0; c < HD / 32; ++c)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[c][r] *= alpha;
      }
#pragma unroll
      for (int tu = 0; tu < 4; ++tu) {
        if (tu + 1 < 4) ldv(tu + 1, fb[(tu + 1) & 1]);
        __builtin_amdgcn_sched_barrier(0);
        const bf16x8 pf = pack8(st[tu >> 1], tu & 1);
#pragma unroll
        for (int c = 0; c < HD / 32; ++c) oacc[c] = mfma(fb[tu & 1][c], pf, oacc[c]);
      }
    }
    {
      char* nk = smem + ((kt + 1) & 1) * (kKTile + kVTile);
      ST::store(rk, nk, KS, tid);
      ST::store(rv, nk + kKTile, VS, tid);
    }
    __syncthreads();
  }
  const float l_tot = l_i + __shfl_xor(l_i, 32);
  if (q < T) {
    const float inv = 1.0f / l_tot;
    bf16* orow = o + ((int64_t)b * T + q) * H * HD + a * HD;
#pragma unroll
    for (int c = 0; c < HD / 32; ++c)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 w;
        w.x = pack_bf16(oacc[c][4 * g] * inv, oacc[c][4 * g + 1] * inv);
        w.y = pack_bf16(oacc[c][4 * g + 2] * inv, oacc[c][4 * g + 3] * inv);
        *reinterpret_cast<uint2*>(orow + c * 32 + g * 8 + hh * 4) = w;
      }
    if (hh == 0) lse[((int64_t)b * H + a) * T + q] = (m_i + log2f(l_tot)) * kLn2;
  }
}

// ================================================================================ delta
// delta[b][a][i] = sum_c dO[i][a][c] * O[i][a][c]; one wavefront per 64/HD*8 ... rows: lane = (row, 8 columns)
template <int HD>
__global__ __launch_bounds__(256) void k_flash_delta(const bf16* __restrict__ o, const bf16* __restrict__ dO, int B, int T,
                                                     int H, float* __restrict__ delta) {
  constexpr int LPR = HD / 8;  // lanes per (row, head)
  const int64_t total = (int64_t)B * T * H;
  const int64_t item = ((int64_t)blockIdx.x * 256 + threadIdx.x) / LPR;
  const int part = threadIdx.x % LPR;
  float s = 0.f;
  if (item < total) {
    float x[8], y[8];
    load8(o + item * HD + part * 8, x);
    load8(dO + item * HD + part * 8, y);
#pragma unroll
    for (int j = 0; j < 8; ++j) s += x[j] * y[j];
  }
#pragma unroll
  for (int off = LPR / 2; off > 0; off >>= 1) s += __shfl_xor(s, off);
  if (item < total && part == 0) {
    const int64_t row = item / H;
    const int a = (int)(item - row * H);
    const int64_t bb = row / T, i = row - bb * T;
    delta[(bb * H + a) * T + i] = s;
  }
}

// ================================================================================ backward: dQ
// Same walk as the forward.  Per tile: S^T = K Q^T, P = exp(S - lse), dP^T = V dO^T,
// dS^T = P (dP^T - delta), dQ^T[col][query] += K^T dS^T.  The 1/sqrt(hd) factor is applied at the end.
template <int HD>
__global__ __launch_bounds__(256, 2) void k_flash_bwd_dq(const bf16* __restrict__ qkv, const bf16* __restrict__ dO,
                                                         const float* __restrict__ lse, const float* __restrict__ delta,
                                                         bf16* __restrict__ dqkv, int T, int H, int Hkv, float scale) {
  constexpr int BQ = 128, BKV = 64;
  constexpr int KS = HD * 2 + 16;   // K and V tiles [key][hd]
  constexpr int TS = HD * 2 + 64;   // second copy of K, [key][hd], strided for the transpose read
  constexpr int kKTile = BKV * KS, kTTile = BKV * TS;
  __shared__ __attribute__((aligned(16))) char smem[2 * kKTile + kTTile];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lq = lane & 31, hh = lane >> 5;
  const int qb = gridDim.x - 1 - blockIdx.x, a = blockIdx.y, b = blockIdx.z;
  const int kvh = a / (H / Hkv);
  const int64_t ld = (int64_t)(H + 2 * Hkv) * HD;
  const bf16* Q = qkv + (int64_t)b * T * ld + a * HD;
  const bf16* Kp = qkv + (int64_t)b * T * ld + (H + kvh) * HD;
  const bf16* Vp = qkv + (int64_t)b * T * ld + (H + Hkv + kvh) * HD;
  const int q0 = qb * BQ, qw0 = q0 + wave * 32, q = qw0 + lq, qc = min(q, T - 1);
  const float scale_log2 = scale * kLog2e;

  bf16x8 qf[HD / 16], dof[HD / 16];
  {
    const bf16* qr = Q + (int64_t)qc * ld + hh * 8;
    const bf16* dr = dO + ((int64_t)b * T + qc) * H * HD + a * HD + hh * 8;
#pragma unroll
    for (int kk = 0; kk < HD / 16; ++kk) {
      qf[kk] = *reinterpret_cast<const bf16x8*>(qr + kk * 16);
      dof[kk] = *reinterpret_cast<const bf16x8*>(dr + kk * 16);
    }
  }
  const float lse2 = lse[((int64_t)b * H + a) * T + qc] * kLog2e;
  const float dlt = delta[((int64_t)b * H + a) * T + qc];
  f32x16 dq[HD / 32];
#pragma unroll
  for (int c = 0; c < HD / 32; ++c) dq[c] = zero16();

  char* ks = smem;
  char* vs = smem + kKTile;
  char* kts = smem + 2 * kKTile;
  const int kv_end = min(T, q0 + BQ);
  const int ntiles = (kv_end + BKV - 1) / BKV;
  typedef Stage<HD, BKV> ST;
  u32x4 rk[ST::NCH], rv[ST::NCH];
  ST::load(rk, Kp, ld, 0, T - 1, tid);
  ST::load(rv, Vp, ld, 0, T - 1, tid);
  for (int kt = 0; kt < ntiles; ++kt) {
    const int k0 = kt * BKV;
    ST::store(rk, ks, KS, tid);
    ST::store(rk, kts, TS, tid);
    ST::store(rv, vs, KS, tid);
    __syncthreads();
    {
      const int kn = min(k0 + BKV, (ntiles - 1) * BKV);   // straight-line body, as in the forward kernel
      ST::load(rk, Kp, ld, kn, T - 1, tid);
      ST::load(rv, Vp, ld, kn, T - 1, tid);
    }
    {
      const bool mask = k0 + BKV - 1 > qw0;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        // S^T and dP^T as two independent MFMA chains; K and V fragments fetched two k-steps ahead
        f32x16 st = zero16(), dp = zero16();
        bf16x8 fb[2][4];
        const char* kr = ks + (t * 32 + lq) * KS + hh * 16;
        const char* vr = vs + (t * 32 + lq) * KS + hh * 16;
        auto ldkv = [&](int g, bf16x8 (&f)[4]) {
          f[0] = *reinterpret_cast<const bf16x8*>(kr + (2 * g) * 32);
          f[1] = *reinterpret_cast<const bf16x8*>(vr + (2 * g) * 32);
          f[2] = *reinterpret_cast<const bf16x8*>(kr + (2 * g + 1) * 32);
          f[3] = *reinterpret_cast<const bf16x8*>(vr + (2 * g + 1) * 32);
        };
        auto ldt = [&](int u, bf16x8 (&f)[4]) {
#pragma unroll
          for (int c = 0; c < HD / 32; ++c) f[c] = read_tr(kts, TS, c * 32, t * 32 + 16 * u, lane);
        };
        ldkv(0, fb[0]);
#pragma unroll
        for (int g = 0; g < HD / 32; ++g) {
          if (g + 1 < HD / 32) ldkv(g + 1, fb[(g + 1) & 1]);
          __builtin_amdgcn_sched_barrier(0);
          st = mfma(fb[g & 1][0], qf[2 * g], st);
          dp = mfma(fb[g & 1][1], dof[2 * g], dp);
          st = mfma(fb[g & 1][2], qf[2 * g + 1], st);
          dp = mfma(fb[g & 1][3], dof[2 * g + 1], dp);
          __builtin_amdgcn_sched_barrier(0);
        }
        ldt(0, fb[0]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(st[r], scale_log2, -lse2));
          if (mask) {
            const int key = k0 + t * 32 + (r >> 2) * 8 + hh * 4 + (r & 3);
            if (key > q) pv = 0.f;
          }
          st[r] = pv * (dp[r] - dlt);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          if (u + 1 < 2) ldt(u + 1, fb[(u + 1) & 1]);
          __builtin_amdgcn_sched_barrier(0);
          const bf16x8 dsf = pack8(st, u);
#pragma unroll
          for (int c = 0; c < HD / 32; ++c) dq[c] = mfma(fb[u & 1][c], dsf, dq[c]);
        }
      }
    }
    __syncthreads();
  }
  if (q < T) {
    bf16* row = dqkv + ((int64_t)b * T + q) * ld + a * HD;
#pragma unroll
    for (int c = 0; c < HD / 32; ++c)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 w;
        w.x = pack_bf16(dq[c][4 * g] * scale, dq[c][4 * g + 1] * scale);
        w.y = pack_bf16(dq[c][4 * g + 2] * scale, dq[c][4 * g + 3] * scale);
        *reinterpret_cast<uint2*>(row + c * 32 + g * 8 + hh * 4) = w;
      }
  }
}

// ================================================================================ backward: dK, dV
// Workgroup: 128 keys of one (sequence, kv head), 4 wavefronts x 32 keys, which it owns: their K
// and V fragments stay in registers.  It walks the query heads of its group and, for each, the
// query tiles (32 rows) from its first key onward.  Per tile: S[query][key] = Q K^T,
// P = exp(S - lse[query]), dP = dO V^T, dS = P (dP - delta[query]),
// dV^T[col][key] += dO^T P,  dK^T[col][key] += Q^T dS.
template <int HD>
__global__ __launch_bounds__(256) void k_flash_bwd_dkv(const bf16* __restrict__ qkv, const bf16* __restrict__ dO,
                                                       const float* __restrict__ lse, const float* __restrict__ delta,
                                                       bf16* __restrict__ dqkv, int T, int H, int Hkv, float scale) {
  constexpr int BK = 128, BQ = 32;
  constexpr int QS = HD * 2 + 16;   // Q and dO tiles [query][hd]
  constexpr int TS = HD * 2 + 64;   // second copies of Q and dO, [query][hd], strided for the transpose read
  constexpr int kQTile = BQ * QS, kTTile = BQ * TS;
  constexpr int kBuf = 2 * kQTile + 2 * kTTile + 2 * BQ * 4;
  __shared__ __attribute__((aligned(16))) char smem[2 * kBuf];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lk = lane & 31, hh = lane >> 5;
  const int kb = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int rep = H / Hkv;
  const int64_t ld = (int64_t)(H + 2 * Hkv) * HD;
  const bf16* Kp = qkv + (int64_t)b * T * ld + (H + kvh) * HD;
  const bf16* Vp = qkv + (int64_t)b * T * ld + (H + Hkv + kvh) * HD;
  const int k0 = kb * BK, kw0 = k0 + wave * 32, key = kw0 + lk, keyc = min(key, T - 1);
  const float scale_log2 = scale * kLog2e;

  bf16x8 kf[HD / 16], vf[HD / 16];
  {
    const bf16* kr = Kp + (int64_t)keyc * ld + hh * 8;
    const bf16* vr = Vp + (int64_t)keyc * ld + hh * 8;
#pragma unroll
    for (int kk = 0; kk < HD / 16; ++kk) {
      kf[kk] = *reinterpret_cast<const bf16x8*>(kr + kk * 16);
      vf[kk] = *reinterpret_cast<const bf16x8*>(vr + kk * 16);
    }
  }
  f32x16 dk[HD / 32], dv[HD / 32];
#pragma unroll
  for (int c = 0; c < HD / 32; ++c) { dk[c] = zero16(); dv[c] = zero16(); }

  const int qt0 = k0 / BQ, nqt = (T + BQ - 1) / BQ;   // query tiles that can see a key of this block
  const int per_head = nqt - qt0;
  const int steps = per_head * rep;
  typedef Stage<HD, BQ> SQ;
  u32x4 rq[SQ::NCH], rdo[SQ::NCH];
  float st_lse = 0.f, st_dlt = 0.f;
  auto load_step = [&](int step) {
    const int a = kvh * rep + step / per_head;
    const int qs = (qt0 + step % per_head) * BQ;
    SQ::load(rq, qkv + (int64_t)b * T * ld + a * HD, ld, qs, T - 1, tid);
    SQ::load(rdo, dO + (int64_t)b * T * H * HD + a * HD, (int64_t)H * HD, qs, T - 1, tid);
    if (tid < BQ) {
      const int qi = min(qs + tid, T - 1);
      st_lse = lse[((int64_t)b * H + a) * T + qi] * kLog2e;
      st_dlt = delta[((int64_t)b * H + a) * T + qi];
    }
  };
  auto store_step = [&](int buf) {
    char* base = smem + buf * kBuf;
    SQ::store(rq, base, QS, tid);
    SQ::store(rdo, base + kQTile, QS, tid);
    SQ::store(rq, base + 2 * kQTile, TS, tid);
    SQ::store(rdo, base + 2 * kQTile + kTTile, TS, tid);
    if (tid < BQ) {
      reinterpret_cast<float*>(base + 2 * kQTile + 2 * kTTile)[tid] = st_lse;
      reinterpret_cast<float*>(base + 2 * kQTile + 2 * kTTile + BQ * 4)[tid] = st_dlt;
    }
  };
  if (steps > 0) {
    load_step(0);
    store_step(0);
  }
  __syncthreads();
  for (int step = 0; step < steps; ++step) {
    load_step(min(step + 1, steps - 1));   // straight-line body: after the last step this re-reads it
    const int qs = (qt0 + step % per_head) * BQ;
    const char* base = smem + (step & 1) * kBuf;
    {  // a wavefront none of whose keys is visible to the tile's queries computes zeros
      const char* qsm = base;
      const char* dosm = base + kQTile;
      const char* qts = base + 2 * kQTile;
      const char* dots = qts + kTTile;
      const float* s_lse = reinterpret_cast<const float*>(base + 2 * kQTile + 2 * kTTile);
      const float* s_dlt = s_lse + BQ;
      f32x16 s = zero16(), dp = zero16();
      bf16x8 fb[2][4];
      const char* qr = qsm + lk * QS + hh * 16;     // A operand: row = query lk of the tile
      const char* dr = dosm + lk * QS + hh * 16;
      auto ldq = [&](int g, bf16x8 (&f)[4]) {
        f[0] = *reinterpret_cast<const bf16x8*>(qr + (2 * g) * 32);
        f[1] = *reinterpret_cast<const bf16x8*>(dr + (2 * g) * 32);
        f[2] = *reinterpret_cast<const bf16x8*>(qr + (2 * g + 1) * 32);
        f[3] = *reinterpret_cast<const bf16x8*>(dr + (2 * g + 1) * 32);
      };
      // group w of the second phase: w = 2u + (0: dO^T for dV, 1: Q^T for dK)
      auto ldt = [&](int w, bf16x8 (&f)[4]) {
#pragma unroll
        for (int c = 0; c < HD / 32; ++c) f[c] = read_tr((w & 1) ? qts : dots, TS, c * 32, 16 * (w >> 1), lane);
      };
      ldq(0, fb[0]);
#pragma unroll
      for (int g = 0; g < HD / 32; ++g) {
        if (g + 1 < HD / 32) ldq(g + 1, fb[(g + 1) & 1]);
        __builtin_amdgcn_sched_barrier(0);
        s = mfma(fb[g & 1][0], kf[2 * g], s);
        dp = mfma(fb[g & 1][1], vf[2 * g], dp);
        s = mfma(fb[g & 1][2], kf[2 * g + 1], s);
        dp = mfma(fb[g & 1][3], vf[2 * g + 1], dp);
        __builtin_amdgcn_sched_barrier(0);
      }
      ldt(0, fb[0]);
      __builtin_amdgcn_sched_barrier(0);
      const bool mask = qs < kw0 + 31;
      f32x16 p;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int qi = g * 8 + hh * 4;   // accumulator rows 4g..4g+3 are queries qi..qi+3 of the tile
        const float4 l4 = *reinterpret_cast<const float4*>(s_lse + qi);
        const float4 d4 = *reinterpret_cast<const float4*>(s_dlt + qi);
        const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int r = 4 * g + e;
          float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], scale_log2, -lv[e]));
          if (mask && key > qs + qi + e) pv = 0.f;
          if (qs + qi + e >= T) pv = 0.f;     // rows past the end of the sequence are re-reads of row T-1
          p[r] = pv;
          s[r] = pv * (dp[r] - dv4[e]);
        }
      }
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        if (w + 1 < 4) ldt(w + 1, fb[(w + 1) & 1]);
        __builtin_amdgcn_sched_barrier(0);
        const bf16x8 bf = pack8((w & 1) ? s : p, w >> 1);
#pragma unroll
        for (int c = 0; c < HD / 32; ++c) {
          if (w & 1) dk[c] = mfma(fb[w & 1][c], bf, dk[c]);
          else dv[c] = mfma(fb[w & 1][c], bf, dv[c]);
        }
      }
    }
    store_step((step + 1) & 1);
    __syncthreads();
  }
  if (key < T) {
    bf16* krow = dqkv + ((int64_t)b * T + key) * ld + (H + kvh) * HD;
    bf16* vrow = dqkv + ((int64_t)b * T + key) * ld + (H + Hkv + kvh) * HD;
#pragma unroll
    for (int c = 0; c < HD / 32; ++c)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 w;
        w.x = pack_bf16(dk[c][4 * g] * scale, dk[c][4 * g + 1] * scale);
        w.y = pack_bf16(dk[c][4 * g + 2] * scale, dk[c][4 * g + 3] * scale);
        *reinterpret_cast<uint2*>(krow + c * 32 + g * 8 + hh * 4) = w;
        w.x = pack_bf16(dv[c][4 * g], dv[c][4 * g + 1]);
        w.y = pack_bf16(dv[c][4 * g + 2], dv[c][4 * g + 3]);
        *reinterpret_cast<uint2*>(vrow + c * 32 + g * 8 + hh * 4) = w;
      }
  }
}

}  // namespace

bool attention_flash_supported(int B, int T, int H, int Hkv, int hd) {
  return (hd == 64 || hd == 128) && B >= 1 && T >= 1 && B <= 65535 && H <= 65535 && H % Hkv == 0;
}

void attention_flash_fwd(hipStream_t s, int B, int T, int H, int Hkv, int hd, const void* qkv, void* o, float* lse) {
  const float sl2 = kLog2e / sqrtf((float)hd);
  dim3 grid((T + 127) / 128, H, B);
  if (hd == 128)
    hipLaunchKernelGGL(k_flash_fwd<128>, grid, dim3(256), 0, s, (const bf16*)qkv, (bf16*)o, lse, T, H, Hkv, sl2);
  else
    hipLaunchKernelGGL(k_flash_fwd<64>, grid, dim3(256), 0, s, (const bf16*)qkv, (bf16*)o, lse, T, H, Hkv, sl2);
}

void attention_flash_bwd(hipStream_t s, int B, int T, int H, int Hkv, int hd, const void* qkv, const void* o,
                         const float* lse, const void* do_, void* dqkv, float* delta) {
  const float scale = 1.0f / sqrtf((float)hd);
  const int64_t items = (int64_t)B * T * H;
  dim3 gq((T + 127) / 128, H, B), gk((T + 127) / 128, Hkv, B);
  // algorithmic flops of the backward pass: four products (dV, dP, dQ, dK) over the causal half;
  // dQ is credited to its kernel, the other three to the dK/dV kernel (the recomputed scores are not counted)
  const double unit = (double)B * H * (double)T * (T + 1) * hd;
  int pi = prof_start(PROF_ATTN_DELTA, s);
  if (hd == 128)
    hipLaunchKernelGGL(k_flash_delta<128>, dim3((unsigned)((items * 16 + 255) / 256)), dim3(256), 0, s, (const bf16*)o,
                       (const bf16*)do_, B, T, H, delta);
  else
    hipLaunchKernelGGL(k_flash_delta<64>, dim3((unsigned)((items * 8 + 255) / 256)), dim3(256), 0, s, (const bf16*)o,
                       (const bf16*)do_, B, T, H, delta);
  prof_stop(pi, s, 0.0);
  pi = prof_start(PROF_ATTN_DQ, s);
  if (hd == 128)
    hipLaunchKernelGGL(k_flash_bwd_dq<128>, gq, dim3(256), 0, s, (const bf16*)qkv, (const bf16*)do_, lse, delta,
                       (bf16*)dqkv, T, H, Hkv, scale);
  else
    hipLaunchKernelGGL(k_flash_bwd_dq<64>, gq, dim3(256), 0, s, (const bf16*)qkv, (const bf16*)do_, lse, delta,
                       (bf16*)dqkv, T, H, Hkv, scale);
  prof_stop(pi, s, unit);
  pi = prof_start(PROF_ATTN_DKV, s);
  if (hd == 128)
    hipLaunchKernelGGL(k_flash_bwd_dkv<128>, gk, dim3(256), 0, s, (const bf16*)qkv, (const bf16*)do_, lse, delta,
                       (bf16*)dqkv, T, H, Hkv, scale);
  else
    hipLaunchKernelGGL(k_flash_bwd_dkv<64>, gk, dim3(256), 0, s, (const bf16*)qkv, (const bf16*)do_, lse, delta,
                       (bf16*)dqkv, T, H, Hkv, scale);
  prof_stop(pi, s, 3.0 * unit);
}

}  // namespace sp
