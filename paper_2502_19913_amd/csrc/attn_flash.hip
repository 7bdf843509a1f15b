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
// u32x4 (devutil.h): one staged 16-byte chunk; a native vector, so staged tiles stay in registers

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
  // the same block through a buffer descriptor: voff0(tid) + row0 * row_bytes; rows past the end read as zero
  __device__ __forceinline__ static uint32_t voff0(int tid, int n, uint32_t row_bytes) {
    const int c = tid + 256 * n;
    return (uint32_t)(c / kChunksPerRow) * row_bytes + (uint32_t)(c % kChunksPerRow) * 16u;
  }
  __device__ __forceinline__ static void bload(u32x4 (&reg)[NCH], rsrc_t rsrc, uint32_t row_bytes, uint32_t off, int tid) {
#pragma unroll
    for (int n = 0; n < NCH; ++n)
      if (kChunks % 256 == 0 || tid + 256 * n < kChunks) reg[n] = buffer_load16(rsrc, voff0(tid, n, row_bytes) + off);
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
// query tiles (32 rows) from its first key onward.  Per tile:
//   phase 1  S' = Q K^T - lse/scale + mask bias,  dP' = dO V^T - delta           (2 * hd/16 MFMAs)
//   phase 2  P = exp(scale S'),  dS = P dP'                                      (arithmetic only)
//   phase 3  dV^T[col][key] += dO^T P,  dK^T[col][key] += Q^T dS                 (2 * hd/16 MFMAs)
// The log-sum-exp, the causal mask and delta enter as the initial accumulators of phase 1, so phase 2
// is a product, an exponential, a product and the conversions per element.
// One wavefront per SIMD (the accumulators leave no room for two), so matrix work, arithmetic and
// LDS latency overlap inside the wavefront, by software pipelining over the tiles:
//   first half of an iteration   phase 1 of tile i+1 (operands already in registers), phase 2 of
//                                tile i, LDS reads of tile i's phase 3 operands
//   second half                  phase 3 of tile i, LDS reads of tile i+2's phase 1 operands and
//                                initial accumulators
// with one workgroup barrier between the halves.  Tiles rotate through three LDS buffers: tile i+2 is
// written at the top of iteration i (its buffer was last read before the previous barrier), and the
// global loads of tile i+3 are then in flight for a whole iteration.  Tiles past the end of the walk
// carry lse = +inf, so they multiply through as zeros.
template <int HD>
__global__ __launch_bounds__(256) void k_flash_bwd_dkv(const bf16* __restrict__ qkv, const bf16* __restrict__ dO,
                                                       const float* __restrict__ lse, const float* __restrict__ delta,
                                                       bf16* __restrict__ dqkv, int T, int H, int Hkv, float scale) {
  constexpr int BK = 128, BQ = 32, NK = HD / 16, NC = HD / 32;
  constexpr int QS = HD * 2 + 16;   // Q and dO tiles [query][hd], read along hd
  constexpr int TS = HD * 2 + 64;   // second copies, strided for the transpose read
  constexpr int kDO = BQ * QS, kQT = 2 * BQ * QS, kDOT = kQT + BQ * TS;
  constexpr int kNL = kDOT + BQ * TS;   // -lse / scale per query: 256 slots, the first 32 are read
  constexpr int kND = kNL + 256 * 4;    // -delta per query, likewise
  constexpr int kBuf = kND + 256 * 4;
  __shared__ __attribute__((aligned(16))) char smem[3 * kBuf];
  const int tid = threadIdx.x, lane = tid & 63, lk = lane & 31, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kb = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int rep = H / Hkv;
  const int64_t ld = (int64_t)(H + 2 * Hkv) * HD;
  const bf16* Kp = qkv + (int64_t)b * T * ld + (H + kvh) * HD;
  const bf16* Vp = qkv + (int64_t)b * T * ld + (H + Hkv + kvh) * HD;
  const int k0 = kb * BK, kw0 = k0 + wave * 32, key = kw0 + lk, keyc = min(key, T - 1);
  const float scale_log2 = scale * kLog2e, inv_scale = 1.f / scale;

  bf16x8 kf[NK], vf[NK];
  {
    const bf16* kr = Kp + (int64_t)keyc * ld + hh * 8;
    const bf16* vr = Vp + (int64_t)keyc * ld + hh * 8;
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) {
      kf[kk] = *reinterpret_cast<const bf16x8*>(kr + kk * 16);
      vf[kk] = *reinterpret_cast<const bf16x8*>(vr + kk * 16);
    }
  }
  f32x16 dk[NC], dv[NC];
#pragma unroll
  for (int c = 0; c < NC; ++c) { dk[c] = zero16(); dv[c] = zero16(); }
  // Mask bias.  Accumulator register r = 4g+e of a tile that starts at query qs is query qs + 8g + 4hh + e.
  // On the tile that starts at this wavefront's first key it sees this lane's key iff lk - 4hh <= 8g + e;
  // later tiles see every key, earlier ones none.  bias = diag[r] * sel with diag = -1e30 (hidden on the
  // diagonal tile) or -1e-30, and sel = 0 (later tile), 1 (diagonal: -1e-30 vanishes beside any score) or
  // 1e38 (earlier tile: every entry ends below -1e8, and exp gives 0).
  f32x16 diag;
#pragma unroll
  for (int r = 0; r < 16; ++r) diag[r] = (lk - 4 * hh > 8 * (r / 4) + r % 4) ? -1e30f : -1e-30f;

  // the walk: query heads a of this kv head, for each the query tiles qt0 .. nqt-1
  const int qt0 = k0 / BQ, nqt = (T + BQ - 1) / BQ;
  const int steps = (nqt - qt0) * rep;
  struct Walk { int a, qt, left; };
  auto advance = [&](Walk& w) {
    const bool wrap = w.qt == nqt - 1;
    w.qt = wrap ? qt0 : w.qt + 1;
    w.a = min(wrap ? w.a + 1 : w.a, H - 1);   // past the end: any valid head, the tile counts for nothing
    w.left -= 1;
  };
  typedef Stage<HD, BQ> SQ;
  u32x4 rq[SQ::NCH], rdo[SQ::NCH];
  float st_l = 0.f, st_d = 0.f;
  bool st_live = false;
  // Q and dO of this sequence behind buffer descriptors: rows past T read as zero
  const uint32_t q_row = (uint32_t)ld * 2u, do_row = (uint32_t)H * HD * 2u;
  const rsrc_t q_rs = make_rsrc(qkv + (int64_t)b * T * ld, (uint32_t)(((int64_t)(T - 1) * ld + (int64_t)H * HD) * 2));
  const rsrc_t do_rs = make_rsrc(dO + (int64_t)b * T * H * HD, (uint32_t)((int64_t)T * H * HD * 2));
  // loads only: nothing here may touch a loaded value, or the wavefront would wait for memory on the spot
  auto load_tile = [&](const Walk& w) {
    const int qs = w.qt * BQ;
    SQ::bload(rq, q_rs, q_row, (uint32_t)qs * q_row + (uint32_t)w.a * HD * 2u, tid);
    SQ::bload(rdo, do_rs, do_row, (uint32_t)qs * do_row + (uint32_t)w.a * HD * 2u, tid);
    const int qi = qs + (tid & (BQ - 1));
    const int64_t at = ((int64_t)b * H + w.a) * T + min(qi, T - 1);
    st_l = lse[at];
    st_d = delta[at];
    st_live = qi < T && w.left > 0;
  };
  auto store_tile = [&](int boff) {
    char* base = smem + boff;
    SQ::store(rq, base, QS, tid);
    SQ::store(rdo, base + kDO, QS, tid);
    SQ::store(rq, base + kQT, TS, tid);
    SQ::store(rdo, base + kDOT, TS, tid);
    // a row past the end of the sequence, or a tile past the end of the walk, gets lse = +inf:
    // its probabilities are exactly zero
    const float nl = -st_l * inv_scale;
    reinterpret_cast<float*>(base + kNL)[tid] = st_live ? nl : -INFINITY;
    reinterpret_cast<float*>(base + kND)[tid] = -st_d;
  };
  // phase 1 operands of the tile in buffer boff, which starts at query qs: f[2kk] = Q, f[2kk+1] = dO
  // (A operand: row = query lk), and the initial accumulators
  auto read_phase1 = [&](int boff, int qs, bf16x8 (&f)[2 * NK], f32x16& s, f32x16& dp) {
    const char* base = smem + boff + lk * QS + hh * 16;
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) {
      f[2 * kk] = *reinterpret_cast<const bf16x8*>(base + kk * 32);
      f[2 * kk + 1] = *reinterpret_cast<const bf16x8*>(base + kDO + kk * 32);
    }
    const float sel = qs == kw0 ? 1.f : (qs < kw0 ? 1e38f : 0.f);
    const float* pl = reinterpret_cast<const float*>(smem + boff + kNL) + hh * 4;
    const float* pd = reinterpret_cast<const float*>(smem + boff + kND) + hh * 4;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float4 l = *reinterpret_cast<const float4*>(pl + g * 8);
      const float4 d = *reinterpret_cast<const float4*>(pd + g * 8);
      s[4 * g] = __builtin_fmaf(diag[4 * g], sel, l.x);
      s[4 * g + 1] = __builtin_fmaf(diag[4 * g + 1], sel, l.y);
      s[4 * g + 2] = __builtin_fmaf(diag[4 * g + 2], sel, l.z);
      s[4 * g + 3] = __builtin_fmaf(diag[4 * g + 3], sel, l.w);
      dp[4 * g] = d.x; dp[4 * g + 1] = d.y; dp[4 * g + 2] = d.z; dp[4 * g + 3] = d.w;
    }
  };
  auto phase1 = [&](const bf16x8 (&f)[2 * NK], f32x16& s, f32x16& dp) {
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) {
      s = mfma(f[2 * kk], kf[kk], s);
      dp = mfma(f[2 * kk + 1], vf[kk], dp);
    }
  };

  Walk w_ld = {kvh * rep, qt0, steps}, w_nx = w_ld;   // next tile to load; next tile whose phase 1 operands are read
  int b0 = 0, b1 = kBuf, b2 = 2 * kBuf;
  load_tile(w_ld); advance(w_ld);
  store_tile(b0);
  load_tile(w_ld); advance(w_ld);
  store_tile(b1);
  load_tile(w_ld); advance(w_ld);
  __syncthreads();
  bf16x8 f1[2 * NK];
  f32x16 s_a, dp_a, s_b, dp_b;
  read_phase1(b0, w_nx.qt * BQ, f1, s_a, dp_a); advance(w_nx);
  phase1(f1, s_a, dp_a);
  read_phase1(b1, w_nx.qt * BQ, f1, s_b, dp_b); advance(w_nx);

  // one iteration: tile i's phase 1 result in (s_c, dp_c); tile i+1's initial accumulators in (s_n, dp_n)
  // and its operands in f1.  On return (s_n, dp_n) hold tile i+1's result, (s_c, dp_c) tile i+2's start.
  auto iteration = [&](f32x16& s_c, f32x16& dp_c, f32x16& s_n, f32x16& dp_n) {
    // ---- top: tile i+2 into its buffer, tile i+3 on its way
    store_tile(b2);
    load_tile(w_ld); advance(w_ld);
    __builtin_amdgcn_sched_barrier(0);
    // ---- first half, in NK slots fenced from each other: two MFMAs of tile i+1's phase 1, 16/NK
    // elements of tile i's phase 2, two of the 2 NK operand fragments of tile i's phase 3
    constexpr int EPS = 16 / NK;   // elements per slot: 2 (hd 128) or 4 (hd 64)
    bf16x8 pf[2], dsf[2];
    bf16x8 f3[2 * NK];             // in the order phase 3 uses them
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) {
      s_n = mfma(f1[2 * kk], kf[kk], s_n);
      dp_n = mfma(f1[2 * kk + 1], vf[kk], dp_n);
#pragma unroll
      for (int j = 0; j < EPS; ++j) {
        const int r = EPS * kk + j;
        const float pv = __builtin_amdgcn_exp2f(s_c[r] * scale_log2);
        pf[r / 8][r % 8] = (bf16)pv;
        dsf[r / 8][r % 8] = (bf16)(pv * dp_c[r]);
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        // fragment m = (u * 2 + which) * NC + c: which 0 = dO^T (for dV), 1 = Q^T (for dK)
        const int m = 2 * kk + j, c = m % NC, which = (m / NC) & 1, u = m / (2 * NC);
        f3[m] = read_tr(smem + b0 + (which ? kQT : kDOT), TS, c * 32, 16 * u, lane);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();
    // ---- second half, likewise: two MFMAs of phase 3, two operand fragments of tile i+2's phase 1, and
    // in the first four slots a quarter of its initial accumulators
    {
      const int qs = w_nx.qt * BQ;
      const float sel = qs == kw0 ? 1.f : (qs < kw0 ? 1e38f : 0.f);
      const char* base = smem + b2 + lk * QS + hh * 16;
      const float* pl = reinterpret_cast<const float*>(smem + b2 + kNL) + hh * 4;
      const float* pd = reinterpret_cast<const float*>(smem + b2 + kND) + hh * 4;
      float4 l4[4], d4[4];
      auto init_group = [&](int g) {
        s_c[4 * g] = __builtin_fmaf(diag[4 * g], sel, l4[g].x);
        s_c[4 * g + 1] = __builtin_fmaf(diag[4 * g + 1], sel, l4[g].y);
        s_c[4 * g + 2] = __builtin_fmaf(diag[4 * g + 2], sel, l4[g].z);
        s_c[4 * g + 3] = __builtin_fmaf(diag[4 * g + 3], sel, l4[g].w);
        dp_c[4 * g] = d4[g].x; dp_c[4 * g + 1] = d4[g].y; dp_c[4 * g + 2] = d4[g].z; dp_c[4 * g + 3] = d4[g].w;
      };
#pragma unroll
      for (int kk = 0; kk < NK; ++kk) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int m = 2 * kk + j, c = m % NC, which = (m / NC) & 1, u = m / (2 * NC);
          if (which) dk[c] = mfma(f3[m], dsf[u], dk[c]);
          else dv[c] = mfma(f3[m], pf[u], dv[c]);
        }
        f1[2 * kk] = *reinterpret_cast<const bf16x8*>(base + kk * 32);
        f1[2 * kk + 1] = *reinterpret_cast<const bf16x8*>(base + kDO + kk * 32);
        if (kk < 4) {
          l4[kk] = *reinterpret_cast<const float4*>(pl + kk * 8);
          d4[kk] = *reinterpret_cast<const float4*>(pd + kk * 8);
        }
        if (kk >= 1 && kk <= 4) init_group(kk - 1);   // a slot after its reads: their latency is covered
        __builtin_amdgcn_sched_barrier(0);
      }
      if (NK <= 4) init_group(3);
      advance(w_nx);
    }
    const int t = b0; b0 = b1; b1 = b2; b2 = t;
  };
  for (int step = 0; step < steps; step += 2) {
    iteration(s_a, dp_a, s_b, dp_b);
    iteration(s_b, dp_b, s_a, dp_a);
  }
  if (key < T) {
    bf16* krow = dqkv + ((int64_t)b * T + key) * ld + (H + kvh) * HD;
    bf16* vrow = dqkv + ((int64_t)b * T + key) * ld + (H + Hkv + kvh) * HD;
#pragma unroll
    for (int c = 0; c < NC; ++c)
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
