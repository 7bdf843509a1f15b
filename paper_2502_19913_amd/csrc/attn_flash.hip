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
// the accumulator's own order; the LDS-side operand is read in the matching order.
//
// Layout: qkv rows of (H + 2*Hkv)*hd = queries | keys | values; o rows of H*hd; lse, delta [B][H][T].
#include "devutil.h"
#include "internal.h"

namespace sp {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

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

// LDS operand that pairs with pack8: row `row` of a [*][rows-contiguous] tile, the 8 entries at
// offsets base + hh*4 + {0..3} and base + 8 + hh*4 + {0..3}   (two 8-byte reads)
__device__ __forceinline__ bf16x8 read_slots(const char* tile, int stride_bytes, int row, int base, int hh) {
  const char* p = tile + row * stride_bytes + (base + hh * 4) * 2;
  uint2 a = *reinterpret_cast<const uint2*>(p);
  uint2 b = *reinterpret_cast<const uint2*>(p + 16);
  uint4 w = make_uint4(a.x, a.y, b.x, b.y);
  return __builtin_bit_cast(bf16x8, w);
}

// ---- staging of a [rows x HD] block of a row-major matrix (row stride ld elements) ----------------
// 4 rows x 8 columns per thread.  KQ_FAST: consecutive lanes take consecutive row quads (good for
// the transposed LDS store), else consecutive column blocks (good for the row-major store).
template <int HD, int ROWS, bool KQ_FAST>
struct Stage {
  static constexpr int kColBlocks = HD / 8, kRowQuads = ROWS / 4;
  static constexpr int kBlocks = kColBlocks * kRowQuads;  // may be below or above the thread count
  uint4 reg[(kBlocks + 255) / 256][4];

  __device__ __forceinline__ static void split(int blk, int& rq, int& cb) {
    if (KQ_FAST) { rq = blk % kRowQuads; cb = blk / kRowQuads; } else { cb = blk % kColBlocks; rq = blk / kColBlocks; }
  }
  __device__ __forceinline__ void load(const bf16* __restrict__ X, int64_t ld, int row0, int row_max, int tid) {
#pragma unroll
    for (int n = 0; n < (kBlocks + 255) / 256; ++n) {
      const int blk = tid + 256 * n;
      if (blk < kBlocks) {
        int rq, cb;
        split(blk, rq, cb);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int r = min(row0 + rq * 4 + i, row_max);
          reg[n][i] = *reinterpret_cast<const uint4*>(X + (int64_t)r * ld + cb * 8);
        }
      }
    }
  }
  // tile[row][col], row stride in bytes
  __device__ __forceinline__ void store_rows(char* tile, int stride, int tid) const {
#pragma unroll
    for (int n = 0; n < (kBlocks + 255) / 256; ++n) {
      const int blk = tid + 256 * n;
      if (blk < kBlocks) {
        int rq, cb;
        split(blk, rq, cb);
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4*>(tile + (rq * 4 + i) * stride + cb * 16) = reg[n][i];
      }
    }
  }
  // tile[col][row], row stride in bytes
  __device__ __forceinline__ void store_cols(char* tile, int stride, int tid) const {
#pragma unroll
    for (int n = 0; n < (kBlocks + 255) / 256; ++n) {
      const int blk = tid + 256 * n;
      if (blk < kBlocks) {
        int rq, cb;
        split(blk, rq, cb);
        const uint32_t w[4][4] = {{reg[n][0].x, reg[n][0].y, reg[n][0].z, reg[n][0].w},
                                  {reg[n][1].x, reg[n][1].y, reg[n][1].z, reg[n][1].w},
                                  {reg[n][2].x, reg[n][2].y, reg[n][2].z, reg[n][2].w},
                                  {reg[n][3].x, reg[n][3].y, reg[n][3].z, reg[n][3].w}};
#pragma unroll
        for (int c = 0; c < 8; ++c) {
          const int j = c >> 1;
          uint2 o;
          if (c & 1) {
            o.x = (w[0][j] >> 16) | (w[1][j] & 0xffff0000u);
            o.y = (w[2][j] >> 16) | (w[3][j] & 0xffff0000u);
          } else {
            o.x = (w[0][j] & 0xffffu) | (w[1][j] << 16);
            o.y = (w[2][j] & 0xffffu) | (w[3][j] << 16);
          }
          *reinterpret_cast<uint2*>(tile + (cb * 8 + c) * stride + rq * 8) = o;
        }
      }
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
  constexpr int VS = BKV * 2 + 8;   // V^T tile row stride (bytes): [hd][key]
  constexpr int kKTile = BKV * KS, kVTile = HD * VS;
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
  Stage<HD, BKV, false> sk;
  Stage<HD, BKV, true> sv;
  sk.load(Kp, ld, 0, T - 1, tid);
  sv.load(Vp, ld, 0, T - 1, tid);
  sk.store_rows(smem, KS, tid);
  sv.store_cols(smem + kKTile, VS, tid);
  __syncthreads();
  for (int kt = 0; kt < ntiles; ++kt) {
    const int k0 = kt * BKV;
    const bool more = kt + 1 < ntiles;
    if (more) {
      sk.load(Kp, ld, k0 + BKV, T - 1, tid);
      sv.load(Vp, ld, k0 + BKV, T - 1, tid);
    }
    const char* ks = smem + (kt & 1) * (kKTile + kVTile);
    const char* vs = ks + kKTile;
    if (k0 <= qw0 + 31) {  // the tile holds a key some query of this wavefront may see
      f32x16 st[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        st[t] = zero16();
        const char* kr = ks + (t * 32 + lq) * KS + hh * 16;
#pragma unroll
        for (int kk = 0; kk < HD / 16; ++kk) st[t] = mfma(*reinterpret_cast<const bf16x8*>(kr + kk * 32), qf[kk], st[t]);
      }
      const bool mask = k0 + BKV - 1 > qw0;
      float mx = -INFINITY;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float s = st[t][r] * scale_log2;
          if (mask) {
            const int key = k0 + t * 32 + (r >> 2) * 8 + hh * 4 + (r & 3);
            if (key > q) s = -INFINITY;
          }
          st[t][r] = s;
          mx = fmaxf(mx, s);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_i, mx);           // finite: tile 0 holds key 0, visible to every query
      const float alpha = exp2f(m_i - m_new);
      float rs = 0.f;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = exp2f(st[t][r] - m_new);
          st[t][r] = p;
          rs += p;
        }
      l_i = l_i * alpha + rs;
      m_i = m_new;
#pragma unroll
      for (int c = 0; c < HD / 32; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[c][r] *= alpha;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const bf16x8 pf = pack8(st[t], u);
#pragma unroll
          for (int c = 0; c < HD / 32; ++c)
            oacc[c] = mfma(read_slots(vs, VS, c * 32 + lq, t * 32 + 16 * u, hh), pf, oacc[c]);
        }
    }
    if (more) {
      char* nk = smem + ((kt + 1) & 1) * (kKTile + kVTile);
      sk.store_rows(nk, KS, tid);
      sv.store_cols(nk + kKTile, VS, tid);
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
  constexpr int TS = BKV * 2 + 8;   // K^T tile [hd][key]
  constexpr int kKTile = BKV * KS, kTTile = HD * TS;
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
  Stage<HD, BKV, true> sk;
  Stage<HD, BKV, false> sv;
  sk.load(Kp, ld, 0, T - 1, tid);
  sv.load(Vp, ld, 0, T - 1, tid);
  for (int kt = 0; kt < ntiles; ++kt) {
    const int k0 = kt * BKV;
    sk.store_rows(ks, KS, tid);
    sk.store_cols(kts, TS, tid);
    sv.store_rows(vs, KS, tid);
    __syncthreads();
    if (kt + 1 < ntiles) {
      sk.load(Kp, ld, k0 + BKV, T - 1, tid);
      sv.load(Vp, ld, k0 + BKV, T - 1, tid);
    }
    if (k0 <= qw0 + 31) {
      const bool mask = k0 + BKV - 1 > qw0;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        f32x16 st = zero16(), dp = zero16();
        const char* kr = ks + (t * 32 + lq) * KS + hh * 16;
        const char* vr = vs + (t * 32 + lq) * KS + hh * 16;
#pragma unroll
        for (int kk = 0; kk < HD / 16; ++kk) st = mfma(*reinterpret_cast<const bf16x8*>(kr + kk * 32), qf[kk], st);
#pragma unroll
        for (int kk = 0; kk < HD / 16; ++kk) dp = mfma(*reinterpret_cast<const bf16x8*>(vr + kk * 32), dof[kk], dp);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float p = exp2f(st[r] * scale_log2 - lse2);
          if (mask) {
            const int key = k0 + t * 32 + (r >> 2) * 8 + hh * 4 + (r & 3);
            if (key > q) p = 0.f;
          }
          st[r] = p * (dp[r] - dlt);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const bf16x8 dsf = pack8(st, u);
#pragma unroll
          for (int c = 0; c < HD / 32; ++c)
            dq[c] = mfma(read_slots(kts, TS, c * 32 + lq, t * 32 + 16 * u, hh), dsf, dq[c]);
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
  constexpr int TS = BQ * 2 + 8;    // Q^T and dO^T tiles [hd][query]
  constexpr int kQTile = BQ * QS, kTTile = HD * TS;
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
  Stage<HD, BQ, true> sq, sdo;
  float st_lse = 0.f, st_dlt = 0.f;
  auto load_step = [&](int step) {
    const int a = kvh * rep + step / per_head;
    const int qs = (qt0 + step % per_head) * BQ;
    sq.load(qkv + (int64_t)b * T * ld + a * HD, ld, qs, T - 1, tid);
    sdo.load(dO + (int64_t)b * T * H * HD + a * HD, (int64_t)H * HD, qs, T - 1, tid);
    if (tid < BQ) {
      const int qi = min(qs + tid, T - 1);
      st_lse = lse[((int64_t)b * H + a) * T + qi] * kLog2e;
      st_dlt = delta[((int64_t)b * H + a) * T + qi];
    }
  };
  auto store_step = [&](int buf) {
    char* base = smem + buf * kBuf;
    sq.store_rows(base, QS, tid);
    sdo.store_rows(base + kQTile, QS, tid);
    sq.store_cols(base + 2 * kQTile, TS, tid);
    sdo.store_cols(base + 2 * kQTile + kTTile, TS, tid);
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
    const bool more = step + 1 < steps;
    if (more) load_step(step + 1);
    const int qs = (qt0 + step % per_head) * BQ;
    const char* base = smem + (step & 1) * kBuf;
    if (qs + BQ - 1 >= kw0) {  // some query of the tile sees a key of this wavefront
      const char* qsm = base;
      const char* dosm = base + kQTile;
      const char* qts = base + 2 * kQTile;
      const char* dots = qts + kTTile;
      const float* s_lse = reinterpret_cast<const float*>(base + 2 * kQTile + 2 * kTTile);
      const float* s_dlt = s_lse + BQ;
      f32x16 s = zero16(), dp = zero16();
      const char* qr = qsm + lk * QS + hh * 16;     // A operand: row = query lk of the tile
      const char* dr = dosm + lk * QS + hh * 16;
#pragma unroll
      for (int kk = 0; kk < HD / 16; ++kk) s = mfma(*reinterpret_cast<const bf16x8*>(qr + kk * 32), kf[kk], s);
#pragma unroll
      for (int kk = 0; kk < HD / 16; ++kk) dp = mfma(*reinterpret_cast<const bf16x8*>(dr + kk * 32), vf[kk], dp);
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
          float pv = exp2f(s[r] * scale_log2 - lv[e]);
          if (mask && key > qs + qi + e) pv = 0.f;
          if (qs + qi + e >= T) pv = 0.f;     // rows past the end of the sequence are re-reads of row T-1
          p[r] = pv;
          s[r] = pv * (dp[r] - dv4[e]);
        }
      }
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const bf16x8 pf = pack8(p, u), dsf = pack8(s, u);
#pragma unroll
        for (int c = 0; c < HD / 32; ++c) {
          dv[c] = mfma(read_slots(dots, TS, c * 32 + lk, 16 * u, hh), pf, dv[c]);
          dk[c] = mfma(read_slots(qts, TS, c * 32 + lk, 16 * u, hh), dsf, dk[c]);
        }
      }
    }
    if (more) store_step((step + 1) & 1);
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
