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
#include <type_traits>

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

// LDS operand that pairs with pack8, gathered from a row-major [row][col] tile with the LDS transpose read:
// MFMA row (lane % 32) = tile column col_base + lane % 32, and the 8 k-slots of lane half hh = tile rows
// row_base + hh*4 + {0..3} and row_base + 8 + hh*4 + {0..3}.  (ds_read_b64_tr_b16: within 16 lanes, lane i
// receives element i%4 of the 8-byte pieces addressed by lanes i/4, i/4+4, i/4+8, i/4+12; here piece s of a
// group is row s/4, columns 4*(s%4)..+3.)  The kernels below form the two addresses of such an operand from
// per-lane constants (p3_base) of the permuted tile layout.
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

// Workgroups are dealt to the 8 XCDs (each with its own L2) in turn: linear id L runs on XCD L % 8.
// Longest blocks first over the whole launch: linear id L -> (level, sequence, head) with the level (which
// query or key block of the causal triangle, i.e. how much work) changing slowest, so the heaviest blocks of
// all heads start first and the light ones fill the tail (a launch has a few blocks per CU and their costs differ
// by the number of blocks of the triangle's side).  Within a level, ids that land on one XCD get neighbouring
// heads (the query heads of one kv group when the head count is a multiple of 8): the K/V (or Q/dO) rows a
// head streams are then re-read, level after level, through the same L2.
struct BlockId { int level, b, a; };
__device__ __forceinline__ BlockId heavy_first(int L, int B, int H) {
  const int per_level = B * H, level = L / per_level, j = L - level * per_level;
  if (H % 8 == 0) {
    const int g = j % 8, r = j / 8, hx = H / 8;
    return {level, r / hx, g * hx + r % hx};
  }
  return {level, j / H, j % H};
}

// Gradient of a rotated vector -> gradient of the vector before the rotation, for 4 consecutive columns
// col..col+3 (two pairs) of the head-dimension at position pos: the transpose of the rotation, i.e. a turn
// by the opposite angle.  tab holds (cos, sin) per (position, pair).
__device__ __forceinline__ void unrotate4(float (&v)[4], const float* __restrict__ tab, int pos, int hd, int col) {
  const float4 cs = *reinterpret_cast<const float4*>(tab + ((int64_t)pos * (hd / 2) + col / 2) * 2);
  const float a0 = v[0], b0 = v[1], a1 = v[2], b1 = v[3];
  v[0] = a0 * cs.x + b0 * cs.y;
  v[1] = b0 * cs.x - a0 * cs.y;
  v[2] = a1 * cs.z + b1 * cs.w;
  v[3] = b1 * cs.z - a1 * cs.w;
}

// Geometry of the unpadded row-major [rows][HD] tiles that direct-to-LDS loads fill (used by the ring forward
// kernel for K and V and by the dK/dV kernel for Q and dO), with the chunk permutation that makes row-wise
// and transpose reads of such a tile free of bank conflicts.
template <int HD>
struct DkvGeom {
  static constexpr int BQ = 32, NK = HD / 16, NC = HD / 32;
  static constexpr int RB = HD * 2;            // bytes per tile row
  static constexpr int CPR = HD / 8;           // 16-byte chunks per row
  static constexpr int kTile = BQ * RB;
  static constexpr int NJ = kTile / 4096;      // tile loads per thread and matrix (256 threads x 16 bytes each)
  static constexpr int kDO = kTile, kL = 2 * kTile, kD = kL + 1024, kBuf = kD + 1024;
  static constexpr int kDepth = 4, kRing = kDepth + 1;
  static constexpr int NI = 2 * NJ + 2;        // load instructions per thread and tile
  // chunk permutation key of a row: distinct over 16 consecutive rows (aligned), and over rows 4m..4m+3
  // distinct in the bits above the two lowest
  __device__ __forceinline__ static int key(int row) {
    return HD == 128 ? ((row & 3) << 2) | ((row >> 2) & 3) : (((row >> 1) & 1) << 2) | ((row >> 2) & 3);
  }
};

// ================================================================================ forward
// Workgroup: 128 queries of one (sequence, head), 4 wavefronts x 32 queries; key/value tiles of 64.
// Per tile and wavefront: S^T[key][query] = K Q^T, online softmax down each lane's query,
// O^T[col][query] += V^T P^T.
// The key / value tiles go from memory straight into LDS (buffer loads with the LDS modifier, as in the dK/dV
// kernel below: unpadded row-major tiles whose 16-byte chunks are permuted by DkvGeom::key, which serves the
// row-wise reads of K and the transpose reads of V alike) and are kept in rings, three tiles of K and two of V:
// no staging registers and no LDS stores, and the scores of tile i+1 are formed while tile i goes through its
// softmax, one matrix instruction and its share of the exponentials at a time, so a wavefront has matrix work
// in flight during its arithmetic.  Loads issued in an iteration are waited for (vmcnt, by hand) at its end,
// before the barrier that also frees the buffers read in it.  Keys past the end of the sequence read as zeros
// (offsets beyond the descriptor) and are masked.  Against the kernel this replaced (tiles staged through
// registers into two padded LDS buffers, scores and softmax in sequence): 8 - 10 % faster.
template <int HD>
__global__ __launch_bounds__(256, 2) void k_flash_fwd(const bf16* __restrict__ qkv, bf16* __restrict__ o,
                                                           float* __restrict__ lse, int T, int H, int Hkv, float scale_log2) {
  typedef DkvGeom<HD> G;
  constexpr int BQ = 128, BKV = 64, RB = G::RB, CPR = G::CPR;
  constexpr int kTile = BKV * RB;          // one tile of K or V
  constexpr int NJ = kTile / 4096;         // load instructions per wavefront and tile
  constexpr int NK = HD / 16, NC = HD / 32;
  __shared__ __attribute__((aligned(1024))) char smem[5 * kTile];
  char* const k_ring = smem;               // 3 tiles
  char* const v_ring = smem + 3 * kTile;   // 2 tiles
  const int tid = threadIdx.x, lane = tid & 63, lq = lane & 31, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nqb = (T + 127) / 128;
  const BlockId id = heavy_first(blockIdx.x, (int)gridDim.x / (nqb * H), H);   // heaviest query blocks first
  const int qb = nqb - 1 - id.level, a = id.a, b = id.b;
  const int kvh = a / (H / Hkv);
  const int64_t ld = (int64_t)(H + 2 * Hkv) * HD;
  const bf16* Q = qkv + (int64_t)b * T * ld + a * HD;
  const int q0 = qb * BQ, qw0 = q0 + wave * 32, q = qw0 + lq;

  bf16x8 qf[NK];
  {
    const bf16* qr = Q + (int64_t)min(q, T - 1) * ld + hh * 8;
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qr + kk * 16);
  }
  f32x16 oacc[NC];
#pragma unroll
  for (int c = 0; c < NC; ++c) oacc[c] = zero16();
  float m_i = -INFINITY, l_i = 0.f;

  const int kv_end = min(T, q0 + BQ);
  const int ntiles = (kv_end + BKV - 1) / BKV;

  // ---- tile loads: instruction j of this wavefront fills chunks (4j + wave) * 64 + lane of a tile; the chunk at
  // row, position p holds the row's chunk p ^ key(row)
  const uint32_t row_bytes = (uint32_t)ld * 2u;
  uint32_t ldo[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int c = (4 * j + wave) * 64 + lane, row = c / CPR, pos = c % CPR;
    ldo[j] = (uint32_t)row * row_bytes + (uint32_t)((pos ^ G::key(row)) << 4);
  }
  const u32x4 rs = make_desc(qkv + (int64_t)b * T * ld, (uint32_t)((int64_t)T * ld * 2));   // this sequence's rows
  const uint32_t k_col = (uint32_t)(H + kvh) * HD * 2u, v_col = (uint32_t)(H + Hkv + kvh) * HD * 2u;
  auto load_k = [&](int kt) {
    char* dst = k_ring + (kt % 3) * kTile;
    const uint32_t off = (uint32_t)kt * BKV * row_bytes + k_col;
#pragma unroll
    for (int j = 0; j < NJ; ++j) load_to_lds16(rs, (lds_ptr)(dst + (4 * j + wave) * 1024), ldo[j] + off);
  };
  auto load_v = [&](int kt) {
    char* dst = v_ring + (kt & 1) * kTile;
    const uint32_t off = (uint32_t)kt * BKV * row_bytes + v_col;
#pragma unroll
    for (int j = 0; j < NJ; ++j) load_to_lds16(rs, (lds_ptr)(dst + (4 * j + wave) * 1024), ldo[j] + off);
  };
  auto landed_barrier = [&]() {
    __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (0 << 8));   // vmcnt(0) lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
  };
  // ---- lane constants of the LDS reads
  // K, row-wise: key row lq (+32 for the tile's second half), chunk 2 kk + hh permuted; kk enters by XOR with kk * 32
  const int p1_base = lq * RB + ((hh ^ G::key(lq)) << 4);
  // V, transpose reads (see pack8): rows 16 tu + 8 hi + 4 hh + i, chunks 4 c + w; c enters by XOR with c * 64
  int p3_base[2];
  {
    const int sl = lane & 15, i = sl >> 2, w = ((lane >> 4) & 1) * 2 + ((sl & 3) >> 1), half = sl & 1;
#pragma unroll
    for (int hi = 0; hi < 2; ++hi) {
      const int row = 8 * hi + 4 * hh + i;
      p3_base[hi] = row * RB + (((G::key(row) & 12) | (w ^ (G::key(row) & 3))) << 4) + half * 8;
    }
  }
  typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
  auto read_v = [&](const char* vt, int tu, int c) {
    const char* base = vt + 16 * tu * RB;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(base + (p3_base[0] ^ (c * 64))));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(base + (p3_base[1] ^ (c * 64))));
    const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
  };
  // S^T = K Q^T of tile kt on two accumulators (32 keys each)
  auto scores = [&](int kt, f32x16 (&st)[2]) {
    const char* kt_base = k_ring + (kt % 3) * kTile;
    st[0] = zero16();
    st[1] = zero16();
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) {
      const char* p = kt_base + (p1_base ^ (kk * 32));
      const bf16x8 f0 = *reinterpret_cast<const bf16x8*>(p);
      const bf16x8 f1 = *reinterpret_cast<const bf16x8*>(p + 32 * RB);
      st[0] = mfma(f0, qf[kk], st[0]);
      st[1] = mfma(f1, qf[kk], st[1]);
    }
  };

  load_k(0);
  load_v(0);
  if (ntiles > 1) load_k(1);
  landed_barrier();
  f32x16 s_next[2];
  scores(0, s_next);

  auto tile_step = [&](int kt, auto masked_tag) {
    constexpr bool MASKED = decltype(masked_tag)::value;
    const int k0 = kt * BKV;
    f32x16 st[2] = {s_next[0], s_next[1]};
    // The buffers these go to were last read in the iteration before, which ended at a barrier.  No branches
    // here, so that the compiler may weave the next tile's products into this tile's softmax: past the last
    // tile the loads fetch rows nobody reads (or zeros past the end of the sequence) and the scores are dropped.
    load_v(kt + 1);
    load_k(kt + 2);
    float mx = -INFINITY;
    if (MASKED) {
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
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
      for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[c][r] *= alpha;
    }
    // From here to the barrier one straight block.  First the next tile's products beside this tile's
    // exponentials, in slots of one matrix instruction followed by its share of the arithmetic (a wavefront's
    // arithmetic overlaps only the matrix instruction issued just before it), fenced so the order holds.
    {
      constexpr int EPS = 32 / (2 * NK);   // exponentials per matrix instruction
      const char* kn = k_ring + ((kt + 1) % 3) * kTile;
      s_next[0] = zero16();
      s_next[1] = zero16();
      bf16x8 kf[2][2];
      kf[0][0] = *reinterpret_cast<const bf16x8*>(kn + p1_base);
      kf[0][1] = *reinterpret_cast<const bf16x8*>(kn + p1_base + 32 * RB);
      float rsum = 0.f;
      auto exps = [&](int e0) {
#pragma unroll
        for (int e = e0; e < e0 + EPS; ++e) {
          float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(st[e >> 4][e & 15], scale_log2, -m_new));
          asm volatile("" : "+v"(pv));   // holds the exponential in its slot: arithmetic without side effects is
                                         // otherwise placed where its result is first needed, after all the slots
          st[e >> 4][e & 15] = pv;
          rsum += pv;
        }
      };
#pragma unroll
      for (int kk = 0; kk < NK; ++kk) {
        if (kk + 1 < NK) {
          const char* p = kn + (p1_base ^ ((kk + 1) * 32));
          kf[(kk + 1) & 1][0] = *reinterpret_cast<const bf16x8*>(p);
          kf[(kk + 1) & 1][1] = *reinterpret_cast<const bf16x8*>(p + 32 * RB);
        }
        __builtin_amdgcn_sched_barrier(0);
        s_next[0] = mfma(kf[kk & 1][0], qf[kk], s_next[0]);
        exps(2 * kk * EPS);
        __builtin_amdgcn_sched_barrier(0);
        s_next[1] = mfma(kf[kk & 1][1], qf[kk], s_next[1]);
        exps((2 * kk + 1) * EPS);
        __builtin_amdgcn_sched_barrier(0);
      }
      l_i = l_i * alpha + rsum;
      m_i = m_new;
    }
    const char* vt = v_ring + (kt & 1) * kTile;
#pragma unroll
    for (int tu = 0; tu < 4; ++tu) {
      const bf16x8 pf = pack8(st[tu >> 1], tu & 1);
#pragma unroll
      for (int c = 0; c < NC; ++c) oacc[c] = mfma(read_v(vt, tu, c), pf, oacc[c]);
    }
    landed_barrier();
  };
  // tiles that end before the workgroup's first query need no mask: their arithmetic is a third shorter
  const int n_free = min(ntiles, q0 / BKV);
  for (int kt = 0; kt < n_free; ++kt) tile_step(kt, std::false_type());
  for (int kt = n_free; kt < ntiles; ++kt) tile_step(kt, std::true_type());
  const float l_tot = l_i + __shfl_xor(l_i, 32);
  if (q < T) {
    const float inv = 1.0f / l_tot;
    bf16* orow = o + ((int64_t)b * T + q) * H * HD + a * HD;
#pragma unroll
    for (int c = 0; c < NC; ++c)
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
// K and V tiles arrive as in the forward kernel (direct-to-LDS loads into rings of two tiles each, one barrier per
// tile); the one copy of a K tile serves both the row-wise reads of the first product and the transpose reads of
// the last (DkvGeom::key).
template <int HD>
__global__ __launch_bounds__(256, 2) void k_flash_bwd_dq(const bf16* __restrict__ qkv, const bf16* __restrict__ dO,
                                                         const float* __restrict__ lse, const float* __restrict__ delta,
                                                         bf16* __restrict__ dqkv, int T, int H, int Hkv, float scale,
                                                         const float* __restrict__ rope_tab) {
  typedef DkvGeom<HD> G;
  constexpr int BQ = 128, BKV = 64, RB = G::RB, CPR = G::CPR;
  constexpr int kTile = BKV * RB;
  constexpr int NJ = kTile / 4096;
  constexpr int NK = HD / 16, NC = HD / 32;
  __shared__ __attribute__((aligned(1024))) char smem[4 * kTile];
  char* const k_ring = smem;
  char* const v_ring = smem + 2 * kTile;
  const int tid = threadIdx.x, lane = tid & 63, lq = lane & 31, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nqb = (T + 127) / 128;
  const BlockId id = heavy_first(blockIdx.x, (int)gridDim.x / (nqb * H), H);   // heaviest query blocks first
  const int qb = nqb - 1 - id.level, a = id.a, b = id.b;
  const int kvh = a / (H / Hkv);
  const int64_t ld = (int64_t)(H + 2 * Hkv) * HD;
  const bf16* Q = qkv + (int64_t)b * T * ld + a * HD;
  const int q0 = qb * BQ, qw0 = q0 + wave * 32, q = qw0 + lq, qc = min(q, T - 1);
  const float scale_log2 = scale * kLog2e;

  bf16x8 qf[NK], dof[NK];
  {
    const bf16* qr = Q + (int64_t)qc * ld + hh * 8;
    const bf16* dr = dO + ((int64_t)b * T + qc) * H * HD + a * HD + hh * 8;
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) {
      qf[kk] = *reinterpret_cast<const bf16x8*>(qr + kk * 16);
      dof[kk] = *reinterpret_cast<const bf16x8*>(dr + kk * 16);
    }
  }
  const float lse2 = lse[((int64_t)b * H + a) * T + qc] * kLog2e;
  const float dlt = delta[((int64_t)b * H + a) * T + qc];
  f32x16 dq[NC];
#pragma unroll
  for (int c = 0; c < NC; ++c) dq[c] = zero16();

  const int kv_end = min(T, q0 + BQ);
  const int ntiles = (kv_end + BKV - 1) / BKV;

  // ---- tile loads and LDS read offsets: as in the forward kernel
  const uint32_t row_bytes = (uint32_t)ld * 2u;
  uint32_t ldo[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int c = (4 * j + wave) * 64 + lane, row = c / CPR, pos = c % CPR;
    ldo[j] = (uint32_t)row * row_bytes + (uint32_t)((pos ^ G::key(row)) << 4);
  }
  const u32x4 rs = make_desc(qkv + (int64_t)b * T * ld, (uint32_t)((int64_t)T * ld * 2));   // this sequence's rows
  const uint32_t k_col = (uint32_t)(H + kvh) * HD * 2u, v_col = (uint32_t)(H + Hkv + kvh) * HD * 2u;
  auto load_kv = [&](int kt) {
    char* kd = k_ring + (kt & 1) * kTile;
    char* vd = v_ring + (kt & 1) * kTile;
    const uint32_t off = (uint32_t)kt * BKV * row_bytes;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      load_to_lds16(rs, (lds_ptr)(kd + (4 * j + wave) * 1024), ldo[j] + off + k_col);
      load_to_lds16(rs, (lds_ptr)(vd + (4 * j + wave) * 1024), ldo[j] + off + v_col);
    }
  };
  auto landed_barrier = [&]() {
    __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (0 << 8));   // vmcnt(0) lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
  };
  const int p1_base = lq * RB + ((hh ^ G::key(lq)) << 4);
  int p3_base[2];
  {
    const int sl = lane & 15, i = sl >> 2, w = ((lane >> 4) & 1) * 2 + ((sl & 3) >> 1), half = sl & 1;
#pragma unroll
    for (int hi = 0; hi < 2; ++hi) {
      const int row = 8 * hi + 4 * hh + i;
      p3_base[hi] = row * RB + (((G::key(row) & 12) | (w ^ (G::key(row) & 3))) << 4) + half * 8;
    }
  }
  typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
  // K^T fragment for the last product: tile rows (keys) 16 u2 + .., columns 32 c + ..
  auto read_kt = [&](const char* kt_base, int u2, int c) {
    const char* base = kt_base + 16 * u2 * RB;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(base + (p3_base[0] ^ (c * 64))));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(base + (p3_base[1] ^ (c * 64))));
    const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
  };

  load_kv(0);
  landed_barrier();
  // one tile; MASKED: some key of the tile may lie past some query of the workgroup (its last two tiles)
  auto tile_step = [&](int kt, auto masked_tag) {
    constexpr bool MASKED = decltype(masked_tag)::value;
    const int k0 = kt * BKV;
    // into the buffers read in the iteration before, which ended at a barrier; past the last tile the rows are
    // never read (or zeros past the end of the sequence)
    load_kv(kt + 1);
    const char* kt_base = k_ring + (kt & 1) * kTile;
    const char* vt_base = v_ring + (kt & 1) * kTile;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      // S^T and dP^T as two independent MFMA chains; K and V fragments fetched a k-step pair ahead
      f32x16 st = zero16(), dp = zero16();
      bf16x8 fb[2][4];
      const char* kr = kt_base + t * 32 * RB;
      const char* vr = vt_base + t * 32 * RB;
      auto ldkv = [&](int g, bf16x8 (&f)[4]) {
        f[0] = *reinterpret_cast<const bf16x8*>(kr + (p1_base ^ ((2 * g) * 32)));
        f[1] = *reinterpret_cast<const bf16x8*>(vr + (p1_base ^ ((2 * g) * 32)));
        f[2] = *reinterpret_cast<const bf16x8*>(kr + (p1_base ^ ((2 * g + 1) * 32)));
        f[3] = *reinterpret_cast<const bf16x8*>(vr + (p1_base ^ ((2 * g + 1) * 32)));
      };
      auto ldt = [&](int u, bf16x8 (&f)[4]) {
#pragma unroll
        for (int c = 0; c < NC; ++c) f[c] = read_kt(kt_base, 2 * t + u, c);
      };
      ldkv(0, fb[0]);
#pragma unroll
      for (int g = 0; g < NC; ++g) {
        if (g + 1 < NC) ldkv(g + 1, fb[(g + 1) & 1]);
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
        if (MASKED) {
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
        for (int c = 0; c < NC; ++c) dq[c] = mfma(fb[u & 1][c], dsf, dq[c]);
      }
    }
    landed_barrier();
  };
  const int n_free = min(ntiles, q0 / BKV);   // tiles that end before the workgroup's first query: no mask
  for (int kt = 0; kt < n_free; ++kt) tile_step(kt, std::false_type());
  for (int kt = n_free; kt < ntiles; ++kt) tile_step(kt, std::true_type());
  if (q < T) {
    bf16* row = dqkv + ((int64_t)b * T + q) * ld + a * HD;
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 w;
        float q4[4] = {dq[c][4 * g] * scale, dq[c][4 * g + 1] * scale, dq[c][4 * g + 2] * scale, dq[c][4 * g + 3] * scale};
        if (rope_tab) unrotate4(q4, rope_tab, q, HD, c * 32 + g * 8 + hh * 4);
        w.x = pack_bf16(q4[0], q4[1]);
        w.y = pack_bf16(q4[2], q4[3]);
        *reinterpret_cast<uint2*>(row + c * 32 + g * 8 + hh * 4) = w;
      }
  }
}

// ================================================================================ backward: dK, dV
// Workgroup: 128 keys of one (sequence, kv head), 4 wavefronts x 32 keys, which it owns: their K
// and V fragments stay in registers.  It walks the query heads of its group and, for each, the
// query tiles (32 rows) from its first key onward.  Per tile:
//   phase 1  S' = Q K^T - lse/scale + mask bias,  dP' = delta - dO V^T           (2 * hd/16 MFMAs)
//   phase 2  P = exp(scale S'),  dS' = P dP' = -dS                               (arithmetic only)
//   phase 3  dV^T[col][key] += dO^T P,  -dK^T[col][key] += Q^T dS'               (2 * hd/16 MFMAs)
// The log-sum-exp, the causal mask and delta enter as the initial accumulators of phase 1 (V is
// held negated so that delta enters unchanged), so phase 2 is a product, an exponential, a product and
// the conversions per element.
//
// One wavefront per SIMD (the accumulators leave no room for two), so matrix work, arithmetic and
// LDS latency overlap inside the wavefront, by software pipelining over the tiles:
//   first half of an iteration   phase 1 of tile i+1 (operands already in registers), phase 2 of
//                                tile i, LDS reads of tile i's phase 3 operands
//   second half                  phase 3 of tile i, LDS reads of tile i+2's phase 1 operands and
//                                initial accumulators
// with one workgroup barrier between the halves.  Each half is cut into slots of two MFMAs plus their
// share of the other work, fenced from each other, because a wavefront overlaps arithmetic only with
// the MFMA issued just before it.
//
// Q, dO, lse and delta tiles go from memory straight into LDS (buffer loads with the LDS modifier: no
// staging registers, no LDS store instructions), kDepth tiles ahead, in a ring of kDepth + 1 buffers.
// A load instruction fills 1 KiB of LDS in lane order, so the layout is row-major without padding and
// the 16-byte chunks of a row are permuted by an XOR with bits of the row number, applied on the memory
// side of the copy; the permutation makes both the row-wise reads of phase 1 and the transpose reads
// of phase 3 bank-conflict free.  These loads are issued from assembly, outside the compiler's wait insertion: the
// wavefront waits for its own (vmcnt, counted by hand) before the barrier after which a tile is first read.
// Rows past the end of the sequence and tiles past the end of the walk read as zeros (offsets beyond
// the buffer descriptors), and zero rows of Q and dO contribute nothing to either gradient.

template <int HD>
__global__ __launch_bounds__(256) void k_flash_bwd_dkv(const bf16* __restrict__ qkv, const bf16* __restrict__ dO,
                                                       const float* __restrict__ lse, const float* __restrict__ delta,
                                                       bf16* __restrict__ dqkv, int T, int H, int Hkv, float scale,
                                                       const float* __restrict__ rope_tab) {
  typedef DkvGeom<HD> G;
  constexpr int BK = 128, BQ = G::BQ, NK = G::NK, NC = G::NC, RB = G::RB, CPR = G::CPR, NJ = G::NJ;
  constexpr int kDO = G::kDO, kL = G::kL, kD = G::kD, kBuf = G::kBuf, kRing = G::kRing, kDepth = G::kDepth;
  __shared__ __attribute__((aligned(1024))) char smem[kRing * kBuf];
  const int tid = threadIdx.x, lane = tid & 63, lk = lane & 31, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nkb = (T + BK - 1) / BK;
  const BlockId id = heavy_first(blockIdx.x, (int)gridDim.x / (nkb * Hkv), Hkv);   // heaviest key blocks (the first) first
  const int kb = id.level, kvh = id.a, b = id.b;
  const int rep = H / Hkv;
  const int64_t ld = (int64_t)(H + 2 * Hkv) * HD;
  const bf16* Kp = qkv + (int64_t)b * T * ld + (H + kvh) * HD;
  const bf16* Vp = qkv + (int64_t)b * T * ld + (H + Hkv + kvh) * HD;
  const int k0 = kb * BK, kw0 = k0 + wave * 32, key = kw0 + lk, keyc = min(key, T - 1);
  const float scale_log2 = scale * kLog2e, neg_inv_scale = -1.f / scale;

  bf16x8 kf[NK], vf[NK];   // vf = -V
  {
    const bf16* kr = Kp + (int64_t)keyc * ld + hh * 8;
    const bf16* vr = Vp + (int64_t)keyc * ld + hh * 8;
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) {
      kf[kk] = *reinterpret_cast<const bf16x8*>(kr + kk * 16);
      u32x4 v = *reinterpret_cast<const u32x4*>(vr + kk * 16);
      v ^= 0x80008000u;
      vf[kk] = __builtin_bit_cast(bf16x8, v);
    }
  }
  f32x16 dk[NC], dv[NC];   // dk accumulates -dK / scale
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

  // ---- lane constants of the LDS reads (byte offsets inside a ring buffer)
  // phase 1: row lk, chunk (2 kk + hh) permuted; kk enters by XOR with kk * 32
  const int p1_base = lk * RB + ((hh ^ G::key(lk)) << 4);
  // phase 3 (transpose reads, see pack8): 16-lane group position i = row, w = chunk, half = 8-byte half;
  // rows 16u + 8hi + 4hh + i, chunks 4c + w.  u enters as a constant offset, c by XOR with c * 64.
  int p3_base[2];
  {
    const int sl = lane & 15, i = sl >> 2, w = ((lane >> 4) & 1) * 2 + ((sl & 3) >> 1), half = sl & 1;
#pragma unroll
    for (int hi = 0; hi < 2; ++hi) {
      const int row = 8 * hi + 4 * hh + i;
      p3_base[hi] = row * RB + (((G::key(row) & 12) | (w ^ (G::key(row) & 3))) << 4) + half * 8;
    }
  }
  // ---- lane constants of the tile loads: instruction j of this wavefront fills chunks (4j + wave) * 64 + lane
  // of the tile; a chunk at row, position p holds the row's chunk p ^ key(row)
  const uint32_t q_row = (uint32_t)ld * 2u, do_row = (uint32_t)H * HD * 2u;
  uint32_t ldq[NJ], ldo[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int q = (4 * j + wave) * 64 + lane, row = q / CPR, pos = q % CPR;
    ldq[j] = (uint32_t)row * q_row + (uint32_t)((pos ^ G::key(row)) << 4);
    ldo[j] = (uint32_t)row * do_row + (uint32_t)((pos ^ G::key(row)) << 4);
  }
  const uint32_t ldl = (uint32_t)(lane & (BQ - 1)) * 4u;
  const u32x4 q_rs = make_desc(qkv + (int64_t)b * T * ld, (uint32_t)(((int64_t)(T - 1) * ld + (int64_t)H * HD) * 2));
  const u32x4 do_rs = make_desc(dO + (int64_t)b * T * H * HD, (uint32_t)((int64_t)T * H * HD * 2));
  const u32x4 l_rs = make_desc(lse + (int64_t)b * H * T, (uint32_t)((int64_t)H * T * 4));
  const u32x4 d_rs = make_desc(delta + (int64_t)b * H * T, (uint32_t)((int64_t)H * T * 4));

  // the walk: query heads a of this kv head, for each the query tiles qt0 .. nqt-1
  const int qt0 = k0 / BQ, nqt = (T + BQ - 1) / BQ;
  const int steps = (nqt - qt0) * rep;
  struct Walk { int a, qt, left; };
  auto advance = [&](Walk& w) {
    const bool wrap = w.qt == nqt - 1;
    w.qt = wrap ? qt0 : w.qt + 1;
    w.a = wrap ? w.a + 1 : w.a;
    w.left -= 1;
  };
  auto ring_next = [&](int boff) { return boff + kBuf == kRing * kBuf ? 0 : boff + kBuf; };
  // loads of tile w into the ring buffer at boff; a tile past the end of the walk is fetched from beyond
  // every buffer, i.e. as zeros
  auto load_tile = [&](const Walk& w, int boff) {
    const uint32_t dead = w.left > 0 ? 0u : 0x80000000u;
    const uint32_t qs = (uint32_t)w.qt * BQ;
    const uint32_t oq = (qs * q_row + (uint32_t)w.a * HD * 2u) | dead, od = (qs * do_row + (uint32_t)w.a * HD * 2u) | dead;
    const uint32_t ol = (((uint32_t)w.a * T + qs) * 4u) | dead;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      load_to_lds16(q_rs, (lds_ptr)(smem + boff + (4 * j + wave) * 1024), ldq[j] + oq);
      load_to_lds16(do_rs, (lds_ptr)(smem + boff + kDO + (4 * j + wave) * 1024), ldo[j] + od);
    }
    load_to_lds4(l_rs, (lds_ptr)(smem + boff + kL + wave * 256), ldl + ol);
    load_to_lds4(d_rs, (lds_ptr)(smem + boff + kD + wave * 256), ldl + ol);
  };
  // wait until all but the newest kDepth - 2 tiles of this wavefront's loads and all its LDS reads are
  // done, then meet the other wavefronts
  auto tiles_barrier = [&]() {
    constexpr int n = (kDepth - 2) * G::NI;
    static_assert(n < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((n & 15) | ((n >> 4) << 14) | (7 << 4) | (0 << 8));   // vmcnt(n) lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
  };
  // phase 1 operands of the tile at boff, which starts at query qs: f[2kk] = Q, f[2kk+1] = dO (A operand:
  // row = query lk), and the initial accumulators
  auto read_tr2 = [&](int lo, int hi2) {
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const s16x4 l = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(smem + lo));
    const s16x4 h = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(smem + hi2));
    const s16x8 v = {l[0], l[1], l[2], l[3], h[0], h[1], h[2], h[3]};
    return __builtin_bit_cast(bf16x8, v);
  };
  auto read_f1 = [&](int boff, int kk, bf16x8 (&f)[2 * NK]) {
    const char* p = smem + ((p1_base + boff) ^ (kk * 32));
    f[2 * kk] = *reinterpret_cast<const bf16x8*>(p);
    f[2 * kk + 1] = *reinterpret_cast<const bf16x8*>(p + kDO);
  };
  auto init_group = [&](int g, float sel, const float4& l, const float4& d, f32x16& s, f32x16& dp) {
    s[4 * g] = __builtin_fmaf(diag[4 * g], sel, l.x * neg_inv_scale);
    s[4 * g + 1] = __builtin_fmaf(diag[4 * g + 1], sel, l.y * neg_inv_scale);
    s[4 * g + 2] = __builtin_fmaf(diag[4 * g + 2], sel, l.z * neg_inv_scale);
    s[4 * g + 3] = __builtin_fmaf(diag[4 * g + 3], sel, l.w * neg_inv_scale);
    dp[4 * g] = d.x; dp[4 * g + 1] = d.y; dp[4 * g + 2] = d.z; dp[4 * g + 3] = d.w;
  };
  auto tile_sel = [&](const Walk& w) {
    const int qs = w.qt * BQ;
    return qs == kw0 ? 1.f : (qs < kw0 ? 1e38f : 0.f);
  };
  auto read_phase1 = [&](int boff, float sel, bf16x8 (&f)[2 * NK], f32x16& s, f32x16& dp) {
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) read_f1(boff, kk, f);
    const float* pl = reinterpret_cast<const float*>(smem + boff + kL) + hh * 4;
    const float* pd = reinterpret_cast<const float*>(smem + boff + kD) + hh * 4;
#pragma unroll
    for (int g = 0; g < 4; ++g)
      init_group(g, sel, *reinterpret_cast<const float4*>(pl + g * 8), *reinterpret_cast<const float4*>(pd + g * 8), s, dp);
  };
  auto phase1 = [&](const bf16x8 (&f)[2 * NK], f32x16& s, f32x16& dp) {
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) {
      s = mfma(f[2 * kk], kf[kk], s);
      dp = mfma(f[2 * kk + 1], vf[kk], dp);
    }
  };

  Walk w_ld = {kvh * rep, qt0, steps}, w_nx = w_ld;   // next tile to load; next tile whose phase 1 operands are read
  int b_ld = 0, b_cur = 0, b_nx = 0;                  // their ring buffers, and the current tile's
#pragma unroll
  for (int t = 0; t < kDepth; ++t) { load_tile(w_ld, b_ld); advance(w_ld); b_ld = ring_next(b_ld); }
  tiles_barrier();
  bf16x8 f1[2 * NK];
  f32x16 s_a, dp_a, s_b, dp_b;
  read_phase1(b_nx, tile_sel(w_nx), f1, s_a, dp_a); advance(w_nx); b_nx = ring_next(b_nx);
  phase1(f1, s_a, dp_a);
  read_phase1(b_nx, tile_sel(w_nx), f1, s_b, dp_b); advance(w_nx); b_nx = ring_next(b_nx);

  // one iteration: tile i's phase 1 result in (s_c, dp_c); tile i+1's initial accumulators in (s_n, dp_n)
  // and its operands in f1.  On return (s_n, dp_n) hold tile i+1's result, (s_c, dp_c) tile i+2's start.
  auto iteration = [&](f32x16& s_c, f32x16& dp_c, f32x16& s_n, f32x16& dp_n) {
    // ---- top: tile i + kDepth on its way, into the buffer tile i-1 left at the last barrier
    load_tile(w_ld, b_ld); advance(w_ld); b_ld = ring_next(b_ld);
    int p3[2][NC];   // addresses of the transpose reads of tile i, by (hi, c)
#pragma unroll
    for (int hi = 0; hi < 2; ++hi)
#pragma unroll
      for (int c = 0; c < NC; ++c) p3[hi][c] = (p3_base[hi] + b_cur) ^ (c * 64);
    __builtin_amdgcn_sched_barrier(0);
    // ---- first half, in NK slots: two MFMAs of tile i+1's phase 1, 16/NK elements of tile i's phase 2,
    // two of the 2 NK operand fragments of tile i's phase 3
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
        const int off = (which ? 0 : kDO) + 16 * u * RB;
        f3[m] = read_tr2(p3[0][c] + off, p3[1][c] + off);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    tiles_barrier();   // tile i+2 is complete
    // ---- second half, likewise: two MFMAs of phase 3, two operand fragments of tile i+2's phase 1, and
    // its initial accumulators a slot after their reads
    {
      const float sel = tile_sel(w_nx);
      const float* pl = reinterpret_cast<const float*>(smem + b_nx + kL) + hh * 4;
      const float* pd = reinterpret_cast<const float*>(smem + b_nx + kD) + hh * 4;
      float4 l4[4], d4[4];
#pragma unroll
      for (int kk = 0; kk < NK; ++kk) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int m = 2 * kk + j, c = m % NC, which = (m / NC) & 1, u = m / (2 * NC);
          if (which) dk[c] = mfma(f3[m], dsf[u], dk[c]);
          else dv[c] = mfma(f3[m], pf[u], dv[c]);
        }
        read_f1(b_nx, kk, f1);
        if (kk < 4) {
          l4[kk] = *reinterpret_cast<const float4*>(pl + kk * 8);
          d4[kk] = *reinterpret_cast<const float4*>(pd + kk * 8);
        }
        if (kk >= 1 && kk <= 4) init_group(kk - 1, sel, l4[kk - 1], d4[kk - 1], s_c, dp_c);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (NK <= 4) init_group(3, sel, l4[3], d4[3], s_c, dp_c);
      advance(w_nx); b_nx = ring_next(b_nx);
    }
    b_cur = ring_next(b_cur);
  };
  for (int step = 0; step < steps; step += 2) {
    iteration(s_a, dp_a, s_b, dp_b);
    iteration(s_b, dp_b, s_a, dp_a);
  }
  __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8));   // vmcnt(0): no load may still be writing LDS at the end
  if (key < T) {
    bf16* krow = dqkv + ((int64_t)b * T + key) * ld + (H + kvh) * HD;
    bf16* vrow = dqkv + ((int64_t)b * T + key) * ld + (H + Hkv + kvh) * HD;
    const float ks = -scale;
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 w;
        float k4[4] = {dk[c][4 * g] * ks, dk[c][4 * g + 1] * ks, dk[c][4 * g + 2] * ks, dk[c][4 * g + 3] * ks};
        if (rope_tab) unrotate4(k4, rope_tab, key, HD, c * 32 + g * 8 + hh * 4);
        w.x = pack_bf16(k4[0], k4[1]);
        w.y = pack_bf16(k4[2], k4[3]);
        *reinterpret_cast<uint2*>(krow + c * 32 + g * 8 + hh * 4) = w;
        w.x = pack_bf16(dv[c][4 * g], dv[c][4 * g + 1]);
        w.y = pack_bf16(dv[c][4 * g + 2], dv[c][4 * g + 3]);
        *reinterpret_cast<uint2*>(vrow + c * 32 + g * 8 + hh * 4) = w;
      }
  }
}

}  // namespace

bool attention_flash_supported(int B, int T, int H, int Hkv, int hd) {
  // one sequence's rows of qkv, and its lse block, are addressed with 31-bit byte offsets
  return (hd == 64 || hd == 128) && B >= 1 && T >= 1 && H % Hkv == 0 && (int64_t)((T + 127) / 128) * H * B < (1ll << 31) &&
         (int64_t)T * (H + 2 * Hkv) * hd * 2 < (1ll << 31) && (int64_t)T * H * 4 < (1ll << 31);
}

void attention_flash_fwd(hipStream_t s, int B, int T, int H, int Hkv, int hd, const void* qkv, void* o, float* lse) {
  const float sl2 = kLog2e / sqrtf((float)hd);
  dim3 grid((unsigned)(((T + 127) / 128) * H * B));
  if (hd == 128)
    hipLaunchKernelGGL(k_flash_fwd<128>, grid, dim3(256), 0, s, (const bf16*)qkv, (bf16*)o, lse, T, H, Hkv, sl2);
  else
    hipLaunchKernelGGL(k_flash_fwd<64>, grid, dim3(256), 0, s, (const bf16*)qkv, (bf16*)o, lse, T, H, Hkv, sl2);
}

void attention_flash_bwd(hipStream_t s, int B, int T, int H, int Hkv, int hd, const void* qkv, const void* o,
                         const float* lse, const void* do_, void* dqkv, float* delta, const float* rope_tab) {
  const float scale = 1.0f / sqrtf((float)hd);
  const int64_t items = (int64_t)B * T * H;
  dim3 gq((unsigned)(((T + 127) / 128) * H * B)), gk((unsigned)(((T + 127) / 128) * Hkv * B));
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
  prof_stop(pi, s, (double)items * (2.0 * hd * 2 + 4));   // bytes: o and dO read, delta written
  pi = prof_start(PROF_ATTN_DQ, s);
  if (hd == 128)
    hipLaunchKernelGGL(k_flash_bwd_dq<128>, gq, dim3(256), 0, s, (const bf16*)qkv, (const bf16*)do_, lse, delta,
                       (bf16*)dqkv, T, H, Hkv, scale, rope_tab);
  else
    hipLaunchKernelGGL(k_flash_bwd_dq<64>, gq, dim3(256), 0, s, (const bf16*)qkv, (const bf16*)do_, lse, delta,
                       (bf16*)dqkv, T, H, Hkv, scale, rope_tab);
  prof_stop(pi, s, unit);
  pi = prof_start(PROF_ATTN_DKV, s);
  if (hd == 128)
    hipLaunchKernelGGL(k_flash_bwd_dkv<128>, gk, dim3(256), 0, s, (const bf16*)qkv, (const bf16*)do_, lse, delta,
                       (bf16*)dqkv, T, H, Hkv, scale, rope_tab);
  else
    hipLaunchKernelGGL(k_flash_bwd_dkv<64>, gk, dim3(256), 0, s, (const bf16*)qkv, (const bf16*)do_, lse, delta,
                       (bf16*)dqkv, T, H, Hkv, scale, rope_tab);
  prof_stop(pi, s, 3.0 * unit);
}

}  // namespace sp
