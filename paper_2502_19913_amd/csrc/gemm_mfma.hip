// bf16 matrix products on the CDNA4 matrix cores (v_mfma_f32_32x32x16_bf16), float accumulation.
//
// One workgroup of 8 wavefronts owns a 256x256 tile of the output and walks the reduction
// dimension in steps of 64.  Operand tiles are staged global -> registers -> LDS with buffer loads
// (the hardware range check returns zero past the end of an operand, so ragged edges need no
// branches) two steps ahead of the MFMAs, into two LDS buffers (147 KB of the CU's 160 KB); one
// barrier per step.
//
// LDS layouts, chosen so that every fragment read is conflict free and every global access is a
// full 16-byte chunk of a contiguous run:
//   k-contiguous operand (memory [row][k]): LDS [row][64 k] padded to 144 B; a lane's MFMA fragment
//     (8 consecutive k of one row) is one ds_read_b128.
//   k-strided operand (memory [k][x]):      LDS [64 k][256 x] padded to 576 B, copied as is; the
//     fragment is gathered by two ds_read_b64_tr_b16 (the LDS transpose read: within 16 lanes,
//     lane i receives element i%4 of the 8-byte pieces addressed by lanes i/4, i/4+4, i/4+8, i/4+12).
//
//   op 0  C[M,N]  = A[M,K] B[N,K]^T (+R)   A, B k-contiguous
//   op 1  C[M,N]  = A[M,K] B[K,N]          B k-strided
//   op 2  C[M,N] += A[K,M]^T B[K,N]        both k-strided; float output, added atomically: the k-steps
//                                          of all tiles are dealt out in equal runs, one per CU, whatever
//                                          the number of tiles (a weight gradient has few tiles and a
//                                          long reduction)
//
// For bf16 outputs the MFMA is issued with the tile of B as its row operand and the tile of A as its
// column operand, so a lane's accumulator holds 4 consecutive output columns of one output row; they go
// through LDS ([256][256] padded to 528 B) and leave as coalesced 16-byte stores, the optional
// added matrix R is read the same way.  Wavefront layout inside the tile: 2 (M) x 4 (N), each
// wavefront 128x64.  Workgroup ids are regrouped so that the ids that land on one XCD (id mod 8)
// cover neighbouring tiles and share operand panels in that XCD's L2.
#include "devutil.h"
#include "internal.h"

namespace sp {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int kThreads = 512;
constexpr int kRowBytes = 144;                  // k-contiguous tile: 64 bf16 + 16 bytes of padding per row
constexpr int kKRowBytes = 576;                 // k-strided tile: 256 bf16 + 64 bytes of padding per k
constexpr int kTileBytes = 256 * kRowBytes;     // = 64 * kKRowBytes
constexpr int kLdsBytes = 4 * kTileBytes;       // A and B, two buffers
constexpr int kCRowBytes = 528;                 // output staging: 256 bf16 + 16 bytes
static_assert(64 * kKRowBytes == kTileBytes, "both tile layouts have the same footprint");
static_assert(256 * kCRowBytes <= kLdsBytes, "output staging fits in the operand buffers");

// 16 bytes at byte offset voff; zero if voff is at or past the end of the buffer
__device__ __forceinline__ uint4 bload(rsrc_t rsrc, uint32_t voff) {
  i32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)voff, 0, 0);
  return make_uint4((uint32_t)v[0], (uint32_t)v[1], (uint32_t)v[2], (uint32_t)v[3]);
}

// One operand's share of the staging for one thread: 4 chunks of 16 bytes.
template <bool KSTRIDED>
struct Operand {
  rsrc_t rsrc;
  uint32_t voff0;      // byte offset of this thread's chunk 0 at k = 0
  uint32_t chunk_step; // distance between the thread's consecutive chunks
  uint32_t k_step;     // byte distance of one k element
  int kc8;             // k-contiguous: first k of the thread's chunk inside a step
  int lds_off;         // byte offset of chunk 0 in the LDS tile
  // ld: leading dimension (elements); origin: first tile row (k-contiguous) or first x (k-strided)
  __device__ __forceinline__ void init(const bf16* X, uint32_t bytes, int ld, int origin, int tid) {
    rsrc = make_rsrc(X, bytes);
    if (KSTRIDED) {
      const int krow = tid >> 5, xc = tid & 31;          // chunk c = tid + 512 i: k row c / 32, x chunk c % 32
      voff0 = ((uint32_t)krow * ld + origin + xc * 8) * 2u;
      chunk_step = 16u * ld * 2u;
      k_step = (uint32_t)ld * 2u;
      kc8 = 0;
      lds_off = krow * kKRowBytes + xc * 16;
    } else {
      const int row = tid >> 3, kc = tid & 7;            // chunk c = tid + 512 i: row c / 8, k chunk c % 8
      voff0 = ((uint32_t)(origin + row) * ld + kc * 8) * 2u;
      chunk_step = 64u * ld * 2u;
      k_step = 2u;
      kc8 = kc * 8;
      lds_off = row * kRowBytes + kc * 16;
    }
  }
  // KMASK (k-contiguous only): chunks whose k is at or past kend read as zero
  template <bool KMASK>
  __device__ __forceinline__ void load(int k0, int kend, uint4 (&reg)[4]) const {
    const uint32_t base = voff0 + (uint32_t)k0 * k_step;
    const bool dead = KMASK && !KSTRIDED && (k0 + kc8 >= kend);
#pragma unroll
    for (int i = 0; i < 4; ++i) reg[i] = bload(rsrc, dead ? 0xffffffffu : base + i * chunk_step);
  }
  __device__ __forceinline__ void store(char* tile, const uint4 (&reg)[4]) const {
    constexpr int step = KSTRIDED ? 16 * kKRowBytes : 64 * kRowBytes;
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4*>(tile + lds_off + i * step) = reg[i];
  }
};

// MFMA fragment of tile row `row` (0..255) for k-step ks (16 k): 8 consecutive k, starting at
// ks*16 + (lane/32)*8, of that row.
template <bool KSTRIDED>
__device__ __forceinline__ bf16x8 read_frag(const char* tile, int row_base, int ks, int lane) {
  if (!KSTRIDED) {
    return *reinterpret_cast<const bf16x8*>(tile + (row_base + (lane & 31)) * kRowBytes + ks * 32 + (lane >> 5) * 16);
  } else {
    // group of 16 lanes = 16 consecutive x; lane s of the group addresses k row s/4, x piece s%4
    const int g16 = (lane >> 4) & 1, hh = lane >> 5, s = lane & 15;
    const char* p = tile + (ks * 16 + hh * 8 + (s >> 2)) * kKRowBytes + (row_base + g16 * 16 + (s & 3) * 4) * 2;
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * kKRowBytes));
    typedef __attribute__((ext_vector_type(8))) short s16x8;
    s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
  }
}

template <int OP, bool KMASK>
__global__ __launch_bounds__(kThreads) void k_gemm_mfma(const bf16* __restrict__ A, const bf16* __restrict__ B,
                                                        void* __restrict__ Cv, const bf16* __restrict__ Rr, int M,
                                                        int N, int K, int tiles_m, int tiles_n) {
  constexpr bool AS = OP == 2, BS = OP != 0;   // which operands are k-strided
  __shared__ __attribute__((aligned(16))) char smem[kLdsBytes];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3;

  // ---- the work of this workgroup.  OP 0/1: one output tile, the whole reduction.  OP 2: the k-steps of
  // all tiles form one sequence (tile-major), cut into gridDim.x equal runs; a run covers the end of
  // one tile, whole tiles, the start of another, and every piece is added to the output atomically, so
  // the workgroups finish together whatever the number of tiles.
  // Ids that share an XCD (id mod 8) get consecutive tiles (runs); tiles run down M first inside bands
  // of 8 tile columns so that neighbours share B panels and reuse A panels.
  const int tiles = tiles_m * tiles_n;
  int id = blockIdx.x;
  {
    const int n_ids = gridDim.x, per = n_ids / 8, rem = n_ids % 8, x = id % 8;
    id = x * per + min(x, rem) + id / 8;
  }
  const int ksteps = (K + BK - 1) / BK;
  int64_t u = OP == 2 ? (int64_t)id * tiles * ksteps / gridDim.x : (int64_t)id * ksteps;
  const int64_t u_end = OP == 2 ? (int64_t)(id + 1) * tiles * ksteps / gridDim.x : u + ksteps;
  while (u < u_end) {
  const int tile = (int)(u / ksteps), ks0 = (int)(u - (int64_t)tile * ksteps);
  const int ks1 = (int)min((int64_t)ksteps, ks0 + (u_end - u));
  u += ks1 - ks0;
  constexpr int kBand = 8;
  const int band = tile / (kBand * tiles_m);
  const int band_w = min(kBand, tiles_n - band * kBand);
  const int in_band = tile - band * kBand * tiles_m;
  const int tm = in_band / band_w, tn = band * kBand + in_band % band_w;
  const int m0 = tm * BM, n0 = tn * BN;
  const int kb = ks0 * BK, kend = min(K, ks1 * BK);
  const int nk = ks1 - ks0;

  Operand<AS> opa;
  Operand<BS> opb;
  opa.init(A, (uint32_t)((size_t)M * K * 2), AS ? M : K, m0, tid);
  opb.init(B, (uint32_t)((size_t)N * K * 2), BS ? N : K, n0, tid);

  // acc[j][i]: MFMA rows = 32 output columns n (i of 2), MFMA columns = 32 output rows m (j of 4)
  f32x16 acc[4][2];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

  uint4 ra[2][4], rb[2][4];
  auto compute = [&](const char* base) {
    const char* ta = base;
    const char* tb = base + kTileBytes;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 fa[4], fb[2];
#pragma unroll
      for (int j = 0; j < 4; ++j) fa[j] = read_frag<AS>(ta, wm * 128 + j * 32, ks, lane);
#pragma unroll
      for (int i = 0; i < 2; ++i) fb[i] = read_frag<BS>(tb, wn * 64 + i * 32, ks, lane);
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 2; ++i)
          acc[j][i] = OP == 2 ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[j], fb[i], acc[j][i], 0, 0, 0)
                              : __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[i], fa[j], acc[j][i], 0, 0, 0);
    }
  };
  auto gload = [&](int t, uint4 (&xa)[4], uint4 (&xb)[4]) {
    opa.template load<KMASK>(kb + t * BK, kend, xa);
    opb.template load<KMASK>(kb + t * BK, kend, xb);
  };
  auto sstore = [&](int t, const uint4 (&xa)[4], const uint4 (&xb)[4]) {
    char* d = smem + (t & 1) * 2 * kTileBytes;
    opa.store(d, xa);
    opb.store(d + kTileBytes, xb);
  };

  // tile t of the reduction waits in register set t & 1 until it is written to LDS buffer t & 1
  if (nk > 0) {
    gload(0, ra[0], rb[0]);
    if (nk > 1) gload(1, ra[1], rb[1]);
    sstore(0, ra[0], rb[0]);
  }
  __syncthreads();
  int kt = 0;
  for (; kt + 3 < nk; kt += 2) {   // steady state: no conditionals, so outstanding loads can be counted
    gload(kt + 2, ra[0], rb[0]);
    compute(smem);
    sstore(kt + 1, ra[1], rb[1]);
    __syncthreads();
    gload(kt + 3, ra[1], rb[1]);
    compute(smem + 2 * kTileBytes);
    sstore(kt + 2, ra[0], rb[0]);
    __syncthreads();
  }
  for (; kt < nk; ++kt) {          // the last (up to three) steps
    const bool odd = kt & 1;
    if (kt + 2 < nk) { if (odd) gload(kt + 2, ra[1], rb[1]); else gload(kt + 2, ra[0], rb[0]); }
    compute(smem + (kt & 1) * 2 * kTileBytes);
    if (kt + 1 < nk) { if (odd) sstore(kt + 1, ra[0], rb[0]); else sstore(kt + 1, ra[1], rb[1]); }
    __syncthreads();
  }

  // ---- epilogue.  Accumulator r of lane l: output row m = lane%32, output column n = (r/4)*8 + (l/32)*4 + r%4
  // of its 32x32 tile, i.e. 4 consecutive columns per group of 4 registers.
  const int lm = lane & 31, hh = lane >> 5;
  if (OP == 2) {
    // float output, accumulated in place.  Here the tile of A is the MFMA's row operand: accumulator r of
    // lane l is output row (r/4)*8 + (l/32)*4 + r%4, column l%32, so a wavefront's atomic covers 128
    // contiguous bytes of two rows.
    float* C = reinterpret_cast<float*>(Cv);
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int col = n0 + wn * 64 + i * 32 + lm;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = m0 + wm * 128 + j * 32 + (r >> 2) * 8 + hh * 4 + (r & 3);
          if (row < M && col < N) {
            float* p = C + (int64_t)row * N + col;
            unsafeAtomicAdd(p, acc[j][i][r]);
          }
        }
      }
  } else {
    // all wavefronts are past the last barrier of the loop: the operand buffers are free
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          uint2 w;
          w.x = pack_bf16(acc[j][i][4 * g], acc[j][i][4 * g + 1]);
          w.y = pack_bf16(acc[j][i][4 * g + 2], acc[j][i][4 * g + 3]);
          *reinterpret_cast<uint2*>(smem + (wm * 128 + j * 32 + lm) * kCRowBytes + (wn * 64 + i * 32 + g * 8 + hh * 4) * 2) = w;
        }
    __syncthreads();
    bf16* C = reinterpret_cast<bf16*>(Cv);
    const bool add = OP == 0 && Rr != nullptr;
#pragma unroll 4
    for (int it = 0; it < 16; ++it) {
      const int c = tid + kThreads * it;
      const int row = c >> 5, nc = c & 31;
      const int grow = m0 + row, gcol = n0 + nc * 8;
      if (grow < M && gcol < N) {   // N is a multiple of 8: a chunk is inside or outside as a whole
        uint4 v = *reinterpret_cast<const uint4*>(smem + row * kCRowBytes + nc * 16);
        const int64_t at = (int64_t)grow * N + gcol;
        if (add) {
          // the sum is formed in float from the accumulator's bf16 rounding; one more rounding on the way out
          float x[8], y[8];
          const uint32_t wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) { x[2 * e] = bf16_bits_to_float(wv[e] & 0xffffu); x[2 * e + 1] = bf16_bits_to_float(wv[e] >> 16); }
          load8(Rr + at, y);
#pragma unroll
          for (int e = 0; e < 8; ++e) x[e] += y[e];
          store8(C + at, x);
        } else {
          *reinterpret_cast<uint4*>(C + at) = v;
        }
      }
    }
  }
  }  // next piece of the run
}

inline bool al16(const void* p) { return ((uintptr_t)p & 15) == 0; }

int cu_count() {
  static int n = 0;
  if (!n) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) n = v;
    else n = 256;
  }
  return n;
}

}  // namespace

bool gemm_mfma_supported(int op, int64_t M, int64_t N, int64_t K, const void* A, const void* B, const void* C,
                         const void* R) {
  if (M < 1 || N < 1 || K < 1) return false;
  // buffer descriptors address up to 4 GiB per operand with 32-bit offsets
  if (M * K * 2 >= ((int64_t)1 << 32) || N * K * 2 >= ((int64_t)1 << 32)) return false;
  if (!al16(A) || !al16(B) || !al16(C) || (R && !al16(R))) return false;
  if (((M + BM - 1) / BM) * ((N + BN - 1) / BN) > (1 << 24)) return false;
  if (N % 8) return false;                      // 16-byte output chunks
  switch (op) {
    case 0: return K % 8 == 0;
    case 1: return K % 8 == 0;
    case 2: return M % 8 == 0;
  }
  return false;
}

void gemm_mfma(hipStream_t s, int op, int64_t M, int64_t N, int64_t K, const void* A, const void* B, void* C,
               const void* R) {
  const int tm = (int)((M + BM - 1) / BM), tn = (int)((N + BN - 1) / BN);
  const int tiles = tm * tn;
  int wgs = tiles;
  if (op == 2) {
    // one run of k-steps per CU, but no run shorter than 4 steps
    const int64_t units = (int64_t)tiles * ((K + BK - 1) / BK);
    wgs = (int)std::max<int64_t>(1, std::min<int64_t>(cu_count(), units / 4));
  }
  dim3 grid(wgs);
  const bf16* a = (const bf16*)A;
  const bf16* b = (const bf16*)B;
  const bf16* r = (const bf16*)R;
  const bool kmask = K % BK != 0;
#define SP_LAUNCH(OP, KM) \
  hipLaunchKernelGGL((k_gemm_mfma<OP, KM>), grid, dim3(kThreads), 0, s, a, b, C, r, (int)M, (int)N, (int)K, tm, tn)
  if (op == 0) { if (kmask) SP_LAUNCH(0, true); else SP_LAUNCH(0, false); }
  else if (op == 1) { if (kmask) SP_LAUNCH(1, true); else SP_LAUNCH(1, false); }
  else SP_LAUNCH(2, false);
#undef SP_LAUNCH
}

}  // namespace sp
