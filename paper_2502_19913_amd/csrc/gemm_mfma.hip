// bf16 matrix products on the CDNA4 matrix cores, float accumulation.  Ops 0 and 1 use
// v_mfma_f32_16x16x32_bf16, which on random data sustains more flops per watt than the 32x32x16 form (the chip
// is power-limited here); op 2 keeps v_mfma_f32_32x32x16_bf16, whose accumulator layout gives wider atomics.
//
// One workgroup of 8 wavefronts owns a 256x256 tile of the output (128x128 when the product has too few
// 256-tiles to occupy the CUs) and walks the reduction dimension in steps of 64.  Operand tiles go from
// memory straight into LDS (buffer loads with the LDS modifier: no staging registers, no LDS stores; the
// hardware range check returns zero past the end of an operand, so ragged edges need no branches).  The
// small tile keeps two stages of A and B, loaded one step ahead, with one barrier per step (two workgroups per
// CU overlap each other).  The large tile fills the CU's 160 KB of LDS alone (two tiles of A, three of B) and
// runs the alternating-phase loop described where it stands: the two wavefronts of a SIMD take turns between
// reading fragments and issuing MFMAs, half a step apart.
//
// LDS layouts.  A load instruction fills 1 KiB of LDS in lane order, so tiles are unpadded and the
// 16-byte chunks of a row are permuted by an XOR with bits of the row number (see Operand), which
// makes every fragment read conflict free while every global access stays a full 16-byte chunk of a
// contiguous run:
//   k-contiguous operand (memory [row][k]): LDS [256 rows][64 k]; a lane's MFMA fragment (8 consecutive
//     k of one row) is one ds_read_b128.
//   k-strided operand (memory [k][x]):      LDS [64 k][256 x]; the fragment is gathered by two
//     ds_read_b64_tr_b16 (the LDS transpose read: within 16 lanes, lane i receives element i%4 of the
//     8-byte pieces addressed by lanes i/4, i/4+4, i/4+8, i/4+12).
//
//   op 0  C[M,N]  = A[M,K] B[N,K]^T (+R)   A, B k-contiguous
//   op 1  C[M,N]  = A[M,K] B[K,N]          B k-strided
//   op 2  C[M,N] += A[K,M]^T B[K,N]        both k-strided; float output, added atomically: the k-steps
//                                          of every tile are cut into a whole number of equal runs, one
//                                          workgroup each, so that the rounds of workgroups are full (a
//                                          weight gradient has few tiles and a long reduction)
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
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;

constexpr int BK = 64;
constexpr int kThreads = 512;
// Geometry of a TILE x TILE output tile (TILE = 256, or 128 for products with few tiles)
template <int TILE>
struct Geo {
  static constexpr int kTileBytes = TILE * BK * 2;        // one operand tile, either layout, unpadded
  static constexpr int kStageBytes = 2 * kTileBytes;      // A and B
  static constexpr int kCRowBytes = TILE * 2 + 16;        // output staging row: TILE bf16 + 16 bytes
  static constexpr int kLdsBytes = TILE * kCRowBytes > 2 * kStageBytes ? TILE * kCRowBytes : 2 * kStageBytes;
  static constexpr int kLdsBytesPP = 5 * kTileBytes;     // alternating-phase loop: two tiles of A, three of B
  static constexpr int NJ = kTileBytes / 1024 / 8;        // load instructions per wavefront and operand tile
  static constexpr int XCH = TILE / 8;                    // 16-byte chunks per k row of a k-strided tile
  static constexpr int WM = TILE / 2, WN = TILE / 4;      // a wavefront's share of the tile (2 x 4 wavefronts)
};

constexpr uint32_t kPastEnd = 0x80000000u;      // no descriptor is this large

// Byte offset, from the tile's first row (k-contiguous) or first x (k-strided) at the step's first k, of the
// 16-byte chunk that belongs at position q of the tile in LDS (layouts above); kc8: for k-contiguous tiles, the
// first k of that chunk inside the step.
// split (k-contiguous only): the second half of the tile's rows lies `split` rows further on in memory (the gate
// and up rows of a SwiGLU projection that share one tile).
template <bool KSTRIDED, bool W32, int TILE>
__device__ __forceinline__ uint32_t chunk_offset(int q, int ld, int& kc8, int split = 0) {
  constexpr int XCH = Geo<TILE>::XCH;
  if (KSTRIDED) {
    const int krow = q / XCH, pos = q % XCH;
    const int c = pos ^ (W32 ? (krow & 3) << 2 : ((krow & 3) | (((krow >> 3) & 1) << 2)) << 1);
    return ((uint32_t)krow * ld + c * 8) * 2u;
  }
  const int row = q >> 3, pos = q & 7, c = pos ^ ((row >> 1) & 7);
  kc8 = c * 8;
  return ((uint32_t)(row + (row >= TILE / 2 ? split : 0)) * ld + c * 8) * 2u;
}

// One operand's share of the tile loads for one wavefront: TILE / 64 instructions of 1 KiB per step.
// Instruction j fills the tile's 16-byte chunks (8j + wave) * 64 + lane.
//   k-contiguous tile: [TILE rows][64 k], 8 chunks per row; the chunk at position p of a row holds the row's
//     chunk p ^ ((row >> 1) & 7): the 16 rows a ds_read_b128 touches then fall in 16 different bank groups.
//   k-strided tile: [64 k][TILE x], TILE / 8 chunks per k row; position p of k row k holds chunk p ^ kkey(k).
//     For 16-wide fragments kkey(k) = ((k & 3) | ((k >> 3) & 1) << 2) << 1: the 8 k rows x 32 bytes that 32
//     lanes of a transpose read touch (rows k0..k0+3 and k0+8..k0+11) fall in 8 different 32-byte bank groups.
//     For 32-wide fragments (W32, the weight-gradient product) kkey(k) = (k & 3) << 2: the 4 k rows x 4 chunks
//     that 32 lanes touch fall in 16 different bank groups.
// The permutation is applied on the memory side: a lane fetches the chunk that belongs at its position.
template <bool KSTRIDED, bool W32, int TILE>
struct Operand {
  static constexpr int NJ = Geo<TILE>::NJ, XCH = Geo<TILE>::XCH;
  const char* base;    // first byte of the tile's rows (k-contiguous) or of its first x (k-strided), at k = 0
  int64_t left;        // bytes from base to the end of the operand
  uint32_t voff[NJ];   // byte offset of the lane's chunk from base, per instruction
  uint32_t k_step;     // byte distance of one k element
  int kc8;             // k-contiguous: first k of the lane's chunk inside a step
  // rows x ld elements in memory; origin: first tile row (k-contiguous) or first x (k-strided).
  // Offsets stay below 2^31 for ld < 2^21 (checked by the caller); the operand itself may be larger.
  __device__ __forceinline__ void init(const bf16* X, int64_t rows, int ld, int origin, int wave, int lane, int split = 0) {
    const int64_t first = KSTRIDED ? (int64_t)origin : (int64_t)origin * ld;
    base = reinterpret_cast<const char*>(X + first);
    left = (rows * ld - first) * 2;
    kc8 = 0;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int q = (8 * j + wave) * 64 + lane;
      voff[j] = chunk_offset<KSTRIDED, W32, TILE>(q, ld, kc8, split);   // kc8: the same for every j (lane and wave & 1 only)
    }
    k_step = KSTRIDED ? (uint32_t)ld * 2u : 2u;
  }
  // The step's descriptor starts at the step's first k, so offsets never grow with the operand; its size
  // is what is left of the operand, capped below kPastEnd.
  // KMASK (k-contiguous only): chunks whose k is at or past kend read as zero
  template <bool KMASK>
  __device__ __forceinline__ void load(int k0, int kend, char* tile, int wave) const {
    const bool dead = KMASK && !KSTRIDED && (k0 + kc8 >= kend);
    const int64_t skip = (int64_t)k0 * k_step;
    const int64_t rest = left - skip;
    const u32x4 desc = make_desc(base + skip, (uint32_t)(rest < 0 ? 0 : (rest > 0x7fffffff ? 0x7fffffff : rest)));
#pragma unroll
    for (int j = 0; j < NJ; ++j) load_to_lds16(desc, (lds_ptr)(tile + (8 * j + wave) * 1024), dead ? kPastEnd : voff[j]);
  }
};

// The loads of one wavefront when a workgroup's halves divide the operands between them (the alternating-phase
// loop): wavefronts 0-3 load the tiles of A, wavefronts 4-7 those of B, so a wavefront issues a quarter of one
// operand's tile, instruction j filling chunks (4 j + w4) * 64 + lane.  One set of offsets serves either role.
template <bool AS, bool BS, bool W32, int TILE>
struct HalfLoader {
  static constexpr int NJ = Geo<TILE>::kTileBytes / 1024 / 4;
  const char* base;
  int64_t left;
  uint32_t voff[NJ];
  uint32_t k_step;
  int kc8;
  bool strided;
  __device__ __forceinline__ void init(bool late, const bf16* A, int64_t a_rows, int a_ld, int a_origin, const bf16* B,
                                       int64_t b_rows, int b_ld, int b_origin, int w4, int lane, int b_split = 0) {
    const bf16* X = late ? B : A;
    const int64_t rows = late ? b_rows : a_rows;
    const int ld = late ? b_ld : a_ld, origin = late ? b_origin : a_origin;
    strided = late ? BS : AS;
    const int64_t first = strided ? (int64_t)origin : (int64_t)origin * ld;
    base = reinterpret_cast<const char*>(X + first);
    left = (rows * ld - first) * 2;
    kc8 = 0;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int q = (4 * j + w4) * 64 + lane;
      int kc_a = 0, kc_b = 0;
      const uint32_t oa = chunk_offset<AS, W32, TILE>(q, ld, kc_a);
      const uint32_t ob = (AS == BS && b_split == 0) ? oa : chunk_offset<BS, W32, TILE>(q, ld, kc_b, b_split);
      voff[j] = late ? ob : oa;
      kc8 = late ? ((AS == BS && b_split == 0) ? kc_a : kc_b) : kc_a;
    }
    k_step = strided ? (uint32_t)ld * 2u : 2u;
  }
  template <bool KMASK>
  __device__ __forceinline__ void load(int k0, int kend, char* tile, int w4) const {
    const bool dead = KMASK && !strided && (k0 + kc8 >= kend);
    const int64_t skip = (int64_t)k0 * k_step;
    const int64_t rest = left - skip;
    const u32x4 desc = make_desc(base + skip, (uint32_t)(rest < 0 ? 0 : (rest > 0x7fffffff ? 0x7fffffff : rest)));
#pragma unroll
    for (int j = 0; j < NJ; ++j) load_to_lds16(desc, (lds_ptr)(tile + (4 * j + w4) * 1024), dead ? kPastEnd : voff[j]);
  }
};

// MFMA operand fragment (v_mfma_f32_16x16x32_bf16: lane l holds row l % 16, k = (l / 16) * 8 .. + 7) of tile rows
// row_base .. row_base + 15 for the k32-th group of 32 k of the step.  row_base is a multiple of 16.
template <bool KSTRIDED, int TILE>
__device__ __forceinline__ bf16x8 read_frag(const char* tile, int row_base, int k32, int lane) {
  constexpr int KR = TILE * 2;   // bytes per k row of a k-strided tile
  if (!KSTRIDED) {
    const int lr = lane & 15, kg = lane >> 4;
    // chunk 4 k32 + kg permuted by the row's key; k32 enters by XOR with k32 * 64
    const int lane_off = lr * 128 + ((kg ^ ((lr >> 1) & 7)) << 4);
    return *reinterpret_cast<const bf16x8*>(tile + row_base * 128 + (lane_off ^ (k32 * 64)));
  } else {
    // Two transpose reads.  Within a group of 16 lanes, lane s addresses k row s/4 and the 8-byte piece s%4 of
    // the group's 32 bytes (16 x), and receives x = s, 4 consecutive k.  Group g = lane/16 takes k rows
    // 8g .. 8g+3, then 8g+4 .. 8g+7; both have the same kkey: (s/4) | (g & 1) << 2, shifted left by one.
    const int g = lane >> 4, s = lane & 15;
    const int key = ((s >> 2) | ((g & 1) << 2)) << 1;
    const int lane_off = (g * 8 + (s >> 2)) * KR + (key << 4) + (((s & 3) >> 1) << 4) + (s & 1) * 8;
    const char* p = tile + k32 * 32 * KR + (lane_off ^ (row_base * 2));   // row_base * 2: a multiple of 32 bytes
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * KR));
    typedef __attribute__((ext_vector_type(8))) short s16x8;
    s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
  }
}

// The same for v_mfma_f32_32x32x16_bf16 (the weight-gradient product keeps this form: its accumulator layout
// gives atomics that cover 128 contiguous bytes).  Fragment of tile row `row_base + lane % 32` for k-step ks (16 k): 8 consecutive k, starting at
// ks*16 + (lane/32)*8.  row_base is a multiple of 32.
template <bool KSTRIDED, int TILE>
__device__ __forceinline__ bf16x8 read_frag32(const char* tile, int row_base, int ks, int lane) {
  constexpr int KR = TILE * 2;
  if (!KSTRIDED) {
    const int lr = lane & 31, hh = lane >> 5;
    // chunk 2 ks + hh permuted by the row's key; ks enters by XOR with ks * 32
    const int lane_off = lr * 128 + ((hh ^ ((lr >> 1) & 7)) << 4);
    return *reinterpret_cast<const bf16x8*>(tile + row_base * 128 + (lane_off ^ (ks * 32)));
  } else {
    // group of 16 lanes = 16 consecutive x; lane s of the group addresses k row s/4, x piece s%4:
    // k row ks*16 + hh*8 + i (and + 4), chunk row_base/8 + 2 g16 + (s%4)/2, permuted by i << 2
    const int g16 = (lane >> 4) & 1, hh = lane >> 5, s = lane & 15, i = s >> 2;
    const int lane_off = (hh * 8 + i) * KR + (((i << 2) | (g16 * 2 + ((s & 3) >> 1))) << 4) + (s & 1) * 8;
    const char* p = tile + ks * 16 * KR + (lane_off ^ (row_base * 2));   // row_base * 2 = chunk bits 2.. : multiple of 64
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * KR));
    typedef __attribute__((ext_vector_type(8))) short s16x8;
    s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
  }
}

// What happens to a bf16 output tile on its way out (EPI):
//   kEpiPlain      stored, plus the matrix R if given (op 0)
//   kEpiRope       op 0: the leading rope.rot_cols columns are rotated
//   kEpiSwiglu     op 0, N = 2h, B = [gate rows | up rows]: a tile holds TILE/2 gate columns and the TILE/2 up
//                  columns of the same features (tiles_n = h / (TILE/2)); C receives both at their places and
//                  aux[M, h] receives silu(gate) * up, formed from the rounded values C holds
//   kEpiSwigluBwd  op 1, N = h: the product is d(act); with gate|up read from R[M, 2h], C[M, 2h] receives
//                  d(gate) | d(up); d(act) itself is not stored
enum { kEpiPlain = 0, kEpiRope = 1, kEpiSwiglu = 2, kEpiSwigluBwd = 3 };

template <int OP, bool KMASK, int EPI, int TILE, bool PP = false>
__global__ __launch_bounds__(kThreads) void k_gemm_mfma(const bf16* __restrict__ A, const bf16* __restrict__ B,
                                                        void* __restrict__ Cv, const bf16* __restrict__ Rr, int M,
                                                        int N, int K, int tiles_m, int tiles_n, RopeArgs rope,
                                                        bf16* __restrict__ aux) {
  constexpr bool ROPE = EPI == kEpiRope;
  static_assert(EPI == kEpiPlain || (EPI == kEpiSwigluBwd ? OP == 1 : OP == 0), "epilogue and product do not match");
  constexpr bool AS = OP == 2, BS = OP != 0;   // which operands are k-strided
  typedef Geo<TILE> G;
  constexpr int kTileBytes = G::kTileBytes, kStageBytes = G::kStageBytes, kCRowBytes = G::kCRowBytes;
  constexpr int WM = G::WM, WN = G::WN, BM = TILE, BN = TILE;
  __shared__ __attribute__((aligned(1024))) char smem[PP ? G::kLdsBytesPP : G::kLdsBytes];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2, wn = wave & 3;

  // ---- the work of this workgroup: a sequence of pieces, each a range of k-steps of one output tile.
  // OP 0/1: whole tiles id, id + gridDim.x, ...: the launch has as many workgroups as make its rounds of
  // tiles equally full.  OP 2: the k-steps of all tiles form one sequence (tile-major), cut into gridDim.x
  // equal runs (normally a whole number of runs per tile); every piece is added to the output atomically.
  // Ids that share an XCD (id mod 8) get consecutive tiles (runs); tiles run down M first inside bands
  // of 8 tile columns so that neighbours share B panels and reuse A panels.
  const int tiles = tiles_m * tiles_n;
  int id = blockIdx.x;
  {
    const int n_ids = gridDim.x, per = n_ids / 8, rem = n_ids % 8, x = id % 8;
    id = x * per + min(x, rem) + id / 8;
  }
  const int ksteps = (K + BK - 1) / BK;
  // OP 2: gridDim.x = tiles x s; id -> run id / tiles of tile id % tiles, so that the ids that share an XCD (a
  // contiguous range) work on neighbouring tiles over the same k range and share their operand panels
  const int s_runs = OP == 2 ? (int)gridDim.x / tiles : 1;
  const int run = OP == 2 ? id / tiles : 0;
  int64_t u = OP == 2 ? (int64_t)(id % tiles) * ksteps + (int64_t)run * ksteps / s_runs : (int64_t)id * ksteps;
  const int64_t u_end = OP == 2 ? (int64_t)(id % tiles) * ksteps + (int64_t)(run + 1) * ksteps / s_runs : (int64_t)tiles * ksteps;
  while (u < u_end) {
  const int tile = (int)(u / ksteps), ks0 = (int)(u - (int64_t)tile * ksteps);
  const int ks1 = OP == 2 ? (int)min((int64_t)ksteps, ks0 + (u_end - u)) : ksteps;
  u += OP == 2 ? (int64_t)(ks1 - ks0) : (int64_t)gridDim.x * ksteps;
  constexpr int kBand = 8;
  const int band = tile / (kBand * tiles_m);
  const int band_w = min(kBand, tiles_n - band * kBand);
  const int in_band = tile - band * kBand * tiles_m;
  const int tm = in_band / band_w, tn = band * kBand + in_band % band_w;
  // n0: first output column of the tile (kEpiSwiglu: first gate column; the up columns start at hN + n0)
  const int hN = N / 2;
  const int m0 = tm * BM, n0 = EPI == kEpiSwiglu ? tn * (BN / 2) : tn * BN;
  const int b_split = EPI == kEpiSwiglu ? hN - BN / 2 : 0;
  const int kb = ks0 * BK, kend = min(K, ks1 * BK);
  const int nk = ks1 - ks0;

  constexpr bool W32 = OP == 2;   // which MFMA form (see read_frag32)
  Operand<AS, W32, TILE> opa;
  Operand<BS, W32, TILE> opb;
  opa.init(A, AS ? K : M, AS ? M : K, m0, wave, lane);
  opb.init(B, BS ? K : N, BS ? N : K, n0, wave, lane, b_split);

  // OP 0/1: acc[j][i] = 16 output rows m x 16 output columns n of the wavefront's WM x WN share.
  // OP 2: acc32[j][i] = 32 rows x 32 columns of it.
  constexpr int NJ16 = WM / 16, NI16 = WN / 16, NJ32 = WM / 32, NI32 = WN / 32;
  f32x4 acc[W32 ? 1 : NJ16][W32 ? 1 : NI16];
  f32x16 acc32[W32 ? NJ32 : 1][W32 ? NI32 : 1];
  if (W32) {
#pragma unroll
    for (int j = 0; j < NJ32; ++j)
#pragma unroll
      for (int i = 0; i < NI32; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc32[W32 ? j : 0][W32 ? i : 0][r] = 0.f;
  } else {
#pragma unroll
    for (int j = 0; j < NJ16; ++j)
#pragma unroll
      for (int i = 0; i < NI16; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[W32 ? 0 : j][W32 ? 0 : i][r] = 0.f;
  }

  auto compute = [&](const char* base) {
    const char* ta = base;
    const char* tb = base + kTileBytes;
    if (W32) {
#pragma unroll
      for (int ks = 0; ks < BK / 16; ++ks) {
        bf16x8 fa[NJ32], fb[NI32];
#pragma unroll
        for (int j = 0; j < NJ32; ++j) fa[j] = read_frag32<AS, TILE>(ta, wm * WM + j * 32, ks, lane);
#pragma unroll
        for (int i = 0; i < NI32; ++i) fb[i] = read_frag32<BS, TILE>(tb, wn * WN + i * 32, ks, lane);
#pragma unroll
        for (int j = 0; j < NJ32; ++j)
#pragma unroll
          for (int i = 0; i < NI32; ++i)
            acc32[W32 ? j : 0][W32 ? i : 0] =
                __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[j], fb[i], acc32[W32 ? j : 0][W32 ? i : 0], 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int k32 = 0; k32 < BK / 32; ++k32) {
        bf16x8 fa[NJ16], fb[NI16];
#pragma unroll
        for (int j = 0; j < NJ16; ++j) fa[j] = read_frag<AS, TILE>(ta, wm * WM + j * 16, k32, lane);
#pragma unroll
        for (int i = 0; i < NI16; ++i) fb[i] = read_frag<BS, TILE>(tb, wn * WN + i * 16, k32, lane);
#pragma unroll
        for (int j = 0; j < NJ16; ++j)
#pragma unroll
          for (int i = 0; i < NI16; ++i)
            acc[W32 ? 0 : j][W32 ? 0 : i] =
                __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[i], fa[j], acc[W32 ? 0 : j][W32 ? 0 : i], 0, 0, 0);
      }
    }
  };
  // step t of the reduction goes to stage t & 1
  auto issue = [&](int t) {
    char* st = smem + (t & 1) * kStageBytes;
    opa.template load<KMASK>(kb + t * BK, kend, st, wave);
    opb.template load<KMASK>(kb + t * BK, kend, st + kTileBytes, wave);
  };
  // this wavefront's loads have landed and its LDS reads are done; then the same for the others
  auto landed_barrier = [&]() {
    __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (0 << 8));   // vmcnt(0) lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
  };

  if (!PP) {
    issue(0);
    landed_barrier();
    for (int kt = 0; kt < nk; ++kt) {
      if (kt + 1 < nk) issue(kt + 1);   // into the stage every wavefront left before the last barrier
      compute(smem + (kt & 1) * kStageBytes);
      landed_barrier();
    }
  } else {
    // Two wavefronts share a SIMD (w and w + 4).  They alternate between a memory phase (all fragments of one
    // k-step from LDS into registers, loads of a later step issued) and a compute phase (the step's MFMAs, back
    // to back from registers), half a step apart, so that a SIMD's matrix core always has one wavefront
    // feeding it while the other waits for LDS and for the load queue.  Every phase ends at a workgroup
    // barrier; the late half executes one more barrier before its first phase and the early half one more
    // after its last.  The early half loads the tiles of A one step ahead into two buffers, the late half the
    // tiles of B two steps ahead into three, so every load has two phases to land before anyone waits for it
    // and the load unit sees the same number of instructions in every phase.
    const bool late = wave >= 4;
    const int w4 = wave & 3;
    constexpr int kLgkm0 = 0xC07F, kVm0 = 0x0F70;
    char* const a_ring = smem;                       // 2 tiles
    char* const b_ring = smem + 2 * kTileBytes;      // 3 tiles
    HalfLoader<AS, BS, W32, TILE> mine;
    mine.init(late, A, AS ? K : M, AS ? M : K, m0, B, BS ? K : N, BS ? N : K, n0, w4, lane, b_split);
    auto issue_a = [&](int t) { mine.template load<KMASK>(kb + t * BK, kend, a_ring + (t & 1) * kTileBytes, w4); };
    auto issue_b = [&](int t, int slot) { mine.template load<KMASK>(kb + t * BK, kend, b_ring + slot * kTileBytes, w4); };
    if (!late) issue_a(0);
    else { issue_b(0, 0); if (nk > 1) issue_b(1, 1); }
    __builtin_amdgcn_s_waitcnt(kVm0);
    __builtin_amdgcn_s_barrier();
    if (late) __builtin_amdgcn_s_barrier();
    int bs = 0;   // kt mod 3
    for (int kt = 0; kt < nk; ++kt) {
      const char* ta = a_ring + (kt & 1) * kTileBytes;
      const char* tb = b_ring + bs * kTileBytes;
      if (W32) {
        bf16x8 fa[BK / 16][NJ32], fb[BK / 16][NI32];
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
#pragma unroll
          for (int j = 0; j < NJ32; ++j) fa[ks][j] = read_frag32<AS, TILE>(ta, wm * WM + j * 32, ks, lane);
#pragma unroll
          for (int i = 0; i < NI32; ++i) fb[ks][i] = read_frag32<BS, TILE>(tb, wn * WN + i * 32, ks, lane);
        }
        if (!late) { if (kt + 1 < nk) issue_a(kt + 1); }
        else if (kt + 2 < nk) issue_b(kt + 2, bs == 0 ? 2 : bs - 1);
        __builtin_amdgcn_s_waitcnt(kLgkm0);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks)
#pragma unroll
          for (int j = 0; j < NJ32; ++j)
#pragma unroll
            for (int i = 0; i < NI32; ++i)
              acc32[W32 ? j : 0][W32 ? i : 0] =
                  __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks][j], fb[ks][i], acc32[W32 ? j : 0][W32 ? i : 0], 0, 0, 0);
        __builtin_amdgcn_s_setprio(0);
      } else {
        bf16x8 fa[BK / 32][NJ16], fb[BK / 32][NI16];
#pragma unroll
        for (int k32 = 0; k32 < BK / 32; ++k32) {
#pragma unroll
          for (int j = 0; j < NJ16; ++j) fa[k32][j] = read_frag<AS, TILE>(ta, wm * WM + j * 16, k32, lane);
#pragma unroll
          for (int i = 0; i < NI16; ++i) fb[k32][i] = read_frag<BS, TILE>(tb, wn * WN + i * 16, k32, lane);
        }
        if (!late) { if (kt + 1 < nk) issue_a(kt + 1); }
        else if (kt + 2 < nk) issue_b(kt + 2, bs == 0 ? 2 : bs - 1);
        __builtin_amdgcn_s_waitcnt(kLgkm0);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int k32 = 0; k32 < BK / 32; ++k32)
#pragma unroll
          for (int j = 0; j < NJ16; ++j)
#pragma unroll
            for (int i = 0; i < NI16; ++i)
              acc[W32 ? 0 : j][W32 ? 0 : i] =
                  __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[k32][i], fa[k32][j], acc[W32 ? 0 : j][W32 ? 0 : i], 0, 0, 0);
        __builtin_amdgcn_s_setprio(0);
      }
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_waitcnt(kVm0);   // issued two phases ago
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
      bs = bs == 2 ? 0 : bs + 1;
    }
    if (!late) __builtin_amdgcn_s_barrier();
  }

  // ---- epilogue.  With the tile of B as the MFMA's row operand (OP 0/1), accumulator r of lane l is output
  // row m = l % 16, output column n = (l / 16) * 4 + r of its 16x16 block: 4 consecutive columns.
  const int lm = lane & 15, kg = lane >> 4;
  if (OP == 2) {
    // float output, accumulated in place.  Here the tile of A is the MFMA's row operand: accumulator r of
    // lane l is output row (r/4)*8 + (l/32)*4 + r%4, column l%32, so a wavefront's atomic covers 128
    // contiguous bytes of two rows.
    float* C = reinterpret_cast<float*>(Cv);
#pragma unroll
    for (int j = 0; j < NJ32; ++j)
#pragma unroll
      for (int i = 0; i < NI32; ++i) {
        const int col = n0 + wn * WN + i * 32 + (lane & 31);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = m0 + wm * WM + j * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
          if (row < M && col < N) {
            float* p = C + (int64_t)row * N + col;
            unsafeAtomicAdd(p, acc32[W32 ? j : 0][W32 ? i : 0][r]);
          }
        }
      }
  } else {
    // all wavefronts are past the last barrier of the loop: the operand buffers are free
#pragma unroll
    for (int j = 0; j < NJ16; ++j)
#pragma unroll
      for (int i = 0; i < NI16; ++i) {
        uint2 w;
        w.x = pack_bf16(acc[W32 ? 0 : j][W32 ? 0 : i][0], acc[W32 ? 0 : j][W32 ? 0 : i][1]);
        w.y = pack_bf16(acc[W32 ? 0 : j][W32 ? 0 : i][2], acc[W32 ? 0 : j][W32 ? 0 : i][3]);
        *reinterpret_cast<uint2*>(smem + (wm * WM + j * 16 + lm) * kCRowBytes + (wn * WN + i * 16 + kg * 4) * 2) = w;
      }
    __syncthreads();
    bf16* C = reinterpret_cast<bf16*>(Cv);
    const bool add = OP == 0 && Rr != nullptr;
    if (EPI == kEpiSwiglu) {
      // chunk nc < TILE/16 of a staged row is 8 gate values, chunk nc + TILE/16 the up values of the same features
#pragma unroll 4
      for (int it = 0; it < TILE * TILE / 16 / kThreads; ++it) {
        const int c = tid + kThreads * it;
        const int row = c / (TILE / 16), nc = c % (TILE / 16);
        const int grow = m0 + row, gcol = n0 + nc * 8;
        if (grow < M) {
          const uint4 vg = *reinterpret_cast<const uint4*>(smem + row * kCRowBytes + nc * 16);
          const uint4 vu = *reinterpret_cast<const uint4*>(smem + row * kCRowBytes + (nc + TILE / 16) * 16);
          float g[8], u[8], o[8];
          unpack8(vg, g);
          unpack8(vu, u);
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] = g[e] / (1.0f + expf(-g[e])) * u[e];
          store16_stream(C + (int64_t)grow * N + gcol, vg);
          store16_stream(C + (int64_t)grow * N + hN + gcol, vu);
          store8_stream(aux + (int64_t)grow * hN + gcol, o);
        }
      }
    } else if (EPI == kEpiSwigluBwd) {
#pragma unroll 4
      for (int it = 0; it < TILE * TILE / 8 / kThreads; ++it) {
        const int c = tid + kThreads * it;
        const int row = c / (TILE / 8), nc = c % (TILE / 8);
        const int grow = m0 + row, gcol = n0 + nc * 8;
        if (grow < M && gcol < N) {
          float d[8], g[8], u[8], og[8], ou[8];
          unpack8(*reinterpret_cast<const uint4*>(smem + row * kCRowBytes + nc * 16), d);
          const int64_t at = (int64_t)grow * 2 * N + gcol;
          load8(Rr + at, g);
          load8(Rr + at + N, u);
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float sg = 1.0f / (1.0f + expf(-g[e]));
            og[e] = d[e] * u[e] * sg * (1.0f + g[e] * (1.0f - sg));
            ou[e] = d[e] * g[e] * sg;
          }
          store8_stream(C + at, og);
          store8_stream(C + at + N, ou);
        }
      }
    } else
#pragma unroll 4
    for (int it = 0; it < TILE * TILE / 8 / kThreads; ++it) {
      const int c = tid + kThreads * it;
      const int row = c / (TILE / 8), nc = c % (TILE / 8);
      const int grow = m0 + row, gcol = n0 + nc * 8;
      if (grow < M && gcol < N) {   // N is a multiple of 8: a chunk is inside or outside as a whole
        uint4 v = *reinterpret_cast<const uint4*>(smem + row * kCRowBytes + nc * 16);
        const int64_t at = (int64_t)grow * N + gcol;
        if (ROPE && gcol < rope.rot_cols) {
          // 8 columns = 4 pairs of one head (hd is a multiple of 8); their cos, sin are 32 contiguous bytes
          float x[8];
          const uint32_t wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) { x[2 * e] = bf16_bits_to_float(wv[e] & 0xffffu); x[2 * e + 1] = bf16_bits_to_float(wv[e] >> 16); }
          const float4* cs = reinterpret_cast<const float4*>(rope.table) + ((int64_t)(grow % rope.T) * (rope.hd / 2) + (gcol % rope.hd) / 2) / 2;
          const float4 c01 = cs[0], c23 = cs[1];
          const float c[4] = {c01.x, c01.z, c23.x, c23.z}, sn[4] = {c01.y, c01.w, c23.y, c23.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float a = x[2 * e], b = x[2 * e + 1];
            x[2 * e] = a * c[e] - b * sn[e];
            x[2 * e + 1] = a * sn[e] + b * c[e];
          }
          store8_stream(C + at, x);
        } else if (add) {
          // the sum is formed in float from the accumulator's bf16 rounding; one more rounding on the way out
          float x[8], y[8];
          const uint32_t wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) { x[2 * e] = bf16_bits_to_float(wv[e] & 0xffffu); x[2 * e + 1] = bf16_bits_to_float(wv[e] >> 16); }
          load8(Rr + at, y);
#pragma unroll
          for (int e = 0; e < 8; ++e) x[e] += y[e];
          store8_stream(C + at, x);
        } else {
          store16_stream(C + at, v);
        }
      }
    }
    __syncthreads();   // the staging area becomes the next piece's operand stages
  }
  }  // next piece
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
  // tile-relative byte offsets (up to 256 rows of the leading dimension) stay below 2^31
  if (M >= (1 << 21) || N >= (1 << 21) || K >= (1 << 21)) return false;
  if (!al16(A) || !al16(B) || !al16(C) || (R && !al16(R))) return false;
  if (((M + 127) / 128) * ((N + 127) / 128) > (1 << 24)) return false;
  if (N % 8) return false;                      // 16-byte output chunks
  switch (op) {
    case 0: return K % 8 == 0;
    case 1: return K % 8 == 0;
    case 2: return M % 8 == 0;
  }
  return false;
}

// epi: kEpiPlain (R optional), kEpiRope (rope given), kEpiSwiglu (N = 2h, aux = act out), kEpiSwigluBwd (N = h,
// R = gate|up in, C = d(gate)|d(up) out)
void gemm_mfma(hipStream_t s, int op, int64_t M, int64_t N, int64_t K, const void* A, const void* B, void* C,
               const void* R, const RopeArgs* rope, int epi, void* aux) {
  if (rope) epi = kEpiRope;
  // The chip delivers about the same aggregate rate with two thirds of its CUs busy as with all of them
  // (the kernel is bound by what the L2s and the power budget give), but a nearly empty round is lost time.
  const int cus = cu_count();
  // 256 x 256 tiles move the fewest bytes per flop; a product with too few of them to occupy the CUs
  // (a single microbatch through a narrow layer) takes 128 x 128 tiles instead
  const int64_t big = ((M + 255) / 256) * ((N + 255) / 256);
  int tile = (op != 2 && big * 4 < (int64_t)cus * 3) ? 128 : 256;
  if (epi == kEpiSwiglu && (N / 2) % 128) tile = 128;   // the caller has checked (N/2) % 64 == 0
  const int tm = (int)((M + tile - 1) / tile);
  // kEpiSwiglu: a tile covers tile/2 gate and the matching tile/2 up columns
  const int tn = epi == kEpiSwiglu ? (int)(N / tile) : (int)((N + tile - 1) / tile);
  const int tiles = tm * tn;
  int wgs;
  if (op == 2) {
    // a whole number s of runs per tile, so that the runs of neighbouring tiles walk the same k range
    // together: the smallest s whose last round of s * tiles workgroups is at least 0.65 full
    const int ksteps = (int)((K + BK - 1) / BK);
    int s_best = 1;
    for (int sp = 1; sp <= 8 && ksteps / sp >= 8; ++sp) {
      const int64_t w = (int64_t)tiles * sp;
      const int64_t last = w % cus;
      s_best = sp;
      if (last == 0 || last * 100 >= (int64_t)cus * 65 || w >= 6 * (int64_t)cus) break;
    }
    wgs = tiles * s_best;
  } else {
    // equally full rounds: ceil(tiles / rounds) workgroups, each taking every wgs-th tile
    const int rounds = (tiles + cus - 1) / cus;
    wgs = (tiles + rounds - 1) / rounds;
  }
  dim3 grid(wgs);
  const bf16* a = (const bf16*)A;
  const bf16* b = (const bf16*)B;
  const bf16* r = (const bf16*)R;
  const bool kmask = K % BK != 0;
  const RopeArgs ra = rope ? *rope : RopeArgs{nullptr, 1, 8, 0};
#define SP_LAUNCH(OP, KM, EP, TL) \
  hipLaunchKernelGGL((k_gemm_mfma<OP, KM, EP, TL, TL == 256>), grid, dim3(kThreads), 0, s, a, b, C, r, (int)M, (int)N, (int)K, tm, tn, ra, (bf16*)aux)
#define SP_LAUNCH_K(OP, EP, TL) \
  do { if (kmask) SP_LAUNCH(OP, true, EP, TL); else SP_LAUNCH(OP, false, EP, TL); } while (0)
#define SP_LAUNCH_T(OP, EP) \
  do { if (tile == 128) SP_LAUNCH_K(OP, EP, 128); else SP_LAUNCH_K(OP, EP, 256); } while (0)
  if (op == 0 && epi == kEpiRope) SP_LAUNCH_T(0, kEpiRope);
  else if (op == 0 && epi == kEpiSwiglu) SP_LAUNCH_T(0, kEpiSwiglu);
  else if (op == 0) SP_LAUNCH_T(0, kEpiPlain);
  else if (op == 1 && epi == kEpiSwigluBwd) SP_LAUNCH_T(1, kEpiSwigluBwd);
  else if (op == 1) SP_LAUNCH_T(1, kEpiPlain);
  else SP_LAUNCH(2, false, kEpiPlain, 256);
#undef SP_LAUNCH_T
#undef SP_LAUNCH_K
#undef SP_LAUNCH
}

bool gemm_swiglu_supported(bool bwd, int64_t R, int64_t h, int64_t d, const void* X, const void* W, const void* gu,
                           const void* other) {
  if (h % 64) return false;   // forward: a tile of 128 or 256 columns holds whole halves of gate and up
  if (bwd) return gemm_mfma_supported(1, R, h, d, X, W, other, gu);
  return gemm_mfma_supported(0, R, 2 * h, d, X, W, gu, other);
}

void gemm_mfma_swiglu_fwd(hipStream_t s, int64_t R, int64_t h, int64_t d, const void* hn, const void* wgu, void* gu, void* act) {
  gemm_mfma(s, 0, R, 2 * h, d, hn, wgu, gu, nullptr, nullptr, kEpiSwiglu, act);
}

void gemm_mfma_swiglu_bwd(hipStream_t s, int64_t R, int64_t h, int64_t d, const void* dy, const void* wd, const void* gu, void* dgu) {
  gemm_mfma(s, 1, R, h, d, dy, wd, dgu, gu, nullptr, kEpiSwigluBwd, nullptr);
}

}  // namespace sp
