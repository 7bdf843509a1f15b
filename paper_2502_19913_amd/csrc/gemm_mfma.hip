// bf16 matrix products on the CDNA4 matrix cores (v_mfma_f32_32x32x16_bf16), float accumulation.
//
// One workgroup of 8 wavefronts owns a 256x256 tile of the output and walks the reduction
// dimension in steps of 64.  Both operand tiles live in LDS as [row][k] with rows padded to 144
// bytes, double buffered (147 KB of the CU's 160 KB): a wavefront reads its MFMA fragments with one
// 16-byte LDS load per lane (8 consecutive k for one row), conflict free thanks to the padding.
// The next step's tiles are fetched from global memory into registers before the current step's
// MFMAs are issued and written to the other LDS buffer afterwards, so one barrier per step suffices.
//
// Operand layouts:
//   op 0  C[M,N]  = A[M,K] B[N,K]^T (+R)   both operands k-contiguous: 16-byte chunks go straight to LDS
//   op 1  C[M,N]  = A[M,K] B[K,N]          B is k-strided: 4x8 blocks are transposed in registers
//   op 2  C[M,N] += A[K,M]^T B[K,N]        both k-strided; float output, optional split of K with
//                                          atomic accumulation so that few output tiles still fill the chip
// Wavefront layout inside the tile: 2 (M) x 4 (N), each wavefront 128x64 = 4x2 MFMA tiles, 128
// accumulator registers.  Workgroup ids are regrouped so that the ids that land on one XCD (id mod 8)
// cover neighbouring tiles and share operand panels in that XCD's L2.
#include "devutil.h"
#include "internal.h"

namespace sp {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int kThreads = 512;
constexpr int kRowBytes = 144;                   // 64 bf16 + 16 bytes of padding
constexpr int kTileBytes = 256 * kRowBytes;      // one operand tile
constexpr int kLdsBytes = 4 * kTileBytes;        // A and B, two buffers

__device__ __forceinline__ uint4 zero4() { return make_uint4(0u, 0u, 0u, 0u); }

// ---- global -> registers ------------------------------------------------------------------------
// k-contiguous operand X[rows][ld]: tile rows [r0, r0+256), k in [k0, k0+64).  Thread t takes the
// 16-byte chunks t, t+512, t+1024, t+1536 of the 2048 in the tile (chunk = row*8 + kchunk).
__device__ __forceinline__ void load_kcontig(const bf16* __restrict__ X, int64_t ld, int rows, int r0, int k0, int kend,
                                             int tid, uint4 (&reg)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = tid + kThreads * i;
    const int row = c >> 3, kc = c & 7;
    const int gr = min(r0 + row, rows - 1);     // rows past the edge re-read the last row; never stored
    const int gk = k0 + kc * 8;
    reg[i] = gk < kend ? *reinterpret_cast<const uint4*>(X + (int64_t)gr * ld + gk) : zero4();
  }
}
__device__ __forceinline__ void store_kcontig(char* s, int tid, const uint4 (&reg)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = tid + kThreads * i;
    *reinterpret_cast<uint4*>(s + (c >> 3) * kRowBytes + (c & 7) * 16) = reg[i];
  }
}

// k-strided operand X[k][ld] (the tile's "row" index x runs along memory): x in [x0, x0+256),
// k in [k0, k0+64).  Thread t takes the 4(k) x 8(x) block (kquad = t & 15, xblock = t >> 4).
__device__ __forceinline__ void load_kstrided(const bf16* __restrict__ X, int64_t ld, int xdim, int x0, int k0, int kend,
                                              int tid, uint4 (&reg)[4]) {
  const int kq = tid & 15, xb = tid >> 4;
  const int gx = x0 + xb * 8;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int gk = k0 + kq * 4 + i;
    reg[i] = (gk < kend && gx < xdim) ? *reinterpret_cast<const uint4*>(X + (int64_t)gk * ld + gx) : zero4();
  }
}
// transposes the 4x8 block and writes 8 rows of 4 consecutive k (8 bytes each)
__device__ __forceinline__ void store_kstrided(char* s, int tid, const uint4 (&reg)[4]) {
  const int kq = tid & 15, xb = tid >> 4;
  const uint32_t w[4][4] = {{reg[0].x, reg[0].y, reg[0].z, reg[0].w}, {reg[1].x, reg[1].y, reg[1].z, reg[1].w},
                            {reg[2].x, reg[2].y, reg[2].z, reg[2].w}, {reg[3].x, reg[3].y, reg[3].z, reg[3].w}};
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
    *reinterpret_cast<uint2*>(s + (xb * 8 + c) * kRowBytes + kq * 8) = o;
  }
}

template <int OP>
__global__ __launch_bounds__(kThreads) void k_gemm_mfma(const bf16* __restrict__ A, const bf16* __restrict__ B,
                                                        void* __restrict__ Cv, const bf16* __restrict__ Rr, int M,
                                                        int N, int K, int tiles_m, int tiles_n, int ksplit) {
  __shared__ __attribute__((aligned(16))) char smem[kLdsBytes];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3;

  // ---- which tile: ids that share an XCD (id mod 8) get consecutive tiles; tiles run down M first
  // inside bands of 8 tile columns so that neighbours share B panels and reuse A panels
  const int tiles = tiles_m * tiles_n;
  int id = blockIdx.x;
  const int per_xcd = tiles / 8;
  if (id < per_xcd * 8) id = (id & 7) * per_xcd + (id >> 3);
  constexpr int kBand = 8;
  const int band = id / (kBand * tiles_m);
  const int band_w = min(kBand, tiles_n - band * kBand);
  const int in_band = id - band * kBand * tiles_m;
  const int tm = in_band / band_w, tn = band * kBand + in_band % band_w;
  const int m0 = tm * BM, n0 = tn * BN;
  const int kb = blockIdx.y * ksplit, kend = min(K, kb + ksplit);

  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  uint4 ra[4], rb[4];
  auto load_tiles = [&](int k0) {
    if (OP == 2) load_kstrided(A, M, M, m0, k0, kend, tid, ra); else load_kcontig(A, K, M, m0, k0, kend, tid, ra);
    if (OP == 0) load_kcontig(B, K, N, n0, k0, kend, tid, rb); else load_kstrided(B, N, N, n0, k0, kend, tid, rb);
  };
  auto store_tiles = [&](int buf) {
    char* sa = smem + buf * 2 * kTileBytes;
    char* sb = sa + kTileBytes;
    if (OP == 2) store_kstrided(sa, tid, ra); else store_kcontig(sa, tid, ra);
    if (OP == 0) store_kcontig(sb, tid, rb); else store_kstrided(sb, tid, rb);
  };

  const int nk = (kend - kb + BK - 1) / BK;
  if (nk > 0) {
    load_tiles(kb);
    store_tiles(0);
  }
  __syncthreads();
  const int frag_off = (lane & 31) * kRowBytes + (lane >> 5) * 16;
  for (int kt = 0; kt < nk; ++kt) {
    const bool more = kt + 1 < nk;
    if (more) load_tiles(kb + (kt + 1) * BK);
    const char* sa = smem + (kt & 1) * 2 * kTileBytes + wm * 128 * kRowBytes + frag_off;
    const char* sb = smem + (kt & 1) * 2 * kTileBytes + kTileBytes + wn * 64 * kRowBytes + frag_off;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 af[4], bf[2];
#pragma unroll
      for (int i = 0; i < 4; ++i) af[i] = *reinterpret_cast<const bf16x8*>(sa + i * 32 * kRowBytes + ks * 32);
#pragma unroll
      for (int j = 0; j < 2; ++j) bf[j] = *reinterpret_cast<const bf16x8*>(sb + j * 32 * kRowBytes + ks * 32);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
    if (more) store_tiles((kt + 1) & 1);
    __syncthreads();
  }

  // ---- epilogue.  Accumulator r of lane l sits at row (r/4)*8 + (l/32)*4 + r%4, column l%32 of its 32x32 tile.
  const bool atomic = gridDim.y > 1;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int col = n0 + wn * 64 + j * 32 + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * 128 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        if (row < M && col < N) {
          const int64_t at = (int64_t)row * N + col;
          if (OP == 2) {
            float* C = reinterpret_cast<float*>(Cv);
            if (atomic) unsafeAtomicAdd(C + at, acc[i][j][r]); else C[at] += acc[i][j][r];
          } else {
            bf16* C = reinterpret_cast<bf16*>(Cv);
            float v = acc[i][j][r];
            if (OP == 0 && Rr) v += (float)Rr[at];
            C[at] = (bf16)v;
          }
        }
      }
    }
}

inline bool al16(const void* p) { return ((uintptr_t)p & 15) == 0; }

}  // namespace

bool gemm_mfma_supported(int op, int64_t M, int64_t N, int64_t K, const void* A, const void* B, const void* C,
                         const void* R) {
  if (M < 1 || N < 1 || K < 1 || M > (1 << 30) || N > (1 << 30) || K > (1 << 30)) return false;
  if (!al16(A) || !al16(B) || !al16(C) || (R && !al16(R))) return false;
  if (((M + BM - 1) / BM) * ((N + BN - 1) / BN) > (1 << 24)) return false;
  switch (op) {
    case 0: return K % 8 == 0;
    case 1: return K % 8 == 0 && N % 8 == 0;
    case 2: return M % 8 == 0 && N % 8 == 0;
  }
  return false;
}

void gemm_mfma(hipStream_t s, int op, int64_t M, int64_t N, int64_t K, const void* A, const void* B, void* C,
               const void* R) {
  const int tm = (int)((M + BM - 1) / BM), tn = (int)((N + BN - 1) / BN);
  const int tiles = tm * tn;
  int splits = 1;
  if (op == 2) {
    // few output tiles and a long reduction: cut K so that about two rounds of workgroups fill 256 CUs
    const int ksteps = (int)((K + BK - 1) / BK);
    splits = std::max(1, std::min((512 + tiles - 1) / tiles, ksteps / 8));
    splits = std::min(splits, 64);
  }
  int ksplit = (int)(((K + splits - 1) / splits + BK - 1) / BK * BK);
  splits = (int)((K + ksplit - 1) / ksplit);
  dim3 grid(tiles, splits);
  const bf16* a = (const bf16*)A;
  const bf16* b = (const bf16*)B;
  const bf16* r = (const bf16*)R;
  if (op == 0)
    hipLaunchKernelGGL(k_gemm_mfma<0>, grid, dim3(kThreads), 0, s, a, b, C, r, (int)M, (int)N, (int)K, tm, tn, ksplit);
  else if (op == 1)
    hipLaunchKernelGGL(k_gemm_mfma<1>, grid, dim3(kThreads), 0, s, a, b, C, r, (int)M, (int)N, (int)K, tm, tn, ksplit);
  else
    hipLaunchKernelGGL(k_gemm_mfma<2>, grid, dim3(kThreads), 0, s, a, b, C, r, (int)M, (int)N, (int)K, tm, tn, ksplit);
}

}  // namespace sp
