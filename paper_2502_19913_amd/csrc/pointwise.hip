// Bandwidth-bound kernels of the stage: embedding, slot gather/scatter, RMSNorm, rotary embedding,
// SwiGLU and cross-entropy, each forward and backward.  One wavefront (64 lanes) owns one row
// wherever a row reduction is needed; rows are read with 16-byte loads when the width allows.
#include <algorithm>
#include <type_traits>

#include "devutil.h"
#include "internal.h"

namespace sp {

namespace {

constexpr int kBlock = 256;
constexpr int kWavesPerBlock = kBlock / kWave;

inline int grid_for_rows(int64_t rows, int rows_per_block, int cap = 4096) {
  int64_t g = (rows + rows_per_block - 1) / rows_per_block;
  if (g < 1) g = 1;
  return (int)(g > cap ? cap : g);
}

// ------------------------------------------------------------------------------------------ fill / copy
__global__ __launch_bounds__(kBlock) void k_fill_zero(uint32_t* p, int64_t n_words) {
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n_words; i += (int64_t)gridDim.x * kBlock) p[i] = 0u;
}

// Copies rows of `chunks` units of type U.  Row r of dst comes from row src_row(r) of src.
// mode 0: src row = idx[r] (embedding rows)        mode 1: gather slots        mode 2: scatter slots
// mode 0: an index outside [0, n_src_rows) raises *bad and yields a row of zeros
template <class U>
__global__ __launch_bounds__(kBlock) void k_copy_rows(const U* __restrict__ src, U* __restrict__ dst, int64_t rows,
                                                      int chunks, int mode, const int32_t* __restrict__ idx,
                                                      SlotList sl, int64_t rows_per_slot, int64_t n_src_rows,
                                                      int32_t* __restrict__ bad) {
  const int64_t total = rows * chunks;
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total; i += (int64_t)gridDim.x * kBlock) {
    int64_t r = i / chunks;
    int c = (int)(i - r * chunks);
    int64_t sr = r, dr = r;
    if (mode == 0) {
      sr = idx[r];
      if (sr < 0 || sr >= n_src_rows) {
        if (c == 0) *bad = 1;
        dst[dr * chunks + c] = U{};
        continue;
      }
    } else {
      int64_t g = r / rows_per_slot, w = r - g * rows_per_slot;
      int64_t pr = (int64_t)sl.slot[g] * rows_per_slot + w;
      if (mode == 1) sr = pr; else dr = pr;
    }
    dst[dr * chunks + c] = src[sr * chunks + c];
  }
}

void copy_rows(hipStream_t s, const void* src, void* dst, int64_t rows, int64_t row_bytes, int mode,
               const int32_t* idx, const SlotList& sl, int64_t rows_per_slot, int64_t n_src_rows = 0,
               int32_t* bad = nullptr) {
  if (rows <= 0) return;
  bool al16 = row_bytes % 16 == 0 && ((uintptr_t)src % 16 == 0) && ((uintptr_t)dst % 16 == 0);
  if (al16) {
    int chunks = (int)(row_bytes / 16);
    int grid = grid_for_rows(rows * chunks, kBlock * 4, 8192);
    hipLaunchKernelGGL(k_copy_rows<uint4>, dim3(grid), dim3(kBlock), 0, s, (const uint4*)src, (uint4*)dst, rows,
                       chunks, mode, idx, sl, rows_per_slot, n_src_rows, bad);
  } else {
    int chunks = (int)(row_bytes / 2);
    int grid = grid_for_rows(rows * chunks, kBlock * 4, 8192);
    hipLaunchKernelGGL(k_copy_rows<uint16_t>, dim3(grid), dim3(kBlock), 0, s, (const uint16_t*)src, (uint16_t*)dst,
                       rows, chunks, mode, idx, sl, rows_per_slot, n_src_rows, bad);
  }
}

// dE[tok[r], :] += dx[r, :]; a token outside [0, V) raises *bad and adds nothing
template <class T>
__global__ __launch_bounds__(kBlock) void k_embed_bwd(const T* __restrict__ dx, const int32_t* __restrict__ tok,
                                                      int64_t rows, int d, float* __restrict__ dE, int V,
                                                      int32_t* __restrict__ bad) {
  const int64_t total = rows * d;
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total; i += (int64_t)gridDim.x * kBlock) {
    int64_t r = i / d;
    int c = (int)(i - r * d);
    const int t = tok[r];
    if (t < 0 || t >= V) {
      if (c == 0) *bad = 1;
      continue;
    }
    unsafeAtomicAdd(dE + (int64_t)t * d + c, to_float(dx[i]));
  }
}

// ------------------------------------------------------------------------------------------ RMSNorm
// y = x * rstd * g, rstd = 1/sqrt(mean(x^2) + eps).  One wavefront per row; NV 8-wide vectors per lane.
template <class T, int NV>
__global__ __launch_bounds__(kBlock) void k_rmsnorm_fwd(const T* __restrict__ x, const T* __restrict__ g, int64_t R,
                                                        int d, float eps, T* __restrict__ y, float* __restrict__ rstd) {
  const int lane = threadIdx.x & 63;
  const int64_t nw = (int64_t)gridDim.x * kWavesPerBlock;
  for (int64_t r = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6); r < R; r += nw) {
    float v[NV][8];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      int col = (lane + 64 * i) * 8;
      if (col < d) {
        load8(x + r * d + col, v[i]);
#pragma unroll
        for (int j = 0; j < 8; ++j) ss += v[i][j] * v[i][j];
      }
    }
    ss = wave_sum(ss);
    const float rs = 1.0f / sqrtf(ss / (float)d + eps);
    if (lane == 0) rstd[r] = rs;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      int col = (lane + 64 * i) * 8;
      if (col < d) {
        float gv[8], o[8];
        load8(g + col, gv);
#pragma unroll
        for (int j = 0; j < 8; ++j) o[j] = v[i][j] * rs * gv[j];
        store8(y + r * d + col, o);
      }
    }
  }
}

template <class T>
__global__ __launch_bounds__(kBlock) void k_rmsnorm_fwd_scalar(const T* __restrict__ x, const T* __restrict__ g,
                                                               int64_t R, int d, float eps, T* __restrict__ y,
                                                               float* __restrict__ rstd) {
  const int lane = threadIdx.x & 63;
  const int64_t nw = (int64_t)gridDim.x * kWavesPerBlock;
  for (int64_t r = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6); r < R; r += nw) {
    float ss = 0.f;
    for (int c = lane; c < d; c += 64) { float a = to_float(x[r * d + c]); ss += a * a; }
    ss = wave_sum(ss);
    const float rs = 1.0f / sqrtf(ss / (float)d + eps);
    if (lane == 0) rstd[r] = rs;
    for (int c = lane; c < d; c += 64) y[r * d + c] = from_float<T>(to_float(x[r * d + c]) * rs * to_float(g[c]));
  }
}

// xh = x*rstd ; dxh = dy*g ; dx = rstd*(dxh - xh*mean(dxh*xh)) (+ dres) ; dg += sum_rows dy*xh.
// Each lane keeps the dg partial sums of its columns over all rows its wavefront visits; the block
// folds its four wavefronts in LDS and hands one value per column on: into its own row of part_out when that is
// given (a second kernel adds the rows up: hundreds of blocks adding atomically into the same d addresses
// queue up at a few L2 channels and cost more than the rows' traffic), else as one atomic add per column.
template <class T, int NV>
__global__ __launch_bounds__(kBlock) void k_rmsnorm_bwd(const T* __restrict__ dy, const T* __restrict__ x,
                                                        const T* __restrict__ g, const float* __restrict__ rstd,
                                                        const T* __restrict__ dres, int64_t R, int d,
                                                        T* __restrict__ dx, float* __restrict__ dg,
                                                        float* __restrict__ part_out) {
  extern __shared__ float s_dg[];
  const int lane = threadIdx.x & 63;
  const int64_t nw = (int64_t)gridDim.x * kWavesPerBlock;
  float acc[NV][8];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[i][j] = 0.f;
  }
  for (int64_t r = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6); r < R; r += nw) {
    const float rs = rstd[r];
    float vdy[NV][8], vx[NV][8];
    float m = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      int col = (lane + 64 * i) * 8;
      if (col < d) {
        float gv[8];
        load8(dy + r * d + col, vdy[i]);
        load8(x + r * d + col, vx[i]);
        load8(g + col, gv);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          vx[i][j] *= rs;                       // xh
          acc[i][j] += vdy[i][j] * vx[i][j];    // dg partial
          vdy[i][j] *= gv[j];                   // dxh
          m += vdy[i][j] * vx[i][j];
        }
      }
    }
    m = wave_sum(m) / (float)d;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      int col = (lane + 64 * i) * 8;
      if (col < d) {
        float o[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) o[j] = rs * (vdy[i][j] - vx[i][j] * m);
        if (dres) {
          float rv[8];
          load8(dres + r * d + col, rv);
#pragma unroll
          for (int j = 0; j < 8; ++j) o[j] += rv[j];
        }
        store8(dx + r * d + col, o);
      }
    }
  }
  // fold the block's four wavefronts: each writes its partial sums to its own row of LDS, then every column is
  // added up by one thread and goes out as one atomic
  float* part = s_dg + (size_t)(threadIdx.x >> 6) * d;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    int col = (lane + 64 * i) * 8;
    if (col < d) {
#pragma unroll
      for (int j = 0; j < 8; ++j) part[col + j] = acc[i][j];
    }
  }
  __syncthreads();
  for (int c = threadIdx.x; c < d; c += kBlock) {
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) v += s_dg[(size_t)w * d + c];
    if (part_out) part_out[(size_t)blockIdx.x * d + c] = v;
    else unsafeAtomicAdd(dg + c, v);
  }
}

// The same for bf16, columns instead of rows divided among the wavefronts: the block's four wavefronts share
// each row (wavefront w takes the 512-column pieces w, w + 4, ..), so a lane's gain and its gain-gradient sums
// are NVW x 8 values for the whole kernel and nothing has to be folded across wavefronts at the end.  RPI rows are
// in flight together (dy, x and the added gradient all loaded before the first is used); the four partial sums
// of a row's mean meet in LDS, one barrier per RPI rows (two sets of slots, alternating, so that the next
// round's sums never overwrite one still being read).
template <int NVW, int RPI, bool HAS_RES>
__global__ __launch_bounds__(kBlock) void k_rmsnorm_bwd_cols(const bf16* __restrict__ dy, const bf16* __restrict__ x,
                                                             const bf16* __restrict__ g, const float* __restrict__ rstd,
                                                             const bf16* __restrict__ dres, int64_t R, int d,
                                                             bf16* __restrict__ dx, float* __restrict__ dg,
                                                             float* __restrict__ part_out) {
  __shared__ float s_m[2][RPI][kWavesPerBlock];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int col[NVW];
  uint32_t coff[NVW];   // byte offset of the piece in a row; 0 for a lane past the end of the row (loads stay in bounds, the
                        // lane's gain is zero and nothing of it is stored)
  float gv[NVW][8], acc[NVW][8];
#pragma unroll
  for (int i = 0; i < NVW; ++i) {
    col[i] = ((i * kWavesPerBlock + wave) * 64 + lane) * 8;
    coff[i] = col[i] < d ? (uint32_t)col[i] * 2u : 0u;
#pragma unroll
    for (int j = 0; j < 8; ++j) { acc[i][j] = 0.f; gv[i][j] = 0.f; }
    if (col[i] < d) load8(g + col[i], gv[i]);
  }
  const float inv_d = 1.0f / (float)d;
  // a row's (uniform) byte offset + the lane's 32-bit byte offset: one address register per piece for all streams
  const char* const dyb = reinterpret_cast<const char*>(dy);
  const char* const xb = reinterpret_cast<const char*>(x);
  const char* const resb = reinterpret_cast<const char*>(dres);
  char* const dxb = reinterpret_cast<char*>(dx);
  int par = 0;
#pragma nounroll
  for (int64_t r0 = (int64_t)blockIdx.x * RPI; r0 < R; r0 += (int64_t)gridDim.x * RPI, par ^= 1) {
    // all loads of the round first, unconditionally: a row past the end reads the last row again and counts
    // for nothing (its rstd is taken as zero)
    uint4 qdy[RPI][NVW], qx[RPI][NVW], qres[HAS_RES ? RPI : 1][NVW];
#pragma unroll
    for (int rr = 0; rr < RPI; ++rr) {
      const size_t rb = (size_t)(r0 + rr < R ? r0 + rr : R - 1) * d * 2;
#pragma unroll
      for (int i = 0; i < NVW; ++i) {
        qdy[rr][i] = *reinterpret_cast<const uint4*>(dyb + rb + coff[i]);
        qx[rr][i] = *reinterpret_cast<const uint4*>(xb + rb + coff[i]);
        if (HAS_RES) qres[rr][i] = *reinterpret_cast<const uint4*>(resb + rb + coff[i]);
      }
    }
    float dxh[RPI][NVW][8], xh[RPI][NVW][8], rs[RPI];
#pragma unroll
    for (int rr = 0; rr < RPI; ++rr) {
      rs[rr] = r0 + rr < R ? rstd[r0 + rr] : 0.f;
      float m = 0.f;
#pragma unroll
      for (int i = 0; i < NVW; ++i) {
        unpack8(qdy[rr][i], dxh[rr][i]);
        unpack8(qx[rr][i], xh[rr][i]);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          xh[rr][i][j] *= rs[rr];
          acc[i][j] += dxh[rr][i][j] * xh[rr][i][j];   // dg partial
          dxh[rr][i][j] *= gv[i][j];
          m += dxh[rr][i][j] * xh[rr][i][j];
        }
      }
      m = wave_sum(m);
      if (lane == 0) s_m[par][rr][wave] = m;
    }
    __syncthreads();
#pragma unroll
    for (int rr = 0; rr < RPI; ++rr) {
      const bool row_in = r0 + rr < R;
      const float m = ((s_m[par][rr][0] + s_m[par][rr][1]) + (s_m[par][rr][2] + s_m[par][rr][3])) * inv_d;
      const size_t rb = (size_t)(row_in ? r0 + rr : R - 1) * d * 2;
#pragma unroll
      for (int i = 0; i < NVW; ++i) {
        float o[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) o[j] = rs[rr] * (dxh[rr][i][j] - xh[rr][i][j] * m);
        if (HAS_RES) {
          float rv[8];
          unpack8(qres[rr][i], rv);
#pragma unroll
          for (int j = 0; j < 8; ++j) o[j] += rv[j];
        }
        if (row_in && col[i] < d) store8(reinterpret_cast<bf16*>(dxb + rb + coff[i]), o);
      }
    }
  }
#pragma unroll
  for (int i = 0; i < NVW; ++i) {
    if (col[i] < d) {
      if (part_out) store8(part_out + (size_t)blockIdx.x * d + col[i], acc[i]);
      else {
#pragma unroll
        for (int j = 0; j < 8; ++j) unsafeAtomicAdd(dg + col[i] + j, acc[i][j]);
      }
    }
  }
}

// dg[c] += sum over n rows of part[row][c].  A block takes 64 columns and one of gridDim.y runs of rows: its four
// wavefronts stride the run's rows, fold in LDS, and add one value per column atomically (gridDim.y adds per
// address in all).
__global__ __launch_bounds__(kBlock) void k_colsum_add(const float* __restrict__ part, int n, int d, float* __restrict__ dg) {
  __shared__ float s_part[kWavesPerBlock][64];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, c = blockIdx.x * 64 + lane;
  const int per = (n + gridDim.y - 1) / gridDim.y, r0 = blockIdx.y * per, r1 = min(n, r0 + per);
  float v0 = 0.f, v1 = 0.f;
  if (c < d) {
    int r = r0 + w;
    for (; r + kWavesPerBlock < r1; r += 2 * kWavesPerBlock) {
      v0 += part[(size_t)r * d + c];
      v1 += part[(size_t)(r + kWavesPerBlock) * d + c];
    }
    if (r < r1) v0 += part[(size_t)r * d + c];
  }
  s_part[w][lane] = v0 + v1;
  __syncthreads();
  if (w == 0 && c < d) unsafeAtomicAdd(dg + c, (s_part[0][lane] + s_part[1][lane]) + (s_part[2][lane] + s_part[3][lane]));
}

template <class T>
__global__ __launch_bounds__(kBlock) void k_rmsnorm_bwd_scalar(const T* __restrict__ dy, const T* __restrict__ x,
                                                               const T* __restrict__ g, const float* __restrict__ rstd,
                                                               const T* __restrict__ dres, int64_t R, int d,
                                                               T* __restrict__ dx, float* __restrict__ dg) {
  const int lane = threadIdx.x & 63;
  const int64_t nw = (int64_t)gridDim.x * kWavesPerBlock;
  for (int64_t r = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6); r < R; r += nw) {
    const float rs = rstd[r];
    float m = 0.f;
    for (int c = lane; c < d; c += 64)
      m += to_float(dy[r * d + c]) * to_float(g[c]) * to_float(x[r * d + c]) * rs;
    m = wave_sum(m) / (float)d;
    for (int c = lane; c < d; c += 64) {
      float xh = to_float(x[r * d + c]) * rs, gy = to_float(dy[r * d + c]);
      float o = rs * (gy * to_float(g[c]) - xh * m);
      if (dres) o += to_float(dres[r * d + c]);
      dx[r * d + c] = from_float<T>(o);
      unsafeAtomicAdd(dg + c, gy * xh);
    }
  }
}

// ------------------------------------------------------------------------------------------ rotary embedding
// One thread turns one pair.  pairs_per_row = nheads*hd/2; angle = (row % T) * theta^(-2i/hd).
template <class T>
__global__ __launch_bounds__(kBlock) void k_rope(T* __restrict__ qk, int64_t R, int T_, int pairs_per_row, int hd,
                                                 int row_stride, float log2_theta, float sign) {
  const int64_t total = R * pairs_per_row;
  const int half = hd / 2;
  for (int64_t idx = (int64_t)blockIdx.x * kBlock + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * kBlock) {
    int64_t r = idx / pairs_per_row;
    int pr = (int)(idx - r * pairs_per_row);
    int i = pr % half;
    int p = (int)(r % T_);
    float inv = exp2f(-(float)(2 * i) / (float)hd * log2_theta);
    float sn, cs;
    sincosf((float)p * inv, &sn, &cs);
    sn *= sign;
    T* v = qk + r * row_stride + 2 * pr;
    float a = to_float(v[0]), b = to_float(v[1]);
    v[0] = from_float<T>(a * cs - b * sn);
    v[1] = from_float<T>(a * sn + b * cs);
  }
}

// cos and sin of the same angles, tabulated: entry p * hd/2 + i
__global__ __launch_bounds__(kBlock) void k_rope_table(float2* __restrict__ table, int T_, int hd, float log2_theta) {
  const int half = hd / 2;
  const int idx = blockIdx.x * kBlock + threadIdx.x;
  if (idx >= T_ * half) return;
  const int p = idx / half, i = idx - p * half;
  float inv = exp2f(-(float)(2 * i) / (float)hd * log2_theta);
  float sn, cs;
  sincosf((float)p * inv, &sn, &cs);
  table[idx] = make_float2(cs, sn);
}

// ------------------------------------------------------------------------------------------ SwiGLU
template <class T>
__global__ __launch_bounds__(kBlock) void k_swiglu_fwd(const T* __restrict__ gu, int64_t R, int h, T* __restrict__ a) {
  const int hv = h / 8;
  const int64_t total = R * hv;
  for (int64_t idx = (int64_t)blockIdx.x * kBlock + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * kBlock) {
    int64_t r = idx / hv;
    int c = (int)(idx - r * hv) * 8;
    float g[8], u[8], o[8];
    load8(gu + r * 2 * h + c, g);
    load8(gu + r * 2 * h + h + c, u);
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = g[j] / (1.0f + expf(-g[j])) * u[j];
    store8(a + r * h + c, o);
  }
}

template <class T>
__global__ __launch_bounds__(kBlock) void k_swiglu_bwd(const T* __restrict__ da, const T* __restrict__ gu, int64_t R,
                                                       int h, T* __restrict__ dgu) {
  const int hv = h / 8;
  const int64_t total = R * hv;
  for (int64_t idx = (int64_t)blockIdx.x * kBlock + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * kBlock) {
    int64_t r = idx / hv;
    int c = (int)(idx - r * hv) * 8;
    float g[8], u[8], d[8], og[8], ou[8];
    load8(gu + r * 2 * h + c, g);
    load8(gu + r * 2 * h + h + c, u);
    load8(da + r * h + c, d);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float sg = 1.0f / (1.0f + expf(-g[j]));
      og[j] = d[j] * u[j] * sg * (1.0f + g[j] * (1.0f - sg));
      ou[j] = d[j] * g[j] * sg;
    }
    store8(dgu + r * 2 * h + c, og);
    store8(dgu + r * 2 * h + h + c, ou);
  }
}

template <class T>
__global__ __launch_bounds__(kBlock) void k_swiglu_fwd_scalar(const T* __restrict__ gu, int64_t R, int h,
                                                              T* __restrict__ a) {
  const int64_t total = R * h;
  for (int64_t idx = (int64_t)blockIdx.x * kBlock + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * kBlock) {
    int64_t r = idx / h;
    int c = (int)(idx - r * h);
    float g = to_float(gu[r * 2 * h + c]), u = to_float(gu[r * 2 * h + h + c]);
    a[idx] = from_float<T>(g / (1.0f + expf(-g)) * u);
  }
}

template <class T>
__global__ __launch_bounds__(kBlock) void k_swiglu_bwd_scalar(const T* __restrict__ da, const T* __restrict__ gu,
                                                              int64_t R, int h, T* __restrict__ dgu) {
  const int64_t total = R * h;
  for (int64_t idx = (int64_t)blockIdx.x * kBlock + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * kBlock) {
    int64_t r = idx / h;
    int c = (int)(idx - r * h);
    float g = to_float(gu[r * 2 * h + c]), u = to_float(gu[r * 2 * h + h + c]), d = to_float(da[idx]);
    float sg = 1.0f / (1.0f + expf(-g));
    dgu[r * 2 * h + c] = from_float<T>(d * u * sg * (1.0f + g * (1.0f - sg)));
    dgu[r * 2 * h + h + c] = from_float<T>(d * g * sg);
  }
}

// ------------------------------------------------------------------------------------------ cross-entropy
// A target is a vocabulary entry or -1 (ignored).  Anything else raises *bad and is treated as ignored, here and
// in the loss kernel alike.
__global__ __launch_bounds__(kBlock) void k_count_targets(const int32_t* __restrict__ tgt, int64_t rows_per_mb, int V,
                                                          int32_t* __restrict__ counts, int32_t* __restrict__ bad) {
  __shared__ int s_cnt[kWavesPerBlock];
  const int mb = blockIdx.x;
  int c = 0;
  for (int64_t r = threadIdx.x; r < rows_per_mb; r += kBlock) {
    const int t = tgt[(int64_t)mb * rows_per_mb + r];
    c += t >= 0 && t < V;
    if (t < -1 || t >= V) *bad = 1;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o);
  if ((threadIdx.x & 63) == 0) s_cnt[threadIdx.x >> 6] = c;
  __syncthreads();
  if (threadIdx.x == 0) {
    int t = 0;
    for (int w = 0; w < kWavesPerBlock; ++w) t += s_cnt[w];
    counts[mb] = t;
  }
}

// One block per row: running (max, sum of exp) per thread, folded over the block, then the row is
// rewritten as (softmax - onehot) * scale.  VEC = 8-wide accesses (V % 8 == 0), else element-wise.
template <class T, bool VEC>
__global__ __launch_bounds__(kBlock) void k_cross_entropy(T* __restrict__ logits, const int32_t* __restrict__ tgt,
                                                          int64_t row0, int V, int64_t rows_per_mb,
                                                          const int32_t* __restrict__ counts, float inv_n_mb,
                                                          float* __restrict__ loss_mb) {
  __shared__ float s_m[kWavesPerBlock], s_s[kWavesPerBlock];
  const int64_t r = blockIdx.x;
  T* z = logits + r * (int64_t)V;
  const int64_t grow = row0 + r;
  const int t = tgt[grow];
  const int mb = (int)(grow / rows_per_mb);
  if (t < 0 || t >= V) {  // ignored position: no loss, zero gradient
    if (VEC) {
      float zero[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      for (int c = threadIdx.x * 8; c < V; c += kBlock * 8) store8(z + c, zero);
    } else {
      for (int c = threadIdx.x; c < V; c += kBlock) z[c] = from_float<T>(0.f);
    }
    return;
  }
  float mx = -INFINITY, sm = 0.f;
  if (VEC) {
    for (int c = threadIdx.x * 8; c < V; c += kBlock * 8) {
      float v[8];
      load8(z + c, v);
      float lm = v[0];
#pragma unroll
      for (int j = 1; j < 8; ++j) lm = fmaxf(lm, v[j]);
      if (lm > mx) { sm *= expf(mx - lm); mx = lm; }
#pragma unroll
      for (int j = 0; j < 8; ++j) sm += expf(v[j] - mx);
    }
  } else {
    for (int c = threadIdx.x; c < V; c += kBlock) {
      float v = to_float(z[c]);
      if (v > mx) { sm *= expf(mx - v); mx = v; }
      sm += expf(v - mx);
    }
  }
  // fold (mx, sm) pairs: wavefront, then block
  float wm = wave_max(mx);
  sm = wave_sum(mx == -INFINITY ? 0.f : sm * expf(mx - wm));
  if ((threadIdx.x & 63) == 0) { s_m[threadIdx.x >> 6] = wm; s_s[threadIdx.x >> 6] = sm; }
  __syncthreads();
  float bm = s_m[0];
#pragma unroll
  for (int w = 1; w < kWavesPerBlock; ++w) bm = fmaxf(bm, s_m[w]);
  float bs = 0.f;
#pragma unroll
  for (int w = 0; w < kWavesPerBlock; ++w) bs += s_s[w] * expf(s_m[w] - bm);
  const float lse = bm + logf(bs);
  const float cnt = (float)counts[mb];
  const float scale = inv_n_mb / cnt;
  const float zt = to_float(z[t]);
  __syncthreads();  // every thread has read z[t] before anyone overwrites it
  if (threadIdx.x == 0) unsafeAtomicAdd(loss_mb + mb, (lse - zt) / cnt);
  if (VEC) {
    for (int c = threadIdx.x * 8; c < V; c += kBlock * 8) {
      float v[8];
      load8(z + c, v);
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = (expf(v[j] - lse) - ((c + j) == t ? 1.f : 0.f)) * scale;
      store8(z + c, v);
    }
  } else {
    for (int c = threadIdx.x; c < V; c += kBlock)
      z[c] = from_float<T>((expf(to_float(z[c]) - lse) - (c == t ? 1.f : 0.f)) * scale);
  }
}

// bf16 rows that fit a workgroup's registers (V <= NT * 8 * NCH): the row is read once, as NCH 16-byte pieces per
// thread all in flight together, reduced from registers (block maximum, then the sum of exponentials), and
// written once as (softmax - onehot) * scale: 4 V bytes of traffic per row instead of 6 V, and NCH loads per thread
// outstanding instead of one.  Exponentials by the hardware's exp2 (the results are rounded to bf16).
template <int NT, int NCH>
__global__ __launch_bounds__(NT) void k_cross_entropy_row(bf16* __restrict__ logits, const int32_t* __restrict__ tgt,
                                                          int64_t row0, int V, int64_t rows_per_mb,
                                                          const int32_t* __restrict__ counts, float inv_n_mb,
                                                          float* __restrict__ loss_mb) {
  constexpr int NWV = NT / 64;
  __shared__ float s_m[NWV], s_s[NWV], s_zt;
  const int64_t r = blockIdx.x;
  bf16* z = logits + r * (int64_t)V;
  const int64_t grow = row0 + r;
  const int t = tgt[grow];
  const int mb = (int)(grow / rows_per_mb);
  if (t < 0 || t >= V) {  // ignored position: no loss, zero gradient
    for (int c = threadIdx.x * 8; c < V; c += NT * 8) store16_stream(z + c, make_uint4(0u, 0u, 0u, 0u));
    return;
  }
  uint4 q[NCH];
  char* const zb = reinterpret_cast<char*>(z);
  const uint32_t toff = threadIdx.x * 16u;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = (i * NT + threadIdx.x) * 8;
    // uniform piece base + 32-bit lane offset: one address register for all pieces
    q[i] = c < V ? load16_stream(zb + (size_t)i * NT * 16 + toff) : make_uint4(0xff80ff80u, 0xff80ff80u, 0xff80ff80u, 0xff80ff80u);   // -inf
  }
  float mx = -INFINITY;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    float v[8];
    forget_derived(q[i], mx);
    unpack8(q[i], v);
#pragma unroll
    for (int j = 0; j < 8; ++j) mx = fmaxf(mx, v[j]);
  }
  mx = wave_max(mx);
  if ((threadIdx.x & 63) == 0) s_m[threadIdx.x >> 6] = mx;
  __syncthreads();
  float bm = s_m[0];
#pragma unroll
  for (int w = 1; w < NWV; ++w) bm = fmaxf(bm, s_m[w]);
  float sm = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = (i * NT + threadIdx.x) * 8;
    float v[8];
    forget_derived(q[i], sm);
    unpack8(q[i], v);
#pragma unroll
    for (int j = 0; j < 8; ++j) sm += __expf(v[j] - bm);
    const unsigned jt = (unsigned)(t - c);
    if (jt < 8u) {   // this piece holds the target's logit: one thread of the block, once
      float zt = v[0];
#pragma unroll
      for (int j = 1; j < 8; ++j) zt = jt == (unsigned)j ? v[j] : zt;
      s_zt = zt;
    }
  }
  sm = wave_sum(sm);
  if ((threadIdx.x & 63) == 0) s_s[threadIdx.x >> 6] = sm;
  __syncthreads();
  float bs = 0.f;
#pragma unroll
  for (int w = 0; w < NWV; ++w) bs += s_s[w];
  const float lse = bm + logf(bs);
  const float cnt = (float)counts[mb];
  const float scale = inv_n_mb / cnt;
  if (threadIdx.x == 0) unsafeAtomicAdd(loss_mb + mb, (lse - s_zt) / cnt);
  float last = 0.f;   // a value of the piece before: orders the pieces
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = (i * NT + threadIdx.x) * 8;
    if (c < V) {
      float v[8];
      forget_derived(q[i], last);
      unpack8(q[i], v);
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = __expf(v[j] - lse) * scale;
      const unsigned jt = (unsigned)(t - c);
      if (jt < 8u) {
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] -= jt == (unsigned)j ? scale : 0.f;
      }
      last = v[7];
      store8_stream(reinterpret_cast<bf16*>(zb + (size_t)i * NT * 16 + toff), v);
    }
  }
}

template <class T> bool aligned16(const void* p) { return ((uintptr_t)p % 16) == 0; }

}  // namespace

// ------------------------------------------------------------------------------------------ launchers
void fill_zero(hipStream_t s, void* p, int64_t bytes) {
  if (bytes <= 0) return;
  int64_t words = bytes / 4;  // every buffer this library clears is a whole number of 32-bit words
  hipLaunchKernelGGL(k_fill_zero, dim3(grid_for_rows(words, kBlock * 8, 8192)), dim3(kBlock), 0, s, (uint32_t*)p, words);
}

void embed_fwd(hipStream_t s, int dtype, const void* E, const int32_t* tok, int64_t rows, int d, int V, void* x,
               int32_t* bad) {
  SlotList none{};
  copy_rows(s, E, x, rows, d * elt_size(dtype), 0, tok, none, 1, V, bad);
}

void embed_bwd(hipStream_t s, int dtype, const void* dx, const int32_t* tok, int64_t rows, int d, int V, float* dE,
               int32_t* bad) {
  if (rows <= 0) return;
  int grid = grid_for_rows(rows * d, kBlock * 4, 8192);
  if (dtype == SP_BF16)
    hipLaunchKernelGGL(k_embed_bwd<bf16>, dim3(grid), dim3(kBlock), 0, s, (const bf16*)dx, tok, rows, d, dE, V, bad);
  else
    hipLaunchKernelGGL(k_embed_bwd<float>, dim3(grid), dim3(kBlock), 0, s, (const float*)dx, tok, rows, d, dE, V, bad);
}

void gather_slots(hipStream_t s, int dtype, const void* pool, const SlotList& sl, int64_t rows_per_slot, int d,
                  void* dst) {
  const int pi = prof_start(PROF_COPY_ROWS, s);
  copy_rows(s, pool, dst, sl.n * rows_per_slot, d * elt_size(dtype), 1, nullptr, sl, rows_per_slot);
  prof_stop(pi, s, 2.0 * sl.n * rows_per_slot * d * elt_size(dtype));
}

void scatter_slots(hipStream_t s, int dtype, const void* src, const SlotList& sl, int64_t rows_per_slot, int d,
                   void* pool) {
  const int pi = prof_start(PROF_COPY_ROWS, s);
  copy_rows(s, src, pool, sl.n * rows_per_slot, d * elt_size(dtype), 2, nullptr, sl, rows_per_slot);
  prof_stop(pi, s, 2.0 * sl.n * rows_per_slot * d * elt_size(dtype));
}

template <class T>
static void rmsnorm_fwd_t(hipStream_t s, const T* x, const T* g, int64_t R, int d, float eps, T* y, float* rstd) {
  if (R <= 0) return;
  int grid = grid_for_rows(R, kWavesPerBlock, 16384);
  bool vec = d % 8 == 0 && d <= 8192 && aligned16<T>(x) && aligned16<T>(g) && aligned16<T>(y);
  if (!vec) {
    hipLaunchKernelGGL(k_rmsnorm_fwd_scalar<T>, dim3(grid), dim3(kBlock), 0, s, x, g, R, d, eps, y, rstd);
    return;
  }
  int nv = (d + 511) / 512;
#define SP_CASE(N) hipLaunchKernelGGL((k_rmsnorm_fwd<T, N>), dim3(grid), dim3(kBlock), 0, s, x, g, R, d, eps, y, rstd)
  if (nv <= 1) SP_CASE(1); else if (nv <= 2) SP_CASE(2); else if (nv <= 4) SP_CASE(4); else if (nv <= 8) SP_CASE(8); else SP_CASE(16);
#undef SP_CASE
}

void rmsnorm_fwd(hipStream_t s, int dtype, const void* x, const void* g, int64_t R, int d, float eps, void* y,
                 float* rstd) {
  const int pi = prof_start(PROF_RMSNORM_FWD, s);
  if (dtype == SP_BF16) rmsnorm_fwd_t<bf16>(s, (const bf16*)x, (const bf16*)g, R, d, eps, (bf16*)y, rstd);
  else rmsnorm_fwd_t<float>(s, (const float*)x, (const float*)g, R, d, eps, (float*)y, rstd);
  prof_stop(pi, s, 2.0 * R * d * elt_size(dtype));   // x read, y written
}

template <class T>
static void rmsnorm_bwd_t(hipStream_t s, const T* dy, const T* x, const T* g, const float* rstd, const T* dres,
                          int64_t R, int d, T* dx, float* dg, float* part, int64_t part_floats) {
  if (R <= 0) return;
  // the gain-gradient fold keeps one row of d floats per wavefront in LDS: 64 KB at d = 4096
  bool vec = d % 8 == 0 && d <= 4096 && aligned16<T>(x) && aligned16<T>(g) && aligned16<T>(dy) && aligned16<T>(dx) &&
             (!dres || aligned16<T>(dres));
  if (!vec) {
    int grid = grid_for_rows(R, kWavesPerBlock, 16384);
    hipLaunchKernelGGL(k_rmsnorm_bwd_scalar<T>, dim3(grid), dim3(kBlock), 0, s, dy, x, g, rstd, dres, R, d, dx, dg);
    return;
  }
  int grid = grid_for_rows(R, kWavesPerBlock * 4, 1024);  // >= 4 rows per wavefront amortise the dg fold
  size_t lds = (size_t)d * sizeof(float) * kWavesPerBlock;
  int nv = (d + 511) / 512;
  float* pp = (part && (int64_t)grid * d <= part_floats && grid > 8) ? part : nullptr;
  if constexpr (std::is_same<T, bf16>::value) {
    // d <= 2048: one piece per lane, 4 rows in flight; d <= 4096: two pieces, 2 rows
    const int rpi = d <= 2048 ? 4 : 2;
    // three workgroups fit a CU (registers): one round of 256 x 3 resident workgroups that stride the rows
    int gridc = (int)std::min<int64_t>((R + rpi - 1) / rpi, 768);
    static_assert(768 <= kRmsPartRows, "one partial row per workgroup");
    float* ppc = (part && (int64_t)gridc * d <= part_floats && gridc > 8) ? part : nullptr;
#define SP_COLS(NVW, RPI)                                                                                              \
  do {                                                                                                                 \
    if (dres) hipLaunchKernelGGL((k_rmsnorm_bwd_cols<NVW, RPI, true>), dim3(gridc), dim3(kBlock), 0, s, dy, x, g, rstd, dres, R, d, dx, dg, ppc); \
    else hipLaunchKernelGGL((k_rmsnorm_bwd_cols<NVW, RPI, false>), dim3(gridc), dim3(kBlock), 0, s, dy, x, g, rstd, dres, R, d, dx, dg, ppc);   \
  } while (0)
    if (d <= 2048) SP_COLS(1, 4); else SP_COLS(2, 2);
#undef SP_COLS
    if (ppc) hipLaunchKernelGGL(k_colsum_add, dim3((d + 63) / 64, 8), dim3(kBlock), 0, s, ppc, gridc, d, dg);
    return;
  }
#define SP_CASE(N) hipLaunchKernelGGL((k_rmsnorm_bwd<T, N>), dim3(grid), dim3(kBlock), lds, s, dy, x, g, rstd, dres, R, d, dx, dg, pp)
  if (nv <= 1) SP_CASE(1); else if (nv <= 2) SP_CASE(2); else if (nv <= 4) SP_CASE(4); else if (nv <= 8) SP_CASE(8); else SP_CASE(16);
#undef SP_CASE
  if (pp) hipLaunchKernelGGL(k_colsum_add, dim3((d + 63) / 64, 8), dim3(kBlock), 0, s, pp, grid, d, dg);
}

void rmsnorm_bwd(hipStream_t s, int dtype, const void* dy, const void* x, const void* g, const float* rstd,
                 const void* dres, int64_t R, int d, void* dx, float* dg, float* part, int64_t part_floats) {
  const int pi = prof_start(PROF_RMSNORM_BWD, s);
  if (dtype == SP_BF16)
    rmsnorm_bwd_t<bf16>(s, (const bf16*)dy, (const bf16*)x, (const bf16*)g, rstd, (const bf16*)dres, R, d, (bf16*)dx, dg, part, part_floats);
  else
    rmsnorm_bwd_t<float>(s, (const float*)dy, (const float*)x, (const float*)g, rstd, (const float*)dres, R, d, (float*)dx, dg, part, part_floats);
  prof_stop(pi, s, (dres ? 4.0 : 3.0) * R * d * elt_size(dtype));   // dy, x (, dres) read, dx written
}

void rope(hipStream_t s, int dtype, void* qk, int64_t R, int T, int nheads, int hd, int row_stride, float theta,
          int sign) {
  if (R <= 0) return;
  int pairs = nheads * hd / 2;
  int grid = grid_for_rows(R * pairs, kBlock * 2, 16384);
  float l2 = log2f(theta);
  if (dtype == SP_BF16)
    hipLaunchKernelGGL(k_rope<bf16>, dim3(grid), dim3(kBlock), 0, s, (bf16*)qk, R, T, pairs, hd, row_stride, l2, (float)sign);
  else
    hipLaunchKernelGGL(k_rope<float>, dim3(grid), dim3(kBlock), 0, s, (float*)qk, R, T, pairs, hd, row_stride, l2, (float)sign);
}

void rope_table(hipStream_t s, int T, int hd, float theta, float* table) {
  const int n = T * (hd / 2);
  if (n <= 0) return;
  hipLaunchKernelGGL(k_rope_table, dim3((n + kBlock - 1) / kBlock), dim3(kBlock), 0, s, (float2*)table, T, hd, log2f(theta));
}

template <class T>
static void swiglu_t(hipStream_t s, bool bwd, const T* da, const T* gu, int64_t R, int h, T* out) {
  if (R <= 0) return;
  bool vec = h % 8 == 0 && aligned16<T>(gu) && aligned16<T>(out) && (!bwd || aligned16<T>(da));
  int64_t work = vec ? R * (h / 8) : R * (int64_t)h;
  int grid = grid_for_rows(work, kBlock * 2, 16384);
  if (vec) {
    if (bwd) hipLaunchKernelGGL(k_swiglu_bwd<T>, dim3(grid), dim3(kBlock), 0, s, da, gu, R, h, out);
    else hipLaunchKernelGGL(k_swiglu_fwd<T>, dim3(grid), dim3(kBlock), 0, s, gu, R, h, out);
  } else {
    if (bwd) hipLaunchKernelGGL(k_swiglu_bwd_scalar<T>, dim3(grid), dim3(kBlock), 0, s, da, gu, R, h, out);
    else hipLaunchKernelGGL(k_swiglu_fwd_scalar<T>, dim3(grid), dim3(kBlock), 0, s, gu, R, h, out);
  }
}

void swiglu_fwd(hipStream_t s, int dtype, const void* gu, int64_t R, int h, void* a) {
  const int pi = prof_start(PROF_SWIGLU, s);
  struct Stop { int pi; hipStream_t s; double b; ~Stop() { prof_stop(pi, s, b); } } stop{pi, s, 3.0 * R * h * elt_size(dtype)};
  if (dtype == SP_BF16) swiglu_t<bf16>(s, false, nullptr, (const bf16*)gu, R, h, (bf16*)a);
  else swiglu_t<float>(s, false, nullptr, (const float*)gu, R, h, (float*)a);
}

void swiglu_bwd(hipStream_t s, int dtype, const void* da, const void* gu, int64_t R, int h, void* dgu) {
  const int pi = prof_start(PROF_SWIGLU, s);
  struct Stop { int pi; hipStream_t s; double b; ~Stop() { prof_stop(pi, s, b); } } stop{pi, s, 5.0 * R * h * elt_size(dtype)};
  if (dtype == SP_BF16) swiglu_t<bf16>(s, true, (const bf16*)da, (const bf16*)gu, R, h, (bf16*)dgu);
  else swiglu_t<float>(s, true, (const float*)da, (const float*)gu, R, h, (float*)dgu);
}

void count_targets(hipStream_t s, const int32_t* tgt, int n_mb, int64_t rows_per_mb, int V, int32_t* counts,
                   int32_t* bad) {
  hipLaunchKernelGGL(k_count_targets, dim3(n_mb), dim3(kBlock), 0, s, tgt, rows_per_mb, V, counts, bad);
}

void cross_entropy(hipStream_t s, int dtype, void* logits, const int32_t* tgt, int64_t row0, int64_t R, int V,
                   int64_t rows_per_mb, const int32_t* counts, float inv_n_mb, float* loss_mb) {
  if (R <= 0) return;
  const int pi = prof_start(PROF_CROSS_ENTROPY, s);
  struct Stop { int pi; hipStream_t s; double b; ~Stop() { prof_stop(pi, s, b); } } stop{pi, s, 2.0 * R * V * elt_size(dtype)};   // logits read, dlogits written
  bool vec = V % 8 == 0 && ((uintptr_t)logits % 16) == 0;
  if (dtype == SP_BF16 && vec && V <= 1024 * 8 * 16) {
#define SP_CE_ROW(NT, NCH)                                                                                         \
  hipLaunchKernelGGL((k_cross_entropy_row<NT, NCH>), dim3((unsigned)R), dim3(NT), 0, s, (bf16*)logits, tgt, row0, V, \
                     rows_per_mb, counts, inv_n_mb, loss_mb)
    if (V <= 256 * 8 * 4) SP_CE_ROW(256, 4);
    else if (V <= 256 * 8 * 16) SP_CE_ROW(256, 16);
    else if (V <= 512 * 8 * 16) SP_CE_ROW(512, 16);
    else SP_CE_ROW(1024, 16);
#undef SP_CE_ROW
    return;
  }
#define SP_CE(T, VEC)                                                                                          \
  hipLaunchKernelGGL((k_cross_entropy<T, VEC>), dim3((unsigned)R), dim3(kBlock), 0, s, (T*)logits, tgt, row0, V, \
                     rows_per_mb, counts, inv_n_mb, loss_mb)
  if (dtype == SP_BF16) { if (vec) SP_CE(bf16, true); else SP_CE(bf16, false); }
  else { if (vec) SP_CE(float, true); else SP_CE(float, false); }
#undef SP_CE
}

}  // namespace sp
