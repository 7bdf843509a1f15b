// Declarations shared by the library's translation units (not part of the public boundary).
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "../../include/skippipe.h"

typedef struct ihipStream_t* hipStream_t;

namespace sp {

// ---- error plumbing
int fail(int code, const std::string& msg);
int check_cfg(const sp_cfg* c);
int hip_fail(int hip_error, const char* what);  // records the HIP message, returns SP_EHIP

// ---- flat parameter layout
struct LayerOff { int64_t g1, wqkv, wo, g2, wgu, wd; };
struct Layout {
  int64_t embed = 0, gf = 0, whead = 0, total = 0;
  std::vector<LayerOff> layers;  // local layers, stage-major
  std::vector<sp_tensor_desc> tensors;
};
Layout make_layout(const sp_cfg& c);

// ---- routing
struct Group { int pos, stage; std::vector<int> mb; };
int check_one_path(const sp_cfg& c, const int32_t* p, int len, int mb);
int build_plan(const sp_cfg& c, const int32_t* paths, const int32_t* len, int n_mb, std::vector<Group>& out);

inline int64_t elt_size(int dtype) { return dtype == SP_BF16 ? 2 : 4; }

// Up to this many microbatches may share one group (slot numbers travel as a kernel argument).
constexpr int kMaxGroup = 64;
struct SlotList { int32_t n; int32_t slot[kMaxGroup]; };

// ---- kernel launchers (all asynchronous on `s`; dtype is SP_F32 or SP_BF16)
// A token outside [0, V) sets *bad (device int32) to 1; its row reads as zeros / adds nothing.
void embed_fwd(hipStream_t s, int dtype, const void* E, const int32_t* tok, int64_t rows, int d, int V, void* x,
               int32_t* bad);
void embed_bwd(hipStream_t s, int dtype, const void* dx, const int32_t* tok, int64_t rows, int d, int V, float* dE,
               int32_t* bad);
// dst[g*rows_per_slot + r, :] = pool[slot[g]*rows_per_slot + r, :]   (and the reverse)
void gather_slots(hipStream_t s, int dtype, const void* pool, const SlotList& sl, int64_t rows_per_slot, int d, void* dst);
void scatter_slots(hipStream_t s, int dtype, const void* src, const SlotList& sl, int64_t rows_per_slot, int d, void* pool);
void fill_zero(hipStream_t s, void* p, int64_t bytes);

void rmsnorm_fwd(hipStream_t s, int dtype, const void* x, const void* g, int64_t R, int d, float eps, void* y, float* rstd);
// dx = (dres ? dres : 0) + rmsnorm'(dy) ; dg += sum_rows dy * x * rstd
// part (may be null): scratch of part_floats floats for the per-block partial sums of dg (kRmsPartRows x d is
// enough), which a second kernel adds up
constexpr int kRmsPartRows = 1024;
void rmsnorm_bwd(hipStream_t s, int dtype, const void* dy, const void* x, const void* g, const float* rstd,
                 const void* dres, int64_t R, int d, void* dx, float* dg, float* part = nullptr, int64_t part_floats = 0);
// rotates the first nheads*hd columns of every row (row_stride elements apart); position = row % T
void rope(hipStream_t s, int dtype, void* qk, int64_t R, int T, int nheads, int hd, int row_stride, float theta, int sign);
// table[(p * hd/2 + i) * 2 + {0, 1}] = cos, sin of p * theta^(-2i/hd), the angles rope() uses, for p < T
void rope_table(hipStream_t s, int T, int hd, float theta, float* table);
// Rotation fused into a producer: the leading rot_cols columns of a row are heads of hd columns whose pairs
// (2i, 2i+1) turn by the angle of position (row % T); table as written by rope_table
struct RopeArgs {
  const float* table;
  int T, hd, rot_cols;
};
void swiglu_fwd(hipStream_t s, int dtype, const void* gu, int64_t R, int h, void* a);
void swiglu_bwd(hipStream_t s, int dtype, const void* da, const void* gu, int64_t R, int h, void* dgu);
// counts[mb] = number of targets in [0, V) among the rows of microbatch mb; a target below -1 or >= V sets *bad
void count_targets(hipStream_t s, const int32_t* tgt, int n_mb, int64_t rows_per_mb, int V, int32_t* counts,
                   int32_t* bad);
// rows [row0, row0+R) of the iteration: logits -> dlogits in place, loss_mb[mb] += rowloss / counts[mb]
void cross_entropy(hipStream_t s, int dtype, void* logits, const int32_t* tgt, int64_t row0, int64_t R, int V,
                   int64_t rows_per_mb, const int32_t* counts, float inv_n_mb, float* loss_mb);

// C = A*B^T (+R) | C = A*B | C += A^T*B  (see sp_gemm); returns SP_EINVAL for bad arguments
int gemm(hipStream_t s, int dtype, int op, int64_t M, int64_t N, int64_t K, const void* A, const void* B, void* C,
         const void* R);

int attention_fwd(hipStream_t s, int dtype, int B, int T, int H, int Hkv, int hd, const void* qkv, void* o, float* lse);
// rope_tab (may be null): if given, q and k in qkv are rotated vectors and dqkv is returned with respect to
// the vectors before the rotation (theta is only used when the rotation runs as a pass of its own)
int attention_bwd(hipStream_t s, int dtype, int B, int T, int H, int Hkv, int hd, const void* qkv, const void* o,
                  const float* lse, const void* do_, void* dqkv, float* delta, const float* rope_tab = nullptr,
                  float rope_theta = 0.f);
// C = A*B^T with the rotation applied to C on the way out (same result as gemm op 0 followed by rope)
int gemm_rope(hipStream_t s, int dtype, int64_t M, int64_t N, int64_t K, const void* A, const void* B, void* C,
              const RopeArgs& ra, float rope_theta);

// building blocks the dispatchers choose between
void gemm_simple(hipStream_t s, int dtype, int op, int64_t M, int64_t N, int64_t K, const void* A, const void* B,
                 void* C, const void* R);
bool gemm_mfma_supported(int op, int64_t M, int64_t N, int64_t K, const void* A, const void* B, const void* C,
                         const void* R);
void gemm_mfma(hipStream_t s, int op, int64_t M, int64_t N, int64_t K, const void* A, const void* B, void* C,
               const void* R, const RopeArgs* rope = nullptr, int epi = 0, void* aux = nullptr);
// the feed-forward projections with the SwiGLU arithmetic in their epilogues (bf16, matrix cores):
//   forward   gu[R, 2h] = hn[R, d] wgu[2h, d]^T  and  act[R, h] = silu(gate) * up
//   backward  dgu[R, 2h] = swiglu'(dy[R, d] wd[d, h]; gu)            (d(act) is never stored)
bool gemm_swiglu_supported(bool bwd, int64_t R, int64_t h, int64_t d, const void* X, const void* W, const void* gu,
                           const void* other);
void gemm_mfma_swiglu_fwd(hipStream_t s, int64_t R, int64_t h, int64_t d, const void* hn, const void* wgu, void* gu, void* act);
void gemm_mfma_swiglu_bwd(hipStream_t s, int64_t R, int64_t h, int64_t d, const void* dy, const void* wd, const void* gu, void* dgu);
// the same two steps whatever the dtype and shape: fused where the matrix-core path takes them, else the plain
// product with the pointwise kernel after it; da_tmp [R, h]: scratch for the unfused backward path
int ffn_up_fwd(hipStream_t s, int dtype, int64_t R, int64_t h, int64_t d, const void* hn, const void* wgu, void* gu, void* act);
int ffn_down_bwd(hipStream_t s, int dtype, int64_t R, int64_t h, int64_t d, const void* dy, const void* wd, const void* gu,
                 void* dgu, void* da_tmp);
void attention_simple_fwd(hipStream_t s, int dtype, int B, int T, int H, int Hkv, int hd, const void* qkv, void* o,
                          float* lse);
void attention_simple_bwd(hipStream_t s, int dtype, int B, int T, int H, int Hkv, int hd, const void* qkv,
                          const void* o, const float* lse, const void* do_, void* dqkv, float* delta);
bool attention_flash_supported(int B, int T, int H, int Hkv, int hd);
void attention_flash_fwd(hipStream_t s, int B, int T, int H, int Hkv, int hd, const void* qkv, void* o, float* lse);
void attention_flash_bwd(hipStream_t s, int B, int T, int H, int Hkv, int hd, const void* qkv, const void* o,
                         const float* lse, const void* do_, void* dqkv, float* delta, const float* rope_tab);

// ---- optional per-launch timing (see sp_prof_begin); classes:
enum { PROF_GEMM_NT = 0, PROF_GEMM_NN = 1, PROF_GEMM_TN = 2, PROF_ATTN_FWD = 3, PROF_ATTN_DELTA = 4, PROF_ATTN_DQ = 5,
       PROF_ATTN_DKV = 6, PROF_GEMM_PLAIN = 7, PROF_ATTN_PLAIN = 8,
       // bandwidth-bound kernels: the work recorded is algorithmic bytes, not flops
       PROF_RMSNORM_FWD = 9, PROF_RMSNORM_BWD = 10, PROF_CROSS_ENTROPY = 11, PROF_COPY_ROWS = 12, PROF_SWIGLU = 13,
       PROF_CLASSES = 14 };
int prof_start(int cls, hipStream_t s);
void prof_stop(int idx, hipStream_t s, double flops);

}  // namespace sp
