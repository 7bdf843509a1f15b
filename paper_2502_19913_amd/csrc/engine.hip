// The stage executor: context and workspace, forward and backward of one stage for a group of
// microbatches, the output head with its loss, and the whole-model walk over a route plan.
// Host code only; every arithmetic step is a kernel launched from here on the context's stream.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <string>
#include <vector>

#include "internal.h"

namespace sp {

extern thread_local std::string g_errmsg;

int hip_fail(int e, const char* what) {
  return fail(SP_EHIP, std::string(what) + ": " + hipGetErrorString((hipError_t)e));
}

#define SP_HIP(call)                                      \
  do {                                                    \
    hipError_t e_ = (call);                               \
    if (e_ != hipSuccess) return hip_fail((int)e_, #call); \
  } while (0)

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct LayerSaved {
  char *x, *xn, *qkv, *o, *h, *hn, *gu, *a;
  float *lse, *rstd1, *rstd2;
};

struct Record {
  int stage;
  std::vector<int> mb;
  size_t arena_begin;
  std::vector<LayerSaved> layers;
  bool live;
};

struct Dims {
  int64_t d, H, Hkv, hd, dkv, nq, h, V, T, B, Nmb, E;
  explicit Dims(const sp_cfg& c)
      : d(c.dim), H(c.n_heads), Hkv(c.n_kv_heads), hd(c.dim / c.n_heads), dkv((int64_t)c.n_kv_heads * hd),
        nq(d + 2 * dkv), h(c.hidden), V(c.vocab), T(c.seq_len), B(c.seqs_per_mb), Nmb((int64_t)c.seq_len * c.seqs_per_mb),
        E(elt_size(c.dtype)) {}
};

// bytes of saved activations of one layer for `rows` rows (each tensor 256-byte aligned)
size_t layer_saved_bytes(const Dims& D, int64_t rows) {
  size_t b = 0;
  b += 5 * align_up((size_t)rows * D.d * D.E);           // x, xn, o, h, hn
  b += align_up((size_t)rows * D.nq * D.E);              // qkv
  b += align_up((size_t)rows * 2 * D.h * D.E);           // gu
  b += align_up((size_t)rows * D.h * D.E);               // a
  b += align_up((size_t)rows * D.H * sizeof(float));     // lse
  b += 2 * align_up((size_t)rows * sizeof(float));       // rstd1, rstd2
  return b;
}

// Rows of logits materialised at a time.  Every chunk adds its share of the head's weight gradient into the float
// gradient buffer (vocab x dim x 4 bytes read and written per chunk), so chunks are made large: up to 8 GiB of logits.
int64_t head_chunk_rows(const Dims& D, int64_t total_rows) {
  int64_t ch = ((int64_t)8 << 30) / std::max<int64_t>(1, D.V * D.E);
  ch = ch / 256 * 256;
  if (ch < 256) ch = 256;
  return std::min(ch, total_rows);
}

struct Carve {
  size_t arena, t_y, t_dy[2], t_dh[2], t_d2, t_da, t_dgu[2], t_dqkv[2], t_delta, rope, h_xn, h_rstd, h_logits, h_dxn, pool_a, pool_d,
      loss_mb, counts, bad, dgpart, total;
  size_t arena_bytes;
};

Carve carve(const sp_cfg& c, int n_mb_max, int n_visits_max) {
  const Dims D(c);
  const int64_t Rmax = (int64_t)n_mb_max * D.Nmb;
  Carve w{};
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t at = off; off += align_up(bytes); return at; };
  w.arena_bytes = (size_t)n_visits_max * c.layers_per_stage * layer_saved_bytes(D, D.Nmb);
  w.arena = take(w.arena_bytes);
  w.t_y = take(Rmax * D.d * D.E);
  // two sets of the gradients a weight-gradient product reads: it may still be running (on the side stream)
  // while the next layer's are written
  for (int p = 0; p < 2; ++p) {
    w.t_dy[p] = take(Rmax * D.d * D.E);
    w.t_dh[p] = take(Rmax * D.d * D.E);
    w.t_dgu[p] = take(Rmax * 2 * D.h * D.E);
    w.t_dqkv[p] = take(Rmax * D.nq * D.E);
  }
  w.t_d2 = take(Rmax * D.d * D.E);
  w.t_da = take(Rmax * D.h * D.E);
  w.t_delta = take(Rmax * D.H * sizeof(float));
  w.rope = take((size_t)D.T * (D.hd / 2) * 2 * sizeof(float));   // cos, sin per (position, pair)
  w.dgpart = take((size_t)kRmsPartRows * D.d * sizeof(float));   // per-block partial sums of a norm's gain gradient
  w.bad = take(sizeof(int32_t));   // raised by a kernel that meets a token id or target outside the vocabulary
  if (c.has_head) {
    const int64_t ch = head_chunk_rows(D, Rmax);
    w.h_xn = take(ch * D.d * D.E);
    w.h_rstd = take(ch * sizeof(float));
    w.h_logits = take(ch * D.V * D.E);
    w.h_dxn = take(ch * D.d * D.E);
    w.loss_mb = take(n_mb_max * sizeof(float));
    w.counts = take(n_mb_max * sizeof(int32_t));
  }
  if (c.has_head && c.has_embed) {
    w.pool_a = take(Rmax * D.d * D.E);
    w.pool_d = take(Rmax * D.d * D.E);
  }
  w.total = off;
  return w;
}

}  // namespace
}  // namespace sp

using namespace sp;

struct sp_ctx {
  sp_cfg cfg;
  Layout L;
  hipStream_t stream;
  int n_mb_max, n_visits_max;
  char* base;
  float* rope_tab;   // inside the workspace, filled at creation
  int32_t* bad;      // inside the workspace: input-range flag, cleared at creation and by sp_input_status
  int32_t host_bad;
  // weight-gradient products run on a stream of their own, beside the chain that carries the activation
  // gradient down the layers; events order the two (ready: input written; done: input no longer read)
  hipStream_t side;
  hipEvent_t ready[4], done[2][4], joined;
  bool done_set[2][4];
  int use_side;      // 0: weight gradients run in line on the caller's stream; 1: beside it when that pays; 2: always
  Carve w;
  size_t arena_top;
  std::vector<Record> records;
  std::vector<float> host_loss;
};

namespace {

char* at(sp_ctx* c, size_t off) { return c->base + off; }

int arena_alloc(sp_ctx* c, size_t bytes, char** out) {
  size_t b = align_up(bytes);
  if (c->arena_top + b > c->w.arena_bytes)
    return fail(SP_ENOMEM, "saved-activation arena exhausted: more stage visits alive than n_visits_max");
  *out = at(c, c->w.arena) + c->arena_top;
  c->arena_top += b;
  return SP_OK;
}

void arena_release_dead(sp_ctx* c) {
  while (!c->records.empty() && !c->records.back().live) {
    c->arena_top = c->records.back().arena_begin;
    c->records.pop_back();
  }
}

int check_group(sp_ctx* c, int stage, const int32_t* mb_idx, int n_group, SlotList* sl) {
  const sp_cfg& cfg = c->cfg;
  if (stage < cfg.local_stage_begin || stage >= cfg.local_stage_begin + cfg.local_stage_count)
    return fail(SP_EINVAL, "stage " + std::to_string(stage) + " is not held by this node");
  if (!mb_idx || n_group < 1) return fail(SP_EINVAL, "empty group");
  if (n_group > kMaxGroup || n_group > c->n_mb_max) return fail(SP_EINVAL, "group larger than n_mb_max (or 64)");
  sl->n = n_group;
  for (int g = 0; g < n_group; ++g) {
    if (mb_idx[g] < 0 || mb_idx[g] >= c->n_mb_max) return fail(SP_EINVAL, "microbatch slot outside [0, n_mb_max)");
    for (int k = 0; k < g; ++k)
      if (mb_idx[k] == mb_idx[g]) return fail(SP_EINVAL, "microbatch slot listed twice in one group");
    sl->slot[g] = mb_idx[g];
  }
  return SP_OK;
}

const char* P(const sp_ctx* c, const void* params, int64_t off) { return (const char*)params + off * elt_size(c->cfg.dtype); }

}  // namespace

extern "C" {

int64_t sp_workspace_bytes(const sp_cfg* cfg, int n_mb_max, int n_visits_max) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  if (n_mb_max < 1 || n_visits_max < 0) return fail(SP_EINVAL, "workspace: bad counts");
  return (int64_t)carve(*cfg, n_mb_max, n_visits_max).total;
}

int sp_create(const sp_cfg* cfg, void* hip_stream, int n_mb_max, int n_visits_max, sp_ctx** out) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  if (!out) return fail(SP_EINVAL, "out is null");
  if (n_mb_max < 1 || n_visits_max < 0) return fail(SP_EINVAL, "create: bad counts");
  int ndev = 0;
  hipError_t e = hipGetDeviceCount(&ndev);
  if (e != hipSuccess || ndev < 1) return fail(SP_EHIP, "no HIP device: this library has no CPU path");
  sp_ctx* c = new sp_ctx();
  c->cfg = *cfg;
  c->L = make_layout(*cfg);
  c->stream = (hipStream_t)hip_stream;
  c->n_mb_max = n_mb_max;
  c->n_visits_max = n_visits_max;
  c->w = carve(*cfg, n_mb_max, n_visits_max);
  c->arena_top = 0;
  c->base = nullptr;
  e = hipMalloc((void**)&c->base, c->w.total);
  if (e != hipSuccess) {
    delete c;
    return fail(SP_ENOMEM, std::string("hipMalloc of the workspace failed: ") + hipGetErrorString(e));
  }
  c->side = nullptr;
  c->use_side = 1;
  e = hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking);
  for (int i = 0; i < 4 && e == hipSuccess; ++i) {
    e = hipEventCreateWithFlags(&c->ready[i], hipEventDisableTiming);
    for (int p = 0; p < 2 && e == hipSuccess; ++p) e = hipEventCreateWithFlags(&c->done[p][i], hipEventDisableTiming);
  }
  if (e == hipSuccess) e = hipEventCreateWithFlags(&c->joined, hipEventDisableTiming);
  if (e != hipSuccess) {
    (void)hipFree(c->base);
    delete c;
    return hip_fail((int)e, "side stream / events");
  }
  c->rope_tab = (float*)at(c, c->w.rope);
  c->bad = (int32_t*)at(c, c->w.bad);
  fill_zero(c->stream, c->bad, sizeof(int32_t));
  rope_table(c->stream, (int)Dims(*cfg).T, (int)Dims(*cfg).hd, cfg->rope_theta, c->rope_tab);
  e = hipGetLastError();
  if (e != hipSuccess) {
    (void)hipFree(c->base);
    delete c;
    return hip_fail((int)e, "rope table");
  }
  *out = c;
  return SP_OK;
}

int sp_destroy(sp_ctx* ctx) {
  if (!ctx) return SP_OK;
  hipError_t e = hipStreamSynchronize(ctx->stream);
  (void)hipStreamSynchronize(ctx->side);
  for (int i = 0; i < 4; ++i) {
    (void)hipEventDestroy(ctx->ready[i]);
    for (int p = 0; p < 2; ++p) (void)hipEventDestroy(ctx->done[p][i]);
  }
  (void)hipEventDestroy(ctx->joined);
  (void)hipStreamDestroy(ctx->side);
  hipError_t e2 = hipFree(ctx->base);
  delete ctx;
  if (e != hipSuccess) return hip_fail((int)e, "hipStreamSynchronize");
  if (e2 != hipSuccess) return hip_fail((int)e2, "hipFree");
  return SP_OK;
}

int sp_set_side_stream(sp_ctx* ctx, int enabled) {
  if (!ctx) return fail(SP_EINVAL, "ctx is null");
  if (enabled < 0 || enabled > 2) return fail(SP_EINVAL, "set_side_stream: enabled must be 0, 1 or 2");
  ctx->use_side = enabled;
  return SP_OK;
}

int sp_reset(sp_ctx* ctx) {
  if (!ctx) return fail(SP_EINVAL, "ctx is null");
  ctx->records.clear();
  ctx->arena_top = 0;
  return SP_OK;
}

// Reads and clears the input-range flag; the stream must have been waited for.
static int take_input_flag(sp_ctx* ctx, const char* who) {
  hipError_t e = hipMemcpyAsync(&ctx->host_bad, ctx->bad, sizeof(int32_t), hipMemcpyDeviceToHost, ctx->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return hip_fail((int)e, "reading the input-range flag");
  if (!ctx->host_bad) return SP_OK;
  fill_zero(ctx->stream, ctx->bad, sizeof(int32_t));
  return fail(SP_EINVAL, std::string(who) + ": a token id outside [0, vocab) or a target outside [-1, vocab) was met; "
                                            "such rows were embedded as zeros / left out of loss and gradients");
}

int sp_input_status(sp_ctx* ctx) {
  if (!ctx) return fail(SP_EINVAL, "ctx is null");
  return take_input_flag(ctx, "input_status");
}

int sp_embed_fwd(sp_ctx* ctx, const void* params, const int32_t* tokens, int n_mb, void* act_pool) {
  if (!ctx || !params || !tokens || !act_pool) return fail(SP_EINVAL, "embed_fwd: null argument");
  if (!ctx->cfg.has_embed) return fail(SP_EINVAL, "this node holds no embedding");
  if (n_mb < 1 || n_mb > ctx->n_mb_max) return fail(SP_EINVAL, "embed_fwd: n_mb outside [1, n_mb_max]");
  const Dims D(ctx->cfg);
  embed_fwd(ctx->stream, ctx->cfg.dtype, P(ctx, params, ctx->L.embed), tokens, n_mb * D.Nmb, (int)D.d, (int)D.V, act_pool,
            ctx->bad);
  SP_HIP(hipGetLastError());
  return SP_OK;
}

int sp_embed_bwd(sp_ctx* ctx, const int32_t* tokens, const void* dact_pool, int n_mb, float* grads) {
  if (!ctx || !tokens || !dact_pool || !grads) return fail(SP_EINVAL, "embed_bwd: null argument");
  if (!ctx->cfg.has_embed) return fail(SP_EINVAL, "this node holds no embedding");
  if (n_mb < 1 || n_mb > ctx->n_mb_max) return fail(SP_EINVAL, "embed_bwd: n_mb outside [1, n_mb_max]");
  const Dims D(ctx->cfg);
  embed_bwd(ctx->stream, ctx->cfg.dtype, dact_pool, tokens, n_mb * D.Nmb, (int)D.d, (int)D.V, grads + ctx->L.embed,
            ctx->bad);
  SP_HIP(hipGetLastError());
  return SP_OK;
}

}  // extern "C"

// The stage's first n_layers layers on a group of slots.  keep: the visit stays on record for its backward;
// otherwise its saved tensors are released at once (forward-only evaluation).
static int stage_fwd_impl(sp_ctx* ctx, int stage, const void* params, void* act_pool, const int32_t* mb_idx, int n_group,
                          int n_layers, bool keep) {
  if (!ctx || !params || !act_pool) return fail(SP_EINVAL, "stage_fwd: null argument");
  SlotList sl{};
  int rc = check_group(ctx, stage, mb_idx, n_group, &sl);
  if (rc) return rc;
  const sp_cfg& cfg = ctx->cfg;
  const Dims D(cfg);
  const int64_t R = (int64_t)n_group * D.Nmb;
  const int dt = cfg.dtype;
  hipStream_t s = ctx->stream;

  Record rec;
  rec.stage = stage;
  rec.mb.assign(mb_idx, mb_idx + n_group);
  rec.arena_begin = ctx->arena_top;
  rec.live = true;
  rec.layers.resize(n_layers);
  for (auto& ls : rec.layers) {
    char* p;
#define SP_TAKE(field, bytes)                                   \
  if ((rc = arena_alloc(ctx, (size_t)(bytes), &p)) != SP_OK) {  \
    ctx->arena_top = rec.arena_begin;                           \
    return rc;                                                  \
  }                                                             \
  ls.field = (decltype(ls.field))p;
    SP_TAKE(x, R * D.d * D.E) SP_TAKE(xn, R * D.d * D.E) SP_TAKE(qkv, R * D.nq * D.E) SP_TAKE(o, R * D.d * D.E)
    SP_TAKE(h, R * D.d * D.E) SP_TAKE(hn, R * D.d * D.E) SP_TAKE(gu, R * 2 * D.h * D.E) SP_TAKE(a, R * D.h * D.E)
    SP_TAKE(lse, R * D.H * sizeof(float)) SP_TAKE(rstd1, R * sizeof(float)) SP_TAKE(rstd2, R * sizeof(float))
#undef SP_TAKE
  }

  gather_slots(s, dt, act_pool, sl, D.Nmb, (int)D.d, rec.layers[0].x);
  const int loc = stage - cfg.local_stage_begin;
  const int Bg = (int)(n_group * D.B);
  for (int l = 0; l < n_layers; ++l) {
    const LayerOff& w = ctx->L.layers[(size_t)loc * cfg.layers_per_stage + l];
    LayerSaved& ls = rec.layers[l];
    char* y = l + 1 < n_layers ? rec.layers[l + 1].x : at(ctx, ctx->w.t_y);
    rmsnorm_fwd(s, dt, ls.x, P(ctx, params, w.g1), R, (int)D.d, cfg.rms_eps, ls.xn, ls.rstd1);
    // q, k, v = xn Wqkv^T, the heads of q and k rotated by their positions
    const RopeArgs ra = {ctx->rope_tab, (int)D.T, (int)D.hd, (int)((D.H + D.Hkv) * D.hd)};
    if ((rc = gemm_rope(s, dt, R, D.nq, D.d, ls.xn, P(ctx, params, w.wqkv), ls.qkv, ra, cfg.rope_theta))) return rc;
    if ((rc = attention_fwd(s, dt, Bg, (int)D.T, (int)D.H, (int)D.Hkv, (int)D.hd, ls.qkv, ls.o, ls.lse))) return rc;
    if ((rc = gemm(s, dt, 0, R, D.d, D.d, ls.o, P(ctx, params, w.wo), ls.h, ls.x))) return rc;
    rmsnorm_fwd(s, dt, ls.h, P(ctx, params, w.g2), R, (int)D.d, cfg.rms_eps, ls.hn, ls.rstd2);
    if ((rc = ffn_up_fwd(s, dt, R, D.h, D.d, ls.hn, P(ctx, params, w.wgu), ls.gu, ls.a))) return rc;
    if ((rc = gemm(s, dt, 0, R, D.d, D.h, ls.a, P(ctx, params, w.wd), y, ls.h))) return rc;
  }
  scatter_slots(s, dt, at(ctx, ctx->w.t_y), sl, D.Nmb, (int)D.d, act_pool);
  SP_HIP(hipGetLastError());
  if (keep) ctx->records.push_back(std::move(rec));
  else ctx->arena_top = rec.arena_begin;   // stream order: the next visit's kernels run after this one's
  return SP_OK;
}

extern "C" {

int sp_stage_fwd(sp_ctx* ctx, int stage, const void* params, void* act_pool, const int32_t* mb_idx, int n_group) {
  if (!ctx) return fail(SP_EINVAL, "stage_fwd: null argument");
  return stage_fwd_impl(ctx, stage, params, act_pool, mb_idx, n_group, ctx->cfg.layers_per_stage, true);
}

int sp_stage_bwd(sp_ctx* ctx, int stage, const void* params, void* dact_pool, const int32_t* mb_idx, int n_group,
                 float* grads) {
  if (!ctx || !params || !dact_pool || !grads) return fail(SP_EINVAL, "stage_bwd: null argument");
  SlotList sl{};
  int rc = check_group(ctx, stage, mb_idx, n_group, &sl);
  if (rc) return rc;
  // the newest live forward of exactly this group
  int ri = -1;
  for (int i = (int)ctx->records.size() - 1; i >= 0; --i) {
    const Record& r = ctx->records[i];
    if (r.live && r.stage == stage && (int)r.mb.size() == n_group && std::equal(r.mb.begin(), r.mb.end(), mb_idx)) {
      ri = i;
      break;
    }
  }
  if (ri < 0) return fail(SP_ESTATE, "stage_bwd: no saved forward for this stage and group");
  Record& rec = ctx->records[ri];
  const sp_cfg& cfg = ctx->cfg;
  const Dims D(cfg);
  const int64_t R = (int64_t)n_group * D.Nmb;
  const int dt = cfg.dtype;
  hipStream_t s = ctx->stream;
  const int loc = stage - cfg.local_stage_begin;
  const int Bg = (int)(n_group * D.B);

  char* t = at(ctx, ctx->w.t_d2);
  char* da = at(ctx, ctx->w.t_da);
  float* delta = (float*)at(ctx, ctx->w.t_delta);
  float* dgpart = (float*)at(ctx, ctx->w.dgpart);
  const int64_t dgpart_n = (int64_t)kRmsPartRows * D.d;
  // A second stream pays while the layer's products are short: their partly filled last rounds of tiles take in
  // work of the other stream.  Products of many rounds only get in each other's way (workgroups of two kernels
  // interleave on the CUs and the tiles an XCD holds no longer share panels): measured 3 - 7 % slower from about
  // 2.5 rounds of 256 x 256 tiles of the R x d products on.
  constexpr int64_t kSideMaxTiles = 640;
  const bool side_pays = ((R + 255) / 256) * ((D.d + 255) / 256) < kSideMaxTiles;
  hipStream_t side = ctx->use_side == 2 || (ctx->use_side == 1 && side_pays) ? ctx->side : s;
  for (int p = 0; p < 2; ++p)
    for (int i = 0; i < 4; ++i) ctx->done_set[p][i] = false;
  // weight gradient k of the layer (0: down, 1: gate/up, 2: output, 3: qkv) on the side stream, once its input
  // (just written on the main stream) is ready; `done` marks when that input may be overwritten
  auto side_dw = [&](int k, int par, int64_t M, int64_t N, const void* A, const void* B, float* C) -> int {
    SP_HIP(hipEventRecord(ctx->ready[k], s));
    SP_HIP(hipStreamWaitEvent(side, ctx->ready[k], 0));
    int r = gemm(side, dt, 2, M, N, R, A, B, C, nullptr);
    if (r) return r;
    SP_HIP(hipEventRecord(ctx->done[par][k], side));
    ctx->done_set[par][k] = true;
    return SP_OK;
  };
  auto wait_done = [&](int k, int par) -> int {
    if (ctx->done_set[par][k]) SP_HIP(hipStreamWaitEvent(s, ctx->done[par][k], 0));
    return SP_OK;
  };

  gather_slots(s, dt, dact_pool, sl, D.Nmb, (int)D.d, at(ctx, ctx->w.t_dy[0]));
  int par = 0;
  for (int l = cfg.layers_per_stage - 1; l >= 0; --l, par ^= 1) {
    const LayerOff& w = ctx->L.layers[(size_t)loc * cfg.layers_per_stage + l];
    const LayerSaved& ls = rec.layers[l];
    char* dy = at(ctx, ctx->w.t_dy[par]);
    char* dy_next = at(ctx, ctx->w.t_dy[par ^ 1]);
    char* dh = at(ctx, ctx->w.t_dh[par]);
    char* dgu = at(ctx, ctx->w.t_dgu[par]);
    char* dqkv = at(ctx, ctx->w.t_dqkv[par]);
    // feed-forward: y = h + a Wd^T
    if ((rc = side_dw(0, par, D.d, D.h, dy, ls.a, grads + w.wd))) return rc;
    if ((rc = wait_done(1, par))) return rc;
    if ((rc = ffn_down_bwd(s, dt, R, D.h, D.d, dy, P(ctx, params, w.wd), ls.gu, dgu, da))) return rc;
    if ((rc = side_dw(1, par, 2 * D.h, D.d, dgu, ls.hn, grads + w.wgu))) return rc;
    if ((rc = gemm(s, dt, 1, R, D.d, 2 * D.h, dgu, P(ctx, params, w.wgu), t, nullptr))) return rc;
    if ((rc = wait_done(2, par))) return rc;
    rmsnorm_bwd(s, dt, t, ls.h, P(ctx, params, w.g2), ls.rstd2, dy, R, (int)D.d, dh, grads + w.g2, dgpart, dgpart_n);
    // attention: h = x + o Wo^T
    if ((rc = side_dw(2, par, D.d, D.d, dh, ls.o, grads + w.wo))) return rc;
    if ((rc = gemm(s, dt, 1, R, D.d, D.d, dh, P(ctx, params, w.wo), t, nullptr))) return rc;
    if ((rc = wait_done(3, par))) return rc;
    if ((rc = attention_bwd(s, dt, Bg, (int)D.T, (int)D.H, (int)D.Hkv, (int)D.hd, ls.qkv, ls.o, ls.lse, t, dqkv, delta,
                            ctx->rope_tab, cfg.rope_theta)))
      return rc;
    if ((rc = side_dw(3, par, D.nq, D.d, dqkv, ls.xn, grads + w.wqkv))) return rc;
    if ((rc = gemm(s, dt, 1, R, D.d, D.nq, dqkv, P(ctx, params, w.wqkv), t, nullptr))) return rc;
    if ((rc = wait_done(0, par ^ 1))) return rc;   // the layer above may still read its dy
    rmsnorm_bwd(s, dt, t, ls.x, P(ctx, params, w.g1), ls.rstd1, dh, R, (int)D.d, dy_next, grads + w.g1, dgpart, dgpart_n);
  }
  char* dy = at(ctx, ctx->w.t_dy[par]);
  // the caller's stream continues only after every weight gradient has landed
  SP_HIP(hipEventRecord(ctx->joined, side));
  SP_HIP(hipStreamWaitEvent(s, ctx->joined, 0));
  scatter_slots(s, dt, dy, sl, D.Nmb, (int)D.d, dact_pool);
  SP_HIP(hipGetLastError());
  rec.live = false;
  arena_release_dead(ctx);
  return SP_OK;
}

}  // extern "C"

// final norm, output head, loss; backward: also the gradients (dact_pool, grads), else the loss only
static int head_impl(sp_ctx* ctx, const void* params, const void* act_pool, const int32_t* targets, int n_mb,
                     float* loss_mb, void* dact_pool, float* grads, bool backward) {
  if (!ctx || !params || !act_pool || !targets || !loss_mb || (backward && (!dact_pool || !grads)))
    return fail(SP_EINVAL, "head: null argument");
  const sp_cfg& cfg = ctx->cfg;
  if (!cfg.has_head) return fail(SP_EINVAL, "this node holds no output head");
  if (n_mb < 1 || n_mb > ctx->n_mb_max) return fail(SP_EINVAL, "head: n_mb outside [1, n_mb_max]");
  const Dims D(cfg);
  const int dt = cfg.dtype;
  hipStream_t s = ctx->stream;
  const int64_t Rtot = (int64_t)n_mb * D.Nmb;
  const int64_t CH = head_chunk_rows(D, (int64_t)ctx->n_mb_max * D.Nmb);
  int32_t* counts = (int32_t*)at(ctx, ctx->w.counts);
  char* xn = at(ctx, ctx->w.h_xn);
  float* rstd = (float*)at(ctx, ctx->w.h_rstd);
  char* logits = at(ctx, ctx->w.h_logits);
  char* dxn = at(ctx, ctx->w.h_dxn);
  int rc;
  fill_zero(s, loss_mb, n_mb * sizeof(float));
  count_targets(s, targets, n_mb, D.Nmb, (int)D.V, counts, ctx->bad);
  for (int64_t r0 = 0; r0 < Rtot; r0 += CH) {
    const int64_t R = std::min(CH, Rtot - r0);
    const char* x = (const char*)act_pool + r0 * D.d * D.E;
    char* dx = backward ? (char*)dact_pool + r0 * D.d * D.E : nullptr;
    rmsnorm_fwd(s, dt, x, P(ctx, params, ctx->L.gf), R, (int)D.d, cfg.rms_eps, xn, rstd);
    if ((rc = gemm(s, dt, 0, R, D.V, D.d, xn, P(ctx, params, ctx->L.whead), logits, nullptr))) return rc;
    cross_entropy(s, dt, logits, targets, r0, R, (int)D.V, D.Nmb, counts, 1.0f / (float)n_mb, loss_mb);
    if (!backward) continue;
    if ((rc = gemm(s, dt, 2, D.V, D.d, R, logits, xn, grads + ctx->L.whead, nullptr))) return rc;
    if ((rc = gemm(s, dt, 1, R, D.d, D.V, logits, P(ctx, params, ctx->L.whead), dxn, nullptr))) return rc;
    rmsnorm_bwd(s, dt, dxn, x, P(ctx, params, ctx->L.gf), rstd, nullptr, R, (int)D.d, dx, grads + ctx->L.gf,
                (float*)at(ctx, ctx->w.dgpart), (int64_t)kRmsPartRows * D.d);
  }
  SP_HIP(hipGetLastError());
  return SP_OK;
}

extern "C" {

int sp_head_fwd_bwd(sp_ctx* ctx, const void* params, const void* act_pool, const int32_t* targets, int n_mb,
                    float* loss_mb, void* dact_pool, float* grads) {
  return head_impl(ctx, params, act_pool, targets, n_mb, loss_mb, dact_pool, grads, true);
}

int sp_eval_paths(sp_ctx* ctx, const void* params, const int32_t* tokens, const int32_t* targets, const int32_t* paths,
                  const int32_t* len, const int32_t* half_stage, int n_mb, float* loss_host, float* loss_mb_host) {
  if (!ctx || !params || !tokens || !targets || !paths || !len || !loss_host)
    return fail(SP_EINVAL, "eval_paths: null argument");
  const sp_cfg& cfg = ctx->cfg;
  if (!cfg.has_embed || !cfg.has_head || cfg.local_stage_begin != 0 || cfg.local_stage_count != cfg.n_stages)
    return fail(SP_EINVAL, "eval_paths needs the whole model on this node (all stages, embedding, head)");
  if (n_mb < 1 || n_mb > ctx->n_mb_max) return fail(SP_EINVAL, "eval_paths: n_mb outside [1, n_mb_max]");
  const int s_n = cfg.n_stages, half_layers = cfg.layers_per_stage / 2;
  int rc, lmax = 0;
  for (int mb = 0; mb < n_mb; ++mb) {
    const int32_t* p = paths + (size_t)mb * s_n;
    if ((rc = check_one_path(cfg, p, len[mb], mb))) return rc;   // samples may drop different numbers of stages
    lmax = std::max(lmax, (int)len[mb]);
    if (half_stage && half_stage[mb] >= 0) {
      const int h = half_stage[mb];
      if (h == 0 || half_layers < 1 || std::find(p, p + len[mb], h) == p + len[mb])
        return fail(SP_EPATH, "half_stage of microbatch " + std::to_string(mb) +
                                  ": must be a stage of the path other than stage 0, with at least 2 layers per stage");
    }
  }
  sp_reset(ctx);
  hipStream_t s = ctx->stream;
  char* pool_a = at(ctx, ctx->w.pool_a);
  float* loss_mb = (float*)at(ctx, ctx->w.loss_mb);
  if ((rc = sp_embed_fwd(ctx, params, tokens, n_mb, pool_a))) return rc;
  // route plan: at each path position, one group per (stage, whole or half)
  std::vector<int32_t> g;
  for (int pos = 0; pos < lmax; ++pos)
    for (int st = 0; st < s_n; ++st)
      for (int half = 0; half < 2; ++half) {
        g.clear();
        for (int mb = 0; mb < n_mb; ++mb)
          if (pos < len[mb] && paths[(size_t)mb * s_n + pos] == st &&
              (half == 1) == (half_stage != nullptr && half_stage[mb] == st))
            g.push_back(mb);
        if (g.empty()) continue;
        if ((rc = stage_fwd_impl(ctx, st, params, pool_a, g.data(), (int)g.size(),
                                 half ? half_layers : cfg.layers_per_stage, false)))
          return rc;
      }
  if ((rc = head_impl(ctx, params, pool_a, targets, n_mb, loss_mb, nullptr, nullptr, false))) return rc;
  ctx->host_loss.resize(n_mb);
  SP_HIP(hipMemcpyAsync(ctx->host_loss.data(), loss_mb, n_mb * sizeof(float), hipMemcpyDeviceToHost, s));
  SP_HIP(hipStreamSynchronize(s));
  double tot = 0;
  for (int i = 0; i < n_mb; ++i) tot += ctx->host_loss[i];
  *loss_host = (float)(tot / n_mb);
  if (loss_mb_host) std::memcpy(loss_mb_host, ctx->host_loss.data(), n_mb * sizeof(float));
  return take_input_flag(ctx, "eval_paths");
}

int sp_run_paths(sp_ctx* ctx, const void* params, const int32_t* tokens, const int32_t* targets,
                 const int32_t* paths, const int32_t* len, int n_mb, float* loss_host, float* loss_mb_host,
                 float* grads) {
  if (!ctx || !params || !tokens || !targets || !paths || !len || !loss_host || !grads)
    return fail(SP_EINVAL, "run_paths: null argument");
  const sp_cfg& cfg = ctx->cfg;
  if (!cfg.has_embed || !cfg.has_head || cfg.local_stage_begin != 0 || cfg.local_stage_count != cfg.n_stages)
    return fail(SP_EINVAL, "run_paths needs the whole model on this node (all stages, embedding, head)");
  if (n_mb < 1 || n_mb > ctx->n_mb_max) return fail(SP_EINVAL, "run_paths: n_mb outside [1, n_mb_max]");
  int rc = sp_check_paths(&cfg, paths, len, n_mb);
  if (rc) return rc;
  std::vector<Group> plan;
  build_plan(cfg, paths, len, n_mb, plan);
  sp_reset(ctx);
  hipStream_t s = ctx->stream;
  char* pool_a = at(ctx, ctx->w.pool_a);
  char* pool_d = at(ctx, ctx->w.pool_d);
  float* loss_mb = (float*)at(ctx, ctx->w.loss_mb);
  fill_zero(s, grads, ctx->L.total * (int64_t)sizeof(float));
  if ((rc = sp_embed_fwd(ctx, params, tokens, n_mb, pool_a))) return rc;
  for (const Group& g : plan)
    if ((rc = sp_stage_fwd(ctx, g.stage, params, pool_a, g.mb.data(), (int)g.mb.size()))) return rc;
  if ((rc = sp_head_fwd_bwd(ctx, params, pool_a, targets, n_mb, loss_mb, pool_d, grads))) return rc;
  for (auto it = plan.rbegin(); it != plan.rend(); ++it)
    if ((rc = sp_stage_bwd(ctx, it->stage, params, pool_d, it->mb.data(), (int)it->mb.size(), grads))) return rc;
  if ((rc = sp_embed_bwd(ctx, tokens, pool_d, n_mb, grads))) return rc;
  ctx->host_loss.resize(n_mb);
  SP_HIP(hipMemcpyAsync(ctx->host_loss.data(), loss_mb, n_mb * sizeof(float), hipMemcpyDeviceToHost, s));
  SP_HIP(hipStreamSynchronize(s));
  double tot = 0;
  for (int i = 0; i < n_mb; ++i) tot += ctx->host_loss[i];
  *loss_host = (float)(tot / n_mb);
  if (loss_mb_host) std::memcpy(loss_mb_host, ctx->host_loss.data(), n_mb * sizeof(float));
  return take_input_flag(ctx, "run_paths");
}

int sp_gemm(void* hip_stream, int dtype, int op, int M, int N, int K, const void* A, const void* B, void* C,
            const void* R) {
  if (dtype != SP_F32 && dtype != SP_BF16) return fail(SP_EINVAL, "gemm: unknown dtype");
  int rc = gemm((hipStream_t)hip_stream, dtype, op, M, N, K, A, B, C, R);
  if (rc) return rc;
  SP_HIP(hipGetLastError());
  return SP_OK;
}

int sp_ffn_up_fwd(void* hip_stream, int dtype, int R, int h, int d, const void* hn, const void* wgu, void* gu, void* act) {
  if (dtype != SP_F32 && dtype != SP_BF16) return fail(SP_EINVAL, "ffn: unknown dtype");
  int rc = ffn_up_fwd((hipStream_t)hip_stream, dtype, R, h, d, hn, wgu, gu, act);
  if (rc) return rc;
  SP_HIP(hipGetLastError());
  return SP_OK;
}

int sp_ffn_down_bwd(void* hip_stream, int dtype, int R, int h, int d, const void* dy, const void* wd, const void* gu,
                    void* dgu, void* da_scratch) {
  if (dtype != SP_F32 && dtype != SP_BF16) return fail(SP_EINVAL, "ffn: unknown dtype");
  int rc = ffn_down_bwd((hipStream_t)hip_stream, dtype, R, h, d, dy, wd, gu, dgu, da_scratch);
  if (rc) return rc;
  SP_HIP(hipGetLastError());
  return SP_OK;
}

int sp_attention_fwd(void* hip_stream, int dtype, int B, int T, int H, int Hkv, int hd, const void* qkv, void* o,
                     float* lse) {
  if (dtype != SP_F32 && dtype != SP_BF16) return fail(SP_EINVAL, "attention: unknown dtype");
  int rc = attention_fwd((hipStream_t)hip_stream, dtype, B, T, H, Hkv, hd, qkv, o, lse);
  if (rc) return rc;
  SP_HIP(hipGetLastError());
  return SP_OK;
}

int sp_attention_bwd(void* hip_stream, int dtype, int B, int T, int H, int Hkv, int hd, const void* qkv,
                     const void* o, const float* lse, const void* do_, void* dqkv, float* delta_scratch) {
  if (dtype != SP_F32 && dtype != SP_BF16) return fail(SP_EINVAL, "attention: unknown dtype");
  int rc = attention_bwd((hipStream_t)hip_stream, dtype, B, T, H, Hkv, hd, qkv, o, lse, do_, dqkv, delta_scratch);
  if (rc) return rc;
  SP_HIP(hipGetLastError());
  return SP_OK;
}

}  // extern "C"
