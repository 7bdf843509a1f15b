// CPU checker for path-routed LLaMa stage training (test infrastructure only).
//
// This file is the slow, plain statement of what the GPU library must compute.
// It is not part of the product: only the tests, the smoke check and the
// benchmark's CPU-baseline leg may build or call it, and it shares no code
// with the GPU path.
//
// What it computes (SkipPipe, sections "System Setting" and "Partial pipeline
// schedule"): a model of L layers is cut into s equal stages of consecutive
// layers.  Every microbatch carries a path, an ordered list of stage indices
// that starts with stage 0; the microbatch is pushed through exactly the
// stages on its path, in path order, and a stage that is not on the path is
// never applied, so the residual stream passes it unchanged.  The loss is
// taken after the last stage on the path (the pipeline is a closed loop that
// returns to stage 0's node, section "Allocating Nodes to Stages"), the
// backward pass walks the same stages in reverse, and gradients of all
// microbatches of the iteration are accumulated before any update (section
// "Throughput", gradient accumulation; "System Setting", synchronous update).
//
// The layers are LLaMa decoder blocks (appendix "Model Configurations"):
// pre-norm RMSNorm, rotary embedding on interleaved pairs, causal softmax
// attention with grouped kv heads, SwiGLU feed-forward, residual adds; no
// biases; untied embedding and output head; cross-entropy on next tokens.
//
// Readings taken where the paper is silent: loss of a microbatch = mean over
// its non-ignored target positions; iteration loss = mean over microbatches;
// a stage's gradient is the plain sum over the microbatches that visited it
// (no rescale by visit count); a stage no path visits gets exactly zero.
//
// Everything runs one microbatch at a time, one stage at a time, one op at a
// time, with a hand-written backward for each op.  The scalar type is a
// template parameter: float is the reference precision, double exists for
// finite-difference checks and as the high-precision side of parity tests.
//
// Pins: see tests/test_oracle_*.py (library-routine model with autograd,
// finite differences, closed-form special cases, routing invariants).  The
// absolute fp32 loss value for a given seed has no printed counterpart in the
// paper: parity unpinned beyond those checks.

#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>
#include <algorithm>

namespace {

struct Cfg {
  int32_t dim, n_heads, n_kv_heads, hidden, vocab;
  int32_t n_stages, layers_per_stage;
  int32_t seq_len, seqs_per_mb;
  float rms_eps, rope_theta;
  int32_t local_stage_begin, local_stage_count;
  int32_t has_embed, has_head;
};

template <class F> using Vec = std::vector<F>;

// ---------------------------------------------------------------- RMSNorm
// y = x * r * g,  r = 1/sqrt(mean(x^2) + eps)
template <class F>
void rmsnorm_fwd(const F* x, const F* g, int R, int d, F eps, F* y, F* rstd) {
#pragma omp parallel for
  for (int r = 0; r < R; ++r) {
    F ss = 0;
    for (int c = 0; c < d; ++c) ss += x[(size_t)r * d + c] * x[(size_t)r * d + c];
    F rs = F(1) / std::sqrt(ss / F(d) + eps);
    rstd[r] = rs;
    for (int c = 0; c < d; ++c) y[(size_t)r * d + c] = x[(size_t)r * d + c] * rs * g[c];
  }
}

// xh = x*r ; dxh = dy*g ; dx = r*(dxh - xh*mean(dxh*xh)) ; dg += sum_rows dy*xh
template <class F>
void rmsnorm_bwd(const F* dy, const F* x, const F* g, const F* rstd, int R, int d, F* dx, F* dg) {
#pragma omp parallel for
  for (int r = 0; r < R; ++r) {
    F rs = rstd[r];
    F m = 0;
    for (int c = 0; c < d; ++c) m += dy[(size_t)r * d + c] * g[c] * x[(size_t)r * d + c] * rs;
    m /= F(d);
    for (int c = 0; c < d; ++c) {
      F xh = x[(size_t)r * d + c] * rs;
      dx[(size_t)r * d + c] = rs * (dy[(size_t)r * d + c] * g[c] - xh * m);
    }
  }
#pragma omp parallel for
  for (int c = 0; c < d; ++c) {
    F a = 0;
    for (int r = 0; r < R; ++r) a += dy[(size_t)r * d + c] * x[(size_t)r * d + c] * rstd[r];
    dg[c] += a;
  }
}

// ---------------------------------------------------------------- Linear (no bias), W is [N out, K in]
template <class F>
void linear_fwd(const F* x, const F* W, int R, int K, int N, F* y) {
#pragma omp parallel for collapse(2)
  for (int r = 0; r < R; ++r)
    for (int n = 0; n < N; ++n) {
      const F* xr = x + (size_t)r * K;
      const F* wn = W + (size_t)n * K;
      F a = 0;
#pragma omp simd reduction(+ : a)
      for (int k = 0; k < K; ++k) a += xr[k] * wn[k];
      y[(size_t)r * N + n] = a;
    }
}

// dx = dy W ;  dW += dy^T x
template <class F>
void linear_bwd(const F* dy, const F* x, const F* W, int R, int K, int N, F* dx, F* dW) {
  if (dx) {
#pragma omp parallel for
    for (int r = 0; r < R; ++r) {
      F* dxr = dx + (size_t)r * K;
      for (int k = 0; k < K; ++k) dxr[k] = 0;
      for (int n = 0; n < N; ++n) {
        F g = dy[(size_t)r * N + n];
        const F* wn = W + (size_t)n * K;
        for (int k = 0; k < K; ++k) dxr[k] += g * wn[k];
      }
    }
  }
#pragma omp parallel for
  for (int n = 0; n < N; ++n) {
    F* dwn = dW + (size_t)n * K;
    for (int r = 0; r < R; ++r) {
      F g = dy[(size_t)r * N + n];
      const F* xr = x + (size_t)r * K;
      for (int k = 0; k < K; ++k) dwn[k] += g * xr[k];
    }
  }
}

// ---------------------------------------------------------------- RoPE
// Pair (2i, 2i+1) of every head at position p turns by angle p * theta^(-2i/hd).
// sign = +1 forward, -1 for the backward pass (the transpose of a rotation).
template <class F>
void rope(F* q, int R, int T, int nh, int hd, int row_stride, F theta, int sign) {
#pragma omp parallel for
  for (int r = 0; r < R; ++r) {
    int p = r % T;
    for (int h = 0; h < nh; ++h)
      for (int i = 0; i < hd / 2; ++i) {
        F ang = F(p) * std::pow(theta, -F(2 * i) / F(hd));
        F c = std::cos(ang), s = F(sign) * std::sin(ang);
        F* v = q + (size_t)r * row_stride + h * hd + 2 * i;
        F a = v[0], b = v[1];
        v[0] = a * c - b * s;
        v[1] = a * s + b * c;
      }
  }
}

// ---------------------------------------------------------------- causal attention
// q [R, H*hd], k/v [R, Hkv*hd] with their own row strides; rows are B sequences of T.
// o_i = sum_{j<=i} softmax_j(q_i.k_j / sqrt(hd)) v_j ; q head a reads kv head a / (H/Hkv).
template <class F>
void attention_fwd(const F* q, const F* k, const F* v, int sq, int sk, int sv, int B, int T, int H, int Hkv, int hd,
                   F* o /*[R, H*hd]*/) {
  const F scale = F(1) / std::sqrt(F(hd));
  const int rep = H / Hkv;
#pragma omp parallel for collapse(2)
  for (int b = 0; b < B; ++b)
    for (int a = 0; a < H; ++a) {
      Vec<F> p(T);
      int kvh = a / rep;
      for (int i = 0; i < T; ++i) {
        const F* qi = q + (size_t)(b * T + i) * sq + a * hd;
        F mx = -INFINITY;
        for (int j = 0; j <= i; ++j) {
          const F* kj = k + (size_t)(b * T + j) * sk + kvh * hd;
          F s = 0;
          for (int c = 0; c < hd; ++c) s += qi[c] * kj[c];
          p[j] = s * scale;
          mx = std::max(mx, p[j]);
        }
        F den = 0;
        for (int j = 0; j <= i; ++j) { p[j] = std::exp(p[j] - mx); den += p[j]; }
        F* oi = o + (size_t)(b * T + i) * (H * hd) + a * hd;
        for (int c = 0; c < hd; ++c) oi[c] = 0;
        for (int j = 0; j <= i; ++j) {
          const F* vj = v + (size_t)(b * T + j) * sv + kvh * hd;
          F w = p[j] / den;
          for (int c = 0; c < hd; ++c) oi[c] += w * vj[c];
        }
      }
    }
}

// dV = P^T dO ; dP = dO V^T ; dS = P*(dP - rowsum(dP*P)) ; dQ = dS K/sqrt(hd) ; dK = dS^T Q/sqrt(hd)
// dq/dk/dv must be zero on entry (kv heads receive the sum over their q heads).
template <class F>
void attention_bwd(const F* dO, const F* q, const F* k, const F* v, int sq, int sk, int sv, int B, int T, int H,
                   int Hkv, int hd, F* dq, F* dk, F* dv) {
  const F scale = F(1) / std::sqrt(F(hd));
  const int rep = H / Hkv;
  // parallel over (sequence, kv head): every dk/dv element has one owner thread
#pragma omp parallel for collapse(2)
  for (int b = 0; b < B; ++b)
    for (int kvh = 0; kvh < Hkv; ++kvh) {
      Vec<F> p(T), dp(T);
      for (int a = kvh * rep; a < (kvh + 1) * rep; ++a)
        for (int i = 0; i < T; ++i) {
          const F* qi = q + (size_t)(b * T + i) * sq + a * hd;
          const F* doi = dO + (size_t)(b * T + i) * (H * hd) + a * hd;
          F mx = -INFINITY;
          for (int j = 0; j <= i; ++j) {
            const F* kj = k + (size_t)(b * T + j) * sk + kvh * hd;
            F s = 0;
            for (int c = 0; c < hd; ++c) s += qi[c] * kj[c];
            p[j] = s * scale;
            mx = std::max(mx, p[j]);
          }
          F den = 0;
          for (int j = 0; j <= i; ++j) { p[j] = std::exp(p[j] - mx); den += p[j]; }
          F dot = 0;
          for (int j = 0; j <= i; ++j) {
            p[j] /= den;
            const F* vj = v + (size_t)(b * T + j) * sv + kvh * hd;
            F s = 0;
            for (int c = 0; c < hd; ++c) s += doi[c] * vj[c];
            dp[j] = s;
            dot += s * p[j];
          }
          F* dqi = dq + (size_t)(b * T + i) * sq + a * hd;
          for (int j = 0; j <= i; ++j) {
            F ds = p[j] * (dp[j] - dot) * scale;
            const F* kj = k + (size_t)(b * T + j) * sk + kvh * hd;
            F* dkj = dk + (size_t)(b * T + j) * sk + kvh * hd;
            F* dvj = dv + (size_t)(b * T + j) * sv + kvh * hd;
            for (int c = 0; c < hd; ++c) {
              dqi[c] += ds * kj[c];
              dkj[c] += ds * qi[c];
              dvj[c] += p[j] * doi[c];
            }
          }
        }
    }
}

// ---------------------------------------------------------------- SwiGLU
// gu [R, 2h] = [gate | up] ; a = silu(gate) * up
template <class F>
void swiglu_fwd(const F* gu, int R, int h, F* a) {
#pragma omp parallel for
  for (int r = 0; r < R; ++r)
    for (int c = 0; c < h; ++c) {
      F g = gu[(size_t)r * 2 * h + c], u = gu[(size_t)r * 2 * h + h + c];
      a[(size_t)r * h + c] = g / (F(1) + std::exp(-g)) * u;
    }
}

template <class F>
void swiglu_bwd(const F* da, const F* gu, int R, int h, F* dgu) {
#pragma omp parallel for
  for (int r = 0; r < R; ++r)
    for (int c = 0; c < h; ++c) {
      F g = gu[(size_t)r * 2 * h + c], u = gu[(size_t)r * 2 * h + h + c];
      F sg = F(1) / (F(1) + std::exp(-g));
      F d = da[(size_t)r * h + c];
      dgu[(size_t)r * 2 * h + c] = d * u * sg * (F(1) + g * (F(1) - sg));
      dgu[(size_t)r * 2 * h + h + c] = d * g * sg;
    }
}

// ---------------------------------------------------------------- cross entropy
// loss = (1/count) sum_{t: target>=0} (logsumexp(logits_t) - logits_t[target_t])
// dlogits_t = (softmax(logits_t) - onehot) * w / count,  zero rows where target < 0
template <class F>
F cross_entropy(const F* logits, const int32_t* tgt, int R, int V, F w, F* dlogits) {
  int count = 0;
  for (int r = 0; r < R; ++r) count += tgt[r] >= 0;
  if (count == 0) {
    for (size_t i = 0; i < (size_t)R * V; ++i) dlogits[i] = 0;
    return 0;
  }
  Vec<F> rowloss(R, 0);
#pragma omp parallel for
  for (int r = 0; r < R; ++r) {
    const F* z = logits + (size_t)r * V;
    F* dz = dlogits + (size_t)r * V;
    if (tgt[r] < 0) {
      for (int c = 0; c < V; ++c) dz[c] = 0;
      continue;
    }
    F mx = z[0];
    for (int c = 1; c < V; ++c) mx = std::max(mx, z[c]);
    F den = 0;
    for (int c = 0; c < V; ++c) den += std::exp(z[c] - mx);
    F lse = mx + std::log(den);
    rowloss[r] = lse - z[tgt[r]];
    for (int c = 0; c < V; ++c) dz[c] = std::exp(z[c] - lse) * w / F(count);
    dz[tgt[r]] -= w / F(count);
  }
  F tot = 0;
  for (int r = 0; r < R; ++r) tot += rowloss[r];
  return tot / F(count);
}

// ---------------------------------------------------------------- parameter layout
// [embed V*d]? then per local stage, per layer: g1(d) wqkv((d+2dkv)*d) wo(d*d) g2(d) wgu(2h*d) wd(d*h);
// then [gf(d)] [whead V*d]?
struct LayerOff { size_t g1, wqkv, wo, g2, wgu, wd; };
struct Layout {
  size_t embed = 0, gf = 0, whead = 0, total = 0;
  std::vector<LayerOff> layers;  // local layers, stage-major
};

Layout make_layout(const Cfg& c) {
  Layout L;
  size_t d = c.dim, h = c.hidden, hd = c.dim / c.n_heads, dkv = (size_t)c.n_kv_heads * hd, V = c.vocab;
  size_t off = 0;
  if (c.has_embed) { L.embed = off; off += V * d; }
  for (int s = 0; s < c.local_stage_count; ++s)
    for (int l = 0; l < c.layers_per_stage; ++l) {
      LayerOff o;
      o.g1 = off; off += d;
      o.wqkv = off; off += (d + 2 * dkv) * d;
      o.wo = off; off += d * d;
      o.g2 = off; off += d;
      o.wgu = off; off += 2 * h * d;
      o.wd = off; off += d * h;
      L.layers.push_back(o);
    }
  if (c.has_head) { L.gf = off; off += d; L.whead = off; off += V * d; }
  L.total = off;
  return L;
}

// ---------------------------------------------------------------- one decoder block
template <class F>
struct BlockCache {
  Vec<F> x, xn, rstd1, qkv, o, h, hn, rstd2, gu, a;
};

template <class F>
void block_fwd(const Cfg& c, const F* P, const LayerOff& w, const F* x, int B, F* y, BlockCache<F>& S) {
  const int d = c.dim, H = c.n_heads, Hkv = c.n_kv_heads, hd = d / H, dkv = Hkv * hd, hh = c.hidden, T = c.seq_len;
  const int R = B * T, nq = d + 2 * dkv;
  S.x.assign(x, x + (size_t)R * d);
  S.xn.resize((size_t)R * d); S.rstd1.resize(R);
  rmsnorm_fwd<F>(x, P + w.g1, R, d, F(c.rms_eps), S.xn.data(), S.rstd1.data());
  S.qkv.resize((size_t)R * nq);
  linear_fwd<F>(S.xn.data(), P + w.wqkv, R, d, nq, S.qkv.data());
  rope<F>(S.qkv.data(), R, T, H, hd, nq, F(c.rope_theta), +1);
  rope<F>(S.qkv.data() + d, R, T, Hkv, hd, nq, F(c.rope_theta), +1);
  S.o.resize((size_t)R * d);
  attention_fwd<F>(S.qkv.data(), S.qkv.data() + d, S.qkv.data() + d + dkv, nq, nq, nq, B, T, H, Hkv, hd, S.o.data());
  S.h.resize((size_t)R * d);
  linear_fwd<F>(S.o.data(), P + w.wo, R, d, d, S.h.data());
  for (size_t i = 0; i < (size_t)R * d; ++i) S.h[i] += x[i];
  S.hn.resize((size_t)R * d); S.rstd2.resize(R);
  rmsnorm_fwd<F>(S.h.data(), P + w.g2, R, d, F(c.rms_eps), S.hn.data(), S.rstd2.data());
  S.gu.resize((size_t)R * 2 * hh);
  linear_fwd<F>(S.hn.data(), P + w.wgu, R, d, 2 * hh, S.gu.data());
  S.a.resize((size_t)R * hh);
  swiglu_fwd<F>(S.gu.data(), R, hh, S.a.data());
  linear_fwd<F>(S.a.data(), P + w.wd, R, hh, d, y);
  for (size_t i = 0; i < (size_t)R * d; ++i) y[i] += S.h[i];
}

// dy -> dx (may alias), parameter gradients accumulated into G (same layout as P)
template <class F>
void block_bwd(const Cfg& c, const F* P, F* G, const LayerOff& w, const F* dy, int B, F* dx, const BlockCache<F>& S) {
  const int d = c.dim, H = c.n_heads, Hkv = c.n_kv_heads, hd = d / H, dkv = Hkv * hd, hh = c.hidden, T = c.seq_len;
  const int R = B * T, nq = d + 2 * dkv;
  Vec<F> da((size_t)R * hh), dgu((size_t)R * 2 * hh), dhn((size_t)R * d), dh((size_t)R * d), t((size_t)R * d);
  linear_bwd<F>(dy, S.a.data(), P + w.wd, R, hh, d, da.data(), G + w.wd);
  swiglu_bwd<F>(da.data(), S.gu.data(), R, hh, dgu.data());
  linear_bwd<F>(dgu.data(), S.hn.data(), P + w.wgu, R, d, 2 * hh, dhn.data(), G + w.wgu);
  rmsnorm_bwd<F>(dhn.data(), S.h.data(), P + w.g2, S.rstd2.data(), R, d, t.data(), G + w.g2);
  for (size_t i = 0; i < (size_t)R * d; ++i) dh[i] = dy[i] + t[i];
  Vec<F> dO((size_t)R * d), dqkv((size_t)R * nq, F(0)), dxn((size_t)R * d);
  linear_bwd<F>(dh.data(), S.o.data(), P + w.wo, R, d, d, dO.data(), G + w.wo);
  attention_bwd<F>(dO.data(), S.qkv.data(), S.qkv.data() + d, S.qkv.data() + d + dkv, nq, nq, nq, B, T, H, Hkv, hd,
                   dqkv.data(), dqkv.data() + d, dqkv.data() + d + dkv);
  rope<F>(dqkv.data(), R, T, H, hd, nq, F(c.rope_theta), -1);
  rope<F>(dqkv.data() + d, R, T, Hkv, hd, nq, F(c.rope_theta), -1);
  linear_bwd<F>(dqkv.data(), S.xn.data(), P + w.wqkv, R, d, nq, dxn.data(), G + w.wqkv);
  rmsnorm_bwd<F>(dxn.data(), S.x.data(), P + w.g1, S.rstd1.data(), R, d, t.data(), G + w.g1);
  for (size_t i = 0; i < (size_t)R * d; ++i) dx[i] = dh[i] + t[i];
}

// ---------------------------------------------------------------- a stage = its layers in order
template <class F>
struct StageCache { std::vector<BlockCache<F>> blocks; };

template <class F>
void stage_fwd(const Cfg& c, const Layout& L, const F* P, int local_stage, F* x, int B, StageCache<F>& S) {
  const size_t n = (size_t)B * c.seq_len * c.dim;
  Vec<F> y(n);
  S.blocks.resize(c.layers_per_stage);
  for (int l = 0; l < c.layers_per_stage; ++l) {
    block_fwd<F>(c, P, L.layers[(size_t)local_stage * c.layers_per_stage + l], x, B, y.data(), S.blocks[l]);
    std::copy(y.begin(), y.end(), x);
  }
}

template <class F>
void stage_bwd(const Cfg& c, const Layout& L, const F* P, F* G, int local_stage, F* dx, int B,
               const StageCache<F>& S) {
  for (int l = c.layers_per_stage - 1; l >= 0; --l)
    block_bwd<F>(c, P, G, L.layers[(size_t)local_stage * c.layers_per_stage + l], dx, B, dx, S.blocks[l]);
}

// ---------------------------------------------------------------- head: final norm, output projection, loss
template <class F>
F head_fwd_bwd(const Cfg& c, const Layout& L, const F* P, F* G, const F* x, const int32_t* tgt, int B, F w, F* dx) {
  const int d = c.dim, V = c.vocab, R = B * c.seq_len;
  Vec<F> xn((size_t)R * d), rstd(R), logits((size_t)R * V), dlogits((size_t)R * V), dxn((size_t)R * d);
  rmsnorm_fwd<F>(x, P + L.gf, R, d, F(c.rms_eps), xn.data(), rstd.data());
  linear_fwd<F>(xn.data(), P + L.whead, R, d, V, logits.data());
  F loss = cross_entropy<F>(logits.data(), tgt, R, V, w, dlogits.data());
  linear_bwd<F>(dlogits.data(), xn.data(), P + L.whead, R, d, V, dxn.data(), G + L.whead);
  rmsnorm_bwd<F>(dxn.data(), x, P + L.gf, rstd.data(), R, d, dx, G + L.gf);
  return loss;
}

// ---------------------------------------------------------------- the iteration: every microbatch along its path
template <class F>
int run_paths(const Cfg& c, const F* P, const int32_t* tokens, const F* x_in, const int32_t* targets, const F* dy_in,
              const int32_t* paths, const int32_t* len, int n_mb, F* loss_mb, F* loss_total, F* y_out, F* dx_out,
              F* G) {
  const Layout L = make_layout(c);
  const int d = c.dim, B = c.seqs_per_mb, T = c.seq_len, R = B * T;
  const size_t n = (size_t)R * d;
  for (size_t i = 0; i < L.total; ++i) G[i] = 0;
  F total = 0;
  for (int mb = 0; mb < n_mb; ++mb) {
    const int32_t* p = paths + (size_t)mb * c.n_stages;
    Vec<F> x(n);
    if (c.has_embed) {
      for (int r = 0; r < R; ++r) {
        int tk = tokens[(size_t)mb * R + r];
        if (tk < 0 || tk >= c.vocab) return -1;
        for (int k = 0; k < d; ++k) x[(size_t)r * d + k] = P[L.embed + (size_t)tk * d + k];
      }
    } else {
      std::copy(x_in + mb * n, x_in + (mb + 1) * n, x.begin());
    }
    // forward: the stages on the path, in path order; stages held elsewhere are not simulated
    std::vector<StageCache<F>> caches(len[mb]);
    for (int j = 0; j < len[mb]; ++j) {
      int st = p[j];
      if (st < 0 || st >= c.n_stages) return -2;
      int loc = st - c.local_stage_begin;
      if (loc < 0 || loc >= c.local_stage_count) continue;
      stage_fwd<F>(c, L, P, loc, x.data(), B, caches[j]);
    }
    if (y_out) std::copy(x.begin(), x.end(), y_out + mb * n);
    Vec<F> dx(n);
    if (c.has_head) {
      loss_mb[mb] = head_fwd_bwd<F>(c, L, P, G, x.data(), targets + (size_t)mb * R, B, F(1) / F(n_mb), dx.data());
      total += loss_mb[mb];
    } else {
      std::copy(dy_in + mb * n, dy_in + (mb + 1) * n, dx.begin());
      if (loss_mb) loss_mb[mb] = 0;
    }
    // backward: the same stages, reversed
    for (int j = len[mb] - 1; j >= 0; --j) {
      int loc = p[j] - c.local_stage_begin;
      if (loc < 0 || loc >= c.local_stage_count) continue;
      stage_bwd<F>(c, L, P, G, loc, dx.data(), B, caches[j]);
    }
    if (c.has_embed) {
      for (int r = 0; r < R; ++r) {
        int tk = tokens[(size_t)mb * R + r];
        for (int k = 0; k < d; ++k) G[L.embed + (size_t)tk * d + k] += dx[(size_t)r * d + k];
      }
    }
    if (dx_out) std::copy(dx.begin(), dx.end(), dx_out + mb * n);
  }
  if (loss_total) *loss_total = total / F(n_mb);
  return 0;
}

// ---------------------------------------------------------------- evaluation under stage drops, forward only
// Section "Fault Tolerant Inference": every sample runs the stages of its path (stage 0 is never dropped);
// where the number of stages to drop is not whole, one stage of the path runs only the first half of its
// layers.  half[mb] names that stage (-1: none); "the first half" of an odd count is read as the first
// floor(layers_per_stage / 2) layers.  Returns each microbatch's mean loss; perplexity is its exponential.
template <class F>
int eval_paths(const Cfg& c, const F* P, const int32_t* tokens, const int32_t* targets, const int32_t* paths,
               const int32_t* len, const int32_t* half, int n_mb, F* loss_mb, F* loss_total) {
  if (!c.has_embed || !c.has_head || c.local_stage_begin != 0 || c.local_stage_count != c.n_stages) return -3;
  const Layout L = make_layout(c);
  const int d = c.dim, B = c.seqs_per_mb, T = c.seq_len, R = B * T, V = c.vocab;
  const size_t n = (size_t)R * d;
  F total = 0;
  for (int mb = 0; mb < n_mb; ++mb) {
    const int32_t* p = paths + (size_t)mb * c.n_stages;
    Vec<F> x(n), y(n);
    for (int r = 0; r < R; ++r) {
      int tk = tokens[(size_t)mb * R + r];
      if (tk < 0 || tk >= V) return -1;
      for (int k = 0; k < d; ++k) x[(size_t)r * d + k] = P[L.embed + (size_t)tk * d + k];
    }
    for (int j = 0; j < len[mb]; ++j) {
      const int st = p[j];
      if (st < 0 || st >= c.n_stages) return -2;
      const int n_layers = (half && half[mb] == st) ? c.layers_per_stage / 2 : c.layers_per_stage;
      for (int l = 0; l < n_layers; ++l) {
        BlockCache<F> scratch;
        block_fwd<F>(c, P, L.layers[(size_t)st * c.layers_per_stage + l], x.data(), B, y.data(), scratch);
        x.swap(y);
      }
    }
    Vec<F> xn(n), rstd(R), logits((size_t)R * V), dlogits((size_t)R * V);
    rmsnorm_fwd<F>(x.data(), P + L.gf, R, d, F(c.rms_eps), xn.data(), rstd.data());
    linear_fwd<F>(xn.data(), P + L.whead, R, d, V, logits.data());
    loss_mb[mb] = cross_entropy<F>(logits.data(), targets + (size_t)mb * R, R, V, F(1), dlogits.data());
    total += loss_mb[mb];
  }
  if (loss_total) *loss_total = total / F(n_mb);
  return 0;
}

}  // namespace

// ---------------------------------------------------------------- C entry points (ctypes)
#define ORC_EXPORT(F, SUF)                                                                                          \
  extern "C" size_t orc_param_count##SUF(const Cfg* c) { return make_layout(*c).total; }                            \
  extern "C" int orc_run_paths##SUF(const Cfg* c, const F* P, const int32_t* tokens, const F* x_in,                 \
                                    const int32_t* targets, const F* dy_in, const int32_t* paths,                   \
                                    const int32_t* len, int n_mb, F* loss_mb, F* loss_total, F* y_out, F* dx_out,   \
                                    F* G) {                                                                         \
    return run_paths<F>(*c, P, tokens, x_in, targets, dy_in, paths, len, n_mb, loss_mb, loss_total, y_out, dx_out,  \
                        G);                                                                                         \
  }                                                                                                                 \
  extern "C" int orc_eval_paths##SUF(const Cfg* c, const F* P, const int32_t* tokens, const int32_t* targets,       \
                                     const int32_t* paths, const int32_t* len, const int32_t* half, int n_mb,       \
                                     F* loss_mb, F* loss_total) {                                                   \
    return eval_paths<F>(*c, P, tokens, targets, paths, len, half, n_mb, loss_mb, loss_total);                      \
  }                                                                                                                 \
  extern "C" void orc_rmsnorm_fwd##SUF(const F* x, const F* g, int R, int d, F eps, F* y, F* rstd) {                \
    rmsnorm_fwd<F>(x, g, R, d, eps, y, rstd);                                                                       \
  }                                                                                                                 \
  extern "C" void orc_rmsnorm_bwd##SUF(const F* dy, const F* x, const F* g, const F* rstd, int R, int d, F* dx,     \
                                       F* dg) {                                                                     \
    rmsnorm_bwd<F>(dy, x, g, rstd, R, d, dx, dg);                                                                   \
  }                                                                                                                 \
  extern "C" void orc_linear_fwd##SUF(const F* x, const F* W, int R, int K, int N, F* y) {                          \
    linear_fwd<F>(x, W, R, K, N, y);                                                                                \
  }                                                                                                                 \
  extern "C" void orc_linear_bwd##SUF(const F* dy, const F* x, const F* W, int R, int K, int N, F* dx, F* dW) {     \
    linear_bwd<F>(dy, x, W, R, K, N, dx, dW);                                                                       \
  }                                                                                                                 \
  extern "C" void orc_rope##SUF(F* q, int R, int T, int nh, int hd, F theta, int sign) {                            \
    rope<F>(q, R, T, nh, hd, nh * hd, theta, sign);                                                                 \
  }                                                                                                                 \
  extern "C" void orc_attention_fwd##SUF(const F* q, const F* k, const F* v, int B, int T, int H, int Hkv, int hd,  \
                                         F* o) {                                                                    \
    attention_fwd<F>(q, k, v, H * hd, Hkv * hd, Hkv * hd, B, T, H, Hkv, hd, o);                                     \
  }                                                                                                                 \
  extern "C" void orc_attention_bwd##SUF(const F* dO, const F* q, const F* k, const F* v, int B, int T, int H,      \
                                         int Hkv, int hd, F* dq, F* dk, F* dv) {                                    \
    attention_bwd<F>(dO, q, k, v, H * hd, Hkv * hd, Hkv * hd, B, T, H, Hkv, hd, dq, dk, dv);                        \
  }                                                                                                                 \
  extern "C" void orc_swiglu_fwd##SUF(const F* gu, int R, int h, F* a) { swiglu_fwd<F>(gu, R, h, a); }              \
  extern "C" void orc_swiglu_bwd##SUF(const F* da, const F* gu, int R, int h, F* dgu) {                             \
    swiglu_bwd<F>(da, gu, R, h, dgu);                                                                               \
  }                                                                                                                 \
  extern "C" F orc_cross_entropy##SUF(const F* logits, const int32_t* tgt, int R, int V, F w, F* dlogits) {         \
    return cross_entropy<F>(logits, tgt, R, V, w, dlogits);                                                         \
  }

ORC_EXPORT(float, _f32)
ORC_EXPORT(double, _f64)
