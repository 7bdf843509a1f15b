// Host-side logic: configuration checks, flat parameter layout, seeded path generation, path
// validation and the route plan.  Plain C++; nothing here touches the GPU.
#include "internal.h"

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <numeric>
#include <string>
#include <vector>

namespace sp {

thread_local std::string g_errmsg;

int fail(int code, const std::string& msg) {
  g_errmsg = msg;
  return code;
}

int check_cfg(const sp_cfg* c) {
  if (!c) return fail(SP_EINVAL, "cfg is null");
  if (c->dim <= 0 || c->n_heads <= 0 || c->n_kv_heads <= 0 || c->hidden <= 0 || c->n_stages <= 0 ||
      c->layers_per_stage <= 0 || c->seq_len <= 0 || c->seqs_per_mb <= 0)
    return fail(SP_EINVAL, "cfg: sizes must be positive");
  if (c->dim % c->n_heads) return fail(SP_EINVAL, "cfg: dim not divisible by n_heads");
  if ((c->dim / c->n_heads) % 2) return fail(SP_EINVAL, "cfg: head dimension must be even (rotary pairs)");
  if (c->n_heads % c->n_kv_heads) return fail(SP_EINVAL, "cfg: n_heads not divisible by n_kv_heads");
  if ((c->has_embed || c->has_head) && c->vocab <= 0) return fail(SP_EINVAL, "cfg: vocab must be positive");
  if (c->dtype != SP_F32 && c->dtype != SP_BF16) return fail(SP_EINVAL, "cfg: unknown dtype");
  if (c->local_stage_begin < 0 || c->local_stage_count < 0 ||
      c->local_stage_begin + c->local_stage_count > c->n_stages)
    return fail(SP_EINVAL, "cfg: local stage range outside [0, n_stages)");
  if (!(c->rms_eps >= 0.f) || !(c->rope_theta > 0.f)) return fail(SP_EINVAL, "cfg: rms_eps / rope_theta");
  if (c->path_flags < 0 || c->path_flags > 2) return fail(SP_EINVAL, "cfg: unknown path_flags");
  return SP_OK;
}

Layout make_layout(const sp_cfg& c) {
  Layout L;
  const int64_t d = c.dim, h = c.hidden, hd = c.dim / c.n_heads, dkv = (int64_t)c.n_kv_heads * hd, V = c.vocab;
  int64_t off = 0;
  auto add = [&](const std::string& name, int stage, int layer, int64_t rows, int64_t cols) {
    sp_tensor_desc t;
    std::memset(&t, 0, sizeof t);
    std::snprintf(t.name, sizeof t.name, "%s", name.c_str());
    t.stage = stage; t.layer = layer; t.offset = off; t.rows = rows; t.cols = cols;
    L.tensors.push_back(t);
    int64_t at = off;
    off += rows * cols;
    return at;
  };
  if (c.has_embed) L.embed = add("embed", -1, -1, V, d);
  for (int s = c.local_stage_begin; s < c.local_stage_begin + c.local_stage_count; ++s)
    for (int l = 0; l < c.layers_per_stage; ++l) {
      const std::string p = "s" + std::to_string(s) + ".l" + std::to_string(l) + ".";
      LayerOff o;
      o.g1 = add(p + "g1", s, l, 1, d);
      o.wqkv = add(p + "wqkv", s, l, d + 2 * dkv, d);
      o.wo = add(p + "wo", s, l, d, d);
      o.g2 = add(p + "g2", s, l, 1, d);
      o.wgu = add(p + "wgu", s, l, 2 * h, d);
      o.wd = add(p + "wd", s, l, d, h);
      L.layers.push_back(o);
    }
  if (c.has_head) {
    L.gf = add("gf", -1, -1, 1, d);
    L.whead = add("whead", -1, -1, V, d);
  }
  L.total = off;
  return L;
}

// splitmix64: the generator's whole state is one counter
struct Rng {
  uint64_t s;
  explicit Rng(uint64_t seed) : s(seed * 0x9E3779B97F4A7C15ull + 0x1234567ull) {}
  uint64_t next() {
    uint64_t z = (s += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
  }
  uint64_t below(uint64_t n) { return next() % n; }
};

template <class T>
void shuffle(std::vector<T>& v, Rng& r) {
  for (size_t i = v.size(); i > 1; --i) std::swap(v[i - 1], v[r.below(i)]);
}

int check_one_path(const sp_cfg& c, const int32_t* p, int len, int mb) {
  const int s = c.n_stages;
  const std::string who = "path of microbatch " + std::to_string(mb) + ": ";
  if (len < 1 || len > s) return fail(SP_EPATH, who + "length outside [1, n_stages]");
  if (p[0] != 0) return fail(SP_EPATH, who + "does not open with stage 0 (CC1)");
  std::vector<char> seen(s, 0);
  for (int j = 0; j < len; ++j) {
    if (p[j] < 0 || p[j] >= s) return fail(SP_EPATH, who + "stage index out of range");
    if (seen[p[j]]) return fail(SP_EPATH, who + "a stage appears twice");
    seen[p[j]] = 1;
  }
  if (c.path_flags == SP_ALLOW_ANY_ORDER) return SP_OK;
  int desc = -1;
  for (int j = 0; j + 1 < len; ++j)
    if (p[j + 1] < p[j]) {
      if (desc >= 0) return fail(SP_EPATH, who + "more than one swap (CC2)");
      desc = j;
    }
  if (desc >= 0) {
    // undoing the exchange must give an increasing list
    std::vector<int32_t> q(p, p + len);
    std::swap(q[desc], q[desc + 1]);
    if (!std::is_sorted(q.begin(), q.end())) return fail(SP_EPATH, who + "order is not one adjacent exchange (CC2)");
    if (c.path_flags == SP_STRICT_CC && p[desc] - p[desc + 1] != 1)
      return fail(SP_EPATH, who + "exchanged stages are not consecutive stages (CC2)");
  }
  return SP_OK;
}

int build_plan(const sp_cfg& c, const int32_t* paths, const int32_t* len, int n_mb, std::vector<Group>& out) {
  out.clear();
  const int s = c.n_stages;
  int lmax = 0;
  for (int mb = 0; mb < n_mb; ++mb) lmax = std::max(lmax, (int)len[mb]);
  for (int pos = 0; pos < lmax; ++pos)
    for (int st = c.local_stage_begin; st < c.local_stage_begin + c.local_stage_count; ++st) {
      Group g;
      g.pos = pos; g.stage = st;
      for (int mb = 0; mb < n_mb; ++mb)
        if (pos < len[mb] && paths[(size_t)mb * s + pos] == st) g.mb.push_back(mb);
      if (!g.mb.empty()) out.push_back(std::move(g));
    }
  return SP_OK;
}

}  // namespace sp

using namespace sp;

extern "C" {

const char* sp_strerror(int status) {
  static thread_local std::string buf;
  const char* base = "unknown status";
  switch (status) {
    case SP_OK: return "ok";
    case SP_EINVAL: base = "invalid argument"; break;
    case SP_EPATH: base = "path violates the constraints"; break;
    case SP_ENOMEM: base = "out of workspace memory"; break;
    case SP_EHIP: base = "HIP runtime error"; break;
    case SP_ESTATE: base = "call order"; break;
  }
  buf = base;
  if (!g_errmsg.empty()) buf += ": " + g_errmsg;
  return buf.c_str();
}

int64_t sp_param_count(const sp_cfg* cfg) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  return make_layout(*cfg).total;
}

int sp_param_layout(const sp_cfg* cfg, sp_tensor_desc* out, int cap, int* n) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  if (!n) return fail(SP_EINVAL, "n is null");
  Layout L = make_layout(*cfg);
  *n = (int)L.tensors.size();
  if (!out || cap < *n) return fail(SP_EINVAL, "layout: capacity too small");
  std::copy(L.tensors.begin(), L.tensors.end(), out);
  return SP_OK;
}

int sp_make_paths(int n_stages, int n_mb, int skip_num, int skip_den, int allow_swap, uint64_t seed,
                  int32_t* paths, int32_t* len) {
  const int s = n_stages;
  if (s < 1 || n_mb < 1 || skip_den < 1 || skip_num < 0 || !paths || !len)
    return fail(SP_EINVAL, "make_paths: bad argument");
  const int64_t num = (int64_t)n_mb * s * skip_num;
  const int64_t total = (2 * num + skip_den) / (2 * (int64_t)skip_den);  // round(n_mb * s * k)
  const int lo = (int)(((int64_t)s * skip_num) / skip_den);
  const int64_t extra = total - (int64_t)lo * n_mb;
  if (extra < 0 || extra > n_mb) return fail(SP_EINVAL, "make_paths: inconsistent skip ratio");
  if (lo + (extra > 0 ? 1 : 0) > s - 1) return fail(SP_EINVAL, "make_paths: ratio leaves no stage besides stage 0");
  Rng rng(seed);
  std::vector<int> order(n_mb);
  std::iota(order.begin(), order.end(), 0);
  shuffle(order, rng);
  std::vector<int> q(n_mb, lo);
  for (int64_t i = 0; i < extra; ++i) q[order[i]] += 1;
  std::vector<int> perm(s > 1 ? s - 1 : 0);
  std::iota(perm.begin(), perm.end(), 1);
  shuffle(perm, rng);
  size_t cur = 0;
  for (int mb = 0; mb < n_mb; ++mb) {
    std::vector<char> skipped(s, 0);
    for (int j = 0; j < q[mb]; ++j) skipped[perm[(cur + j) % perm.size()]] = 1;
    cur += q[mb];
    std::vector<int32_t> kept;
    for (int st = 0; st < s; ++st)
      if (!skipped[st]) kept.push_back(st);
    if (allow_swap) {
      const bool coin = rng.next() >> 63;
      const uint64_t pick = rng.next();
      std::vector<int> elig;
      for (int j = 1; j + 1 < (int)kept.size(); ++j)
        if (kept[j + 1] - kept[j] == 1) elig.push_back(j);
      if (coin && !elig.empty()) {
        int j = elig[pick % elig.size()];
        std::swap(kept[j], kept[j + 1]);
      }
    }
    for (int j = 0; j < s; ++j) paths[(size_t)mb * s + j] = j < (int)kept.size() ? kept[j] : -1;
    len[mb] = (int32_t)kept.size();
  }
  return SP_OK;
}

int sp_check_paths(const sp_cfg* cfg, const int32_t* paths, const int32_t* len, int n_mb) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  if (!paths || !len || n_mb < 1) return fail(SP_EINVAL, "check_paths: bad argument");
  for (int mb = 0; mb < n_mb; ++mb) {
    if (len[mb] < 1 || len[mb] > cfg->n_stages) return fail(SP_EPATH, "path length outside [1, n_stages]");
    rc = check_one_path(*cfg, paths + (size_t)mb * cfg->n_stages, len[mb], mb);
    if (rc) return rc;
  }
  return SP_OK;
}

int sp_route_plan(const sp_cfg* cfg, const int32_t* paths, const int32_t* len, int n_mb, int32_t* group_pos,
                  int32_t* group_stage, int32_t* group_begin, int32_t* group_mb, int cap_groups, int* n_groups) {
  int rc = sp_check_paths(cfg, paths, len, n_mb);
  if (rc) return rc;
  if (!group_pos || !group_stage || !group_begin || !group_mb || !n_groups)
    return fail(SP_EINVAL, "route_plan: null output");
  std::vector<Group> plan;
  build_plan(*cfg, paths, len, n_mb, plan);
  *n_groups = (int)plan.size();
  if ((int)plan.size() > cap_groups) return fail(SP_EINVAL, "route_plan: capacity too small");
  int at = 0;
  for (size_t g = 0; g < plan.size(); ++g) {
    group_pos[g] = plan[g].pos;
    group_stage[g] = plan[g].stage;
    group_begin[g] = at;
    for (int mb : plan[g].mb) group_mb[at++] = mb;
  }
  group_begin[plan.size()] = at;
  return SP_OK;
}

}  // extern "C"
