// Host path scheduler: which node of which stage every microbatch of the first wave visits, and when.
// Plain C++; nothing here touches the GPU.
//
// Sections "Partial and Reordered Pipelining" and "Path finding", appendix "Detailed Path Selection
// Algorithm".  The setting is continuous-time multi-agent path finding: a microbatch (agent) starts on
// its node of stage 0, moves through one node of each stage on its path (a move costs the link's
// transfer time, a visit the node's forward time), returns to its start node where the loss is taken,
// and walks back; its end-to-end latency is the time its backward pass ends.  The search is
// conflict-based: a high level keeps sets of per-agent constraints "agent a may not occupy node n
// during [t0, t1)", a low level finds each agent's fastest closed path under its constraints.
//
//   low level   best-first search over (node, set of visited stages, exchange used), time as the
//               cost.  A visit that would overlap a forbidden interval is delayed to the interval's
//               end.  Order rule (CC2): stages ascend, with at most one exchange of two consecutive
//               stages.  The agent visits exactly its number of stages, then closes the loop; the
//               backward pass is added as an estimate without conflicts (only the first forward pass
//               is optimised, as the paper says of its own solution).
//   high level  phase 1 (HR1): resolve CC3 - every stage but the first is left out by the same number
//               of agents, up to one - by forbidding the over-visited stage's nodes to the fastest
//               paths through it (HR2: the slowest quarter of the agents is never constrained), until
//               a number of solutions (32 in the paper) is collected.  Phase 2, best solution first:
//               TC1 - at most m paths through a node: forbid the node to the fastest paths through it
//               (never to the slowest one); then TC2 - two agents on one node at the same time: the
//               faster agent (either, as two branches, if their latencies differ by less than delta) is
//               forbidden the node for the other's stay.  Conflicts with the slowest agent are taken first.  The first
//               solution without conflicts is returned.
//
// Readings where the paper is silent: an agent's latency counts from time 0; forward occupancy of a node
// is [arrival, arrival + forward time); links are full duplex and never conflict; an agent's number of
// kept stages is given by the caller (the rounding of s * k is the caller's, as in sp_make_paths).
#include "internal.h"

#include <algorithm>
#include <cmath>
#include <limits>
#include <map>
#include <queue>
#include <string>
#include <tuple>
#include <vector>

namespace sp {
namespace {

constexpr double kInf = std::numeric_limits<double>::infinity();

struct Constraint { int node; double t0, t1; };

struct AgentPath {
  std::vector<int> nodes;          // visited nodes, in order (nodes[0] = start node)
  std::vector<double> arrive;      // start of the forward stay at each
  double e2e = kInf;
};

struct Problem {
  int s, N, A, m, strict, no_swap;
  const int32_t* node_stage;
  const float *fwd, *bwd, *comm;
  const int32_t *start, *keep;
  std::vector<std::vector<int>> stage_nodes;
  double link(int a, int b) const { return comm[(size_t)a * N + b]; }
};

// earliest start >= t of a stay of length dur on `node` that avoids the agent's forbidden intervals
double earliest_stay(const std::vector<Constraint>& cs, int node, double t, double dur) {
  bool moved = true;
  while (moved) {
    moved = false;
    for (const Constraint& c : cs)
      if (c.node == node && t < c.t1 && t + dur > c.t0) {
        if (c.t1 == kInf) return kInf;
        t = c.t1;
        moved = true;
      }
  }
  return t;
}

struct SearchState {
  double time;      // end of the forward stay on `node`
  double past;      // what the visited nodes will cost on the way back: their backward times and the links between them
  int node, swap;
  uint32_t mask;    // stages visited
  int parent;       // index into the pool
  double arrive;
};

// fastest closed path of one agent under its constraints; false if none exists
bool plan_agent(const Problem& P, int a, const std::vector<Constraint>& cs, AgentPath* out) {
  const int n0 = P.start[a], keep = P.keep[a];
  std::vector<SearchState> pool;
  typedef std::pair<double, int> QE;   // (time + past: a lower bound of the closed path's latency, index in pool)
  std::priority_queue<QE, std::vector<QE>, std::greater<QE>> open;
  // states with the same node, stages and exchange flag: one that is no earlier and no cheaper on the way back
  // than another can be dropped (waiting is always allowed, so an earlier arrival is never worse)
  std::map<std::tuple<int, uint32_t, int>, std::vector<std::pair<double, double>>> seen;
  const double t_first = earliest_stay(cs, n0, 0.0, P.fwd[n0]);
  if (t_first == kInf) return false;
  pool.push_back({t_first + P.fwd[n0], (double)P.bwd[n0], n0, 0, 1u, -1, t_first});
  open.push({pool[0].time + pool[0].past, 0});
  double best_total = kInf;
  int best_idx = -1;
  while (!open.empty()) {
    const QE top = open.top();
    open.pop();
    if (top.first >= best_total) break;   // nothing left can close the loop sooner
    const SearchState cur = pool[top.second];
    int count = 0, mx = 0, second = -1;
    for (int st = 0; st < P.s; ++st)
      if (cur.mask >> st & 1) { ++count; second = mx; mx = st; }
    if (count == 1) second = -1;
    if (count == keep) {
      // close the loop: back to the start node for the loss, out again, and the backward pass along the path
      const double total = cur.time + (cur.node == n0 ? 0.0 : P.link(cur.node, n0) + P.link(n0, cur.node)) + cur.past;
      if (total < best_total) { best_total = total; best_idx = top.second; }
      continue;
    }
    const int last = P.node_stage[cur.node];
    for (int st = 1; st < P.s; ++st) {
      if (cur.mask >> st & 1) continue;
      int swap = cur.swap;
      if (st < mx) {
        // the second half of the one exchange (CC2): straight after the largest stage so far, a stage between
        // it and the next largest (in the strict form: the stage just below it); stage 0 is never exchanged
        if (P.no_swap || cur.swap || last != mx || st <= second || count < 2 || (P.strict && mx - st != 1)) continue;
        swap = 1;
      }
      for (int nd : P.stage_nodes[st]) {
        const double arr = earliest_stay(cs, nd, cur.time + P.link(cur.node, nd), P.fwd[nd]);
        if (arr == kInf) continue;
        const double done = arr + P.fwd[nd];
        const double past = cur.past + P.bwd[nd] + P.link(nd, cur.node);
        std::vector<std::pair<double, double>>& front = seen[std::make_tuple(nd, cur.mask | (1u << st), swap)];
        bool dominated = false;
        for (const auto& f : front)
          if (f.first <= done && f.second <= past) { dominated = true; break; }
        if (dominated) continue;
        front.push_back({done, past});
        pool.push_back({done, past, nd, swap, cur.mask | (1u << st), top.second, arr});
        open.push({done + past, (int)pool.size() - 1});
      }
    }
  }
  if (best_idx < 0) return false;
  out->nodes.clear(); out->arrive.clear();
  for (int idx = best_idx; idx >= 0; idx = pool[idx].parent) {
    out->nodes.push_back(pool[idx].node);
    out->arrive.push_back(pool[idx].arrive);
  }
  std::reverse(out->nodes.begin(), out->nodes.end());
  std::reverse(out->arrive.begin(), out->arrive.end());
  out->e2e = best_total;
  return true;
}

struct Solution {
  std::vector<std::vector<Constraint>> cons;   // per agent
  std::vector<AgentPath> paths;
  double cost = 0;
  int collisions = 0;   // pairs of forward stays that overlap on a node
  void recost() { cost = 0; for (const AgentPath& p : paths) cost = std::max(cost, p.e2e); }
};
struct ByCost {
  bool operator()(const Solution* a, const Solution* b) const { return a->cost > b->cost; }
};

bool visits_stage(const Problem& P, const AgentPath& p, int st) {
  for (int nd : p.nodes) if (P.node_stage[nd] == st) return true;
  return false;
}

// agents ordered fastest first
std::vector<int> by_speed(const Solution& T, const std::vector<int>& agents) {
  std::vector<int> v = agents;
  std::stable_sort(v.begin(), v.end(), [&](int x, int y) { return T.paths[x].e2e < T.paths[y].e2e; });
  return v;
}

int count_collisions(const Problem& P, const Solution& S) {
  int n = 0;
  for (int x = 0; x < P.A; ++x)
    for (int y = x + 1; y < P.A; ++y) {
      const AgentPath &pi = S.paths[x], &pj = S.paths[y];
      for (size_t u = 0; u < pi.nodes.size(); ++u)
        for (size_t v = 0; v < pj.nodes.size(); ++v)
          if (pi.nodes[u] == pj.nodes[v]) {
            const double a0 = pi.arrive[u], a1 = a0 + P.fwd[pi.nodes[u]], b0 = pj.arrive[v], b1 = b0 + P.fwd[pj.nodes[v]];
            n += a0 < b1 - 1e-9 && b0 < a1 - 1e-9;
          }
    }
  return n;
}

bool replan(const Problem& P, Solution* S, const std::vector<int>& agents) {
  for (int a : agents)
    if (!plan_agent(P, a, S->cons[a], &S->paths[a])) return false;
  S->recost();
  S->collisions = count_collisions(P, *S);
  return true;
}

// Open list of the second phase: the paper takes the cheapest solution next; among the solutions within
// `slack` of the cheapest this one takes the one with the fewest collisions left (a focal search), which
// reaches a collision-free schedule in far fewer expansions when many agents share few nodes.
struct Focal {
  std::vector<Solution*> v;
  double slack;
  bool empty() const { return v.empty(); }
  void push(Solution* s) { v.push_back(s); }
  Solution* pop() {
    double best = kInf;
    for (Solution* s : v) best = std::min(best, s->cost);
    size_t pick = 0;
    bool have = false;
    for (size_t i = 0; i < v.size(); ++i) {
      if (v[i]->cost > best * (1.0 + slack) + 1e-12) continue;
      if (!have || v[i]->collisions < v[pick]->collisions ||
          (v[i]->collisions == v[pick]->collisions && v[i]->cost < v[pick]->cost)) { pick = i; have = true; }
    }
    Solution* s = v[pick];
    v[pick] = v.back();
    v.pop_back();
    return s;
  }
};

}  // namespace
}  // namespace sp

using namespace sp;

// Eq. 1 of "Allocating Nodes to Stages": |S_i| = |S_0| (1 - s/(s-1) k) for i >= 1, with all n_nodes used.
extern "C" int sp_stage_sizes(int n_nodes, int n_stages, int skip_num, int skip_den, int32_t* sizes) {
  if (!sizes || n_stages < 1 || n_nodes < n_stages || skip_den <= 0 || skip_num < 0)
    return fail(SP_EINVAL, "stage_sizes: bad arguments");
  if (n_stages == 1) { sizes[0] = n_nodes; return SP_OK; }
  const double s = n_stages, k = (double)skip_num / skip_den;
  const double r = 1.0 - s / (s - 1.0) * k;   // |S_i| / |S_0|
  if (!(r > 0.0)) return fail(SP_EINVAL, "stage_sizes: the skip ratio leaves the later stages no node");
  const double first = n_nodes / (1.0 + (s - 1.0) * r);
  // nearest whole numbers that use every node: later stages get round(first * r), stage 0 the rest
  int later = (int)std::lround(first * r);
  later = std::max(1, std::min(later, (n_nodes - 1) / (n_stages - 1)));
  sizes[0] = n_nodes - later * (n_stages - 1);
  for (int i = 1; i < n_stages; ++i) sizes[i] = later;
  return SP_OK;
}

extern "C" int sp_schedule_paths(const sp_sched_problem* q, int32_t* path_nodes, int32_t* path_stages, int32_t* len,
                                 float* arrive, float* e2e, float* max_e2e) {
  if (!q || !path_nodes || !path_stages || !len) return fail(SP_EINVAL, "schedule: null argument");
  if (q->n_stages < 1 || q->n_stages > 30 || q->n_nodes < 1 || q->n_agents < 1 || q->mem_limit < 1 ||
      !q->node_stage || !q->compute_fwd || !q->compute_bwd || !q->comm || !q->start_node || !q->n_keep)
    return fail(SP_EINVAL, "schedule: bad sizes or null arrays");
  Problem P;
  P.s = q->n_stages; P.N = q->n_nodes; P.A = q->n_agents; P.m = q->mem_limit; P.strict = q->strict_swap; P.no_swap = q->no_swap;
  P.node_stage = q->node_stage; P.fwd = q->compute_fwd; P.bwd = q->compute_bwd; P.comm = q->comm;
  P.start = q->start_node; P.keep = q->n_keep;
  P.stage_nodes.assign(P.s, {});
  for (int n = 0; n < P.N; ++n) {
    if (P.node_stage[n] < 0 || P.node_stage[n] >= P.s) return fail(SP_EINVAL, "schedule: node_stage out of range");
    if (!(P.fwd[n] >= 0.f) || !(P.bwd[n] >= 0.f)) return fail(SP_EINVAL, "schedule: negative compute time");
    P.stage_nodes[P.node_stage[n]].push_back(n);
  }
  for (size_t i = 0; i < (size_t)P.N * P.N; ++i)
    if (!(P.comm[i] >= 0.f)) return fail(SP_EINVAL, "schedule: negative transfer time");
  long total_skips = 0;
  for (int a = 0; a < P.A; ++a) {
    if (P.start[a] < 0 || P.start[a] >= P.N || P.node_stage[P.start[a]] != 0)
      return fail(SP_EINVAL, "schedule: a start node is not a node of stage 0");
    if (P.keep[a] < 1 || P.keep[a] > P.s) return fail(SP_EINVAL, "schedule: n_keep outside [1, n_stages]");
    total_skips += P.s - P.keep[a];
  }
  for (int st = 1; st < P.s; ++st)
    if (P.stage_nodes[st].empty()) return fail(SP_EINVAL, "schedule: a stage has no node");
  const int n_solutions = q->n_solutions > 0 ? q->n_solutions : 32;
  const int max_expansions = q->max_expansions > 0 ? q->max_expansions : 20000;
  const double delta = q->delta >= 0.f ? q->delta : 0.0;
  // CC3: every later stage is left out by floor or ceil of the mean number of skips, so it is visited by at
  // most A - floor(total_skips / (s - 1)) agents
  const int cap_visits = P.s > 1 ? P.A - (int)(total_skips / (P.s - 1)) : P.A;
  const int protect = P.A / 4;   // HR2: the slowest quarter is never constrained

  int expansions = 0;
  std::vector<Solution*> all;   // owns every node of the search tree
  auto make = [&](const Solution* from) { Solution* n = new Solution(*from); all.push_back(n); return n; };
  auto cleanup = [&]() { for (Solution* p : all) delete p; };
  Solution* root = new Solution();
  all.push_back(root);
  root->cons.assign(P.A, {});
  root->paths.assign(P.A, {});
  {
    std::vector<int> everyone(P.A);
    for (int a = 0; a < P.A; ++a) everyone[a] = a;
    if (!replan(P, root, everyone)) { cleanup(); return fail(SP_EPATH, "schedule: an agent has no path at all"); }
  }
  std::priority_queue<Solution*, std::vector<Solution*>, ByCost> open;
  Focal done{{}, q->focal_slack >= 0.f ? (double)q->focal_slack : 0.5};
  open.push(root);
  // CC3 on solution T: false if it holds; else pushes children into `into`, each with the over-visited stage
  // forbidden to `excess` of the paths through it: first the fastest ones (the paper's choice; never the
  // slowest quarter of the agents unless nobody else is left), then the same window moved on by one and by
  // two paths, so that a choice that leaves some agent without a path is not the end of the search
  auto resolve_cc3 = [&](Solution* T, auto* into) -> bool {
    int bad = -1;
    std::vector<int> through;
    for (int st = 1; st < P.s && bad < 0; ++st) {
      through.clear();
      for (int a = 0; a < P.A; ++a) if (visits_stage(P, T->paths[a], st)) through.push_back(a);
      if ((int)through.size() > cap_visits) bad = st;
    }
    if (bad < 0) return false;
    ++expansions;
    const int excess = (int)through.size() - cap_visits;
    std::vector<int> order(P.A);
    for (int a = 0; a < P.A; ++a) order[a] = a;
    order = by_speed(*T, order);
    std::vector<char> shielded(P.A, 0);
    for (int i = 0; i < protect; ++i) shielded[order[P.A - 1 - i]] = 1;
    // among equally fast paths, the agents that have been turned away from the fewest nodes so far go first:
    // with equal nodes everywhere the fastest-first rule alone would keep picking the same agents until they
    // have no stage left
    auto barred = [&](int a) {
      int n = 0;
      for (const Constraint& c : T->cons[a]) n += c.t1 == kInf && c.t0 == -kInf;
      return n;
    };
    std::vector<int> sorted = by_speed(*T, through);
    std::stable_sort(sorted.begin(), sorted.end(), [&](int x, int y) {
      if (std::fabs(T->paths[x].e2e - T->paths[y].e2e) > 1e-9) return false;   // keep the speed order
      return barred(x) < barred(y);
    });
    // an agent that already has as many stages barred as it leaves out cannot give up another one
    auto can_give_up = [&](int a) {
      int barred_stages = 0;
      for (int st = 1; st < P.s; ++st) {
        bool all = true;
        for (int nd : P.stage_nodes[st]) {
          bool found = false;
          for (const Constraint& c : T->cons[a]) found = found || (c.node == nd && c.t0 == -kInf && c.t1 == kInf);
          all = all && found;
        }
        barred_stages += all;
      }
      return barred_stages < P.s - P.keep[a];
    };
    std::vector<int> cand;
    for (int a : sorted) if (!shielded[a] && can_give_up(a)) cand.push_back(a);
    for (int a : sorted) if (shielded[a] && can_give_up(a)) cand.push_back(a);
    for (int shift = 0; shift < 3 && shift + excess <= (int)cand.size(); ++shift) {
      std::vector<int> pick(cand.begin() + shift, cand.begin() + shift + excess);
      Solution* S = make(T);
      for (int a : pick)
        for (int nd : P.stage_nodes[bad]) S->cons[a].push_back({nd, -kInf, kInf});
      if (replan(P, S, pick)) into->push(S);
    }
    return true;
  };
  // ---- phase 1: solutions that honour CC1-CC3
  int collected = 0;
  while (!open.empty() && collected < n_solutions && expansions < max_expansions) {
    Solution* T = open.top();
    open.pop();
    if (!resolve_cc3(T, &open)) { done.push(T); ++collected; }
  }
  // ---- phase 2: TC1, then TC2.  Re-planning under the new constraints can move an agent to other stages, so
  // CC3 is checked again first (the paper's listing does not say so; without it the result could break CC3)
  int rc = SP_EPATH;
  const Solution* found = nullptr;
  while (!done.empty() && expansions < max_expansions) {
    Solution* T = done.pop();
    if (resolve_cc3(T, &done)) continue;
    // TC1: at most m paths through a node
    int over = -1;
    std::vector<int> through;
    for (int n = 0; n < P.N && over < 0; ++n) {
      through.clear();
      for (int a = 0; a < P.A; ++a)
        if (std::find(T->paths[a].nodes.begin(), T->paths[a].nodes.end(), n) != T->paths[a].nodes.end())
          through.push_back(a);
      if ((int)through.size() > P.m) over = n;
    }
    if (over >= 0) {
      ++expansions;
      if (P.node_stage[over] == 0) continue;   // start nodes are given: nothing to move (an infeasible m)
      std::vector<int> fast = by_speed(*T, through);
      fast.pop_back();   // never the slowest path through the node
      fast.resize(std::min(fast.size(), through.size() - (size_t)P.m));
      Solution* S = make(T);
      for (int a : fast) S->cons[a].push_back({over, -kInf, kInf});
      if (replan(P, S, fast)) done.push(S);
      continue;
    }
    // TC2: two agents on one node at the same time (forward stays); conflicts with the slowest agent first
    int ci = -1, cj = -1, cn = -1;
    double is = 0, ie = 0, js = 0, je = 0;
    std::vector<int> order(P.A);
    for (int a = 0; a < P.A; ++a) order[a] = a;
    order = by_speed(*T, order);
    std::reverse(order.begin(), order.end());   // slowest first
    for (int x = 0; x < P.A && ci < 0; ++x)
      for (int y = x + 1; y < P.A && ci < 0; ++y) {
        const AgentPath &pi = T->paths[order[x]], &pj = T->paths[order[y]];
        for (size_t u = 0; u < pi.nodes.size() && ci < 0; ++u)
          for (size_t v = 0; v < pj.nodes.size(); ++v) {
            if (pi.nodes[u] != pj.nodes[v]) continue;
            const double a0 = pi.arrive[u], a1 = a0 + P.fwd[pi.nodes[u]], b0 = pj.arrive[v], b1 = b0 + P.fwd[pj.nodes[v]];
            if (a0 < b1 - 1e-9 && b0 < a1 - 1e-9) {
              ci = order[x]; cj = order[y]; cn = pi.nodes[u]; is = a0; ie = a1; js = b0; je = b1;
              break;
            }
          }
      }
    if (ci < 0) { found = T; rc = SP_OK; break; }
    ++expansions;
    const double ei = T->paths[ci].e2e, ej = T->paths[cj].e2e;
    const bool close = std::fabs(ei - ej) < delta;
    // the faster one waits; if the two are within delta of each other either may, and the two choices become
    // two children (were both constrained in one child, two identical agents would stay in step for ever)
    if (ei >= ej || close) {
      Solution* S = make(T);
      S->cons[cj].push_back({cn, is, ie});
      if (replan(P, S, {cj})) done.push(S);
    }
    if (ei < ej || close) {
      Solution* S = make(T);
      S->cons[ci].push_back({cn, js, je});
      if (replan(P, S, {ci})) done.push(S);
    }
  }
  if (rc != SP_OK) {
    cleanup();
    return fail(SP_EPATH, std::string(expansions >= max_expansions ? "schedule: expansion limit reached" : "schedule: search exhausted") +
                              " without a conflict-free solution (" + std::to_string(collected) +
                              " solutions passed the first phase, " + std::to_string(expansions) + " expansions)");
  }
  double worst = 0;
  for (int a = 0; a < P.A; ++a) {
    const AgentPath& p = found->paths[a];
    len[a] = (int32_t)p.nodes.size();
    for (int j = 0; j < P.s; ++j) {
      const bool in = j < (int)p.nodes.size();
      path_nodes[(size_t)a * P.s + j] = in ? p.nodes[j] : -1;
      path_stages[(size_t)a * P.s + j] = in ? P.node_stage[p.nodes[j]] : -1;
      if (arrive) arrive[(size_t)a * P.s + j] = in ? (float)p.arrive[j] : -1.f;
    }
    if (e2e) e2e[a] = (float)p.e2e;
    worst = std::max(worst, p.e2e);
  }
  if (max_e2e) *max_e2e = (float)worst;
  cleanup();
  return SP_OK;
}
