"""Independent checks of a schedule (test helper, plain Python): the constraints of the paper's scheduler
recomputed from the returned paths and times, and an exhaustive single-agent optimum for small graphs."""
import itertools

import numpy as np


def order_ok(stages, strict):
    """CC1 + CC2: opens with stage 0, no repeats, increasing apart from one exchange of two neighbours."""
    st = list(stages)
    if not st or st[0] != 0 or len(set(st)) != len(st):
        return False
    desc = [j for j in range(len(st) - 1) if st[j + 1] < st[j]]
    if not desc:
        return True
    if len(desc) > 1 or desc[0] == 0:
        return False
    j = desc[0]
    q = st[:]
    q[j], q[j + 1] = q[j + 1], q[j]
    return q == sorted(q) and (not strict or st[j] - st[j + 1] == 1)


def latency(nodes, arrive, fwd, bwd, comm):
    """End of the backward pass of a path whose forward stays start at `arrive`."""
    t = arrive[-1] + fwd[nodes[-1]]
    n0 = nodes[0]
    if nodes[-1] != n0:
        t += comm[nodes[-1], n0] + comm[n0, nodes[-1]]
    for j in range(len(nodes) - 1, -1, -1):
        t += bwd[nodes[j]]
        if j:
            t += comm[nodes[j], nodes[j - 1]]
    return t


def check_schedule(res, node_stage, fwd, bwd, comm, start, keep, mem_limit, strict=True, tol=1e-4):
    node_stage = np.asarray(node_stage); A = len(start); s = int(node_stage.max()) + 1
    visits = np.zeros(s, int); through = np.zeros(len(node_stage), int)
    stays = []
    for a in range(A):
        n = int(res["len"][a]); nodes = [int(x) for x in res["path_nodes"][a, :n]]; arr = res["arrive"][a, :n]
        assert n == keep[a] and nodes[0] == start[a]
        assert (res["path_nodes"][a, n:] == -1).all() and (res["path_stages"][a, n:] == -1).all()
        stages = [int(node_stage[x]) for x in nodes]
        assert stages == [int(x) for x in res["path_stages"][a, :n]]
        assert order_ok(stages, strict), stages
        t = 0.0
        for j, nd in enumerate(nodes):
            earliest = t if j == 0 else t + comm[nodes[j - 1], nd]
            assert arr[j] >= earliest - tol, (a, j, arr[j], earliest)     # no stay starts before the agent can be there
            t = arr[j] + fwd[nd]
            stays.append((nd, float(arr[j]), float(t), a))
            visits[stages[j]] += 1; through[nd] += 1
        assert abs(latency(nodes, arr, fwd, bwd, comm) - res["e2e"][a]) < tol * max(1.0, res["e2e"][a])
    assert abs(max(res["e2e"]) - res["max_e2e"]) < tol * max(1.0, res["max_e2e"])
    # CC3: later stages are left out by the same number of agents, up to one
    total_skips = sum(s - k for k in keep)
    if s > 1:
        assert visits[1:].max() <= A - total_skips // (s - 1), visits
    # TC1
    later = node_stage != 0
    assert (through[later] <= mem_limit).all(), through
    # TC2: no two agents on one node at the same time
    for (n1, a0, a1, x), (n2, b0, b1, y) in itertools.combinations(stays, 2):
        if n1 == n2 and x != y:
            assert a1 <= b0 + tol or b1 <= a0 + tol, (n1, x, y, a0, a1, b0, b1)


def single_agent_optimum(node_stage, fwd, bwd, comm, start, keep, strict=True):
    """Exhaustive: every admissible stage order and node choice of one unconstrained agent."""
    node_stage = np.asarray(node_stage); s = int(node_stage.max()) + 1
    by_stage = [[n for n in range(len(node_stage)) if node_stage[n] == st] for st in range(s)]
    best = np.inf
    for later in itertools.permutations(range(1, s), keep - 1):
        stages = [0] + list(later)
        if not order_ok(stages, strict):
            continue
        for choice in itertools.product(*[by_stage[st] for st in later]):
            nodes = [start] + list(choice)
            arr, t = [], 0.0
            for j, nd in enumerate(nodes):
                t = t if j == 0 else t + comm[nodes[j - 1], nd]
                arr.append(t); t += fwd[nd]
            best = min(best, latency(nodes, arr, fwd, bwd, comm))
    return best
