"""The host path scheduler: its low level against an exhaustive optimum, its output against the constraints
recomputed independently (CC1-CC3, TC1, TC2), and its error paths.  CPU only."""
import os

import numpy as np
import pytest

from paper_2502_19913_amd import binding as sp
from paper_2502_19913_amd import synth
from tests import pathcheck
from tests.schedcheck import check_schedule, single_agent_optimum


def world(s, per_stage, seed, first=None):
    """Nodes in stages (stage 0 may be larger, as Eq. 1 asks), seeded compute and transfer times."""
    sizes = [first or per_stage] + [per_stage] * (s - 1)
    node_stage = np.concatenate([[st] * n for st, n in enumerate(sizes)]).astype(np.int32)
    N = len(node_stage)
    u = synth.uniform(seed, "sched", N * N + 2 * N).astype(np.float64)
    fwd = (0.5 + u[:N]).astype(np.float32)
    bwd = (2.0 * fwd).astype(np.float32)
    comm = (0.1 + 2.0 * u[2 * N:].reshape(N, N)).astype(np.float32)
    comm = ((comm + comm.T) / 2).astype(np.float32); np.fill_diagonal(comm, 0)
    return node_stage, fwd, bwd, comm


@pytest.mark.parametrize("s,per,keep,strict", [(4, 2, 3, True), (5, 3, 4, True), (6, 2, 4, False), (4, 3, 4, True),
                                               (5, 2, 2, True)])
def test_one_agent_takes_the_exhaustive_optimum(s, per, keep, strict):
    ns, fwd, bwd, comm = world(s, per, 100 + s + per)
    res = sp.schedule_paths(ns, fwd, bwd, comm, [0], [keep], mem_limit=8, strict_swap=strict)
    want = single_agent_optimum(ns, fwd, bwd, comm, 0, keep, strict)
    assert abs(res["max_e2e"] - want) < 1e-4 * want
    check_schedule(res, ns, fwd, bwd, comm, [0], [keep], 8, strict)


@pytest.mark.parametrize("s,per,first,A,skip,m", [(4, 2, 3, 3, 1, 2), (6, 3, 5, 5, 2, 2), (4, 4, 6, 6, 1, 2),
                                                  (8, 2, 4, 4, 2, 3), (6, 2, 2, 4, 2, 4), (6, 3, 5, 10, 2, 4),
                                                  (6, 3, 5, 20, 2, 12), (8, 4, 6, 24, 2, 12)])
def test_schedule_honours_every_constraint(s, per, first, A, skip, m):
    ns, fwd, bwd, comm = world(s, per, 7 * s + A, first=first)
    start = [a % first for a in range(A)]
    keep = [s - skip] * A
    res = sp.schedule_paths(ns, fwd, bwd, comm, start, keep, mem_limit=m, delta=0.05)
    check_schedule(res, ns, fwd, bwd, comm, start, keep, m)
    # the stage lists are paths the training entry points accept
    for a in range(A):
        pathcheck.check_one(res["path_stages"][a, :res["len"][a]], s, strict=True)
    # no schedule beats the slowest agent's own unconstrained optimum
    lower = max(single_agent_optimum(ns, fwd, bwd, comm, start[a], keep[a]) for a in range(A))
    assert res["max_e2e"] >= lower - 1e-4


def test_two_agents_on_one_chain_take_turns():
    # one node per stage, two agents from the same start: the second waits for the first everywhere (TC2)
    ns = np.array([0, 1, 2], np.int32); fwd = np.array([1, 1, 1], np.float32); bwd = 2 * fwd
    comm = np.full((3, 3), 0.5, np.float32); np.fill_diagonal(comm, 0)
    res = sp.schedule_paths(ns, fwd, bwd, comm, [0, 0], [3, 3], mem_limit=2)
    check_schedule(res, ns, fwd, bwd, comm, [0, 0], [3, 3], 2)
    alone = single_agent_optimum(ns, fwd, bwd, comm, 0, 3)
    assert sorted(np.round(res["e2e"], 4)) == [round(alone, 4), round(alone + 1.0, 4)]   # one forward stay later


def test_worked_chain_example_of_the_paper():
    # appendix "Path Coarsening": A-B-C with 1, 2, 1 seconds per microbatch and 1 second per transfer; two
    # microbatches keep A busy for 2 s, B for 4 s, and leave C idle for 1 s between them
    rows = [l.split() for l in open(os.path.join(os.path.dirname(__file__), "golden", "abc_chain_example.txt"))
            if l.strip() and not l.startswith("#")]
    fwd = np.array([float(r[1]) for r in rows[:3]], np.float32)
    tr, n_mb, busy_a, busy_b, gap_c = (float(x) for x in rows[3])
    ns = np.array([0, 1, 2], np.int32)
    comm = np.full((3, 3), tr, np.float32); np.fill_diagonal(comm, 0)
    res = sp.schedule_paths(ns, fwd, fwd, comm, [0] * int(n_mb), [3] * int(n_mb), mem_limit=int(n_mb), allow_swap=False)
    check_schedule(res, ns, fwd, fwd, comm, [0] * int(n_mb), [3] * int(n_mb), int(n_mb))
    stays = {n: sorted((float(res["arrive"][a, n]), float(res["arrive"][a, n]) + float(fwd[n])) for a in range(int(n_mb)))
             for n in range(3)}
    assert stays[0][-1][1] - stays[0][0][0] == pytest.approx(busy_a)        # back to back on A
    assert stays[1][-1][1] - stays[1][0][0] == pytest.approx(busy_b)        # back to back on B
    assert stays[1][1][0] == pytest.approx(stays[1][0][1])
    assert stays[2][1][0] - stays[2][0][1] == pytest.approx(gap_c)          # C waits for B
    # with the one exchange CC2 allows, the second microbatch visits C before B and nobody waits: the slowest
    # microbatch finishes earlier than in the in-order schedule
    swapped = sp.schedule_paths(ns, fwd, fwd, comm, [0] * int(n_mb), [3] * int(n_mb), mem_limit=int(n_mb))
    check_schedule(swapped, ns, fwd, fwd, comm, [0] * int(n_mb), [3] * int(n_mb), int(n_mb))
    assert sorted(map(tuple, swapped["path_stages"].tolist())) == [(0, 1, 2), (0, 2, 1)]
    assert swapped["max_e2e"] < res["max_e2e"]


def test_identical_nodes_spread_the_agents():
    # two nodes per stage, equal costs: two agents from two start nodes need not collide at all
    ns = np.array([0, 0, 1, 1, 2, 2], np.int32); fwd = np.ones(6, np.float32); bwd = 2 * fwd
    comm = np.full((6, 6), 0.25, np.float32); np.fill_diagonal(comm, 0)
    res = sp.schedule_paths(ns, fwd, bwd, comm, [0, 1], [3, 3], mem_limit=1)
    check_schedule(res, ns, fwd, bwd, comm, [0, 1], [3, 3], 1)
    assert res["max_e2e"] == pytest.approx(single_agent_optimum(ns, fwd, bwd, comm, 0, 3), rel=1e-5)


def test_identical_agents_from_one_start_node_do_not_stay_in_step():
    # two agents with the same start node and equal latencies collide at time 0; whichever waits, they part
    ns = np.array([0, 1, 1, 2, 2], np.int32); fwd = np.ones(5, np.float32); bwd = 2 * fwd
    comm = np.full((5, 5), 0.5, np.float32); np.fill_diagonal(comm, 0)
    res = sp.schedule_paths(ns, fwd, bwd, comm, [0, 0], [3, 3], mem_limit=2, delta=0.5, max_expansions=100)
    check_schedule(res, ns, fwd, bwd, comm, [0, 0], [3, 3], 2)


def test_rejects_bad_problems():
    ns = np.array([0, 1, 2], np.int32); one = np.ones(3, np.float32); comm = np.zeros((3, 3), np.float32)
    with pytest.raises(sp.SpError):
        sp.schedule_paths(ns, one, one, comm, [1], [3], mem_limit=1)            # start node outside stage 0
    with pytest.raises(sp.SpError):
        sp.schedule_paths(ns, one, one, comm, [0], [4], mem_limit=1)            # more stages than exist
    with pytest.raises(sp.SpError):
        sp.schedule_paths(np.array([0, 2, 2], np.int32), one, one, comm, [0], [2], mem_limit=1)   # stage 1 has no node
    with pytest.raises(sp.SpError):
        sp.schedule_paths(ns, -one, one, comm, [0], [3], mem_limit=1)
    # three agents, one node per later stage, one path allowed through each node: no solution
    with pytest.raises(sp.SpError):
        sp.schedule_paths(np.array([0, 0, 0, 1, 2], np.int32), np.ones(5, np.float32), np.ones(5, np.float32),
                          np.zeros((5, 5), np.float32), [0, 1, 2], [3, 3, 3], mem_limit=1, max_expansions=200)


def test_cheapest_first_and_focal_orders_agree_where_both_finish():
    # focal_slack 0 is the paper's order (cheapest solution next); a wider focus may only cost latency
    ns, fwd, bwd, comm = world(6, 3, 41, first=5)
    start = [a % 5 for a in range(8)]; keep = [4] * 8
    strict = sp.schedule_paths(ns, fwd, bwd, comm, start, keep, mem_limit=4, delta=0.05, focal_slack=0.0)
    focal = sp.schedule_paths(ns, fwd, bwd, comm, start, keep, mem_limit=4, delta=0.05, focal_slack=0.5)
    check_schedule(strict, ns, fwd, bwd, comm, start, keep, 4)
    check_schedule(focal, ns, fwd, bwd, comm, start, keep, 4)
    assert focal["max_e2e"] <= 1.5 * strict["max_e2e"] + 1e-4


def test_stage_sizes_reproduce_the_papers_set_ups():
    # appendix "Test Configurations": 18 nodes / 4 stages / 25 % -> (6,4,4,4); 20 nodes / 6 stages / 33 % -> (5,3,3,3,3,3)
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "eq1_stage_sizes.txt")):
        if not line.strip() or line.startswith("#"):
            continue
        s, num, den, n0, ni = (int(x) for x in line.split())
        assert sp.stage_sizes(n0 + ni * (s - 1), s, num, den) == [n0] + [ni] * (s - 1)
    assert sp.stage_sizes(7, 1, 0, 1) == [7]
    assert sum(sp.stage_sizes(23, 6, 1, 3)) == 23                      # every node is used
    with pytest.raises(sp.SpError):
        sp.stage_sizes(3, 4, 1, 4)
    with pytest.raises(sp.SpError):
        sp.stage_sizes(10, 2, 1, 2)                                    # 1 - 2 * 1/2 = 0: nothing left for stage 1
