"""The seeded path recipe used for all synthetic workloads, pinned by Eq. 1 and the constraints CC1-CC3."""
import os

import numpy as np
import pytest

from paper_2502_19913_amd import synth
from tests import pathcheck

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [[int(x) for x in ln.split()] for ln in f if ln.strip() and not ln.startswith("#")]


def test_eq1_reproduces_the_printed_stage_sizes():
    for s, num, den, n0, ni in rows("eq1_stage_sizes.txt"):
        assert n0 * (1 - s / (s - 1) * num / den) == pytest.approx(ni, abs=1e-12)


def test_token_table_arithmetic():
    # nodes in stage 0 (Eq. 1 instances) send the same number of microbatches each; context 4096
    for nodes, spm, printed_k, n_mb in rows("batch_tokens.txt"):
        tokens = n_mb * spm * 4096
        assert tokens // 1000 == printed_k
        assert n_mb % {20: 5, 18: 6}[nodes] == 0


@pytest.mark.parametrize("seed", range(20))
def test_visits_per_stage_follow_eq1(seed):
    # one path per stage-0 node: the number of paths visiting each later stage is Eq. 1's |S_i|
    for s, num, den, n0, ni in rows("eq1_stage_sizes.txt"):
        paths, lens = synth.make_paths(s, n0, num, den, allow_swap=bool(seed % 2), seed=seed)
        cnt = pathcheck.check_set(paths, lens, s, num, den)
        assert list(n0 - cnt) == [n0] + [ni] * (s - 1)


@pytest.mark.parametrize("s,n,num,den", [(4, 2, 1, 4), (6, 8, 1, 3), (8, 16, 1, 4), (8, 16, 1, 3), (6, 7, 1, 3),
                                         (5, 9, 2, 5), (8, 3, 1, 2), (4, 5, 0, 1), (2, 4, 1, 2)])
def test_constraints_hold_for_many_seeds(s, n, num, den):
    saw_swap = False
    for seed in range(40):
        paths, lens = synth.make_paths(s, n, num, den, allow_swap=True, seed=seed)
        pathcheck.check_set(paths, lens, s, num, den)
        saw_swap |= any(pathcheck.n_swaps(list(p[:l])) for p, l in zip(paths, lens))
        p2, l2 = synth.make_paths(s, n, num, den, allow_swap=True, seed=seed)
        assert np.array_equal(paths, p2) and np.array_equal(lens, l2)
        p3, _ = synth.make_paths(s, n, num, den, allow_swap=False, seed=seed)
        assert all(pathcheck.n_swaps(list(p[:l])) == 0 for p, l in zip(p3, lens))
    if s >= 4 and s - (s * num) // den >= 3:
        assert saw_swap


def test_non_divisible_ratio_uses_floor_and_ceil():
    # 8 stages at 1/3: 16 paths skip 43 stages in total, eleven paths skip 3 and five skip 2
    paths, lens = synth.make_paths(8, 16, 1, 3, True, seed=1)
    q = 8 - lens
    assert q.sum() == 43 and sorted(set(q)) == [2, 3] and (q == 3).sum() == 11


def test_validator_rejects_violations():
    with pytest.raises(AssertionError):
        pathcheck.check_one([1, 2, 3], 4)            # CC1
    with pytest.raises(AssertionError):
        pathcheck.check_one([0, 2, 2], 4)            # repeat
    with pytest.raises(AssertionError):
        pathcheck.check_one([0, 3, 2, 1], 4)         # two descents
    with pytest.raises(AssertionError):
        pathcheck.check_one([0, 3, 1], 4)            # exchanged stages not consecutive (strict)
    pathcheck.check_one([0, 3, 1], 4, strict=False)
    pathcheck.check_one([0, 1, 3, 2], 4)             # the paper's swap example
    with pytest.raises(AssertionError):
        pathcheck.check_one([0, 2, 3, 1], 4, strict=False)   # a rotation, not one adjacent exchange


def test_eval_paths_drop_counts_and_half_stage():
    # 6 stages: 25 % = 1.5 stages (one dropped, one half), 1/3 = 2, 50 % = 3; stage 0 is never touched
    for (num, den), (whole, part) in {(1, 4): (1, 1), (1, 3): (2, 0), (1, 2): (3, 0), (0, 1): (0, 0)}.items():
        paths, lens, half = synth.make_eval_paths(6, 32, num, den, 11)
        assert (lens == 6 - whole).all() and (paths[:, 0] == 0).all()
        for mb in range(32):
            kept = list(paths[mb, :lens[mb]])
            assert kept == sorted(kept) and len(set(kept)) == len(kept) and (paths[mb, lens[mb]:] == -1).all()
            assert (half[mb] >= 1 and half[mb] in kept) if part else half[mb] == -1
        # drops differ between samples (a per-sample draw) and depend on the seed alone
        assert len({tuple(p) for p in paths}) > 1 or whole == 0
        again = synth.make_eval_paths(6, 32, num, den, 11)
        assert all((a == b).all() for a, b in zip((paths, lens, half), again))
    with pytest.raises(ValueError):
        synth.make_eval_paths(2, 4, 3, 4, 1)
