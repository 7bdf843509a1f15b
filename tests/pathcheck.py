"""Independent statement of the path constraints (section "Guideline for Partial Pipelining Scheduler").

CC1: every path opens with stage 0.  No stage appears twice.  Length = stages minus the skipped count.
CC2 (reading taken: the printed inequality cannot hold on a path with a skip): the path is increasing
except for at most one exchange of two neighbouring entries, never touching position 0; in the strict
form the two exchanged stages are also neighbours in the model.
CC3: every stage i >= 1 is left out by the same number of paths (differing by at most one when the
counts do not divide).
"""
import numpy as np


def n_swaps(path):
    """Number of adjacent descents; a single adjacent exchange in an increasing list gives exactly one."""
    return sum(1 for a, b in zip(path[:-1], path[1:]) if b < a)


def check_one(path, n_stages, strict=True):
    path = [int(s) for s in path]
    assert path[0] == 0, "CC1"
    assert len(set(path)) == len(path), "repeat"
    assert all(0 <= s < n_stages for s in path)
    desc = [j for j in range(len(path) - 1) if path[j + 1] < path[j]]
    assert len(desc) <= 1, "CC2: more than one swap"
    if desc:
        j = desc[0]
        assert j >= 1, "CC2: swap touches stage 0"
        fixed = path[:j] + [path[j + 1], path[j]] + path[j + 2:]
        assert fixed == sorted(fixed), "CC2: not a single adjacent exchange"
        if strict:
            assert path[j] - path[j + 1] == 1, "CC2: exchanged stages are not consecutive"


def skip_counts(paths, lens, n_stages):
    cnt = np.zeros(n_stages, dtype=int)
    for p, l in zip(paths, lens):
        kept = set(int(s) for s in p[:l])
        for s in range(n_stages):
            cnt[s] += s not in kept
    return cnt


def check_set(paths, lens, n_stages, skip_num, skip_den, strict=True):
    n = len(lens)
    for p, l in zip(paths, lens):
        check_one(p[:l], n_stages, strict)
        assert all(int(x) == -1 for x in p[l:])
    cnt = skip_counts(paths, lens, n_stages)
    assert cnt[0] == 0
    if n_stages > 1:
        assert cnt[1:].max() - cnt[1:].min() <= 1, "CC3"
    total = int(cnt.sum())
    want = n * n_stages * skip_num / skip_den
    assert abs(total - want) <= 0.5 + 1e-9, "skip fraction"
    lo = (n_stages * skip_num) // skip_den
    for l in lens:
        assert n_stages - int(l) in (lo, lo + 1) if (n_stages * skip_num) % skip_den else n_stages - int(l) == lo
    return cnt
