"""Host logic of the library that needs no GPU: symbol table, layout, path generator, validator, route plan."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2502_19913_amd import binding as sp
from paper_2502_19913_amd import synth
from tests import pathcheck

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "skippipe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sp_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = sp.lib()
    names = declared_symbols()
    assert len(names) >= 15
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(sp.EXPORTS) == names


def test_param_layout_matches_shapes_and_is_dense():
    for key in ("c1", "c2", "c3", "c5"):
        cfg = synth.CONFIGS[key]
        lay = sp.param_layout(cfg)
        want = synth.param_shapes(cfg)
        assert [l[0] for l in lay] == [w[0] for w in want]
        off = 0
        for (name, stage, layer, o, rows, cols), (_, shape) in zip(lay, want):
            assert o == off
            assert rows * cols == int(np.prod(shape))
            if len(shape) == 2:
                assert (rows, cols) == shape
            off += rows * cols
        assert off == sp.param_count(cfg)


def test_param_counts_of_the_named_shapes():
    # per-stage parameter counts of the 1.5B and 8B stage configurations
    assert sp.param_count(synth.CONFIGS["c3"]) == 4 * (2 * 2048 + 3 * 2048 * 2048 + 2048 * 2048 + 3 * 2048 * 5632)
    c5 = synth.CONFIGS["c5"]
    per_layer = 2 * 4096 + (4096 + 2 * 1024) * 4096 + 4096 * 4096 + 3 * 4096 * 14336
    assert sp.param_count(c5) == 4 * per_layer + 4096 + 128256 * 4096


def test_bad_cfg_is_rejected():
    bad = dict(synth.CONFIGS["c1"], n_heads=5)
    with pytest.raises(sp.SpError) as e:
        sp.param_count(bad)
    assert e.value.code == -1
    with pytest.raises(sp.SpError):
        sp.param_count(dict(synth.CONFIGS["c1"], local_stage_count=9))


@pytest.mark.parametrize("seed", range(20))
def test_generated_paths_follow_eq1(seed):
    # |S_i| = |S_0| (1 - s/(s-1) k): 6 -> 4 at s=4, k=1/4 and 5 -> 3 at s=6, k=1/3 (the paper's two set-ups)
    for s, num, den, n0, ni in [(4, 1, 4, 6, 4), (6, 1, 3, 5, 3)]:
        paths, lens = sp.make_paths(s, n0, num, den, bool(seed % 2), seed)
        cnt = pathcheck.check_set(paths, lens, s, num, den)
        assert list(n0 - cnt) == [n0] + [ni] * (s - 1)


@pytest.mark.parametrize("s,n,num,den", [(4, 2, 1, 4), (6, 8, 1, 3), (8, 16, 1, 4), (8, 16, 1, 3), (6, 7, 1, 3),
                                         (5, 9, 2, 5), (8, 3, 1, 2), (4, 5, 0, 1), (2, 4, 1, 2), (1, 3, 0, 1)])
def test_generated_paths_hold_the_constraints(s, n, num, den):
    saw_swap = False
    for seed in range(40):
        paths, lens = sp.make_paths(s, n, num, den, True, seed)
        pathcheck.check_set(paths, lens, s, num, den)
        saw_swap |= any(pathcheck.n_swaps(list(p[:l])) for p, l in zip(paths, lens))
        p2, l2 = sp.make_paths(s, n, num, den, True, seed)
        assert np.array_equal(paths, p2) and np.array_equal(lens, l2)
        cfg = dict(synth.CONFIGS["c1"], n_stages=s, local_stage_count=s)
        sp.check_paths(cfg, paths, lens)
    if s >= 4 and s - (s * num) // den >= 3:
        assert saw_swap


def test_skip_fraction_matches_request():
    paths, lens = sp.make_paths(8, 16, 1, 3, True, 1)
    assert (8 - lens).sum() == 43                 # round(16 * 8 / 3)
    paths, lens = sp.make_paths(6, 8, 1, 3, True, 1)
    assert np.all(lens == 4)
    with pytest.raises(sp.SpError):
        sp.make_paths(4, 2, 1, 1, False, 0)       # would skip stage 0 as well


def test_validator_names_each_violation():
    cfg = dict(synth.CONFIGS["c1"])

    def rej(path, flags=sp.SP_STRICT_CC):
        p = np.full((1, 4), -1, np.int32); p[0, :len(path)] = path
        with pytest.raises(sp.SpError) as e:
            sp.check_paths(dict(cfg, path_flags=flags), p, np.array([len(path)], np.int32))
        assert e.value.code == -2
        return str(e.value)

    def ok(path, flags=sp.SP_STRICT_CC):
        p = np.full((1, 4), -1, np.int32); p[0, :len(path)] = path
        sp.check_paths(dict(cfg, path_flags=flags), p, np.array([len(path)], np.int32))

    assert "CC1" in rej([1, 2, 3])
    assert "twice" in rej([0, 2, 2])
    assert "range" in rej([0, 4])
    assert "CC2" in rej([0, 3, 2, 1])
    assert "CC2" in rej([0, 3, 1])
    ok([0, 3, 1], sp.SP_SWAP_ANY_GAP)
    assert "CC2" in rej([0, 2, 3, 1], sp.SP_SWAP_ANY_GAP)
    ok([0, 2, 3, 1], sp.SP_ALLOW_ANY_ORDER)
    ok([0, 1, 3, 2])                              # the paper's swap example
    ok([0, 1, 3])                                 # a skip
    ok([0])


def test_route_plan_groups_by_position_and_stage():
    cfg = dict(synth.CONFIGS["c1"])
    paths = np.array([[0, 1, 2, 3], [0, 1, 3, -1], [0, 3, 2, -1], [0, 2, 3, -1]], np.int32)
    lens = np.array([4, 3, 3, 3], np.int32)
    plan = sp.route_plan(cfg, paths, lens)
    assert plan == [(0, 0, [0, 1, 2, 3]), (1, 1, [0, 1]), (1, 2, [3]), (1, 3, [2]), (2, 2, [0, 2]), (2, 3, [1, 3]),
                    (3, 3, [0])]
    # every (microbatch, stage) visit appears exactly once
    seen = sorted((mb, st) for _, st, mbs in plan for mb in mbs)
    want = sorted((mb, int(st)) for mb in range(4) for st in paths[mb, :lens[mb]])
    assert seen == want
    # a node holding only stage 2
    share = dict(cfg, local_stage_begin=2, local_stage_count=1, has_embed=0, has_head=0)
    assert sp.route_plan(share, paths, lens) == [(1, 2, [3]), (2, 2, [0, 2])]


def test_workspace_bytes_grows_with_visits():
    cfg = synth.CONFIGS["c3"]
    a = sp.workspace_bytes(cfg, 8, 8)
    b = sp.workspace_bytes(cfg, 8, 4)
    assert a > b > 0
    per_visit = (a - b) // 4
    d, h, T = 2048, 5632, 4096
    est = 4 * T * ((6 * d + 2 * d + 3 * h) * 2 + 16 * 4 + 8)
    assert 0.98 * est < per_visit < 1.05 * est


def test_product_path_refuses_to_run_without_a_gpu():
    # there is no CPU fallback: a context cannot be made where no HIP device is present
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(RuntimeError):
        sp.Context(synth.CONFIGS["c1"], 1, 1)
    # and nothing in the product imports the CPU checker
    import os, re
    pkg = os.path.join(ROOT, "paper_2502_19913_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle|#include\s+\".*oracle", text, re.M), (dirpath, f)
