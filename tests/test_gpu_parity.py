"""GPU library against the CPU checker, element by element, on seeded synthetic inputs.

Tolerances: float mode 1e-4 relative on the loss and on every gradient
tensor (L2-relative per tensor); bfloat16 mode 1e-2 relative on the loss and per-tensor gradient cosine
>= 0.999, with the checker fed the bf16-rounded parameters widened to float.  Beside the per-tensor norms every
tensor also meets an element-wise bound, max|got - ref| <= tol * max|ref| (float: 1e-4; bfloat16: 5e-2, a few
roundings of 2^-9 accumulated over the ops of a layer, taken at the tail of their distribution over millions of
elements), so a handful of wrong elements in a large tensor cannot hide behind its norm.
"""
import math

import numpy as np
import pytest
import torch

from oracle import skippipe_oracle as orc
from paper_2502_19913_amd import binding as sp
from paper_2502_19913_amd import synth
from tests.gpuharness import cosine, maxerr, relerr, round_bf16, run, n_visits

pytestmark = pytest.mark.gpu

F32_TOL = 1e-4
BF16_LOSS_TOL = 1e-2
BF16_COS = 0.999
BF16_MAX = 5e-2      # element-wise, relative to the tensor's largest magnitude


def inputs(cfg, seed, std=0.02, jitter=0.02, bf16=False):
    named = synth.make_params(cfg, seed, gain_jitter=jitter, std=std)
    if bf16:
        named = {k: round_bf16(v) for k, v in named.items()}
    tok, tgt = synth.make_tokens(cfg, seed)
    return named, tok, tgt


def check_f32(got, ref, what=""):
    assert math.isclose(got["loss"], ref["loss"], rel_tol=F32_TOL), (what, got["loss"], ref["loss"])
    assert np.allclose(got["loss_mb"], ref["loss_mb"], rtol=F32_TOL)
    for name, g in ref["grads"].items():
        if np.all(g == 0):
            assert np.all(got["grads"][name] == 0), (what, name)
        else:
            assert relerr(got["grads"][name], g) < F32_TOL, (what, name, relerr(got["grads"][name], g))
            assert maxerr(got["grads"][name], g) < F32_TOL, (what, name, maxerr(got["grads"][name], g))


def check_bf16(got, ref, what="", has_loss=True):
    if has_loss:
        assert math.isclose(got["loss"], ref["loss"], rel_tol=BF16_LOSS_TOL), (what, got["loss"], ref["loss"])
    for name, g in ref["grads"].items():
        if np.all(g == 0):
            assert np.all(got["grads"][name] == 0), (what, name)
        else:
            c = cosine(got["grads"][name], g)
            assert c >= BF16_COS, (what, name, c)
            assert maxerr(got["grads"][name], g) < BF16_MAX, (what, name, maxerr(got["grads"][name], g))


# ------------------------------------------------------------------ whole model, float mode
def test_c1_full_shape_f32():
    cfg = synth.CONFIGS["c1"]
    named, tok, tgt = inputs(cfg, synth.BASE_SEED)
    # paths from the library's own generator (the exported sp_make_paths), not from the harness twin
    paths, lens = sp.make_paths(cfg["n_stages"], cfg["n_mb"], *cfg["skip"], cfg["swap"], synth.BASE_SEED)
    assert (lens == 3).all() and (paths[:, 0] == 0).all()
    ref = orc.run_paths(cfg, named, paths, lens, tokens=tok, targets=tgt, dtype=np.float64)
    got = run(cfg, named, paths, lens, tokens=tok, targets=tgt)
    check_f32(got, ref, "c1")
    assert abs(ref["loss"] - math.log(cfg["vocab"])) < 0.1


SMALL = dict(synth.CONFIGS["c1"], dim=64, n_heads=4, n_kv_heads=2, hidden=96, vocab=200, n_stages=4,
             layers_per_stage=2, seq_len=24, seqs_per_mb=2, n_mb=5)
PATHS5 = np.array([[0, 1, 2, 3], [0, 1, 3, -1], [0, 3, 2, -1], [0, 2, 3, -1], [0, 1, 2, -1]], np.int32)
LENS5 = np.array([4, 3, 3, 3, 3], np.int32)


@pytest.mark.parametrize("whole_call", [True, False])
def test_small_f32_skip_swap_gqa(whole_call):
    cfg = dict(SMALL, path_flags=sp.SP_SWAP_ANY_GAP)
    named, tok, tgt = inputs(cfg, 3, std=0.08, jitter=0.1)
    tgt[1, 0, :5] = -1                                   # some ignored targets
    ref = orc.run_paths(cfg, named, PATHS5, LENS5, tokens=tok, targets=tgt)
    got = run(cfg, named, PATHS5, LENS5, tokens=tok, targets=tgt, whole_call=whole_call)
    check_f32(got, ref, f"small whole_call={whole_call}")
    if not whole_call:
        assert relerr(got["y"], ref["y"]) < F32_TOL


def test_odd_shapes_take_the_scalar_kernels_f32():
    # nothing divisible by 8: dim 36 (hd 6), hidden 50, vocab 77, T 13
    cfg = dict(SMALL, dim=36, n_heads=6, n_kv_heads=3, hidden=50, vocab=77, seq_len=13, seqs_per_mb=3, layers_per_stage=1,
               path_flags=sp.SP_SWAP_ANY_GAP)
    named, tok, tgt = inputs(cfg, 4, std=0.1, jitter=0.1)
    ref = orc.run_paths(cfg, named, PATHS5, LENS5, tokens=tok, targets=tgt)
    got = run(cfg, named, PATHS5, LENS5, tokens=tok, targets=tgt)
    check_f32(got, ref, "odd")


def test_grouping_does_not_change_the_result_f32():
    cfg = dict(SMALL, path_flags=sp.SP_SWAP_ANY_GAP)
    named, tok, tgt = inputs(cfg, 5, std=0.08)
    a = run(cfg, named, PATHS5, LENS5, tokens=tok, targets=tgt, whole_call=False)
    single = lambda plan: [(pos, st, [mb]) for pos, st, mbs in plan for mb in mbs]
    b = run(cfg, named, PATHS5, LENS5, tokens=tok, targets=tgt, whole_call=False, regroup=single)
    assert math.isclose(a["loss"], b["loss"], rel_tol=1e-6)
    assert np.array_equal(a["y"], b["y"])                # forward is row-wise: identical bits
    for k in a["grads"]:
        assert relerr(a["grads"][k], b["grads"][k]) < 1e-5, k


def test_skipped_slots_are_untouched_and_unvisited_stage_gets_zero():
    cfg = dict(SMALL)
    named, tok, tgt = inputs(cfg, 6)
    paths = np.array([[0, 1, 3, -1]] * 5, np.int32)
    lens = np.array([3] * 5, np.int32)
    got = run(cfg, named, paths, lens, tokens=tok, targets=tgt)
    ref = orc.run_paths(cfg, named, paths, lens, tokens=tok, targets=tgt)
    check_f32(got, ref, "skip stage 2")
    for name, g in got["grads"].items():
        if name.startswith("s2."):
            assert np.all(g == 0), name


def test_stage_share_f32():
    cfg = dict(SMALL, local_stage_begin=2, local_stage_count=1, has_embed=0, has_head=0)
    named = synth.make_params(cfg, 7, 0.1, 0.08)
    x = synth.make_activations(cfg, 7)
    dy = synth.make_upstream_grad(cfg, 7)
    ref = orc.run_paths(cfg, named, PATHS5, LENS5, x_in=x, dy_in=dy)
    got = run(dict(cfg, path_flags=sp.SP_SWAP_ANY_GAP), named, PATHS5, LENS5, x_in=x, dy_in=dy)
    assert relerr(got["y"], ref["y"]) < F32_TOL
    assert relerr(got["dx"], ref["dx"]) < F32_TOL
    # microbatch 1 never visits stage 2: its slots must be bit-identical to the inputs
    assert np.array_equal(got["y"][1], x[1]) and np.array_equal(got["dx"][1], dy[1])
    for name, g in ref["grads"].items():
        assert relerr(got["grads"][name], g) < F32_TOL, name


def test_all_targets_ignored_in_one_microbatch():
    cfg = dict(SMALL)
    named, tok, tgt = inputs(cfg, 8)
    tgt[2] = -1
    ref = orc.run_paths(cfg, named, PATHS5[:, :], LENS5, tokens=tok, targets=tgt) if False else \
        orc.run_paths(dict(cfg), named, np.array([[0, 1, 2, 3]] * 5, np.int32), np.array([4] * 5, np.int32),
                      tokens=tok, targets=tgt)
    got = run(cfg, named, np.array([[0, 1, 2, 3]] * 5, np.int32), np.array([4] * 5, np.int32), tokens=tok, targets=tgt)
    check_f32(got, ref, "ignored mb")
    assert got["loss_mb"][2] == 0.0


# ------------------------------------------------------------------ bfloat16 mode
def test_c1_full_shape_bf16():
    cfg = dict(synth.CONFIGS["c1"], dtype="bf16")
    named, tok, tgt = inputs(cfg, synth.BASE_SEED, bf16=True)
    paths, lens = synth.make_paths(cfg["n_stages"], cfg["n_mb"], *cfg["skip"], cfg["swap"], synth.BASE_SEED)
    ref = orc.run_paths(cfg, named, paths, lens, tokens=tok, targets=tgt, dtype=np.float32)
    got = run(cfg, named, paths, lens, tokens=tok, targets=tgt)
    check_bf16(got, ref, "c1 bf16")


def test_small_bf16_row_counts_that_fill_no_round():
    # 25 tokens per microbatch: groups of 25, 50 and 75 rows, none a multiple of the rows a workgroup of the
    # norm backward takes per round, nor of any tile height
    cfg = dict(SMALL, dtype="bf16", seq_len=25, seqs_per_mb=1)
    named, tok, tgt = inputs(cfg, 33, bf16=True)
    ref = orc.run_paths(cfg, named, PATHS5, LENS5, tokens=tok, targets=tgt, dtype=np.float32)
    got = run(cfg, named, PATHS5, LENS5, tokens=tok, targets=tgt)
    check_bf16(got, ref, "ragged rows bf16")


@pytest.mark.parametrize("vocab", [8200, 40000, 70000, 131080])
def test_head_and_loss_over_vocabulary_sizes_bf16(vocab):
    # the loss kernel holds a row of logits in the registers of 256, 512 or 1024 threads, by the row's length;
    # beyond 131072 entries it reads the row twice instead
    cfg = dict(SMALL, vocab=vocab, dtype="bf16", n_stages=2, local_stage_count=2, layers_per_stage=1, n_mb=2)
    named, tok, tgt = inputs(cfg, 21, bf16=True)
    tgt = np.array(tgt)
    tgt[0, 1, 5] = vocab - 1          # the last column, and the first, as targets
    tgt[1, 0, 7] = 0
    paths = np.array([[0, 1], [0, 1]], np.int32)
    lens = np.array([2, 2], np.int32)
    ref = orc.run_paths(cfg, named, paths, lens, tokens=tok, targets=tgt, dtype=np.float32)
    got = run(cfg, named, paths, lens, tokens=tok, targets=tgt)
    check_bf16(got, ref, f"vocab {vocab}")


@pytest.mark.parametrize("name,shape", [
    ("c2", dict(seq_len=256, seqs_per_mb=2, n_mb=4, layers_per_stage=1, vocab=4096)),
])
def test_c2_reduced_bf16(name, shape):
    # full model dimensions of the 500M shape (dim 1024, 16 heads of 64, hidden 2816), fewer tokens and layers
    cfg = synth.shrink(synth.CONFIGS[name], **shape)
    named, tok, tgt = inputs(cfg, 9, bf16=True)
    paths, lens = synth.make_paths(cfg["n_stages"], cfg["n_mb"], *cfg["skip"], cfg["swap"], 9)
    ref = orc.run_paths(cfg, named, paths, lens, tokens=tok, targets=tgt, dtype=np.float32)
    got = run(cfg, named, paths, lens, tokens=tok, targets=tgt)
    check_bf16(got, ref, "c2 reduced")


def test_c2_full_depth_and_vocabulary_bf16():
    # the 500M shape as configured: 6 stages x 4 layers, vocabulary 32000, 1/3 of the stages skipped, exchanges
    # allowed; only the token count is cut (4 microbatches x 2 sequences x 256) so the checker finishes in seconds
    cfg = synth.shrink(synth.CONFIGS["c2"], seq_len=256, seqs_per_mb=2, n_mb=4)
    assert cfg["layers_per_stage"] == 4 and cfg["vocab"] == 32000 and cfg["n_stages"] == 6
    named, tok, tgt = inputs(cfg, 14, bf16=True)
    paths, lens = sp.make_paths(cfg["n_stages"], cfg["n_mb"], *cfg["skip"], cfg["swap"], 14)
    assert any(list(paths[mb, :lens[mb]]) != sorted(paths[mb, :lens[mb]]) for mb in range(cfg["n_mb"])), paths
    ref = orc.run_paths(cfg, named, paths, lens, tokens=tok, targets=tgt, dtype=np.float32)
    got = run(cfg, named, paths, lens, tokens=tok, targets=tgt)
    check_bf16(got, ref, "c2 full depth")
    assert np.allclose(got["loss_mb"], ref["loss_mb"], rtol=BF16_LOSS_TOL)


@pytest.mark.parametrize("key", ["c3", "c5"])
def test_one_layer_full_width_full_sequence_bf16(key):
    # one decoder layer at the full width of the 1.5B / 8B stage (the 8B one with grouped kv heads and rotary
    # base 5e5) on one sequence of the full 4096 tokens, forward and backward through the stage entry points:
    # every position of the rotary table, every tile of the causal triangle, every gradient tensor, y and dx
    cfg = synth.shrink(synth.CONFIGS[key], n_mb=1, layers_per_stage=1, has_head=0, vocab=512)
    assert cfg["seq_len"] == 4096
    stage = cfg["local_stage_begin"]
    named = {k: round_bf16(v) for k, v in synth.make_params(cfg, 21).items()}
    x = round_bf16(synth.make_activations(cfg, 21))
    dy = round_bf16(synth.make_upstream_grad(cfg, 21))
    paths = np.full((1, cfg["n_stages"]), -1, np.int32); paths[0, :2] = (0, stage)
    lens = np.array([2], np.int32)
    ref = orc.run_paths(cfg, named, paths, lens, x_in=x, dy_in=dy, dtype=np.float32)
    got = run(cfg, named, paths, lens, x_in=x, dy_in=dy)
    for name in ("y", "dx"):
        assert cosine(got[name], ref[name]) >= BF16_COS, name
        assert relerr(got[name], ref[name]) < 2e-2, (name, relerr(got[name], ref[name]))
        assert maxerr(got[name], ref[name]) < BF16_MAX, (name, maxerr(got[name], ref[name]))
    # the late positions on their own: a rotation that went wrong beyond some position shows here
    late = slice(3 * cfg["seq_len"] // 4, None)
    assert cosine(got["dx"][0, late], ref["dx"][0, late]) >= BF16_COS
    assert cosine(got["y"][0, late] - x[0, late], ref["y"][0, late] - x[0, late]) >= BF16_COS
    check_bf16(got, ref, key + " one layer", has_loss=False)


@pytest.mark.parametrize("key,shape", [
    ("c3", dict(seq_len=384, n_mb=4, layers_per_stage=2)),
    ("c4", dict(seq_len=256, n_mb=4, layers_per_stage=1)),
])
def test_stage_share_reduced_bf16(key, shape):
    # full width of the 1.5B / 7B stage (dim, heads, hidden), fewer tokens; arrivals at several path positions
    cfg = synth.shrink(synth.CONFIGS[key], **shape)
    named = {k: round_bf16(v) for k, v in synth.make_params(cfg, 10).items()}
    x = round_bf16(synth.make_activations(cfg, 10))
    dy = round_bf16(synth.make_upstream_grad(cfg, 10))
    paths, lens = synth.make_paths(cfg["n_stages"], cfg["n_mb"], *cfg["skip"], cfg["swap"], 10)
    assert n_visits(cfg, paths, lens) >= 2
    ref = orc.run_paths(cfg, named, paths, lens, x_in=x, dy_in=dy, dtype=np.float32)
    got = run(cfg, named, paths, lens, x_in=x, dy_in=dy)
    assert cosine(got["y"], ref["y"]) >= BF16_COS
    assert relerr(got["y"], ref["y"]) < 2e-2
    assert cosine(got["dx"], ref["dx"]) >= BF16_COS
    check_bf16(got, ref, key, has_loss=False)


def test_c5_reduced_gqa_head_bf16():
    # 8B shape: dim 4096, 32 q heads / 8 kv heads, hidden 14336; one layer, short sequences, reduced vocabulary
    cfg = synth.shrink(synth.CONFIGS["c5"], seq_len=128, n_mb=6, layers_per_stage=1, vocab=8016)
    named = {k: round_bf16(v) for k, v in synth.make_params(cfg, 12).items()}
    x = round_bf16(synth.make_activations(cfg, 12))
    tok, tgt = synth.make_tokens(cfg, 12)
    paths, lens = synth.make_paths(cfg["n_stages"], cfg["n_mb"], *cfg["skip"], cfg["swap"], 12)
    ref = orc.run_paths(cfg, named, paths, lens, x_in=x, targets=tgt, dtype=np.float32)
    got = run(cfg, named, paths, lens, x_in=x, targets=tgt)
    check_bf16(got, ref, "c5")
    assert cosine(got["dx"], ref["dx"]) >= BF16_COS


# ------------------------------------------------------------------ error paths (host-side checks only)
def test_call_order_and_argument_errors():
    cfg = dict(SMALL)
    ctx = sp.Context(cfg, 5, 4)
    try:
        params = sp.pack_params(cfg, synth.make_params(cfg, 1))
        act = torch.zeros(5 * 48 * 64, device="cuda")
        grads = torch.zeros(params.numel(), device="cuda")
        with pytest.raises(sp.SpError) as e:
            ctx.stage_bwd(1, params, act, [0, 1], grads)
        assert e.value.code == -5
        with pytest.raises(sp.SpError) as e:
            ctx.stage_fwd(1, params, act, [0, 0])
        assert e.value.code == -1
        with pytest.raises(sp.SpError) as e:
            ctx.set_side_stream(3)
        assert e.value.code == -1
        with pytest.raises(sp.SpError):
            ctx.stage_fwd(7, params, act, [0])
        with pytest.raises(sp.SpError):
            ctx.stage_fwd(1, params, act, [5])
        ctx.stage_fwd(1, params, act, [0, 1])
        with pytest.raises(sp.SpError) as e:
            ctx.stage_bwd(1, params, act, [1, 0], grads)      # same set, different order
        assert e.value.code == -5
        for _ in range(2):
            ctx.stage_fwd(2, params, act, [2])
        with pytest.raises(sp.SpError) as e:                  # five visits alive, room for four
            ctx.stage_fwd(3, params, act, [3])
        assert e.value.code == -3
        ctx.reset()
        ctx.stage_fwd(3, params, act, [3])
        ctx.stage_bwd(3, params, act, [3], grads)
        torch.cuda.synchronize()
    finally:
        ctx.close()
    with pytest.raises(sp.SpError) as e:
        bad = np.array([[0, 2, 1, 3]] + [[0, 1, 2, 3]] * 4, np.int32)
        bad[0] = [1, 0, 2, 3]
        run(cfg, synth.make_params(cfg, 1), bad, np.array([4] * 5, np.int32), *synth.make_tokens(cfg, 1))
    assert e.value.code == -2


def test_out_of_range_token_ids_and_targets_are_reported_not_followed():
    # a token id outside the vocabulary would index outside the embedding (forward) and its gradient (backward),
    # a target outside it outside the logits: the kernels skip such rows and raise a flag the call returns
    cfg = dict(SMALL)
    named, tok, tgt = inputs(cfg, 15)
    full = np.array([[0, 1, 2, 3]] * 5, np.int32); lens = np.array([4] * 5, np.int32)
    clean = run(cfg, named, full, lens, tokens=tok, targets=tgt)
    for what in ("token", "negative token", "target", "target below -1"):
        t2, g2 = tok.copy(), tgt.copy()
        if what == "token":
            t2[1, 0, 3] = cfg["vocab"]
        elif what == "negative token":
            t2[4, 1, 0] = -1
        elif what == "target":
            g2[0, 1, 2] = cfg["vocab"] + 7
        else:
            g2[3, 0, 0] = -2
        with pytest.raises(sp.SpError) as e:
            run(cfg, named, full, lens, tokens=t2, targets=g2)
        assert e.value.code == -1 and "vocab" in str(e.value), what
    # the asynchronous entry points report through sp_input_status, and reading the flag clears it
    ctx = sp.Context(cfg, 5, 4)
    try:
        params = sp.pack_params(cfg, named)
        act = torch.zeros(5 * 48 * 64, device="cuda")
        bad = tok.copy(); bad[2, 1, 5] = 10 ** 6
        ctx.embed_fwd(params, torch.from_numpy(bad.reshape(-1)).cuda(), 5, act)
        with pytest.raises(sp.SpError) as e:
            ctx.input_status()
        assert e.value.code == -1
        ctx.input_status()
        row = (2 * 2 + 1) * 24 + 5
        assert float(act.view(-1, 64)[row].abs().max()) == 0.0       # the bad row was embedded as zeros
        assert float(act.view(-1, 64)[row - 1].abs().max()) > 0.0
        ctx.embed_fwd(params, torch.from_numpy(tok.reshape(-1)).cuda(), 5, act)
        ctx.input_status()
    finally:
        ctx.close()
    again = run(cfg, named, full, lens, tokens=tok, targets=tgt)       # a clean run afterwards is unaffected
    assert math.isclose(again["loss"], clean["loss"], rel_tol=1e-6)      # float atomics: the order of additions varies


def test_side_stream_changes_nothing_but_the_order_of_float_additions():
    # weight gradients beside the main chain or in line: same results up to the order of the atomic adds
    cfg = synth.shrink(synth.CONFIGS["c3"], seq_len=256, n_mb=4, layers_per_stage=3)
    paths, lens, stage = synth.stage_share_paths("c3")
    paths, lens = paths[:4], lens[:4]
    cfg["local_stage_begin"], cfg["local_stage_count"] = stage, 1
    named = {k: round_bf16(v) for k, v in synth.make_params(cfg, 12).items()}
    x = round_bf16(synth.make_activations(cfg, 12)); dy = round_bf16(synth.make_upstream_grad(cfg, 12))
    a = run(cfg, named, paths, lens, x_in=x, dy_in=dy, side_stream=2)
    b = run(cfg, named, paths, lens, x_in=x, dy_in=dy, side_stream=False)
    np.testing.assert_array_equal(a["dx"], b["dx"])
    for k in a["grads"]:
        assert relerr(a["grads"][k], b["grads"][k]) < 1e-5, k


def test_scheduled_paths_run_through_the_model():
    # the host scheduler's stage lists are paths like any other: C1's four stages on 6 emulated nodes
    cfg = synth.CONFIGS["c1"]
    node_stage = np.array([0, 0, 1, 2, 3, 3], np.int32)
    fwd = np.array([1.0, 1.2, 0.9, 1.1, 1.0, 0.8], np.float32)
    comm = np.full((6, 6), 0.3, np.float32); np.fill_diagonal(comm, 0); comm[0, 2] = comm[2, 0] = 2.5
    plan = sp.schedule_paths(node_stage, fwd, 2 * fwd, comm, [0, 1], [3, 3], mem_limit=1)
    paths, lens = plan["path_stages"], plan["len"]
    named, tok, tgt = inputs(cfg, synth.BASE_SEED)
    ref = orc.run_paths(cfg, named, paths, lens, tokens=tok, targets=tgt, dtype=np.float64)
    got = run(cfg, named, paths, lens, tokens=tok, targets=tgt)
    check_f32(got, ref, "scheduled paths")


def test_contexts_can_be_created_and_destroyed_repeatedly():
    # every context owns a workspace, a side stream and events: none of them may be left behind
    cfg = dict(SMALL, dtype="bf16")
    sp.Context(cfg, 2, 4).close()                 # first use loads code objects and the like
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    for _ in range(40):
        c = sp.Context(cfg, 2, 4)
        c.close()
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] >= free0 - (8 << 20)
