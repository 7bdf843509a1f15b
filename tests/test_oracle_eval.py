"""Pins of the forward-only evaluation under stage drops (section "Fault Tolerant Inference"), CPU only."""
import math

import numpy as np

from oracle import skippipe_oracle as orc
from paper_2502_19913_amd import synth
from tests import libmodel

CFG = dict(synth.CONFIGS["c1"], dim=48, n_heads=4, n_kv_heads=2, hidden=80, vocab=97, n_stages=4, layers_per_stage=4,
           seq_len=12, seqs_per_mb=2, n_mb=5)
PATHS = np.array([[0, 1, 2, 3], [0, 2, 3, -1], [0, 1, -1, -1], [0, 3, -1, -1], [0, 1, 3, -1]], np.int32)
LENS = np.array([4, 3, 2, 2, 3], np.int32)
HALF = np.array([-1, 2, 1, -1, 3], np.int32)     # the stage of the path that runs only its first half


def _inputs(seed=4):
    named = synth.make_params(CFG, seed, std=0.08, gain_jitter=0.1)
    tok, tgt = synth.make_tokens(CFG, seed)
    tgt[2, 0, :3] = -1
    return named, tok, tgt


def test_against_library_model_with_truncated_stage():
    named, tok, tgt = _inputs()
    got = orc.eval_paths(CFG, named, PATHS, LENS, tokens=tok, targets=tgt, half=HALF)
    ref = libmodel.eval_losses(CFG, named, PATHS, LENS, tok, tgt, HALF)
    np.testing.assert_allclose(got["loss_mb"], ref, rtol=1e-10)
    assert abs(got["loss"] - np.mean(ref)) < 1e-10


def test_no_half_stage_equals_the_training_forward():
    named, tok, tgt = _inputs(6)
    a = orc.eval_paths(CFG, named, PATHS, LENS, tokens=tok, targets=tgt, half=None)
    b = orc.run_paths(dict(CFG, path_flags=0), named, PATHS, LENS, tokens=tok, targets=tgt)
    np.testing.assert_allclose(a["loss_mb"], b["loss_mb"], rtol=1e-12)


def test_half_of_a_stage_is_its_first_layers_only():
    # re-cut the same layers into stages of 2: stage 0 becomes stages (0, 1), and the first half of stage 2 is
    # a whole stage of the re-cut model; the path (0, half of 2) must equal the re-cut path (0, 1, 2)
    named, tok, tgt = _inputs(7)
    paths = np.array([[0, 2, -1, -1]], np.int32); lens = np.array([2], np.int32)
    a = orc.eval_paths(CFG, named, paths, lens, tokens=tok[:1], targets=tgt[:1], half=np.array([2], np.int32))
    small = dict(CFG, layers_per_stage=2)
    src = {"s0.l0.": "s0.l0.", "s0.l1.": "s0.l1.", "s1.l0.": "s0.l2.", "s1.l1.": "s0.l3.",
           "s2.l0.": "s2.l0.", "s2.l1.": "s2.l1.", "s3.l0.": "s3.l0.", "s3.l1.": "s3.l1."}
    named2 = {k: v for k, v in named.items() if not k.startswith("s")}
    for dst, frm in src.items():
        for k, v in named.items():
            if k.startswith(frm):
                named2[dst + k[len(frm):]] = v
    b = orc.eval_paths(small, named2, np.array([[0, 1, 2, -1]], np.int32), np.array([3], np.int32),
                       tokens=tok[:1], targets=tgt[:1], half=None)
    np.testing.assert_allclose(a["loss_mb"], b["loss_mb"], rtol=1e-12)


def test_untrained_model_has_perplexity_near_vocab():
    # closed form: with tiny weights the logits vanish and the loss is log(vocab), whatever the path
    named = synth.make_params(CFG, 8, std=1e-4, gain_jitter=0.0)
    _, tok, tgt = _inputs(8)
    r = orc.eval_paths(CFG, named, PATHS, LENS, tokens=tok, targets=tgt, half=HALF)
    assert abs(math.exp(r["loss"]) - CFG["vocab"]) < 0.01 * CFG["vocab"]
