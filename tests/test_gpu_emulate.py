"""Several nodes on one GPU, one stream each: the scheduled iteration gives what the single-stream iteration
gives for the same stage paths (and what the CPU checker gives)."""
import numpy as np
import pytest
import torch

from oracle import skippipe_oracle as orc
from paper_2502_19913_amd import binding as sp
from paper_2502_19913_amd import synth
from paper_2502_19913_amd.emulate import NodeEmulator
from tests.gpuharness import relerr, round_bf16

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_emulated_nodes_match_single_stream_and_checker(dtype):
    cfg = dict(synth.CONFIGS["c1"], dim=64, n_heads=4, n_kv_heads=2, hidden=96, vocab=200, n_stages=4, layers_per_stage=2,
               seq_len=24, seqs_per_mb=2, n_mb=4, dtype=dtype)
    node_stage = np.array([0, 0, 1, 1, 2, 3, 3], np.int32)
    fwd = np.array([1.0, 1.1, 0.9, 1.3, 1.0, 0.8, 1.2], np.float32)
    comm = np.full((7, 7), 0.3, np.float32); np.fill_diagonal(comm, 0); comm[0, 2] = comm[2, 0] = 1.5
    plan = sp.schedule_paths(node_stage, fwd, 2 * fwd, comm, [0, 1, 0, 1], [3, 3, 3, 3], mem_limit=3, delta=0.05)
    named = synth.make_params(cfg, 5, std=0.08, gain_jitter=0.1)
    if dtype == "bf16":
        named = {k: round_bf16(v) for k, v in named.items()}
    tok, tgt = synth.make_tokens(cfg, 5)
    ref = orc.run_paths(cfg, named, plan["path_stages"], plan["len"], tokens=tok, targets=tgt,
                        dtype=np.float64 if dtype == "f32" else np.float32)
    params = sp.pack_params(cfg, named, "cuda")
    dtok = torch.from_numpy(tok.astype(np.int32).reshape(-1)).cuda(); dtgt = torch.from_numpy(tgt.astype(np.int32).reshape(-1)).cuda()
    em = NodeEmulator(cfg, node_stage, cfg["n_mb"])
    try:
        out = em.run(params, dtok, dtgt, plan["path_nodes"], plan["len"], plan["arrive"], fwd, 2 * fwd, comm)
    finally:
        em.close()
    grads = sp.unpack(cfg, out["grads"])
    tol = 1e-4 if dtype == "f32" else 2e-2
    assert abs(out["loss"] - ref["loss"]) < (1e-4 if dtype == "f32" else 1e-2) * abs(ref["loss"])
    for k, g in ref["grads"].items():
        assert relerr(grads[k], g) < tol or np.linalg.norm(g) == 0, (k, relerr(grads[k], g))
    # every node did the work the schedule gave it, and only that
    want = np.zeros(len(node_stage), int)
    for mb in range(cfg["n_mb"]):
        nodes = plan["path_nodes"][mb, :plan["len"][mb]]
        for j, nd in enumerate(nodes):
            want[nd] += 2 + (1 if j == 0 else 0)           # forward, backward, and the head on the start node
    assert out["n_ops"] == list(want)
    assert all(b > 0 for b, n in zip(out["busy_ms"], out["n_ops"]) if n) and out["wall_ms"] > 0
