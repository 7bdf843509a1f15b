"""The benchmark's own workload at full size, in the launch configuration bench.py times: sampled outputs
against the CPU checker (a sequence's first tokens do not depend on its later ones, so the checker runs the
same stage on the prefix alone), and properties that hold at any size (grouping, linearity of the backward
pass).  Plus causal attention at the full sequence length against the checker's attention."""
import os
import sys

import numpy as np
import pytest
import torch

from oracle import skippipe_oracle as orc
from paper_2502_19913_amd import binding as sp
from paper_2502_19913_amd import synth
from tests.gpuharness import cosine, relerr, round_bf16

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
import bench  # noqa: E402

pytestmark = pytest.mark.gpu


def _run(w, plan, dact0):
    w["plan"] = plan
    if dact0 is not None:
        w["dact0"] = dact0
    bench.step(w)
    torch.cuda.synchronize()
    return w["act"].clone(), w["dact"].clone(), w["grads"].clone()


@pytest.mark.parametrize("key", ["c3", "c4", "c5"])
def test_full_size_bench_configuration(key):
    # c3: 8 x 4096 tokens, 4 layers, groups 3/3/2.  c4: the 7B-shape stage with its routed microbatches (11 or 12
    # of 16) as one group.  c5: the 8B-shape stage (grouped kv heads) under its routed
    # microbatches, then final norm, head over 128256 tokens and loss on all 16
    w = bench.build_workload(key, torch, sp, synth)
    cfg = w["cfg"]
    try:
        plan = list(w["plan"])
        if key == "c3":
            assert [len(m) for _, _, m in plan] == [3, 3, 2]
        if key == "c4":
            assert len(plan) == 1 and len(plan[0][2]) >= 11
        routed = sorted(m for _, _, ms in plan for m in ms)
        y, dx, g = _run(w, plan, w.get("dact0"))
        # (1) sampled outputs: the first P tokens of three microbatches against the checker on those P tokens
        P, mbs = 160, [routed[0], routed[len(routed) // 2], routed[-1]]
        Nmb, d = cfg["seq_len"], cfg["dim"]
        small = synth.shrink(cfg, seq_len=P, n_mb=len(mbs), has_head=0)
        named = {k: v for k, v in sp.unpack(cfg, w["params"]).items() if k.startswith("s")}
        x0 = w["act0"].view(cfg["n_mb"], Nmb, d)[mbs, :P].float().cpu().numpy()
        paths = np.full((len(mbs), cfg["n_stages"]), -1, np.int32); paths[:, 0] = 0; paths[:, 1] = w["stage"]
        ref = orc.run_paths(small, named, paths, np.full(len(mbs), 2, np.int32), x_in=x0, dy_in=np.zeros_like(x0),
                            dtype=np.float32)
        got = y.view(cfg["n_mb"], Nmb, d)[mbs, :P].float().cpu().numpy()
        assert cosine(got, ref["y"]) >= 0.999 and relerr(got, ref["y"]) < 2e-2
        # (2) one microbatch per group instead of 3/3/2: same outputs, same gradients up to the order of additions
        singles = [(pos, st, [m]) for pos, st, ms in plan for m in ms]
        y1, dx1, g1 = _run(w, singles, w.get("dact0"))
        assert relerr(y1.float().cpu().numpy(), y.float().cpu().numpy()) < 1e-3
        assert relerr(dx1.float().cpu().numpy(), dx.float().cpu().numpy()) < 1e-3
        assert relerr(g1.cpu().numpy(), g.cpu().numpy()) < 1e-3
        # (3) the backward pass is linear in the gradient that arrives: twice the input, twice every gradient
        # (a factor of two is exact in bfloat16 and float, so only the order of the atomic additions differs)
        if key in ("c3", "c4"):
            y2, dx2, g2 = _run(w, plan, w["dact0"] * 2)
            assert relerr(dx2.float().cpu().numpy(), 2 * dx.float().cpu().numpy()) < 1e-5
            assert relerr(g2.cpu().numpy(), 2 * g.cpu().numpy()) < 1e-5
        else:
            # every microbatch reaches the head, routed or not.  Closed form for random weights: the final norm
            # gives rows of unit mean square, so a logit is N(0, dim * 0.02^2) and the expected loss of a
            # uniformly drawn target is log(vocab) + variance / 2
            want = np.log(cfg["vocab"]) + cfg["dim"] * 0.02 ** 2 / 2
            assert np.allclose(w["loss_mb"].cpu().numpy(), want, rtol=0.01)
        # nothing overflowed or vanished on the way
        assert torch.isfinite(g).all() and float(g.abs().max()) > 0
    finally:
        w["ctx"].close()


def test_attention_full_sequence_length_bf16():
    # one sequence of 4096 tokens, 2 query heads on 1 kv head, head dimension 128: every tile of the causal
    # triangle of the full-size kernels, at a cost the checker still finishes
    B, T, H, Hkv, hd = 1, 4096, 2, 1, 128
    nq = (H + 2 * Hkv) * hd
    qkv = round_bf16(synth.normal(31, "qkv_full", (B * T, nq)))
    do = round_bf16(synth.normal(32, "do_full", (B * T, H * hd)))
    q = np.ascontiguousarray(qkv[:, :H * hd]).reshape(B * T, H, hd).astype(np.float32)
    k = np.ascontiguousarray(qkv[:, H * hd:(H + Hkv) * hd]).reshape(B * T, Hkv, hd).astype(np.float32)
    v = np.ascontiguousarray(qkv[:, (H + Hkv) * hd:]).reshape(B * T, Hkv, hd).astype(np.float32)
    o_ref = orc.attention_fwd(q, k, v, B, T)
    dq, dk, dv = orc.attention_bwd(do.reshape(B * T, H, hd).astype(np.float32), q, k, v, B, T)
    dt = torch.bfloat16
    d_qkv = torch.from_numpy(qkv).cuda().to(dt)
    o = torch.empty((B * T, H * hd), dtype=dt, device="cuda")
    lse = torch.empty((B, H, T), dtype=torch.float32, device="cuda")
    sp.attention_fwd(d_qkv, o, lse, B, T, H, Hkv, hd)
    assert cosine(o.float().cpu().numpy().reshape(B * T, H, hd), o_ref) >= 0.999
    dqkv = torch.empty_like(d_qkv); delta = torch.empty(B * H * T, dtype=torch.float32, device="cuda")
    sp.attention_bwd(d_qkv, o, lse, torch.from_numpy(do).cuda().to(dt), dqkv, delta, B, T, H, Hkv, hd)
    got = dqkv.float().cpu().numpy()
    for name, ref, sl in (("dq", dq, slice(0, H * hd)), ("dk", dk, slice(H * hd, (H + Hkv) * hd)),
                          ("dv", dv, slice((H + Hkv) * hd, nq))):
        assert cosine(got[:, sl], ref.reshape(B * T, -1)) >= 0.999, name
        assert relerr(got[:, sl], ref.reshape(B * T, -1)) < 3e-2, name
