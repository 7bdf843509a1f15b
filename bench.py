#!/usr/bin/env python3
"""Throughput of the path-routed stage forward+backward on one MI355X.

One step = one pass of the whole hot path over one batch of seeded synthetic input that is already
resident in HBM: every group of the route plan through the stage forward, (for the head-holding
workload) final norm + output head + loss, then every group through the stage backward, with the
gradient buffer cleared at the start of the step.  Prints one JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config c3|c2|c4|c5|c1] [--one-group]
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E, published
# HBM-side bytes per launch of the weight-gradient product at the default workload, from rocprofv3 --pmc
# FETCH_SIZE (x 1.998, the factor a plain copy of known size gives) + WRITE_SIZE (x 1.000); see
# profiles/c3_stage_counters_pmc.txt.  Valid for the kernel as it was when the counters were taken: set to None
# when k_gemm_mfma changes.
GEMM_TN_C3_TRAFFIC_BYTES = 599.1e6


def flops_per_token_layer(cfg):
    """Algorithmic forward flops of one decoder layer per token (causal attention counted on (T+1)/2 keys)."""
    d, h, T = cfg["dim"], cfg["hidden"], cfg["seq_len"]
    hd = d // cfg["n_heads"]
    nq = d + 2 * cfg["n_kv_heads"] * hd
    return 2 * d * nq + 2 * d * d + 6 * d * h + 2 * d * (T + 1)


def build_workload(key, torch, sp, synth):
    cfg = dict(synth.CONFIGS[key])
    dev = "cuda"
    dt = sp.torch_dtype(cfg)
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.BASE_SEED)
    n_mb, Nmb, d = cfg["n_mb"], cfg["seqs_per_mb"] * cfg["seq_len"], cfg["dim"]
    whole = bool(cfg["has_embed"] and cfg["has_head"])
    # paths come from the library's exported generator (sp_make_paths)
    if whole:
        paths, lens = sp.make_paths(cfg["n_stages"], n_mb, *cfg["skip"], bool(cfg["swap"]), synth.BASE_SEED)
        stage = None
    else:
        paths, lens, stage = synth.stage_share_paths(key, generator=sp.make_paths)
        cfg["local_stage_begin"], cfg["local_stage_count"] = stage, 1
    plan = sp.route_plan(cfg, paths, lens)
    visits = sum(len(m) for _, _, m in plan)
    # parameters: N(0, 0.02) matrices, unit gains, generated on the device in the layout's order
    params = torch.empty(sp.param_count(cfg), dtype=dt, device=dev)
    for name, _, _, off, rows, cols in sp.param_layout(cfg):
        v = params[off:off + rows * cols]
        if rows == 1:
            v.fill_(1.0)
        else:
            step = 1 << 26
            for lo in range(0, rows * cols, step):
                hi = min(rows * cols, lo + step)
                v[lo:hi] = (torch.randn(hi - lo, generator=gen, device=dev, dtype=torch.float32) * 0.02).to(dt)
    grads = torch.zeros(params.numel(), dtype=torch.float32, device=dev)
    w = dict(cfg=cfg, key=key, paths=paths, lens=lens, plan=plan, visits=visits, params=params, grads=grads,
             whole=whole, stage=stage)
    if whole:
        tok, tgt = synth.make_tokens(cfg, synth.BASE_SEED)
        w["tok"] = torch.from_numpy(tok.reshape(-1)).to(dev)
        w["tgt"] = torch.from_numpy(tgt.reshape(-1)).to(dev)
    else:
        w["act0"] = torch.randn(n_mb * Nmb * d, generator=gen, device=dev, dtype=torch.float32).to(dt)
        w["act"] = torch.empty_like(w["act0"])
        w["dact"] = torch.empty_like(w["act0"])
        if cfg["has_head"]:
            tok, tgt = synth.make_tokens(cfg, synth.BASE_SEED)
            w["tgt"] = torch.from_numpy(tgt.reshape(-1)).to(dev)
            w["loss_mb"] = torch.empty(n_mb, dtype=torch.float32, device=dev)
        else:
            w["dact0"] = (torch.randn(n_mb * Nmb * d, generator=gen, device=dev, dtype=torch.float32)
                          / float(Nmb * n_mb)).to(dt)
    w["ctx"] = sp.Context(cfg, n_mb, max(1, visits))
    # algorithmic work of one step
    per_tl = flops_per_token_layer(cfg)
    fl = 3.0 * per_tl * cfg["layers_per_stage"] * visits * Nmb
    if cfg["has_head"]:
        fl += 3.0 * 2 * d * cfg["vocab"] * n_mb * Nmb
    w["flops"] = fl
    w["tokens_presented"] = n_mb * Nmb
    w["stage_tokens"] = visits * Nmb
    return w


def step(w):
    ctx, cfg = w["ctx"], w["cfg"]
    if w["whole"]:
        loss, _ = ctx.run_paths(w["params"], w["tok"], w["tgt"], w["paths"], w["lens"], w["grads"])
        return loss
    w["grads"].zero_()
    w["act"].copy_(w["act0"])
    for _, st, mbs in w["plan"]:
        ctx.stage_fwd(st, w["params"], w["act"], mbs)
    if cfg["has_head"]:
        ctx.head_fwd_bwd(w["params"], w["act"], w["tgt"], cfg["n_mb"], w["loss_mb"], w["dact"], w["grads"])
    else:
        w["dact"].copy_(w["dact0"])
    for _, st, mbs in reversed(w["plan"]):
        ctx.stage_bwd(st, w["params"], w["dact"], mbs, w["grads"])
    return None


def optimizer_step(w, torch, sp, iters=5):
    """The clip + AdamW update over this workload's parameters (not part of `value`): HBM-bound, 34 bytes
    per parameter (gradient read twice, m, v and the float master read and written, bf16 copy written)."""
    n = w["params"].numel()
    master = w["params"].float()
    m = torch.zeros_like(master); v = torch.zeros_like(master)
    ws = torch.empty(sp.optim_workspace_bytes(), dtype=torch.uint8, device=master.device)
    out = w["params"] if w["params"].dtype == torch.bfloat16 else None
    f = lambda t: sp.optim_step(master, w["grads"], m, v, t, params_out=out, workspace=ws)
    f(1)
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for t in range(2, 2 + iters):
        f(t)
    e1.record(); torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / iters
    nbytes = n * (32 + (2 if out is not None else 0))
    return dict(ms=round(ms, 3), params=n, bytes_per_param=nbytes // n, achieved_gbs=round(nbytes / ms / 1e6, 1),
                peak_gbs=8000.0, frac=round(nbytes / ms / 1e6 / 8000.0, 4))


def eval_mode(args, w, torch, sp, synth):
    """Forward-only evaluation under stage drops (the fault-tolerant inference setting): one JSON line."""
    cfg = w["cfg"]
    if not w["whole"]:
        print("--eval-skip needs a whole-model workload (c1 or c2)", file=sys.stderr)
        sys.exit(2)
    num, den = (int(x) for x in args.eval_skip.split("/"))
    paths, lens, half = synth.make_eval_paths(cfg["n_stages"], cfg["n_mb"], num, den, synth.BASE_SEED)
    ctx, Nmb = w["ctx"], cfg["seqs_per_mb"] * cfg["seq_len"]
    run = lambda: ctx.eval_paths(w["params"], w["tok"], w["tgt"], paths, lens, half)
    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        loss, _ = run()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / args.steps
    Lps = cfg["layers_per_stage"]
    layers = sum(int(lens[mb]) * Lps - (Lps - Lps // 2 if half[mb] >= 0 else 0) for mb in range(cfg["n_mb"]))
    fl = flops_per_token_layer(cfg) * layers * Nmb + 2.0 * cfg["dim"] * cfg["vocab"] * cfg["n_mb"] * Nmb
    out = {"metric": "forward-only evaluation tokens/sec under per-sample stage drops on 1 MI355X",
           "value": round(cfg["n_mb"] * Nmb / sec, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": round(sec * 1e3, 3), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "bf16" if cfg["dtype"] == "bf16" else "f32",
           "data": "synthetic (seeded): N(0,0.02) weights, uniform tokens, seeded drops",
           "config": {"workload": f"{args.config} whole model, forward only, {args.eval_skip} of the stages dropped per "
                                  f"sample", "id": args.config, "n_mb": cfg["n_mb"], "tokens_per_mb": Nmb,
                      "layers_run": layers, "half_stages": int((half >= 0).sum())},
           "tflops": round(fl / sec / 1e12, 1), "frac_bf16_mfma_peak": round(fl / sec / 1e12 / PEAK_BF16_TFLOPS, 4),
           "loss": round(loss, 4)}
    ctx.close()
    print(json.dumps(out))


def emulate_mode(args, w, torch, sp, synth):
    """Scheduler + one stream per emulated node against the same paths on one stream: one JSON line."""
    import numpy as np
    from paper_2502_19913_amd.emulate import NodeEmulator
    cfg = w["cfg"]
    if not w["whole"]:
        print("--emulate-nodes needs a whole-model workload (c1 or c2)", file=sys.stderr)
        sys.exit(2)
    s, n_mb = cfg["n_stages"], cfg["n_mb"]
    num, den = cfg["skip"]
    # node distribution rule (Eq. 1) over the paper's node counts: 20 nodes for six stages, 18 for four
    sizes = sp.stage_sizes(20 if s >= 6 else (18 if s >= 4 else 3 * s), s, num, den)
    first, later = sizes[0], sizes[1] if s > 1 else 0
    node_stage = np.array([st for st, n in enumerate(sizes) for _ in range(n)], np.int32)
    N = len(node_stage)
    fwd = np.ones(N, np.float32)
    comm = np.full((N, N), 0.2, np.float32); np.fill_diagonal(comm, 0)
    keep = [s - (s * num) // den] * n_mb
    t0 = time.perf_counter()
    plan = sp.schedule_paths(node_stage, fwd, 2 * fwd, comm, [a % first for a in range(n_mb)], keep,
                             mem_limit=max(2, n_mb // later + 1), delta=0.05)
    sched_s = time.perf_counter() - t0
    em = NodeEmulator(cfg, node_stage, n_mb)
    run = lambda: em.run(w["params"], w["tok"], w["tgt"], plan["path_nodes"], plan["len"], plan["arrive"], fwd, 2 * fwd, comm)
    for _ in range(args.warmup):
        run()
    walls, busy = [], None
    for _ in range(args.steps):
        r = run(); walls.append(r["wall_ms"]); busy = r["busy_ms"]
    em.close()
    # the same stage paths on the one stream
    ctx = w["ctx"]
    one = lambda: ctx.run_paths(w["params"], w["tok"], w["tgt"], plan["path_stages"], plan["len"], w["grads"])
    for _ in range(args.warmup):
        one()
    torch.cuda.synchronize(); t0 = time.perf_counter()
    for _ in range(args.steps):
        loss, _ = one()
    torch.cuda.synchronize(); single_ms = (time.perf_counter() - t0) / args.steps * 1e3
    wall = float(np.median(walls)); Nmb = cfg["seqs_per_mb"] * cfg["seq_len"]
    out = {"metric": "tokens/sec of one iteration over emulated pipeline nodes (one stream per node) on 1 MI355X",
           "value": round(n_mb * Nmb / wall * 1e3, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": round(wall, 3), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "bf16" if cfg["dtype"] == "bf16" else "f32",
           "data": "synthetic (seeded): N(0,0.02) weights, uniform tokens; unit node times, 0.2 per transfer",
           "config": {"workload": f"{args.config} whole model over {N} emulated nodes (stage sizes {first}+{later}x{s - 1}), "
                                  f"{n_mb} microbatches scheduled by sp_schedule_paths", "id": args.config,
                      "n_mb": n_mb, "tokens_per_mb": Nmb, "nodes": N},
           "ms_per_step_one_stream_grouped": round(single_ms, 3), "scheduler_seconds": round(sched_s, 4),
           "planned_max_latency": round(plan["max_e2e"], 3),
           "node_busy_fraction": [round(b / wall, 3) for b in busy], "loss": round(loss, 4)}
    ctx.close()
    print(json.dumps(out))


def cpu_baseline(key, synth, full=False):
    """The CPU checker timed on a bounded sample of the same workload (float32 instantiation); full: on the
    whole workload instead (minutes to hours on the larger shapes)."""
    import numpy as np
    from oracle import skippipe_oracle as orc
    whole_shape = full
    full = synth.CONFIGS[key]
    lib = orc.lib()
    try:
        cores = int(ctypes.CDLL("libgomp.so.1").omp_get_max_threads())
    except Exception:
        cores = os.cpu_count() or 1
    if full["has_embed"] and full["has_head"]:
        # whole small model: keep widths and depth, cut tokens
        T = min(full["seq_len"], 128 if full["dim"] > 512 else full["seq_len"])
        cfg = synth.shrink(full, seq_len=T, seqs_per_mb=1, n_mb=min(2, full["n_mb"]),
                           vocab=min(full["vocab"], 4096))
        if whole_shape:
            cfg, T = dict(full), full["seq_len"] * full["seqs_per_mb"]
        paths, lens = synth.make_paths(cfg["n_stages"], cfg["n_mb"], *cfg["skip"], bool(cfg["swap"]), synth.BASE_SEED)
        named = synth.make_params(cfg, synth.BASE_SEED)
        tok, tgt = synth.make_tokens(cfg, synth.BASE_SEED)
        t0 = time.perf_counter()
        orc.run_paths(cfg, named, paths, lens, tokens=tok, targets=tgt, dtype=np.float32)
        dt = time.perf_counter() - t0
        toks = cfg["n_mb"] * T
        sample = (f"{cfg['n_mb']} microbatches x {T} tokens through the whole {full['n_stages']}-stage model "
                  f"(full widths, vocab {cfg['vocab']}), fwd+bwd+loss")
        if whole_shape:
            sample = "the whole workload"
    else:
        T = 2048 if full["dim"] <= 2048 else 512
        cfg = synth.shrink(full, seq_len=T, seqs_per_mb=1, n_mb=1, has_head=0, vocab=1024)
        _, _, stage = synth.stage_share_paths(key)
        cfg["local_stage_begin"], cfg["local_stage_count"] = stage, 1
        paths = np.full((1, cfg["n_stages"]), -1, np.int32)
        paths[0, :2] = (0, stage)
        lens = np.array([2], np.int32)
        if whole_shape:    # every routed microbatch at full length through the stage (the head, if any, left out)
            T = full["seq_len"]
            all_paths, all_lens, stage = synth.stage_share_paths(key)
            routed = [mb for mb in range(full["n_mb"]) if stage in all_paths[mb, :all_lens[mb]]]
            cfg = synth.shrink(full, n_mb=len(routed), has_head=0, vocab=1024)
            cfg["local_stage_begin"], cfg["local_stage_count"] = stage, 1
            paths = np.full((len(routed), cfg["n_stages"]), -1, np.int32)
            paths[:, 0] = 0; paths[:, 1] = stage
            lens = np.full(len(routed), 2, np.int32)
        named = synth.make_params(cfg, synth.BASE_SEED)
        x = synth.make_activations(cfg, synth.BASE_SEED)
        dy = synth.make_upstream_grad(cfg, synth.BASE_SEED)
        t0 = time.perf_counter()
        orc.run_paths(cfg, named, paths, lens, x_in=x, dy_in=dy, dtype=np.float32)
        dt = time.perf_counter() - t0
        toks = T * cfg["n_mb"]
        sample = (f"{cfg['n_mb']} microbatch(es) x {T} tokens through the {cfg['layers_per_stage']}-layer stage (full "
                  f"widths), fwd+bwd, no head")
    return dict(value=toks / dt, unit="tokens/s (of the sample named in `sample`)", cores=cores, kind="oracle",
                sample=sample, seconds=round(dt, 2))


def probe_mfma(torch, sp):
    """Matrix cores alone (sp_probe_mfma_rate), 8 waves on each of the 256 CUs, about 10 ms per launch."""
    g = torch.Generator(device="cuda").manual_seed(7)
    srcs = {"zeros": torch.zeros(1 << 22, dtype=torch.bfloat16, device="cuda"),
            "ones": torch.ones(1 << 22, dtype=torch.bfloat16, device="cuda"),
            "normal": torch.randn(1 << 22, dtype=torch.float32, device="cuda", generator=g).to(torch.bfloat16)}
    sink = torch.empty(256 * 512, dtype=torch.float32, device="cuda")
    out = {}
    for name, src in srcs.items():
        iters = 10000
        for _ in range(2):
            sp.probe_mfma_rate(src, 256, iters, sink)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 10
        a.record()
        for _ in range(reps):
            fl = sp.probe_mfma_rate(src, 256, iters, sink)
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / reps
        tf = fl / (ms * 1e-3) / 1e12
        # 1024 SIMDs x 1024 flops per cycle each at the rate of one 16x16x32 product per 16 cycles
        out[name] = dict(ms_per_launch=round(ms, 3), tflops=round(tf, 1), frac_peak=round(tf / PEAK_BF16_TFLOPS, 4),
                         implied_clock_ghz=round(tf * 1e12 / (1024 * 1024.0) / 1e9, 3))
    print(json.dumps(dict(metric="mfma_only_rate", unit="TFLOP/s", peak=PEAK_BF16_TFLOPS, blocks=256,
                          waves_per_block=8, operands=out)))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="c3", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--oracle-full", action="store_true",
                    help="time the CPU checker on the whole workload instead of the bounded sample (c1: seconds; c2 "
                         "and c3: minutes; c4 and c5: hours)")
    ap.add_argument("--eval-skip", default=None, metavar="NUM/DEN",
                    help="whole-model workloads (c1, c2): time forward-only evaluation with this share of the "
                         "stages dropped per sample (a half stage where the count ends in .5) instead of training")
    ap.add_argument("--serial", action="store_true",
                    help="keep the weight-gradient products in line on the one stream (no side stream) for the "
                         "whole run; by default only the per-launch timing pass runs that way")
    ap.add_argument("--side-always", action="store_true",
                    help="weight-gradient products on the side stream for every group (by default only for groups "
                         "whose products are short enough to gain from it)")
    ap.add_argument("--emulate-nodes", action="store_true",
                    help="whole-model workloads (c1, c2): schedule the microbatches over emulated nodes (stage sizes "
                         "by the paper's node-distribution rule) and run them one stream per node")
    ap.add_argument("--one-group", action="store_true",
                    help="stage-share workloads: all routed microbatches as one group (upper bound of the rate)")
    ap.add_argument("--probe-mfma", action="store_true",
                    help="instead of a workload: the rate the matrix cores sustain on a registers-only loop of the "
                         "product kernel's k-step, for zero, constant and random operands (one JSON line)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the library has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2502_19913_amd import binding as sp
    from paper_2502_19913_amd import synth
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    if args.probe_mfma:
        return probe_mfma(torch, sp)
    w = build_workload(args.config, torch, sp, synth)
    if args.eval_skip:
        return eval_mode(args, w, torch, sp, synth)
    if args.emulate_nodes:
        return emulate_mode(args, w, torch, sp, synth)
    if args.one_group and not w["whole"]:
        mbs = sorted(m for _, _, g in w["plan"] for m in g)
        w["plan"] = [(w["plan"][0][0], w["stage"], mbs)]
    w["ctx"].set_side_stream(0 if args.serial else 2 if args.side_always else 1)
    for _ in range(args.warmup):
        step(w)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(w)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    sec = (t1 - t0) / args.steps

    # second pass of the same steps with HIP events around every matrix-product and attention launch, all on
    # the one stream: a launch's duration is then its own, not that of two kernels sharing the GPU
    w["ctx"].set_side_stream(False)
    sp.prof_begin()
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for _ in range(args.steps):
        step(w)
    torch.cuda.synchronize()
    sec_serial = (time.perf_counter() - t2) / args.steps
    prof = sp.prof_end()
    gemm_cls = [k for k in ("gemm_nt", "gemm_nn", "gemm_tn") if prof[k]["launches"]]
    roof = None
    if gemm_cls:
        dom = max(gemm_cls, key=lambda k: prof[k]["ms"])
        p = prof[dom]
        achieved = p["flops"] / (p["ms"] * 1e-3) / 1e12
        roof = dict(bound="mfma", kernel={"gemm_nt": "k_gemm_mfma<0>", "gemm_nn": "k_gemm_mfma<1>",
                                          "gemm_tn": "k_gemm_mfma<2>"}[dom],
                    achieved=round(achieved, 1), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                    frac=round(achieved / PEAK_BF16_TFLOPS, 4),
                    traffic=(GEMM_TN_C3_TRAFFIC_BYTES if dom == "gemm_tn" and args.config == "c3" and not args.one_group
                             else None),
                    avg_launch_ms=round(p["ms"] / p["launches"], 4), launches_per_step=p["launches"] // args.steps,
                    share_of_step=round(p["ms"] / args.steps / (sec * 1e3), 3))
    kernels = {}
    for k, v in prof.items():
        if not v["launches"]:
            continue
        e = dict(ms_per_step=round(v["ms"] / args.steps, 3), launches_per_step=v["launches"] // args.steps)
        if k in sp.PROF_BYTES_CLASSES:     # bandwidth-bound: algorithmic bytes against the HBM peak
            gbs = v["flops"] / (v["ms"] * 1e-3) / 1e9 if v["ms"] > 0 else 0.0
            e.update(algorithmic_gbs=round(gbs, 1), frac_hbm_peak=round(gbs / PEAK_HBM_GBS, 4))
        else:
            e["tflops"] = round(v["flops"] / (v["ms"] * 1e-3) / 1e12, 1) if v["ms"] > 0 else None
        kernels[k] = e

    cfg = w["cfg"]
    tflops = w["flops"] / sec / 1e12
    out = {
        "metric": "path-routed stage fwd+bwd tokens/sec on 1 MI355X; % bf16 MFMA peak",
        "value": round(w["tokens_presented"] / sec, 1),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 3),
        "ms_per_step_one_stream_timed_launches": round(sec_serial * 1e3, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg["dtype"] == "bf16" else "f32",
        "data": "synthetic (seeded): N(0,0.02) weights, N(0,1) activations or uniform tokens, seeded paths",
        "config": {"workload": {
            "c1": "50M-shape whole model, 4 stages x 3 layers, 2 microbatches x 64 tokens, keep 3 of 4 stages",
            "c2": "500M-shape whole model, 6 stages x 4 layers, 8 microbatches x 4 x 1024 tokens, 1/3 skip with swaps",
            "c3": "1.5B-shape single stage of 4 layers (dim 2048, 16 heads, hidden 5632), 8 microbatches x 4096 tokens "
                  "arriving at path positions 1/2/3 in groups of 3/3/2, stage fwd+bwd only",
            "c4": "LLaMa-2-7B-shape single stage of 4 layers, 16 microbatches x 4096 tokens under 25% skip",
            "c5": "LLaMa-3-8B-shape single stage of 4 layers (GQA) + final norm + LM head + CE, 16 microbatches x 4096 "
                  "tokens under 1/3 skip with swaps",
        }[args.config], "id": args.config, "n_mb": cfg["n_mb"], "tokens_per_mb": cfg["seqs_per_mb"] * cfg["seq_len"],
            "stage_visits": w["visits"], "groups": [len(m) for _, _, m in w["plan"]],
            "one_group": bool(args.one_group)},
        "stage_tokens_per_s": round(w["stage_tokens"] / sec, 1),
        "tflops": round(tflops, 1),
        "frac_bf16_mfma_peak": round(tflops / PEAK_BF16_TFLOPS, 4),
        "roofline": roof,
        "kernels": kernels,
    }
    out["optimizer_step"] = optimizer_step(w, torch, sp)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.config, synth, full=args.oracle_full)
    w["ctx"].close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
