"""Drives the GPU library through its C boundary for the parity tests (argument marshalling only)."""
import numpy as np
import torch

from paper_2502_19913_amd import binding as sp


def round_bf16(a: np.ndarray) -> np.ndarray:
    """The caller-side rounding of float master values to bfloat16, widened back to float32."""
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(torch.bfloat16).float().numpy()


def n_visits(cfg, paths, lens):
    lo, hi = cfg["local_stage_begin"], cfg["local_stage_begin"] + cfg["local_stage_count"]
    return int(sum(1 for mb in range(len(lens)) for s in paths[mb, :lens[mb]] if lo <= s < hi))


def run(cfg, named, paths, lens, tokens=None, targets=None, x_in=None, dy_in=None, whole_call=True, regroup=None,
        side_stream=True):
    """Same contract as the CPU checker's run_paths.  whole_call: use sp_run_paths when the node holds the
    whole model; otherwise (or for stage shares) walk the route plan through the stage entry points.
    regroup: optional function plan -> plan (e.g. split every group into single microbatches).
    side_stream: weight-gradient products beside the main chain (the default) or in line."""
    dev = "cuda"
    dt = sp.torch_dtype(cfg)
    n_mb = len(lens)
    R = cfg["seqs_per_mb"] * cfg["seq_len"]
    d = cfg["dim"]
    params = sp.pack_params(cfg, named, dev)
    grads = torch.zeros(params.numel(), dtype=torch.float32, device=dev)
    whole = cfg["has_embed"] and cfg["has_head"] and cfg["local_stage_count"] == cfg["n_stages"]
    ctx = sp.Context(cfg, n_mb, max(1, n_visits(cfg, paths, lens)))
    ctx.set_side_stream(side_stream)
    out = {}
    try:
        tok = None if tokens is None else torch.from_numpy(np.ascontiguousarray(tokens, np.int32).reshape(-1)).to(dev)
        tgt = None if targets is None else torch.from_numpy(np.ascontiguousarray(targets, np.int32).reshape(-1)).to(dev)
        if whole and whole_call and regroup is None:
            loss, loss_mb = ctx.run_paths(params, tok, tgt, paths, lens, grads)
            out.update(loss=loss, loss_mb=loss_mb, y=None, dx=None)
        else:
            plan = sp.route_plan(cfg, paths, lens)
            if regroup is not None:
                plan = regroup(plan)
            if cfg["has_embed"]:
                act = torch.empty(n_mb * R * d, dtype=dt, device=dev)
                ctx.embed_fwd(params, tok, n_mb, act)
            else:
                act = torch.from_numpy(np.ascontiguousarray(x_in, np.float32).reshape(-1)).to(dev).to(dt)
            for pos, st, mbs in plan:
                ctx.stage_fwd(st, params, act, mbs)
            out["y"] = act.float().cpu().numpy().reshape(n_mb, R, d)
            if cfg["has_head"]:
                dact = torch.empty(n_mb * R * d, dtype=dt, device=dev)
                loss_mb = torch.empty(n_mb, dtype=torch.float32, device=dev)
                ctx.head_fwd_bwd(params, act, tgt, n_mb, loss_mb, dact, grads)
                out["loss_mb"] = loss_mb.cpu().numpy()
                out["loss"] = float(out["loss_mb"].astype(np.float64).mean())
            else:
                dact = torch.from_numpy(np.ascontiguousarray(dy_in, np.float32).reshape(-1)).to(dev).to(dt)
                out["loss"], out["loss_mb"] = 0.0, np.zeros(n_mb, np.float32)
            for pos, st, mbs in reversed(plan):
                ctx.stage_bwd(st, params, dact, mbs, grads)
            if cfg["has_embed"]:
                ctx.embed_bwd(tok, dact, n_mb, grads)
            out["dx"] = dact.float().cpu().numpy().reshape(n_mb, R, d)
        torch.cuda.synchronize()
        out["grads"] = sp.unpack(cfg, grads)
    finally:
        ctx.close()
    return out


def relerr(a, b):
    a = np.asarray(a, np.float64); b = np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def cosine(a, b):
    a = np.asarray(a, np.float64).ravel(); b = np.asarray(b, np.float64).ravel()
    na, nb = np.linalg.norm(a), np.linalg.norm(b)
    if na == 0 and nb == 0:
        return 1.0
    return float(a @ b / max(na * nb, 1e-300))


def maxerr(a, b):
    """Largest element-wise difference relative to the largest reference magnitude: max|a - b| / max|b|."""
    a = np.asarray(a, np.float64); b = np.asarray(b, np.float64)
    return float(np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300))
