"""A LLaMa stack written with PyTorch CPU library routines and autograd.

Used only to pin the CPU checker: forward ops are library calls
(``scaled_dot_product_attention``, ``rms_norm``, ``silu``, ``cross_entropy``,
``embedding``, complex multiplication for the rotary embedding) and every
gradient comes from autograd, so it shares neither forward code nor backward
formulas with the checker.  A path is expressed here as "the ordinary model
built from the layers of the stages on the path, in that order".
"""
import torch
import torch.nn.functional as Fn


def _rope(x, T, theta):
    # x [B, T, nh, hd]
    hd = x.shape[-1]
    inv = theta ** (-torch.arange(0, hd, 2, dtype=x.dtype) / hd)
    ang = torch.arange(T, dtype=x.dtype)[:, None] * inv[None, :]
    rot = torch.polar(torch.ones_like(ang), ang)                 # e^{i*angle}
    xc = torch.view_as_complex(x.reshape(*x.shape[:-1], hd // 2, 2).contiguous())
    return torch.view_as_real(xc * rot[None, :, None, :]).reshape(x.shape)


def layer(cfg, p, pre, x, B):
    d, H, Hkv = cfg["dim"], cfg["n_heads"], cfg["n_kv_heads"]
    hd = d // H
    T = cfg["seq_len"]
    dkv = Hkv * hd
    xn = Fn.rms_norm(x, (d,), p[pre + "g1"], cfg["rms_eps"])
    qkv = xn @ p[pre + "wqkv"].T
    q = _rope(qkv[:, :d].reshape(B, T, H, hd), T, cfg["rope_theta"])
    k = _rope(qkv[:, d:d + dkv].reshape(B, T, Hkv, hd), T, cfg["rope_theta"])
    v = qkv[:, d + dkv:].reshape(B, T, Hkv, hd)
    rep = H // Hkv
    k = k.repeat_interleave(rep, dim=2)
    v = v.repeat_interleave(rep, dim=2)
    o = Fn.scaled_dot_product_attention(q.transpose(1, 2), k.transpose(1, 2), v.transpose(1, 2), is_causal=True)
    o = o.transpose(1, 2).reshape(B * T, d)
    h = x + o @ p[pre + "wo"].T
    hn = Fn.rms_norm(h, (d,), p[pre + "g2"], cfg["rms_eps"])
    gu = hn @ p[pre + "wgu"].T
    hh = cfg["hidden"]
    a = Fn.silu(gu[:, :hh]) * gu[:, hh:]
    return h + a @ p[pre + "wd"].T


def run(cfg, named, paths, lens, tokens=None, targets=None, x_in=None, dy_in=None, dtype=torch.float64):
    """Same contract as the checker's run_paths; returns loss, loss_mb, grads, y, dx."""
    p = {k: torch.tensor(v, dtype=dtype, requires_grad=True) for k, v in named.items()}
    n_mb = paths.shape[0]
    B, T, d = cfg["seqs_per_mb"], cfg["seq_len"], cfg["dim"]
    lo, hi = cfg["local_stage_begin"], cfg["local_stage_begin"] + cfg["local_stage_count"]
    total = 0.0
    loss_mb, ys, xs = [], [], []
    for mb in range(n_mb):
        if cfg["has_embed"]:
            x = Fn.embedding(torch.tensor(tokens[mb].reshape(-1), dtype=torch.long), p["embed"])
        else:
            x = torch.tensor(x_in[mb].reshape(B * T, d), dtype=dtype, requires_grad=True)
            xs.append(x)
        layers = [f"s{s}.l{l}." for s in paths[mb, :lens[mb]] if lo <= s < hi for l in range(cfg["layers_per_stage"])]
        for pre in layers:
            x = layer(cfg, p, pre, x, B)
        ys.append(x)
        if cfg["has_head"]:
            xn = Fn.rms_norm(x, (d,), p["gf"], cfg["rms_eps"])
            logits = xn @ p["whead"].T
            l = Fn.cross_entropy(logits, torch.tensor(targets[mb].reshape(-1), dtype=torch.long), ignore_index=-1)
            loss_mb.append(l)
            total = total + l / n_mb
        else:
            total = total + (x * torch.tensor(dy_in[mb].reshape(B * T, d), dtype=dtype)).sum()
    total.backward()
    grads = {k: (v.grad.numpy() if v.grad is not None else torch.zeros_like(v).numpy()) for k, v in p.items()}
    return dict(loss=float(total.detach()) if cfg["has_head"] else 0.0,
                loss_mb=[float(l.detach()) for l in loss_mb], grads=grads,
                y=torch.stack([y.detach() for y in ys]).numpy(),
                dx=None if cfg["has_embed"] else torch.stack([x.grad for x in xs]).numpy())


def eval_losses(cfg, named, paths, lens, tokens, targets, half=None, dtype=torch.float64):
    """Forward only: per-microbatch loss of the ordinary model built from the layers of the stages on the
    path, the stage half[mb] contributing only its first layers_per_stage // 2 layers."""
    p = {k: torch.tensor(v, dtype=dtype) for k, v in named.items()}
    B, T, d, Lps = cfg["seqs_per_mb"], cfg["seq_len"], cfg["dim"], cfg["layers_per_stage"]
    out = []
    for mb in range(paths.shape[0]):
        x = Fn.embedding(torch.tensor(tokens[mb].reshape(-1), dtype=torch.long), p["embed"])
        for s in paths[mb, :lens[mb]]:
            n = Lps // 2 if half is not None and half[mb] == s else Lps
            for l in range(n):
                x = layer(cfg, p, f"s{s}.l{l}.", x, B)
        xn = Fn.rms_norm(x, (d,), p["gf"], cfg["rms_eps"])
        out.append(float(Fn.cross_entropy(xn @ p["whead"].T, torch.tensor(targets[mb].reshape(-1), dtype=torch.long),
                                          ignore_index=-1)))
    return out
