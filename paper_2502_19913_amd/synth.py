"""Seeded synthetic inputs: tokens, weights, activations and microbatch paths.

Everything here is index bookkeeping and random numbers.  None of the model's
arithmetic lives in this module; the CPU checker and the GPU library are both
handed the arrays made here and neither of them imports it.

Random numbers come from a counter-based generator: element ``i`` of the tensor
named ``name`` under ``seed`` is a fixed function of ``(seed, name, i)``, so any
slice can be regenerated anywhere without state.
"""
from __future__ import annotations

import zlib
from typing import Dict, List, Sequence, Tuple

import numpy as np

BASE_SEED = 20250219

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _mix64(z: np.ndarray) -> np.ndarray:
    """64-bit finaliser (the splitmix64 output function) applied elementwise."""
    z = z.astype(np.uint64, copy=True)
    with np.errstate(over="ignore"):
        z ^= z >> np.uint64(30)
        z *= np.uint64(0xBF58476D1CE4E5B9)
        z ^= z >> np.uint64(27)
        z *= np.uint64(0x94D049BB133111EB)
        z ^= z >> np.uint64(31)
    return z


def _stream_key(seed: int, name: str) -> np.uint64:
    tid = zlib.crc32(name.encode("utf-8")) & 0xFFFFFFFF
    k = (int(seed) * 0x9E3779B97F4A7C15 + tid * 0xD1B54A32D192ED03 + 0x632BE59BD9B4E019) & 0xFFFFFFFFFFFFFFFF
    return _mix64(np.array([k], dtype=np.uint64))[0]


def raw_u64(seed: int, name: str, n: int, offset: int = 0) -> np.ndarray:
    """``n`` 64-bit words of the stream ``(seed, name)`` starting at ``offset``."""
    key = _stream_key(seed, name)
    ctr = np.arange(offset, offset + n, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (ctr + np.uint64(1)) * np.uint64(0x9E3779B97F4A7C15) + key
    return _mix64(z)


def uniform(seed: int, name: str, n: int) -> np.ndarray:
    """float64 uniforms in (0, 1]."""
    r = raw_u64(seed, name, n)
    return ((r >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)


def normal(seed: int, name: str, shape: Sequence[int], std: float = 1.0, mean: float = 0.0) -> np.ndarray:
    """float32 normals (Box-Muller on consecutive uniform pairs)."""
    n = int(np.prod(shape)) if len(shape) else 1
    m = (n + 1) // 2
    chunks = []
    step = 1 << 22
    for lo in range(0, m, step):
        hi = min(m, lo + step)
        r = raw_u64(seed, name, 2 * (hi - lo), offset=2 * lo)
        u = ((r >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)
        rad = np.sqrt(-2.0 * np.log(u[0::2]))
        ang = (2.0 * np.pi) * u[1::2]
        z = np.empty(2 * (hi - lo), dtype=np.float64)
        z[0::2] = rad * np.cos(ang)
        z[1::2] = rad * np.sin(ang)
        chunks.append((z * std + mean).astype(np.float32))
    out = np.concatenate(chunks)[:n] if chunks else np.zeros(0, np.float32)
    return out.reshape(tuple(shape))


def integers(seed: int, name: str, shape: Sequence[int], high: int) -> np.ndarray:
    """int32 uniform in [0, high)."""
    n = int(np.prod(shape)) if len(shape) else 1
    r = raw_u64(seed, name, n)
    return (r % np.uint64(high)).astype(np.int32).reshape(tuple(shape))


# ----------------------------------------------------------------------------
# Workload shapes (dim / heads / layers / context follow the paper's model
# table in the appendix "Model Configurations"; hidden, vocab and kv heads are
# the standard values of the cited LLaMa checkpoints).
# ----------------------------------------------------------------------------

def _cfg(**kw) -> dict:
    base = dict(rms_eps=1e-5, rope_theta=10000.0, local_stage_begin=0, has_embed=1, has_head=1)
    base.update(kw)
    if "local_stage_count" not in base:
        base["local_stage_count"] = base["n_stages"]
    return base


CONFIGS: Dict[str, dict] = {
    # 50M shape, whole model, keep 3 of 4 stages
    "c1": _cfg(dim=288, n_heads=6, n_kv_heads=6, hidden=768, vocab=512, n_stages=4, layers_per_stage=3,
               seq_len=64, seqs_per_mb=1, n_mb=2, skip=(1, 4), swap=0, dtype="f32"),
    # 500M shape, whole model, skip 1/3, swaps allowed
    "c2": _cfg(dim=1024, n_heads=16, n_kv_heads=16, hidden=2816, vocab=32000, n_stages=6, layers_per_stage=4,
               seq_len=1024, seqs_per_mb=4, n_mb=8, skip=(1, 3), swap=1, dtype="bf16"),
    # 1.5B shape, one node's stage (stage 3 of 6), 8 microbatches all routed here (see stage_share_paths)
    "c3": _cfg(dim=2048, n_heads=16, n_kv_heads=16, hidden=5632, vocab=32000, n_stages=6, layers_per_stage=4,
               seq_len=4096, seqs_per_mb=1, n_mb=8, skip=(1, 3), swap=1, dtype="bf16",
               local_stage_begin=3, local_stage_count=1, has_embed=0, has_head=0),
    # LLaMa-2 7B shape, one stage of 8, 16 microbatches, 25 % skip
    "c4": _cfg(dim=4096, n_heads=32, n_kv_heads=32, hidden=11008, vocab=32000, n_stages=8, layers_per_stage=4,
               seq_len=4096, seqs_per_mb=1, n_mb=16, skip=(1, 4), swap=0, dtype="bf16",
               local_stage_begin=1, local_stage_count=1, has_embed=0, has_head=0),
    # LLaMa-3 8B shape (GQA), one stage + final norm + LM head + loss
    "c5": _cfg(dim=4096, n_heads=32, n_kv_heads=8, hidden=14336, vocab=128256, n_stages=8, layers_per_stage=4,
               seq_len=4096, seqs_per_mb=1, n_mb=16, skip=(1, 3), swap=1, dtype="bf16", rope_theta=500000.0,
               local_stage_begin=1, local_stage_count=1, has_embed=0, has_head=1),
}


def shrink(cfg: dict, **kw) -> dict:
    """A copy of ``cfg`` with some fields replaced (reduced-size parity cases)."""
    c = dict(cfg)
    c.update(kw)
    return c


def param_shapes(cfg: dict) -> List[Tuple[str, Tuple[int, ...]]]:
    """Named parameter tensors a node holds under ``cfg``, in storage order.

    Matrices are ``[out_features, in_features]``.  ``wqkv`` stacks the query,
    key and value projections by rows; ``wgu`` stacks gate then up.
    """
    d, h = cfg["dim"], cfg["hidden"]
    hd = d // cfg["n_heads"]
    dkv = cfg["n_kv_heads"] * hd
    out: List[Tuple[str, Tuple[int, ...]]] = []
    if cfg["has_embed"]:
        out.append(("embed", (cfg["vocab"], d)))
    for s in range(cfg["local_stage_begin"], cfg["local_stage_begin"] + cfg["local_stage_count"]):
        for l in range(cfg["layers_per_stage"]):
            p = f"s{s}.l{l}."
            out += [(p + "g1", (d,)), (p + "wqkv", (d + 2 * dkv, d)), (p + "wo", (d, d)),
                    (p + "g2", (d,)), (p + "wgu", (2 * h, d)), (p + "wd", (d, h))]
    if cfg["has_head"]:
        out += [("gf", (d,)), ("whead", (cfg["vocab"], d))]
    return out


def make_params(cfg: dict, seed: int = BASE_SEED, gain_jitter: float = 0.02, std: float = 0.02) -> Dict[str, np.ndarray]:
    """N(0, std) matrices; gains 1 + N(0, gain_jitter) (jitter 0 gives exact ones)."""
    out = {}
    for name, shape in param_shapes(cfg):
        if len(shape) == 1:
            out[name] = normal(seed, "param." + name, shape, std=gain_jitter, mean=1.0) if gain_jitter else \
                np.ones(shape, np.float32)
        else:
            out[name] = normal(seed, "param." + name, shape, std=std)
    return out


def make_tokens(cfg: dict, seed: int = BASE_SEED) -> Tuple[np.ndarray, np.ndarray]:
    """Uniform token ids ``[n_mb, B, T]`` and next-token targets (last position of a sequence = -1)."""
    n_mb, B, T = cfg["n_mb"], cfg["seqs_per_mb"], cfg["seq_len"]
    tok = integers(seed, "tokens", (n_mb, B, T), cfg["vocab"])
    tgt = np.full_like(tok, -1)
    tgt[..., :-1] = tok[..., 1:]
    return tok, tgt


def make_activations(cfg: dict, seed: int = BASE_SEED) -> np.ndarray:
    """Residual-stream inputs ``[n_mb, B*T, dim]`` ~ N(0,1) for a node that holds no embedding."""
    n_mb, n = cfg["n_mb"], cfg["seqs_per_mb"] * cfg["seq_len"]
    return normal(seed, "act_in", (n_mb, n, cfg["dim"]), std=1.0)


def make_upstream_grad(cfg: dict, seed: int = BASE_SEED) -> np.ndarray:
    """Gradient arriving from downstream ``[n_mb, B*T, dim]`` ~ N(0,1)/(tokens per iteration)."""
    n_mb, n = cfg["n_mb"], cfg["seqs_per_mb"] * cfg["seq_len"]
    return normal(seed, "dact_in", (n_mb, n, cfg["dim"]), std=1.0 / (n * n_mb))


def make_paths(n_stages: int, n_mb: int, skip_num: int, skip_den: int, allow_swap: bool,
               seed: int = BASE_SEED) -> Tuple[np.ndarray, np.ndarray]:
    """Seeded microbatch paths, ``paths[mb, pos]`` padded with -1, and their lengths.

    Stage 0 opens every path.  The stages a path leaves out are consecutive
    entries of a seeded permutation of ``1..s-1`` repeated end to end, so every
    later stage is left out by the same number of paths up to one.  A path may
    then have one pair of neighbouring entries exchanged, if the two stages are
    neighbours in the model as well.
    """
    s = n_stages
    total = (2 * n_mb * s * skip_num + skip_den) // (2 * skip_den)      # round(n_mb*s*k)
    lo = (s * skip_num) // skip_den
    q = np.full(n_mb, lo, dtype=np.int64)
    extra = total - lo * n_mb
    r = raw_u64(seed, "paths", 4 * n_mb + 2 * s + 8)
    ri = 0
    # which paths take one more skip: a seeded subset
    order = np.argsort(r[ri:ri + n_mb], kind="stable"); ri += n_mb
    q[order[:extra]] += 1
    if q.max() > s - 1:
        raise ValueError("skip ratio leaves no room for stage 0")
    perm = 1 + np.argsort(r[ri:ri + s - 1], kind="stable"); ri += s - 1
    paths = np.full((n_mb, s), -1, dtype=np.int32)
    lens = np.zeros(n_mb, dtype=np.int32)
    cur = 0
    for mb in range(n_mb):
        skipped = set(int(perm[(cur + j) % (s - 1)]) for j in range(int(q[mb]))) if s > 1 else set()
        cur += int(q[mb])
        kept = [st for st in range(s) if st not in skipped]
        if allow_swap:
            coin = int(r[ri] >> np.uint64(63)); pick = int(r[ri + 1] % np.uint64(1 << 30)); ri += 2
            elig = [j for j in range(1, len(kept) - 1) if kept[j + 1] - kept[j] == 1]
            if coin and elig:
                j = elig[pick % len(elig)]
                kept[j], kept[j + 1] = kept[j + 1], kept[j]
        paths[mb, :len(kept)] = kept
        lens[mb] = len(kept)
    return paths, lens


def make_eval_paths(n_stages: int, n_mb: int, skip_num: int, skip_den: int,
                    seed: int = BASE_SEED) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Per-sample paths for evaluation under stage drops: ``(paths, lens, half)``.

    Every sample drops ``n_stages * skip_num / skip_den`` stages chosen at random among stages ``1..s-1``
    (its own seeded draw); when that number ends in a half, one more stage of the sample runs only the first
    half of its layers and is named in ``half[mb]`` (else -1).  Kept stages stay in model order.
    """
    s = n_stages
    twice = (2 * s * skip_num) // skip_den                   # number of half stages to drop
    whole, part = twice // 2, twice % 2
    if whole + part > s - 1:
        raise ValueError("skip ratio leaves no room for stage 0")
    r = raw_u64(seed, "eval_paths", n_mb * max(1, s - 1))
    paths = np.full((n_mb, s), -1, dtype=np.int32)
    lens = np.zeros(n_mb, dtype=np.int32)
    half = np.full(n_mb, -1, dtype=np.int32)
    for mb in range(n_mb):
        order = 1 + np.argsort(r[mb * (s - 1):(mb + 1) * (s - 1)], kind="stable") if s > 1 else np.zeros(0, np.int64)
        dropped = set(int(x) for x in order[:whole])
        if part:
            half[mb] = int(order[whole])
        kept = [st for st in range(s) if st not in dropped]
        paths[mb, :len(kept)] = kept
        lens[mb] = len(kept)
    return paths, lens, half


# The eight microbatches a stage-3 node of the 6-stage, 1/3-skip set-up serves in one wave: each path keeps 4
# of 6 stages and holds stage 3, which they reach at path position 1, 2 or 3 (groups of 3, 3 and 2), three of
# them through an exchanged pair of neighbouring stages.
C3_PATHS = [(0, 3, 4, 5), (0, 3, 2, 5), (0, 3, 4, 5), (0, 2, 3, 5), (0, 1, 3, 4), (0, 4, 3, 5), (0, 1, 2, 3),
            (0, 1, 4, 3)]


def stage_share_paths(key: str, seed: int = BASE_SEED, generator=None) -> Tuple[np.ndarray, np.ndarray, int]:
    """Paths of a stage-share workload and the stage the node holds.

    c3: the fixed set above.  c4 / c5: the seeded recipe over all 8 stages; the node holds the later stage
    that most paths visit (ties: the lowest index).  generator: a function with make_paths' signature to draw
    the paths with instead (the GPU library exports one)."""
    cfg = CONFIGS[key]
    s = cfg["n_stages"]
    if key == "c3":
        paths = np.full((len(C3_PATHS), s), -1, np.int32)
        for i, p in enumerate(C3_PATHS):
            paths[i, :len(p)] = p
        return paths, np.array([len(p) for p in C3_PATHS], np.int32), 3
    paths, lens = (generator or make_paths)(s, cfg["n_mb"], *cfg["skip"], bool(cfg["swap"]), seed)
    visits = np.zeros(s, int)
    for mb in range(cfg["n_mb"]):
        for st in paths[mb, :lens[mb]]:
            visits[st] += 1
    stage = 1 + int(np.argmax(visits[1:]))
    return paths, lens, stage
