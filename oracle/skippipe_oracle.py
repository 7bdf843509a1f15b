"""ctypes front end of the CPU checker (test infrastructure, never the product path).

Only ``tests/``, the smoke check and the benchmark's CPU-baseline leg import this.
It builds ``skippipe_oracle.cpp`` with g++ on first use and exposes the iteration
(:func:`run_paths`) plus the single ops, each in float32 and float64.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "skippipe_oracle.cpp")
_LIB = os.path.join(_HERE, "libskippipe_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O3", "-mavx2", "-mfma", "-fopenmp", "-shared", "-fPIC", "-std=c++17", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


class OrcCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("dim", "n_heads", "n_kv_heads", "hidden", "vocab", "n_stages",
                                         "layers_per_stage", "seq_len", "seqs_per_mb")] + \
               [("rms_eps", C.c_float), ("rope_theta", C.c_float)] + \
               [(n, C.c_int32) for n in ("local_stage_begin", "local_stage_count", "has_embed", "has_head")]


def _cfg(cfg: dict) -> OrcCfg:
    return OrcCfg(**{n: cfg[n] for n, _ in OrcCfg._fields_})


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        for suf, ft in (("_f32", C.c_float), ("_f64", C.c_double)):
            getattr(_lib, "orc_param_count" + suf).restype = C.c_size_t
            getattr(_lib, "orc_cross_entropy" + suf).restype = ft
    return _lib


def _suf(dtype):
    dtype = np.dtype(dtype)
    if dtype == np.float32:
        return "_f32", C.c_float
    if dtype == np.float64:
        return "_f64", C.c_double
    raise TypeError(dtype)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


# ------------------------------------------------------------------ parameter packing (this side's own layout)
def _names(cfg: dict):
    d, h = cfg["dim"], cfg["hidden"]
    hd = d // cfg["n_heads"]
    dkv = cfg["n_kv_heads"] * hd
    out = []
    if cfg["has_embed"]:
        out.append(("embed", (cfg["vocab"], d)))
    for s in range(cfg["local_stage_begin"], cfg["local_stage_begin"] + cfg["local_stage_count"]):
        for l in range(cfg["layers_per_stage"]):
            p = f"s{s}.l{l}."
            out += [(p + "g1", (d,)), (p + "wqkv", (d + 2 * dkv, d)), (p + "wo", (d, d)), (p + "g2", (d,)),
                    (p + "wgu", (2 * h, d)), (p + "wd", (d, h))]
    if cfg["has_head"]:
        out += [("gf", (d,)), ("whead", (cfg["vocab"], d))]
    return out


def pack(cfg: dict, named: Dict[str, np.ndarray], dtype) -> np.ndarray:
    n = lib().orc_param_count_f32(C.byref(_cfg(cfg)))
    flat = np.empty(n, dtype=dtype)
    off = 0
    for name, shape in _names(cfg):
        k = int(np.prod(shape))
        a = named[name]
        assert tuple(a.shape) == tuple(shape), (name, a.shape, shape)
        flat[off:off + k] = a.reshape(-1)
        off += k
    assert off == n
    return flat


def unpack(cfg: dict, flat: np.ndarray) -> Dict[str, np.ndarray]:
    out, off = {}, 0
    for name, shape in _names(cfg):
        k = int(np.prod(shape))
        out[name] = flat[off:off + k].reshape(shape)
        off += k
    assert off == flat.size
    return out


# ------------------------------------------------------------------ the iteration
def run_paths(cfg: dict, named_params: Dict[str, np.ndarray], paths: np.ndarray, lens: np.ndarray, *,
              tokens: Optional[np.ndarray] = None, targets: Optional[np.ndarray] = None,
              x_in: Optional[np.ndarray] = None, dy_in: Optional[np.ndarray] = None, dtype=np.float64) -> dict:
    """Push every microbatch along its path, forward and backward.

    Returns ``loss`` (mean over microbatches), ``loss_mb``, ``grads`` (dict by name), ``y`` (residual stream
    after the last local stage, per microbatch) and ``dx`` (gradient w.r.t. the incoming residual stream).
    """
    suf, ft = _suf(dtype)
    n_mb = int(paths.shape[0])
    R = cfg["seqs_per_mb"] * cfg["seq_len"]
    d = cfg["dim"]
    P = pack(cfg, named_params, dtype)
    G = np.zeros_like(P)
    paths = np.ascontiguousarray(paths, np.int32)
    assert paths.shape == (n_mb, cfg["n_stages"])
    lens = np.ascontiguousarray(lens, np.int32)
    tok = None if tokens is None else np.ascontiguousarray(tokens, np.int32).reshape(n_mb, R)
    tgt = None if targets is None else np.ascontiguousarray(targets, np.int32).reshape(n_mb, R)
    xi = None if x_in is None else np.ascontiguousarray(x_in, dtype).reshape(n_mb, R, d)
    dyi = None if dy_in is None else np.ascontiguousarray(dy_in, dtype).reshape(n_mb, R, d)
    if cfg["has_embed"]:
        assert tok is not None
    else:
        assert xi is not None
    if cfg["has_head"]:
        assert tgt is not None
    else:
        assert dyi is not None
    loss_mb = np.zeros(n_mb, dtype)
    loss = np.zeros(1, dtype)
    y = np.zeros((n_mb, R, d), dtype)
    dx = np.zeros((n_mb, R, d), dtype)
    rc = getattr(lib(), "orc_run_paths" + suf)(C.byref(_cfg(cfg)), _p(P), _p(tok), _p(xi), _p(tgt), _p(dyi),
                                               _p(paths), _p(lens), C.c_int(n_mb), _p(loss_mb), _p(loss), _p(y),
                                               _p(dx), _p(G))
    if rc != 0:
        raise ValueError(f"oracle rejected its input (code {rc})")
    return dict(loss=float(loss[0]), loss_mb=loss_mb, grads=unpack(cfg, G), y=y, dx=dx)


# ------------------------------------------------------------------ single ops (for the pins)
def rmsnorm_fwd(x, g, eps):
    suf, ft = _suf(x.dtype)
    R, d = x.shape
    y = np.empty_like(x); rstd = np.empty(R, x.dtype)
    getattr(lib(), "orc_rmsnorm_fwd" + suf)(_p(x), _p(g), R, d, ft(eps), _p(y), _p(rstd))
    return y, rstd


def rmsnorm_bwd(dy, x, g, rstd):
    suf, ft = _suf(x.dtype)
    R, d = x.shape
    dx = np.empty_like(x); dg = np.zeros(d, x.dtype)
    getattr(lib(), "orc_rmsnorm_bwd" + suf)(_p(dy), _p(x), _p(g), _p(rstd), R, d, _p(dx), _p(dg))
    return dx, dg


def eval_paths(cfg: dict, named_params: Dict[str, np.ndarray], paths: np.ndarray, lens: np.ndarray, *,
               tokens: np.ndarray, targets: np.ndarray, half: Optional[np.ndarray] = None, dtype=np.float64) -> dict:
    """Forward only: every microbatch along its path, the stage half[mb] (if >= 0) with only the first half
    of its layers; returns ``loss`` (mean over microbatches) and ``loss_mb``."""
    suf, ft = _suf(dtype)
    n_mb = int(paths.shape[0])
    R = cfg["seqs_per_mb"] * cfg["seq_len"]
    P = pack(cfg, named_params, dtype)
    paths = np.ascontiguousarray(paths, np.int32)
    assert paths.shape == (n_mb, cfg["n_stages"])
    lens = np.ascontiguousarray(lens, np.int32)
    tok = np.ascontiguousarray(tokens, np.int32).reshape(n_mb, R)
    tgt = np.ascontiguousarray(targets, np.int32).reshape(n_mb, R)
    hf = None if half is None else np.ascontiguousarray(half, np.int32).reshape(n_mb)
    loss_mb = np.zeros(n_mb, dtype)
    loss = np.zeros(1, dtype)
    rc = getattr(lib(), "orc_eval_paths" + suf)(C.byref(_cfg(cfg)), _p(P), _p(tok), _p(tgt), _p(paths), _p(lens),
                                                _p(hf), C.c_int(n_mb), _p(loss_mb), _p(loss))
    if rc != 0:
        raise ValueError(f"oracle rejected its input (code {rc})")
    return dict(loss=float(loss[0]), loss_mb=loss_mb)


def linear_fwd(x, W):
    suf, ft = _suf(x.dtype)
    R, K = x.shape; N = W.shape[0]
    y = np.empty((R, N), x.dtype)
    getattr(lib(), "orc_linear_fwd" + suf)(_p(x), _p(W), R, K, N, _p(y))
    return y


def linear_bwd(dy, x, W):
    suf, ft = _suf(x.dtype)
    R, K = x.shape; N = W.shape[0]
    dx = np.empty_like(x); dW = np.zeros_like(W)
    getattr(lib(), "orc_linear_bwd" + suf)(_p(dy), _p(x), _p(W), R, K, N, _p(dx), _p(dW))
    return dx, dW


def rope(q, T, theta, sign=1):
    """q [R, nh, hd] -> rotated copy."""
    suf, ft = _suf(q.dtype)
    R, nh, hd = q.shape
    out = np.ascontiguousarray(q).copy()
    getattr(lib(), "orc_rope" + suf)(_p(out), R, T, nh, hd, ft(theta), sign)
    return out


def attention_fwd(q, k, v, B, T):
    """q [B*T, H, hd], k/v [B*T, Hkv, hd] -> o [B*T, H, hd]."""
    suf, ft = _suf(q.dtype)
    R, H, hd = q.shape; Hkv = k.shape[1]
    o = np.empty_like(q)
    getattr(lib(), "orc_attention_fwd" + suf)(_p(q), _p(k), _p(v), B, T, H, Hkv, hd, _p(o))
    return o


def attention_bwd(dO, q, k, v, B, T):
    suf, ft = _suf(q.dtype)
    R, H, hd = q.shape; Hkv = k.shape[1]
    dq = np.zeros_like(q); dk = np.zeros_like(k); dv = np.zeros_like(v)
    getattr(lib(), "orc_attention_bwd" + suf)(_p(dO), _p(q), _p(k), _p(v), B, T, H, Hkv, hd, _p(dq), _p(dk), _p(dv))
    return dq, dk, dv


def swiglu_fwd(gu):
    suf, ft = _suf(gu.dtype)
    R, h2 = gu.shape
    a = np.empty((R, h2 // 2), gu.dtype)
    getattr(lib(), "orc_swiglu_fwd" + suf)(_p(gu), R, h2 // 2, _p(a))
    return a


def swiglu_bwd(da, gu):
    suf, ft = _suf(gu.dtype)
    R, h2 = gu.shape
    dgu = np.empty_like(gu)
    getattr(lib(), "orc_swiglu_bwd" + suf)(_p(da), _p(gu), R, h2 // 2, _p(dgu))
    return dgu


def cross_entropy(logits, tgt, w=1.0):
    suf, ft = _suf(logits.dtype)
    R, V = logits.shape
    dl = np.empty_like(logits)
    tgt = np.ascontiguousarray(tgt, np.int32)
    loss = getattr(lib(), "orc_cross_entropy" + suf)(_p(logits), _p(tgt), R, V, ft(w), _p(dl))
    return float(loss), dl
