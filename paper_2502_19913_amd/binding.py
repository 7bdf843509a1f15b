"""ctypes binding of libskippipe.so: argument marshalling only.

Every step of the method runs inside the library's HIP kernels; PyTorch is used here for device
memory (tensors whose ``data_ptr()`` is handed over) and for the stream.  There is no CPU path:
if the shared library is missing it is built, and if that fails the import of a symbol raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIBPATH = os.path.join(_HERE, "libskippipe.so")
_lib = None

SP_F32, SP_BF16 = 0, 1
SP_STRICT_CC, SP_SWAP_ANY_GAP, SP_ALLOW_ANY_ORDER = 0, 1, 2

EXPORTS = ["sp_param_count", "sp_param_layout", "sp_workspace_bytes", "sp_make_paths", "sp_check_paths",
           "sp_route_plan", "sp_schedule_paths", "sp_stage_sizes", "sp_strerror", "sp_create", "sp_destroy", "sp_reset", "sp_set_side_stream", "sp_embed_fwd", "sp_embed_bwd",
           "sp_stage_fwd", "sp_stage_bwd", "sp_head_fwd_bwd", "sp_run_paths", "sp_eval_paths", "sp_gemm", "sp_attention_fwd",
           "sp_attention_bwd", "sp_optim_workspace_bytes", "sp_optim_step", "sp_prof_begin", "sp_prof_end", "sp_input_status",
           "sp_grad_reduce", "sp_optim_step_noalloc", "sp_ffn_up_fwd", "sp_ffn_down_bwd", "sp_probe_mfma_rate"]


class SpCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("dim", "n_heads", "n_kv_heads", "hidden", "vocab", "n_stages",
                                         "layers_per_stage", "seq_len", "seqs_per_mb")] + \
               [("rms_eps", C.c_float), ("rope_theta", C.c_float)] + \
               [(n, C.c_int32) for n in ("dtype", "local_stage_begin", "local_stage_count", "has_embed", "has_head",
                                         "path_flags")]


class SpTensorDesc(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("stage", C.c_int32), ("layer", C.c_int32), ("offset", C.c_int64),
                ("rows", C.c_int64), ("cols", C.c_int64)]


class SpError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"[{code}] {msg}")
        self.code = code


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIBPATH):
            from . import build as _build
            _build.build()
        _lib = C.CDLL(_LIBPATH)
        _lib.sp_strerror.restype = C.c_char_p
        _lib.sp_param_count.restype = C.c_int64
        _lib.sp_optim_workspace_bytes.restype = C.c_int64
        _lib.sp_workspace_bytes.restype = C.c_int64
        _lib.sp_make_paths.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_uint64, C.c_void_p, C.c_void_p]
    return _lib


def _check(rc: int) -> int:
    if rc < 0:
        raise SpError(rc, lib().sp_strerror(C.c_int(rc)).decode())
    return rc


def make_cfg(cfg: dict) -> SpCfg:
    dt = cfg.get("dtype", "bf16")
    dt = {"f32": SP_F32, "bf16": SP_BF16}.get(dt, dt)
    vals = {n: cfg[n] for n, _ in SpCfg._fields_ if n not in ("dtype", "path_flags")}
    return SpCfg(dtype=int(dt), path_flags=int(cfg.get("path_flags", SP_STRICT_CC)), **vals)


def _iptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _dptr(t) -> C.c_void_p:
    return C.c_void_p(0 if t is None else t.data_ptr())


# ------------------------------------------------------------------ host helpers
def param_count(cfg: dict) -> int:
    c = make_cfg(cfg)
    return _check(lib().sp_param_count(C.byref(c)))


def param_layout(cfg: dict) -> List[Tuple[str, int, int, int, int, int]]:
    """[(name, stage, layer, offset, rows, cols)] in storage order."""
    c = make_cfg(cfg)
    n = C.c_int(0)
    cap = 8 + 6 * cfg["local_stage_count"] * cfg["layers_per_stage"]
    arr = (SpTensorDesc * cap)()
    _check(lib().sp_param_layout(C.byref(c), arr, C.c_int(cap), C.byref(n)))
    return [(arr[i].name.decode(), arr[i].stage, arr[i].layer, arr[i].offset, arr[i].rows, arr[i].cols)
            for i in range(n.value)]


def workspace_bytes(cfg: dict, n_mb_max: int, n_visits_max: int) -> int:
    c = make_cfg(cfg)
    return _check(lib().sp_workspace_bytes(C.byref(c), C.c_int(n_mb_max), C.c_int(n_visits_max)))


def make_paths(n_stages: int, n_mb: int, skip_num: int, skip_den: int, allow_swap: bool, seed: int):
    paths = np.full((n_mb, n_stages), -7, np.int32)
    lens = np.zeros(n_mb, np.int32)
    _check(lib().sp_make_paths(n_stages, n_mb, skip_num, skip_den, int(allow_swap), seed, _iptr(paths), _iptr(lens)))
    return paths, lens


def check_paths(cfg: dict, paths: np.ndarray, lens: np.ndarray) -> None:
    c = make_cfg(cfg)
    paths = np.ascontiguousarray(paths, np.int32)
    lens = np.ascontiguousarray(lens, np.int32)
    _check(lib().sp_check_paths(C.byref(c), _iptr(paths), _iptr(lens), C.c_int(len(lens))))


def route_plan(cfg: dict, paths: np.ndarray, lens: np.ndarray) -> List[Tuple[int, int, List[int]]]:
    """[(pos, stage, [microbatches])] in forward execution order."""
    c = make_cfg(cfg)
    paths = np.ascontiguousarray(paths, np.int32)
    lens = np.ascontiguousarray(lens, np.int32)
    n_mb, s = paths.shape
    cap = n_mb * s
    gp, gs, gb, gm = (np.zeros(cap + 1, np.int32) for _ in range(4))
    n = C.c_int(0)
    _check(lib().sp_route_plan(C.byref(c), _iptr(paths), _iptr(lens), C.c_int(n_mb), _iptr(gp), _iptr(gs), _iptr(gb),
                               _iptr(gm), C.c_int(cap), C.byref(n)))
    return [(int(gp[g]), int(gs[g]), [int(x) for x in gm[gb[g]:gb[g + 1]]]) for g in range(n.value)]


# ------------------------------------------------------------------ parameter packing by the library's layout
def torch_dtype(cfg: dict):
    import torch
    return torch.bfloat16 if make_cfg(cfg).dtype == SP_BF16 else torch.float32


def pack_params(cfg: dict, named: Dict[str, np.ndarray], device="cuda"):
    """Flat parameter tensor in the library's layout and dtype (bf16 = round-to-nearest of the float values)."""
    import torch
    flat = torch.empty(param_count(cfg), dtype=torch_dtype(cfg), device=device)
    for name, _, _, off, rows, cols in param_layout(cfg):
        a = named[name]
        assert a.size == rows * cols, (name, a.shape, rows, cols)
        flat[off:off + rows * cols] = torch.from_numpy(np.ascontiguousarray(a, np.float32).reshape(-1)).to(
            device=device, dtype=flat.dtype)
    return flat


def unpack(cfg: dict, flat) -> Dict[str, np.ndarray]:
    """Flat tensor in the parameter layout -> dict of float32 numpy arrays."""
    host = flat.detach().float().cpu().numpy()
    out = {}
    for name, _, _, off, rows, cols in param_layout(cfg):
        a = host[off:off + rows * cols]
        out[name] = a.reshape(cols) if rows == 1 and name.split(".")[-1] in ("g1", "g2", "gf") else a.reshape(rows, cols)
    return out


class SpSchedProblem(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_stages", "n_nodes", "n_agents", "mem_limit", "strict_swap", "no_swap", "n_solutions",
                                         "max_expansions")] + [("delta", C.c_float), ("focal_slack", C.c_float)] + \
               [(n, C.c_void_p) for n in ("node_stage", "compute_fwd", "compute_bwd", "comm", "start_node", "n_keep")]


def stage_sizes(n_nodes: int, n_stages: int, skip_num: int, skip_den: int) -> List[int]:
    out = np.zeros(n_stages, np.int32)
    _check(lib().sp_stage_sizes(C.c_int(n_nodes), C.c_int(n_stages), C.c_int(skip_num), C.c_int(skip_den), _iptr(out)))
    return [int(x) for x in out]


def schedule_paths(node_stage, compute_fwd, compute_bwd, comm, start_node, n_keep, mem_limit, strict_swap=True,
                   n_solutions=32, max_expansions=20000, delta=0.0, focal_slack=-1.0, allow_swap=True) -> dict:
    """Path scheduler (host only): returns path_nodes, path_stages [A][s] (-1 padded), len, arrive, e2e, max_e2e."""
    ns = np.ascontiguousarray(node_stage, np.int32)
    cf = np.ascontiguousarray(compute_fwd, np.float32); cb = np.ascontiguousarray(compute_bwd, np.float32)
    cm = np.ascontiguousarray(comm, np.float32)
    st = np.ascontiguousarray(start_node, np.int32); kp = np.ascontiguousarray(n_keep, np.int32)
    N, A = len(ns), len(st)
    assert cm.shape == (N, N) and len(cf) == N and len(cb) == N and len(kp) == A
    s = int(ns.max()) + 1
    pr = SpSchedProblem(s, N, A, mem_limit, 1 if strict_swap else 0, 0 if allow_swap else 1, n_solutions, max_expansions,
                        delta, focal_slack,
                        *(a.ctypes.data_as(C.c_void_p) for a in (ns, cf, cb, cm, st, kp)))
    nodes = np.full((A, s), -1, np.int32); stages = np.full((A, s), -1, np.int32); ln = np.zeros(A, np.int32)
    arrive = np.zeros((A, s), np.float32); e2e = np.zeros(A, np.float32); mx = np.zeros(1, np.float32)
    _check(lib().sp_schedule_paths(C.byref(pr), _iptr(nodes), _iptr(stages), _iptr(ln), _iptr(arrive), _iptr(e2e),
                                   _iptr(mx)))
    return dict(path_nodes=nodes, path_stages=stages, len=ln, arrive=arrive, e2e=e2e, max_e2e=float(mx[0]))


# ------------------------------------------------------------------ device context
class Context:
    """Owns one sp_ctx.  Tensors passed in must live on the context's device and be contiguous."""

    def __init__(self, cfg: dict, n_mb_max: int, n_visits_max: int, stream=None):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("skippipe needs a GPU: there is no CPU path")
        self.cfg = dict(cfg)
        self._c = make_cfg(cfg)
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        self._h = C.c_void_p()
        _check(lib().sp_create(C.byref(self._c), C.c_void_p(self.stream.cuda_stream), C.c_int(n_mb_max),
                               C.c_int(n_visits_max), C.byref(self._h)))

    def close(self):
        if self._h:
            _check(lib().sp_destroy(self._h))
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def reset(self):
        _check(lib().sp_reset(self._h))

    def embed_fwd(self, params, tokens, n_mb, act_pool):
        _check(lib().sp_embed_fwd(self._h, _dptr(params), _dptr(tokens), C.c_int(n_mb), _dptr(act_pool)))

    def embed_bwd(self, tokens, dact_pool, n_mb, grads):
        _check(lib().sp_embed_bwd(self._h, _dptr(tokens), _dptr(dact_pool), C.c_int(n_mb), _dptr(grads)))

    def stage_fwd(self, stage: int, params, act_pool, mb_idx: Sequence[int]):
        idx = np.ascontiguousarray(mb_idx, np.int32)
        _check(lib().sp_stage_fwd(self._h, C.c_int(stage), _dptr(params), _dptr(act_pool), _iptr(idx), C.c_int(len(idx))))

    def stage_bwd(self, stage: int, params, dact_pool, mb_idx: Sequence[int], grads):
        idx = np.ascontiguousarray(mb_idx, np.int32)
        _check(lib().sp_stage_bwd(self._h, C.c_int(stage), _dptr(params), _dptr(dact_pool), _iptr(idx),
                                  C.c_int(len(idx)), _dptr(grads)))

    def head_fwd_bwd(self, params, act_pool, targets, n_mb, loss_mb, dact_pool, grads):
        _check(lib().sp_head_fwd_bwd(self._h, _dptr(params), _dptr(act_pool), _dptr(targets), C.c_int(n_mb),
                                     _dptr(loss_mb), _dptr(dact_pool), _dptr(grads)))

    def run_paths(self, params, tokens, targets, paths: np.ndarray, lens: np.ndarray, grads):
        paths = np.ascontiguousarray(paths, np.int32)
        lens = np.ascontiguousarray(lens, np.int32)
        n_mb = len(lens)
        loss = np.zeros(1, np.float32)
        loss_mb = np.zeros(n_mb, np.float32)
        _check(lib().sp_run_paths(self._h, _dptr(params), _dptr(tokens), _dptr(targets), _iptr(paths), _iptr(lens),
                                  C.c_int(n_mb), _iptr(loss), _iptr(loss_mb), _dptr(grads)))
        return float(loss[0]), loss_mb

    def input_status(self):
        """Waits for the stream; raises SpError(SP_EINVAL) if a kernel met a token id or target out of range."""
        _check(lib().sp_input_status(self._h))

    def set_side_stream(self, enabled):
        """0 / False: weight gradients in line; 1 / True: on the second stream where that pays (default); 2: always."""
        _check(lib().sp_set_side_stream(self._h, C.c_int(int(enabled))))

    def eval_paths(self, params, tokens, targets, paths: np.ndarray, lens: np.ndarray, half=None):
        paths = np.ascontiguousarray(paths, np.int32)
        lens = np.ascontiguousarray(lens, np.int32)
        n_mb = len(lens)
        hf = None if half is None else np.ascontiguousarray(half, np.int32)
        loss = np.zeros(1, np.float32)
        loss_mb = np.zeros(n_mb, np.float32)
        _check(lib().sp_eval_paths(self._h, _dptr(params), _dptr(tokens), _dptr(targets), _iptr(paths), _iptr(lens),
                                   _iptr(hf) if hf is not None else None, C.c_int(n_mb), _iptr(loss), _iptr(loss_mb)))
        return float(loss[0]), loss_mb


def _stream_ptr(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def _dt(t):
    import torch
    return SP_BF16 if t.dtype == torch.bfloat16 else SP_F32


def gemm(op: int, A, B, C_out, R=None, stream=None):
    """op 0: C = A B^T (+R); op 1: C = A B; op 2: C(float) += A^T B."""
    if op == 0:
        M, K = A.shape; N = B.shape[0]
    elif op == 1:
        M, K = A.shape; N = B.shape[1]
    else:
        K, M = A.shape; N = B.shape[1]
    _check(lib().sp_gemm(_stream_ptr(stream), C.c_int(_dt(A)), C.c_int(op), C.c_int(M), C.c_int(N), C.c_int(K),
                         _dptr(A), _dptr(B), _dptr(C_out), _dptr(R)))


def ffn_up_fwd(hn, wgu, gu, act, stream=None):
    """gu = hn wgu^T and act = silu(gate) * up in one call."""
    R, d = hn.shape; h = act.shape[1]
    _check(lib().sp_ffn_up_fwd(_stream_ptr(stream), C.c_int(_dt(hn)), C.c_int(R), C.c_int(h), C.c_int(d), _dptr(hn),
                               _dptr(wgu), _dptr(gu), _dptr(act)))


def ffn_down_bwd(dy, wd, gu, dgu, da_scratch, stream=None):
    """dgu = gradient of [gate | up] for d(act) = dy wd and the saved gu."""
    R, d = dy.shape; h = wd.shape[1]
    _check(lib().sp_ffn_down_bwd(_stream_ptr(stream), C.c_int(_dt(dy)), C.c_int(R), C.c_int(h), C.c_int(d), _dptr(dy),
                                 _dptr(wd), _dptr(gu), _dptr(dgu), _dptr(da_scratch)))


def attention_fwd(qkv, o, lse, B, T, H, Hkv, hd, stream=None):
    _check(lib().sp_attention_fwd(_stream_ptr(stream), C.c_int(_dt(qkv)), B, T, H, Hkv, hd, _dptr(qkv), _dptr(o),
                                  _dptr(lse)))


def attention_bwd(qkv, o, lse, do, dqkv, delta, B, T, H, Hkv, hd, stream=None):
    _check(lib().sp_attention_bwd(_stream_ptr(stream), C.c_int(_dt(qkv)), B, T, H, Hkv, hd, _dptr(qkv), _dptr(o),
                                  _dptr(lse), _dptr(do), _dptr(dqkv), _dptr(delta)))


class SpAdamW(C.Structure):
    _fields_ = [(n, C.c_float) for n in ("lr", "beta1", "beta2", "eps", "weight_decay", "clip_norm")]


def optim_workspace_bytes() -> int:
    return int(lib().sp_optim_workspace_bytes())


def optim_step(master, grads, m, v, step: int, params_out=None, workspace=None, grad_norm=None, lr=3e-4, beta1=0.9,
               beta2=0.999, eps=1e-8, weight_decay=0.01, clip_norm=1.0, stream=None):
    """Clip + AdamW update of the float master copy (in place); params_out receives its low-precision copy."""
    h = SpAdamW(lr, beta1, beta2, eps, weight_decay, clip_norm)
    n = master.numel()
    od = _dt(params_out) if params_out is not None else SP_F32
    _check(lib().sp_optim_step(_stream_ptr(stream), C.byref(h), C.c_int64(n), C.c_int(step), _dptr(master), _dptr(grads),
                               _dptr(m), _dptr(v), _dptr(params_out), C.c_int(od), _dptr(workspace), _dptr(grad_norm)))


def optim_step_noalloc(master, grads, m, v, step: int, params_out=None, grad_norm=None, lr=3e-4, beta1=0.9, beta2=0.999,
                       eps=1e-8, weight_decay=0.01, clip_norm=1.0, stream=None):
    """optim_step without a workspace argument: the library's static device scratch is used; allocates nothing."""
    h = SpAdamW(lr, beta1, beta2, eps, weight_decay, clip_norm)
    od = _dt(params_out) if params_out is not None else SP_F32
    _check(lib().sp_optim_step_noalloc(_stream_ptr(stream), C.byref(h), C.c_int64(master.numel()), C.c_int(step),
                                       _dptr(master), _dptr(grads), _dptr(m), _dptr(v), _dptr(params_out), C.c_int(od),
                                       _dptr(grad_norm)))


def grad_reduce(replica_grads, out, scale: float = 1.0, stream=None):
    """out = scale * sum of the replica gradient buffers (float tensors of equal length)."""
    n = out.numel()
    assert all(g.numel() == n for g in replica_grads)
    ptrs = (C.c_void_p * len(replica_grads))(*[g.data_ptr() for g in replica_grads])
    _check(lib().sp_grad_reduce(_stream_ptr(stream), ptrs, C.c_int(len(replica_grads)), C.c_int64(n), C.c_float(scale),
                                _dptr(out)))


def probe_mfma_rate(src, n_blocks, iters, sink, stream=None):
    """sp_probe_mfma_rate: enqueue the registers-only matrix-core loop; returns the flops of the launch."""
    import torch
    assert src.is_cuda and sink.is_cuda and sink.dtype == torch.float32 and sink.numel() >= n_blocks * 512
    fl = C.c_double(0.0)
    _check(lib().sp_probe_mfma_rate(_stream_ptr(stream), _dptr(src), C.c_int64(src.numel() * src.element_size()),
                                    C.c_int(n_blocks), C.c_int(iters), _dptr(sink), C.byref(fl)))
    return fl.value


PROF_CLASSES = ["gemm_nt", "gemm_nn", "gemm_tn", "attn_fwd", "attn_delta", "attn_dq", "attn_dkv", "gemm_plain",
                "attn_plain", "rmsnorm_fwd", "rmsnorm_bwd", "cross_entropy", "copy_rows", "swiglu"]
PROF_BYTES_CLASSES = ("attn_delta", "rmsnorm_fwd", "rmsnorm_bwd", "cross_entropy", "copy_rows", "swiglu")   # "flops" holds bytes


def prof_begin():
    _check(lib().sp_prof_begin())


def prof_end() -> Dict[str, dict]:
    n = len(PROF_CLASSES)
    ms = np.zeros(n, np.float64); fl = np.zeros(n, np.float64); cnt = np.zeros(n, np.int64)
    _check(lib().sp_prof_end(C.c_int(n), _iptr(ms), _iptr(fl), _iptr(cnt)))
    return {PROF_CLASSES[i]: dict(ms=float(ms[i]), flops=float(fl[i]), launches=int(cnt[i])) for i in range(n)}
