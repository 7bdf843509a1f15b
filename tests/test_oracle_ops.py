"""Pins for the single ops of the CPU checker: closed forms, textbook special cases, library routines."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as Fn

from oracle import skippipe_oracle as orc

RNG = np.random.default_rng(7)


def t64(a):
    return torch.tensor(a, dtype=torch.float64)


# ---------------------------------------------------------------- RMSNorm
def test_rmsnorm_constant_row_closed_form():
    d, c, eps = 24, 3.0, 1e-5
    x = np.full((2, d), c)
    g = np.linspace(0.5, 1.5, d)
    y, rstd = orc.rmsnorm_fwd(x, g, eps)
    want = c / math.sqrt(c * c + eps) * g
    assert np.allclose(y[0], want, rtol=1e-14)
    assert np.allclose(rstd, 1 / math.sqrt(c * c + eps), rtol=1e-14)


def test_rmsnorm_matches_library_and_autograd():
    R, d, eps = 5, 16, 1e-5
    x, g, dy = RNG.normal(size=(R, d)), 1 + 0.1 * RNG.normal(size=d), RNG.normal(size=(R, d))
    y, rstd = orc.rmsnorm_fwd(x, g, eps)
    xt, gt = t64(x).requires_grad_(), t64(g).requires_grad_()
    yt = Fn.rms_norm(xt, (d,), gt, eps)
    yt.backward(t64(dy))
    assert np.allclose(y, yt.detach().numpy(), rtol=1e-12, atol=1e-14)
    dx, dg = orc.rmsnorm_bwd(dy, x, g, rstd)
    assert np.allclose(dx, xt.grad.numpy(), rtol=1e-10, atol=1e-13)
    assert np.allclose(dg, gt.grad.numpy(), rtol=1e-10, atol=1e-13)


def test_rmsnorm_scale_invariance():
    # without eps the output does not change when a row is scaled
    x, g = RNG.normal(size=(3, 32)), np.ones(32)
    y1, _ = orc.rmsnorm_fwd(x, g, 0.0)
    y2, _ = orc.rmsnorm_fwd(7.5 * x, g, 0.0)
    assert np.allclose(y1, y2, rtol=1e-13)
    assert np.allclose((y1 ** 2).mean(axis=1), 1.0, rtol=1e-13)


# ---------------------------------------------------------------- linear
def test_linear_is_x_wT_and_its_adjoints():
    R, K, N = 7, 12, 9                      # non-square so a transposed operand fails
    x, W, dy = RNG.normal(size=(R, K)), RNG.normal(size=(N, K)), RNG.normal(size=(R, N))
    assert np.allclose(orc.linear_fwd(x, W), x @ W.T, rtol=1e-13)
    dx, dW = orc.linear_bwd(dy, x, W)
    assert np.allclose(dx, dy @ W, rtol=1e-13)
    assert np.allclose(dW, dy.T @ x, rtol=1e-13)


def test_linear_f32_close_to_f64():
    R, K, N = 6, 64, 10
    x, W = RNG.normal(size=(R, K)), RNG.normal(size=(N, K))
    y32 = orc.linear_fwd(x.astype(np.float32), W.astype(np.float32))
    assert np.allclose(y32, x @ W.T, rtol=1e-4, atol=1e-5)


# ---------------------------------------------------------------- RoPE
def test_rope_closed_form_angles():
    # hd = 4, theta = 10000: pair 0 turns by p radians, pair 1 by p / 100 radians
    T = 3
    q = np.zeros((T, 1, 4)); q[:, 0, 0] = 1.0; q[:, 0, 2] = 1.0
    out = orc.rope(q, T, 10000.0)
    for p in range(T):
        assert np.allclose(out[p, 0], [math.cos(p), math.sin(p), math.cos(p / 100), math.sin(p / 100)], atol=1e-14)


def test_rope_position_restarts_per_sequence_and_preserves_norm():
    B, T, nh, hd = 2, 5, 3, 8
    q = RNG.normal(size=(B * T, nh, hd))
    out = orc.rope(q, T, 10000.0)
    assert np.allclose(out[0], q[0]) and np.allclose(out[T], q[T])          # position 0 of both sequences
    assert np.allclose(np.linalg.norm(out, axis=-1), np.linalg.norm(q, axis=-1), rtol=1e-13)
    # pairs are (2i, 2i+1): each pair's norm is preserved on its own
    assert np.allclose(np.hypot(out[..., 0::2], out[..., 1::2]), np.hypot(q[..., 0::2], q[..., 1::2]), rtol=1e-12)


def test_rope_scores_depend_on_relative_position_only():
    T, hd = 9, 8
    qv, kv = RNG.normal(size=hd), RNG.normal(size=hd)
    q = np.tile(qv, (T, 1, 1)); k = np.tile(kv, (T, 1, 1))
    qr, kr = orc.rope(q, T, 500.0), orc.rope(k, T, 500.0)
    s = qr[:, 0] @ kr[:, 0].T
    for off in range(-3, 4):
        diag = np.diagonal(s, offset=off)
        assert np.allclose(diag, diag[0], rtol=1e-11, atol=1e-12)
    assert not np.allclose(np.diagonal(s, 1)[0], np.diagonal(s, -1)[0])


def test_rope_backward_is_the_inverse_rotation():
    T = 6
    q = RNG.normal(size=(T, 2, 8))
    assert np.allclose(orc.rope(orc.rope(q, T, 10000.0, 1), T, 10000.0, -1), q, atol=1e-13)


# ---------------------------------------------------------------- attention
def test_attention_single_token_returns_v():
    q, k, v = RNG.normal(size=(3, 2, 4)), RNG.normal(size=(3, 2, 4)), RNG.normal(size=(3, 2, 4))
    assert np.allclose(orc.attention_fwd(q, k, v, 3, 1), v, rtol=1e-14)


def test_attention_zero_query_is_prefix_mean():
    T = 6
    q = np.zeros((T, 1, 4)); k = RNG.normal(size=(T, 1, 4)); v = RNG.normal(size=(T, 1, 4))
    o = orc.attention_fwd(q, k, v, 1, T)
    want = np.cumsum(v, axis=0) / np.arange(1, T + 1)[:, None, None]
    assert np.allclose(o, want, rtol=1e-13)


def test_attention_is_causal_and_sequences_do_not_mix():
    B, T, H, hd = 2, 6, 2, 4
    q, k, v = (RNG.normal(size=(B * T, H, hd)) for _ in range(3))
    o = orc.attention_fwd(q, k, v, B, T)
    k2, v2 = k.copy(), v.copy()
    k2[4] += 1.0; v2[4] -= 2.0                       # touch position 4 of sequence 0
    o2 = orc.attention_fwd(q, k2, v2, B, T)
    assert np.array_equal(o[:4], o2[:4])             # earlier positions unchanged
    assert not np.allclose(o[4:T], o2[4:T])
    assert np.array_equal(o[T:], o2[T:])             # the other sequence unchanged


@pytest.mark.parametrize("H,Hkv", [(4, 4), (4, 2), (4, 1)])
def test_attention_matches_library_sdpa_and_autograd(H, Hkv):
    B, T, hd = 2, 7, 8
    q = RNG.normal(size=(B * T, H, hd)); k = RNG.normal(size=(B * T, Hkv, hd)); v = RNG.normal(size=(B * T, Hkv, hd))
    dO = RNG.normal(size=(B * T, H, hd))
    qt, kt, vt = (t64(a).requires_grad_() for a in (q, k, v))
    rep = H // Hkv
    o_t = Fn.scaled_dot_product_attention(
        qt.reshape(B, T, H, hd).transpose(1, 2),
        kt.reshape(B, T, Hkv, hd).repeat_interleave(rep, dim=2).transpose(1, 2),
        vt.reshape(B, T, Hkv, hd).repeat_interleave(rep, dim=2).transpose(1, 2), is_causal=True)
    o_t = o_t.transpose(1, 2).reshape(B * T, H, hd)
    o_t.backward(t64(dO))
    o = orc.attention_fwd(q, k, v, B, T)
    assert np.allclose(o, o_t.detach().numpy(), rtol=1e-11, atol=1e-13)
    dq, dk, dv = orc.attention_bwd(dO, q, k, v, B, T)
    assert np.allclose(dq, qt.grad.numpy(), rtol=1e-9, atol=1e-12)
    assert np.allclose(dk, kt.grad.numpy(), rtol=1e-9, atol=1e-12)
    assert np.allclose(dv, vt.grad.numpy(), rtol=1e-9, atol=1e-12)


def test_gqa_equals_mha_with_repeated_kv_heads():
    B, T, H, Hkv, hd = 1, 5, 4, 2, 4
    q = RNG.normal(size=(B * T, H, hd)); k = RNG.normal(size=(B * T, Hkv, hd)); v = RNG.normal(size=(B * T, Hkv, hd))
    o1 = orc.attention_fwd(q, k, v, B, T)
    o2 = orc.attention_fwd(q, np.repeat(k, 2, axis=1), np.repeat(v, 2, axis=1), B, T)
    assert np.allclose(o1, o2, rtol=1e-14)


# ---------------------------------------------------------------- SwiGLU
def test_swiglu_matches_library_and_autograd():
    R, h = 4, 6
    gu, da = RNG.normal(size=(R, 2 * h)) * 3, RNG.normal(size=(R, h))
    gt = t64(gu).requires_grad_()
    at = Fn.silu(gt[:, :h]) * gt[:, h:]
    at.backward(t64(da))
    assert np.allclose(orc.swiglu_fwd(gu), at.detach().numpy(), rtol=1e-13)
    assert np.allclose(orc.swiglu_bwd(da, gu), gt.grad.numpy(), rtol=1e-11, atol=1e-14)


def test_swiglu_gate_zero_and_large():
    gu = np.array([[0.0, 40.0, -40.0, 2.0, 3.0, 5.0]])     # gate | up
    a = orc.swiglu_fwd(gu)
    assert a[0, 0] == 0.0
    assert np.isclose(a[0, 1], 40.0 * 3.0, rtol=1e-12)      # silu(x) -> x for large x
    assert abs(a[0, 2]) < 1e-14                             # silu(x) -> 0 for very negative x


# ---------------------------------------------------------------- cross entropy
def test_ce_equal_logits_is_log_vocab():
    R, V = 3, 50
    loss, dl = orc.cross_entropy(np.full((R, V), 1.7), np.array([0, 7, 49]))
    assert math.isclose(loss, math.log(V), rel_tol=1e-13)
    assert np.allclose(dl.sum(axis=1), 0.0, atol=1e-15)


def test_ce_matches_library_with_ignored_rows_and_weight():
    R, V, w = 6, 11, 0.25
    z = RNG.normal(size=(R, V)) * 4
    tgt = np.array([3, -1, 0, 10, -1, 5])
    zt = t64(z).requires_grad_()
    lt = Fn.cross_entropy(zt, torch.tensor(tgt, dtype=torch.long), ignore_index=-1)
    (lt * w).backward()
    loss, dl = orc.cross_entropy(z, tgt, w)
    assert math.isclose(loss, float(lt.detach()), rel_tol=1e-12)
    assert np.allclose(dl, zt.grad.numpy(), rtol=1e-11, atol=1e-15)
    assert np.all(dl[1] == 0) and np.all(dl[4] == 0)
    assert np.allclose(dl.sum(axis=1), 0.0, atol=1e-15)


def test_ce_huge_logits_do_not_overflow():
    z = np.array([[1000.0, 0.0, -1000.0]])
    loss, dl = orc.cross_entropy(z, np.array([1]))
    assert math.isclose(loss, 1000.0, rel_tol=1e-12)
    assert np.all(np.isfinite(dl))
