"""Pins of the update checker: library routines, closed forms and invariants (CPU only)."""
import numpy as np
import pytest
import torch

from oracle import optim_oracle as opt
from paper_2502_19913_amd import synth


def test_paper_hyperparameters():
    # appendix "Test Configurations": learning rate 3e-4, gradient norms clipped to 1.0
    assert opt.PAPER_LR == 3e-4 and opt.PAPER_CLIP == 1.0


@pytest.mark.parametrize("clip", [1.0, 0.05, 0.0])
@pytest.mark.parametrize("wd", [0.0, 0.01, 0.1])
def test_against_torch_adamw_and_clip_grad_norm(clip, wd):
    # several tensors, several steps: torch clips over all of them with one norm and updates each
    shapes = [(7, 5), (33,), (4, 4, 3)]
    rng = [synth.normal(11, f"p{i}", s).astype(np.float64) for i, s in enumerate(shapes)]
    tp = [torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in rng]
    o = torch.optim.AdamW(tp, lr=3e-4, betas=(0.9, 0.95), eps=1e-8, weight_decay=wd)
    flat = lambda xs: np.concatenate([np.asarray(x, np.float64).reshape(-1) for x in xs])
    p = flat(rng); m = np.zeros_like(p); v = np.zeros_like(p)
    for step in range(1, 6):
        gs = [synth.normal(12, f"g{step}_{i}", s).astype(np.float64) * (0.3 * step) for i, s in enumerate(shapes)]
        for t, g in zip(tp, gs):
            t.grad = torch.tensor(g, dtype=torch.float64)
        if clip > 0:
            tn = float(torch.nn.utils.clip_grad_norm_(tp, clip))
        o.step()
        p, m, v, norm = opt.adamw_step(p, flat(gs), m, v, step, lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8,
                                       weight_decay=wd, clip=clip)
        if clip > 0:
            assert abs(norm - tn) <= 1e-12 * max(1.0, tn)
        np.testing.assert_allclose(p, flat([t.detach().numpy() for t in tp]), rtol=1e-12, atol=1e-15)


def test_first_step_is_lr_against_the_sign():
    # t = 1, no decay, no clipping: m_hat = g, v_hat = g^2, so the step is lr * g / (|g| + eps)
    g = np.array([0.5, -2.0, 1e-3, -7.0])
    p = np.array([1.0, 2.0, 3.0, 4.0])
    pn, m, v, _ = opt.adamw_step(p, g, np.zeros(4), np.zeros(4), 1, lr=0.1, eps=1e-12, weight_decay=0.0, clip=0.0)
    np.testing.assert_allclose(pn, p - 0.1 * np.sign(g), rtol=0, atol=1e-9)
    np.testing.assert_allclose(m, 0.1 * g); np.testing.assert_allclose(v, 1e-3 * g * g)


def test_clip_invariants():
    g = synth.normal(13, "cg", (1000,)).astype(np.float64)
    norm, coef = opt.clip_coefficient(g, 1.0)
    assert abs(norm - np.linalg.norm(g)) < 1e-12 and norm > 1.0
    assert np.linalg.norm(g * coef) <= 1.0 and np.linalg.norm(g * coef) > 0.999
    small = g * (0.5 / norm)
    assert opt.clip_coefficient(small, 1.0)[1] == 1.0          # below the bound: untouched
    assert opt.clip_coefficient(g, 0.0)[1] == 1.0              # clipping off
    assert opt.clip_coefficient(np.zeros(5), 1.0) == (0.0, 1.0)


def test_zero_gradient_is_pure_decay():
    p = np.array([2.0, -4.0])
    pn, m, v, norm = opt.adamw_step(p, np.zeros(2), np.zeros(2), np.zeros(2), 3, lr=0.1, weight_decay=0.5)
    np.testing.assert_allclose(pn, p * (1 - 0.05)); assert norm == 0.0 and not m.any() and not v.any()


def test_a_dropped_bias_correction_would_show():
    # planted mistakes in a copy of the arithmetic: each must move the result past the pin's tolerance
    g = np.array([0.3, -0.2]); p = np.array([1.0, 1.0]); m = np.array([0.1, 0.0]); v = np.array([0.01, 0.02])
    good = opt.adamw_step(p, g, m, v, 4, clip=0.0)[0]
    m2 = 0.9 * m + 0.1 * g; v2 = 0.999 * v + 0.001 * g * g
    no_bias = p * (1 - 3e-4 * 0.01) - 3e-4 * m2 / (np.sqrt(v2) + 1e-8)
    assert np.max(np.abs(no_bias - good)) > 1e-6
