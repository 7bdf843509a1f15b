"""Single GPU kernels against the CPU checker's ops: matrix products in the three layouts and causal
attention forward/backward, at sizes that span several tiles with ragged edges."""
import numpy as np
import pytest
import torch

from oracle import skippipe_oracle as orc
from paper_2502_19913_amd import binding as sp
from paper_2502_19913_amd import synth
from tests.gpuharness import cosine, maxerr, relerr, round_bf16

pytestmark = pytest.mark.gpu


def dev(a, dt):
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).cuda().to(dt)


GEMM_SHAPES = [
    (256, 256, 64), (512, 768, 256), (300, 520, 136), (64, 288, 288), (1, 8, 8), (257, 264, 72),
    (1000, 40, 1024), (128, 864, 288), (2048, 2048, 512), (72, 1032, 2056),
    (4096, 3848, 136),     # enough 256 x 256 tiles for the large-tile path; the smaller shapes take 128 x 128 tiles
]


@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_gemm_three_layouts(M, N, K, dtype):
    dt = torch.bfloat16 if dtype == "bf16" else torch.float32
    rnd = round_bf16 if dtype == "bf16" else (lambda a: a)
    tol = 4e-3 if dtype == "bf16" else 2e-5
    a = rnd(synth.normal(1, f"a{M}{N}{K}", (M, K)))
    b = rnd(synth.normal(2, f"b{M}{N}{K}", (N, K)))
    r = rnd(synth.normal(3, f"r{M}{N}{K}", (M, N)))
    a64, b64, r64 = a.astype(np.float64), b.astype(np.float64), r.astype(np.float64)
    # op 0 with and without the added matrix; reference is the checker's linear (x W^T)
    ref0 = orc.linear_fwd(a64, b64)
    c = torch.full((M, N), 7.0, dtype=dt, device="cuda")
    sp.gemm(0, dev(a, dt), dev(b, dt), c)
    assert relerr(c.float().cpu().numpy(), ref0) < tol
    sp.gemm(0, dev(a, dt), dev(b, dt), c, dev(r, dt))
    assert relerr(c.float().cpu().numpy(), ref0 + r64) < tol
    # op 1: C = A B with B [K, N]; reference dx = dy W of the checker (dy = a, W = b^T stored [K, N])
    bt = np.ascontiguousarray(b.T)                                   # [K, N]
    ref1 = a64 @ bt.astype(np.float64)
    c1 = torch.full((M, N), -3.0, dtype=dt, device="cuda")
    sp.gemm(1, dev(a, dt), dev(bt, dt), c1)
    assert relerr(c1.float().cpu().numpy(), ref1) < tol
    # op 2: C += A^T B with A [K, M], B [K, N]; the checker's dW = dy^T x
    at = np.ascontiguousarray(a.T)                                   # [K, M]
    init = synth.normal(4, f"i{M}{N}{K}", (M, N))
    _, ref2 = orc.linear_bwd(at.astype(np.float64), bt.astype(np.float64), np.zeros((M, N)))
    c2 = dev(init, torch.float32)
    sp.gemm(2, dev(at, dt), dev(bt, dt), c2)
    got2 = c2.cpu().numpy().astype(np.float64) - init
    assert relerr(got2, ref2) < (2e-5 if dtype == "f32" else 2e-5), (relerr(got2, ref2))


def test_gemm_long_reduction_split():
    # the weight-gradient shape: reduction over tokens, few output tiles
    K, M, N = 8192, 512, 264
    a = round_bf16(synth.normal(5, "la", (K, M))); b = round_bf16(synth.normal(6, "lb", (K, N)))
    c = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    sp.gemm(2, dev(a, torch.bfloat16), dev(b, torch.bfloat16), c)
    ref = a.astype(np.float64).T @ b.astype(np.float64)
    assert relerr(c.cpu().numpy(), ref) < 1e-5
    sp.gemm(2, dev(a, torch.bfloat16), dev(b, torch.bfloat16), c)       # accumulates
    assert relerr(c.cpu().numpy(), 2 * ref) < 1e-5


def test_gemm_operand_larger_than_2gib():
    # the widest activations of the 7B-shape stage: 12 microbatches x 4096 tokens x 2 x 11008 hidden is 2.16 GB.
    # Inputs from the device's seeded generator (a host draw of a billion normals would take minutes); sampled
    # output rows are checked against the checker's products on the matching slices.
    R, W, N = 49152 + 8, 22016, 264
    g = torch.Generator(device="cuda"); g.manual_seed(77)
    big = torch.randn((R, W), generator=g, device="cuda", dtype=torch.bfloat16)
    assert big.numel() * 2 > (1 << 31)
    # op 1: C[R, N] = big[R, W] * B[W, N]
    b = round_bf16(synth.normal(7, "bigb", (W, N)))
    c = torch.empty((R, N), dtype=torch.bfloat16, device="cuda")
    sp.gemm(1, big, dev(b, torch.bfloat16), c)
    rows = [0, 255, 256, 30001, 48000, R - 9, R - 1]
    ref = big[rows].float().cpu().numpy().astype(np.float64) @ b.astype(np.float64)
    assert relerr(c[rows].float().cpu().numpy(), ref) < 4e-3
    # op 2: C[W, N] += big[R, W]^T * D[R, N] (big is the k-strided operand)
    d = round_bf16(synth.normal(8, "bigd", (R, N)))
    c2 = torch.zeros((W, N), dtype=torch.float32, device="cuda")
    sp.gemm(2, big, dev(d, torch.bfloat16), c2)
    cols = [0, 7, 300, 11008, 22000, W - 1]
    _, ref2 = orc.linear_bwd(big[:, cols].float().cpu().numpy().astype(np.float64), d.astype(np.float64),
                             np.zeros((len(cols), N)))
    assert relerr(c2[cols].cpu().numpy(), ref2) < 2e-5


FFN_SHAPES = [  # R, h, d: tiles of 256 (h % 128 == 0) and of 128 (h % 64 == 0), ragged rows, ragged reduction,
    (1000, 1280, 264),      # and shapes the fused kernels do not take (h % 64 != 0)
    (4096, 2816, 1024), (300, 192, 72), (5000, 1152, 520), (77, 96, 40), (2560, 5632, 128), (3000, 5632, 200),
]


@pytest.mark.parametrize("R,h,d", FFN_SHAPES)
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_feed_forward_steps_with_swiglu_in_the_epilogue(R, h, d, dtype):
    dt = torch.bfloat16 if dtype == "bf16" else torch.float32
    rnd = round_bf16 if dtype == "bf16" else (lambda a: a)
    tol = 6e-3 if dtype == "bf16" else 3e-5
    hn = rnd(synth.normal(11, f"hn{R}{h}{d}", (R, d)))
    wgu = rnd(synth.normal(12, f"wgu{R}{h}{d}", (2 * h, d), std=2.0 / np.sqrt(d)))
    gu_ref = orc.linear_fwd(hn.astype(np.float64), wgu.astype(np.float64))
    gu = torch.full((R, 2 * h), 9.0, dtype=dt, device="cuda"); act = torch.full((R, h), 9.0, dtype=dt, device="cuda")
    sp.ffn_up_fwd(dev(hn, dt), dev(wgu, dt), gu, act)
    gu_got = gu.float().cpu().numpy()
    assert relerr(gu_got, gu_ref) < tol
    # act is formed from the gu the kernel stored (rounded in bf16 mode): one more rounding on the way out
    assert relerr(act.float().cpu().numpy(), orc.swiglu_fwd(gu_got.astype(np.float64))) < (4e-3 if dtype == "bf16" else 1e-5)
    # backward: d(act) = dy wd, then the SwiGLU gradient against the saved gu
    dy = rnd(synth.normal(13, f"dy{R}{h}{d}", (R, d)))
    wd = rnd(synth.normal(14, f"wd{R}{h}{d}", (d, h), std=1.0 / np.sqrt(d)))
    da_ref = dy.astype(np.float64) @ wd.astype(np.float64)
    dgu_ref = orc.swiglu_bwd(da_ref, gu_got.astype(np.float64))
    dgu = torch.full((R, 2 * h), 9.0, dtype=dt, device="cuda"); scratch = torch.empty((R, h), dtype=dt, device="cuda")
    sp.ffn_down_bwd(dev(dy, dt), dev(wd, dt), gu, dgu, scratch)
    got = dgu.float().cpu().numpy()
    assert relerr(got, dgu_ref) < (8e-3 if dtype == "bf16" else 3e-5), relerr(got, dgu_ref)
    assert maxerr(got, dgu_ref) < (3e-2 if dtype == "bf16" else 1e-4)


def test_gemm_rejects_bad_arguments():
    a = torch.zeros((8, 8), device="cuda")
    with pytest.raises(sp.SpError):
        sp._check(sp.lib().sp_gemm(None, 0, 5, 8, 8, 8, sp._dptr(a), sp._dptr(a), sp._dptr(a), None))
    with pytest.raises(sp.SpError):
        sp._check(sp.lib().sp_gemm(None, 0, 0, 8, 8, 8, None, sp._dptr(a), sp._dptr(a), None))


def test_matrix_core_probe_counts_what_it_runs():
    # all-ones operands: every accumulator entry grows by 32 per MFMA of 32 k, 2 per k-step repeat, and a lane's
    # result is the sum of its 128 accumulator entries
    iters, blocks = 3, 5
    src = torch.ones(4096, dtype=torch.bfloat16, device="cuda")
    sink = torch.zeros(blocks * 512, dtype=torch.float32, device="cuda")
    flops = sp.probe_mfma_rate(src, blocks, iters, sink)
    torch.cuda.synchronize()
    assert flops == blocks * 8 * iters * 64 * 2.0 * 16 * 16 * 32
    assert torch.all(sink == 128.0 * iters * 2 * 32).item()
    with pytest.raises(sp.SpError):
        sp._check(sp.lib().sp_probe_mfma_rate(None, sp._dptr(src), 8192, 0, 1, sp._dptr(sink), None))


ATTN_CASES = [  # B, T, H, Hkv, hd
    (2, 64, 6, 6, 48), (1, 200, 4, 2, 64), (2, 333, 4, 1, 128), (1, 1, 2, 2, 64), (3, 17, 2, 1, 10),
    (1, 512, 2, 2, 128), (1, 640, 4, 4, 64),
]


@pytest.mark.parametrize("B,T,H,Hkv,hd", ATTN_CASES)
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_attention_forward_backward(B, T, H, Hkv, hd, dtype):
    dt = torch.bfloat16 if dtype == "bf16" else torch.float32
    rnd = round_bf16 if dtype == "bf16" else (lambda a: a)
    nq = (H + 2 * Hkv) * hd
    qkv = rnd(synth.normal(7, f"qkv{B}{T}{H}{hd}", (B * T, nq)))
    do = rnd(synth.normal(8, f"do{B}{T}{H}{hd}", (B * T, H * hd)))
    q = np.ascontiguousarray(qkv[:, :H * hd]).reshape(B * T, H, hd).astype(np.float64)
    k = np.ascontiguousarray(qkv[:, H * hd:(H + Hkv) * hd]).reshape(B * T, Hkv, hd).astype(np.float64)
    v = np.ascontiguousarray(qkv[:, (H + Hkv) * hd:]).reshape(B * T, Hkv, hd).astype(np.float64)
    o_ref = orc.attention_fwd(q, k, v, B, T)
    dq, dk, dv = orc.attention_bwd(do.reshape(B * T, H, hd).astype(np.float64), q, k, v, B, T)
    dqkv_ref = np.concatenate([dq.reshape(B * T, -1), dk.reshape(B * T, -1), dv.reshape(B * T, -1)], axis=1)

    d_qkv = dev(qkv, dt)
    o = torch.empty((B * T, H * hd), dtype=dt, device="cuda")
    lse = torch.empty((B, H, T), dtype=torch.float32, device="cuda")
    sp.attention_fwd(d_qkv, o, lse, B, T, H, Hkv, hd)
    o_got = o.float().cpu().numpy().reshape(B * T, H, hd)
    # log-sum-exp against its definition on a few rows
    sc = np.einsum("thd,shd->hts", q[:T], np.repeat(k[:T], H // Hkv, axis=1)) / np.sqrt(hd)
    for i in (0, T // 2, T - 1):
        want = np.log(np.exp(sc[:, i, :i + 1] - sc[:, i, :i + 1].max(-1, keepdims=True)).sum(-1)) + sc[:, i, :i + 1].max(-1)
        assert np.allclose(lse[0, :, i].cpu().numpy(), want, rtol=2e-2 if dtype == "bf16" else 1e-4, atol=2e-2 if dtype == "bf16" else 1e-5)
    if dtype == "f32":
        assert relerr(o_got, o_ref) < 1e-5
    else:
        assert relerr(o_got, o_ref) < 1e-2 and cosine(o_got, o_ref) > 0.9999
    # backward uses the forward's own o (as the stage does)
    dqkv = torch.empty((B * T, nq), dtype=dt, device="cuda")
    delta = torch.empty((B * H * T,), dtype=torch.float32, device="cuda")
    sp.attention_bwd(d_qkv, o, lse, dev(do, dt), dqkv, delta, B, T, H, Hkv, hd)
    got = dqkv.float().cpu().numpy()
    if dtype == "f32":
        assert relerr(got, dqkv_ref) < 2e-5
    else:
        for lo, hi, nm in [(0, H * hd, "dq"), (H * hd, (H + Hkv) * hd, "dk"), ((H + Hkv) * hd, nq, "dv")]:
            if not np.any(dqkv_ref[:, lo:hi]):     # T = 1: dq and dk vanish; only rounding noise may remain
                assert np.abs(got[:, lo:hi]).max() <= 1e-2 * np.abs(dqkv_ref).max(), nm
                continue
            assert cosine(got[:, lo:hi], dqkv_ref[:, lo:hi]) > 0.9995, nm
            assert relerr(got[:, lo:hi], dqkv_ref[:, lo:hi]) < 2e-2, nm
