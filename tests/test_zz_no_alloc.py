"""The allocation-free variant of the update, sp_optim_step_noalloc, against sp_optim_step through the C
boundary: same kernels on the library's static device scratch, so every output must agree bit for bit (the
norm is summed in a fixed order).  Two calls in a row, the second on a smaller input, so that what the first
call left in the shared scratch is seen not to leak into the second."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2502_19913_amd import binding as sp
from paper_2502_19913_amd import synth

pytestmark = pytest.mark.gpu


def _state(n, seed):
    g = torch.from_numpy(synth.normal(seed, "g", (n,), std=0.3)).cuda()
    p = torch.from_numpy(synth.normal(seed, "p", (n,), std=0.02)).cuda()
    m = torch.from_numpy(synth.normal(seed, "m", (n,), std=0.01)).cuda()
    v = torch.from_numpy(synth.normal(seed, "v", (n,), std=0.01)).cuda().abs()
    return p, g, m, v


def _both(n, seed, step, out_dtype):
    ws = torch.empty(sp.optim_workspace_bytes(), dtype=torch.uint8, device="cuda")
    res = []
    for noalloc in (False, True):
        p, g, m, v = _state(n, seed)
        lp = torch.zeros(n, dtype=out_dtype, device="cuda")
        norm = torch.zeros(1, device="cuda")
        if noalloc:
            sp.optim_step_noalloc(p, g, m, v, step, params_out=lp, grad_norm=norm, clip_norm=1.0)
        else:
            sp.optim_step(p, g, m, v, step, params_out=lp, workspace=ws, grad_norm=norm, clip_norm=1.0)
        torch.cuda.synchronize()
        res.append((p.cpu(), m.cpu(), v.cpu(), lp.float().cpu(), norm.cpu()))
    return res


def test_noalloc_update_matches_the_workspace_entry_point_twice_in_a_row():
    # first call: 3 000 003 elements (ragged tail, 2048 norm partials in use); second: 1 237 (5 partials), so
    # most of the scratch still holds the first call's partials when the second runs
    for n, seed, step, dt in ((3_000_003, 41, 1, torch.bfloat16), (1_237, 42, 7, torch.float32)):
        a, b = _both(n, seed, step, dt)
        for x, y, what in zip(a, b, ("master", "m", "v", "low-precision copy", "norm")):
            assert torch.equal(x, y), (n, what)
        assert float(a[4]) > 1.0          # the clip was active: the norm entered the update


def test_noalloc_update_rejects_sizes_beyond_its_maximum_and_bad_arguments():
    p, g, m, v = _state(16, 43)
    h = sp.SpAdamW(3e-4, 0.9, 0.999, 1e-8, 0.01, 1.0)
    rc = sp.lib().sp_optim_step_noalloc(C.c_void_p(0), C.byref(h), C.c_int64((1 << 32) + 1), C.c_int(1), sp._dptr(p),
                                        sp._dptr(g), sp._dptr(m), sp._dptr(v), C.c_void_p(0), C.c_int(0), C.c_void_p(0))
    assert rc == -1 and b"2^32" in sp.lib().sp_strerror(C.c_int(rc))
    with pytest.raises(sp.SpError):
        sp.optim_step_noalloc(p, g, m, v, 0)
    before = p.clone()
    sp.optim_step_noalloc(p, g, m, v, 1)
    torch.cuda.synchronize()
    assert not torch.equal(p, before)
