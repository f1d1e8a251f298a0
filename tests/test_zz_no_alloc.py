"""The norm backward entry point that allocates nothing (its partial sums live in a fixed device array of the
library) against the existing entry point with caller-provided scratch: same kernels, so the outputs must be
identical bit for bit -- on two calls in a row, the second on a smaller input, which also shows that the shared array
needs no clearing between calls.  The file name sorts last on purpose: a failure here must not hide the other GPU tests."""
import ctypes as C

import numpy as np
import pytest

from paper_2507_00217_amd import synth
from tests.gpu_util import rnd, to_dev

pytestmark = pytest.mark.gpu
DT = {"fp32": 0, "bf16": 1}


def L():
    from paper_2507_00217_amd import stage as S
    lib = S.lib()
    vp, i = C.c_void_p, C.c_int
    lib.stage_kernel_norm_fwd.argtypes = [i, i, i, i, C.c_float, vp, vp, vp, vp, vp, vp]
    lib.stage_kernel_norm_bwd.argtypes = [i, i, i, i] + [vp] * 10
    lib.stage_kernel_norm_bwd_noalloc.argtypes = [i, i, i, i] + [vp] * 9
    lib.stage_kernel_norm_partial_bytes.restype = C.c_size_t
    return lib


def P(t):
    return None if t is None else t.data_ptr()


def _both(dtype, kind, rows, d, seed):
    """Runs the two entry points on the same inputs; returns (dx, dgamma, dbeta) of each."""
    import torch
    x = rnd(synth.normal(seed, 1, (rows, d), mean=0.3, std=2.0), dtype)
    gamma = rnd(synth.normal(seed, 2, (d,), mean=1.0, std=0.1), dtype); beta = rnd(synth.normal(seed, 3, (d,), std=0.1), dtype)
    dout = rnd(synth.normal(seed, 4, (rows, d)), dtype); resid = rnd(synth.normal(seed, 5, (rows, d)), dtype)
    dg0, db0 = synth.normal(seed, 6, (d,)), synth.normal(seed, 7, (d,))
    xd, gd, bd, doutd, residd = (to_dev(t, dtype) for t in (x, gamma, beta, dout, resid))
    st = torch.zeros((rows, 2), dtype=torch.float32, device="cuda:0")
    outd = torch.zeros_like(xd)
    assert L().stage_kernel_norm_fwd(DT[dtype], kind, rows, d, 1e-5, P(xd), P(gd), P(bd), P(outd), P(st), None) == 0
    res = []
    for noalloc in (False, True):
        dxd = torch.zeros_like(xd)
        dgd, dbd = to_dev(dg0, "fp32"), to_dev(db0, "fp32")
        if noalloc:
            rc = L().stage_kernel_norm_bwd_noalloc(DT[dtype], kind, rows, d, P(xd), P(st), P(gd), P(doutd), P(residd), P(dxd),
                                                   P(dgd), P(dbd), None)
        else:
            part = torch.zeros(L().stage_kernel_norm_partial_bytes(d) // 4, dtype=torch.float32, device="cuda:0")
            rc = L().stage_kernel_norm_bwd(DT[dtype], kind, rows, d, P(xd), P(st), P(gd), P(doutd), P(residd), P(dxd),
                                           P(dgd), P(dbd), P(part), None)
        assert rc == 0
        torch.cuda.synchronize()
        res.append((dxd, dgd, dbd))
    return res, (dg0, db0)


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("norm", ["layernorm", "rmsnorm"])
def test_norm_bwd_noalloc_matches_the_workspace_entry_point(dtype, norm):
    import torch
    kind = {"layernorm": 0, "rmsnorm": 1}[norm]
    big_d = 8192 if dtype == "bf16" else 4096
    for rows, d, seed in ((1500, big_d, 11), (333, 1024, 12)):        # two calls in a row, the second smaller
        (ref, got), (dg0, db0) = _both(dtype, kind, rows, d, seed)
        for a, b in zip(ref, got):
            assert torch.equal(a, b)
        # and the call did something: gradients moved away from their initial values
        assert not np.array_equal(got[1].cpu().numpy(), dg0)
        if norm == "layernorm":
            assert not np.array_equal(got[2].cpu().numpy(), db0)


def test_norm_bwd_noalloc_rejects_rows_wider_than_its_scratch():
    import torch
    t = torch.zeros(16384, dtype=torch.float32, device="cuda:0")
    assert L().stage_kernel_norm_bwd_noalloc(1, 1, 1, 8192 + 8, P(t), P(t), P(t), P(t), None, P(t), P(t), P(t), None) == -1
    assert L().stage_kernel_norm_bwd_noalloc(1, 1, 1, 512, None, P(t), P(t), P(t), None, P(t), P(t), P(t), None) == -1
