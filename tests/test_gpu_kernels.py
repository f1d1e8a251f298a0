"""Each step of the path, called alone through the C ABI, against the oracle's
building block for that step."""
import ctypes as C
import math

import numpy as np
import pytest

from oracle import stage_oracle as so
from paper_2507_00217_amd import synth
from tests.gpu_util import rnd, to_dev, to_np

pytestmark = pytest.mark.gpu
DT = {"fp32": 0, "bf16": 1}
KTOL = {"fp32": 2e-5, "bf16": 1e-2}


def L():
    from paper_2507_00217_amd import stage as S
    lib = S.lib()
    if not hasattr(lib, "_ksig"):
        vp, i, i64, fl = C.c_void_p, C.c_int, C.c_int64, C.c_float
        lib.stage_kernel_gemm.argtypes = [i, i, i, i, i, vp, i64, vp, i64, vp, i64, vp, i64, i, i, vp]
        lib.stage_kernel_gemm_act.argtypes = [i, i, i, i, i, vp, i64, vp, i64, vp, i64, vp, i64, i, vp]
        lib.stage_kernel_gemm_act_bwd.argtypes = [i, i, i, i, i, vp, i64, vp, i64, vp, i64, vp, i, vp]
        lib.stage_kernel_wgrad_group.argtypes = [i, i] + [vp] * 9 + [i, vp]
        lib.stage_kernel_rope_table.argtypes = [i, i, fl, vp, vp]
        lib.stage_kernel_rope.argtypes = [i, i, i, i, i, i, vp, i64, vp, vp]
        lib.stage_kernel_attention_fwd.argtypes = [i] * 7 + [vp, vp, vp, i, vp]
        lib.stage_kernel_attention_bwd.argtypes = [i] * 7 + [vp] * 6 + [i, vp]
        lib.stage_kernel_attention_bwd_ws.argtypes = [i] * 7 + [vp] * 7 + [C.c_size_t, i, vp]
        lib.stage_kernel_attention_bwd_scratch_bytes.argtypes = [i] * 5
        lib.stage_kernel_attention_bwd_scratch_bytes.restype = C.c_size_t
        lib.stage_kernel_norm_fwd.argtypes = [i, i, i, i, fl, vp, vp, vp, vp, vp, vp]
        lib.stage_kernel_norm_bwd.argtypes = [i, i, i, i] + [vp] * 10
        lib.stage_kernel_norm_partial_bytes.restype = C.c_size_t
        lib.stage_kernel_bias_grad.argtypes = [i, i, i, vp, i64, vp, vp, vp]
        lib.stage_kernel_bias_grad_scratch_bytes.argtypes = [i]
        lib.stage_kernel_bias_grad_scratch_bytes.restype = C.c_size_t
        lib.stage_kernel_act_fwd.argtypes = [i, i, i, i, vp, vp, vp]
        lib.stage_kernel_act_bwd.argtypes = [i, i, i, i, vp, vp, vp]
        lib._ksig = True
    return lib


def P(t):
    return None if t is None else t.data_ptr()


GEMM_SHAPES = [(128, 256, 768), (200, 192, 136), (328, 1088, 512), (512, 512, 2048), (257, 320, 72), (1024, 768, 264),
               (136, 72, 64), (72, 136, 128), (264, 136, 192),      # one, two and three K tiles (the pipeline's start-up and tail alone)
               (200, 136, 256), (136, 264, 320)]                    # four and five: the 128 x 128 tile's ring is four K tiles deep


@pytest.mark.parametrize("dtype,kernel_set", [("fp32", 0), ("fp32", 1), ("bf16", 0), ("bf16", 1), ("bf16", 2), ("bf16", 3), ("bf16", 4)])
@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm(dtype, mode, kernel_set, M, N, K):
    """kernel_set 2 / 3 / 4: the tuned kernel with full 256 x 256 tiles only / half-height tiles only / 128 x 128 tiles only
    (0 picks by shape; weight gradients have full tiles only)."""
    import torch
    a_shape = (K, M) if mode == 2 else (M, K)
    b_shape = (N, K) if mode == 1 else (K, N)
    A = rnd(synth.normal(1, 1, a_shape), dtype); Bm = rnd(synth.normal(1, 2, b_shape), dtype)
    R = rnd(synth.normal(1, 3, (M, N)), dtype)
    C0 = synth.normal(1, 4, (M, N))
    Ad, Bd, Rd = to_dev(A, dtype), to_dev(Bm, dtype), to_dev(R, dtype)
    A64, B64 = A.astype(np.float64), Bm.astype(np.float64)
    prod = (A64.T if mode == 2 else A64) @ (B64.T if mode == 1 else B64)
    if mode == 2:
        Cd = to_dev(C0, "fp32")
        ref = C0.astype(np.float64) + prod
        rc = L().stage_kernel_gemm(DT[dtype], mode, M, N, K, P(Ad), M, P(Bd), N, P(Cd), N, None, 0, 1, kernel_set, None)
    else:
        use_r = mode == 0
        Cd = torch.zeros((M, N), dtype=Ad.dtype, device="cuda:0")
        ref = prod + (R if use_r else 0)
        rc = L().stage_kernel_gemm(DT[dtype], mode, M, N, K, P(Ad), K, P(Bd), K if mode == 1 else N, P(Cd), N,
                                   P(Rd) if use_r else None, N, 0, kernel_set, None)
    assert rc == 0
    torch.cuda.synchronize()
    assert so.max_rel_err(to_np(Cd), ref) <= (KTOL[dtype] if mode != 2 else 2e-5 if dtype == "fp32" else 1e-5 * math.sqrt(K))


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("M,N,K", [(1160, 2304, 320), (520, 1088, 512), (1280, 5376, 192), (4352, 4104, 128)])
def test_gemm_tile_shapes_agree_bitwise(mode, M, N, K):
    """Full tiles, half-height tiles, 128 x 128 tiles and the mix chosen from the shape give the same bits: every output
    element is the same sequence of MFMAs over K whichever tile it falls in.  (The third shape has 105 full tiles and the first 45:
    with forced shapes both kernels see ragged edges in M and N; the last one has 17 x 17 = 289 full tiles on 256 CUs, so the
    rule gives its last 33 tiles to the 128 x 128 kernel.)"""
    import torch
    A = rnd(synth.normal(11, 1, (M, K)), "bf16"); Bm = rnd(synth.normal(11, 2, (N, K) if mode == 1 else (K, N)), "bf16")
    R = rnd(synth.normal(11, 3, (M, N)), "bf16")
    Ad, Bd, Rd = to_dev(A, "bf16"), to_dev(Bm, "bf16"), to_dev(R, "bf16")
    outs = []
    for ks in (2, 3, 4, 0):
        Cd = torch.zeros((M, N), dtype=Ad.dtype, device="cuda:0")
        rc = L().stage_kernel_gemm(DT["bf16"], mode, M, N, K, P(Ad), K, P(Bd), K if mode == 1 else N, P(Cd), N,
                                   P(Rd) if mode == 0 else None, N, 0, ks, None)
        assert rc == 0
        outs.append(Cd)
    torch.cuda.synchronize()
    assert all(torch.equal(outs[0], o) for o in outs[1:])


@pytest.mark.parametrize("dtype,kernel_set", [("fp32", 0), ("bf16", 0), ("bf16", 1), ("bf16", 2), ("bf16", 3)])
@pytest.mark.parametrize("act", ["gelu", "swiglu"])
@pytest.mark.parametrize("M,f,K", [(128, 256, 128), (200, 192, 192), (328, 1088, 512), (257, 1408, 64), (512, 64, 256), (1024, 704, 320)])
def test_gemm_with_fused_activation(dtype, kernel_set, act, M, f, K):
    """The forward FFN-in product and its activation in one call: Z against the product's definition, Aout against the
    oracle's activation of the exact product (the tuned kernel forms it from fp32 accumulators; the plain kernels from
    the stored Z).  Ragged tiles in every dimension; kernel_set 2 / 3 force full / half-height tiles."""
    import torch
    kind = {"gelu": 0, "swiglu": 1}[act]
    fin = 2 * f if act == "swiglu" else f
    A = rnd(synth.normal(7, 1, (M, K)), dtype); Bm = rnd(synth.normal(7, 2, (K, fin), std=1.5 / math.sqrt(K)), dtype)
    Ad, Bd = to_dev(A, dtype), to_dev(Bm, dtype)
    z_ref = A.astype(np.float64) @ Bm.astype(np.float64)
    sh = so.Shape(1, 64, 1, 1, f, 1, 1, act=act)
    a_ref = so.gelu(z_ref) if act == "gelu" else z_ref[:, :f] * so.sigmoid(z_ref[:, :f]) * z_ref[:, f:]
    tdt = torch.float32 if dtype == "fp32" else torch.bfloat16
    Zd = torch.full((M, fin), float("nan"), dtype=tdt, device="cuda:0")
    Aout = torch.full((M, f), float("nan"), dtype=tdt, device="cuda:0")
    rc = L().stage_kernel_gemm_act(DT[dtype], kind, M, f, K, P(Ad), K, P(Bd), fin, P(Zd), fin, P(Aout), f, kernel_set, None)
    assert rc == 0
    torch.cuda.synchronize()
    assert so.max_rel_err(to_np(Zd), z_ref) <= KTOL[dtype]
    assert so.max_rel_err(to_np(Aout), a_ref) <= KTOL[dtype]
    if dtype == "bf16" and kernel_set != 1:
        # one rounding only: the fused activation is the rounded activation of the (fp32) product, not of the rounded Z
        a_once = synth.round_bf16(a_ref.astype(np.float32)).astype(np.float64)
        assert np.mean(to_np(Aout) == a_once) > 0.97
    assert L().stage_kernel_gemm_act(DT[dtype], 5, M, f, K, P(Ad), K, P(Bd), fin, P(Zd), fin, P(Aout), f, kernel_set, None) == -1
    assert L().stage_kernel_gemm_act(DT[dtype], kind, M, f, K, P(Ad), K, P(Bd), fin, None, fin, P(Aout), f, kernel_set, None) == -1


@pytest.mark.parametrize("dtype,kernel_set", [("fp32", 0), ("bf16", 0), ("bf16", 1), ("bf16", 2), ("bf16", 3)])
@pytest.mark.parametrize("act", ["gelu", "swiglu"])
@pytest.mark.parametrize("M,f,K", [(128, 256, 128), (200, 192, 192), (328, 1088, 512), (257, 1408, 64), (512, 64, 256), (1024, 704, 320)])
def test_gemm_with_fused_activation_backward(dtype, kernel_set, act, M, f, K):
    """The FFN-out map's input-gradient product and the activation backward in one call: Z becomes dZ in place, against
    the oracle's act_backward of the exact product.  Ragged tiles in every dimension; both tile shapes."""
    import torch
    kind = {"gelu": 0, "swiglu": 1}[act]
    fin = 2 * f if act == "swiglu" else f
    dY = rnd(synth.normal(9, 1, (M, K)), dtype); Wm = rnd(synth.normal(9, 2, (f, K), std=1.5 / math.sqrt(K)), dtype)
    Z = rnd(synth.normal(9, 3, (M, fin), std=1.5), dtype)
    sh = so.Shape(1, 64, 1, 1, f, 1, 1, act=act)
    da_ref = dY.astype(np.float64) @ Wm.astype(np.float64).T
    dz_ref = so.act_backward(sh, Z.astype(np.float64), da_ref)
    tdt = torch.float32 if dtype == "fp32" else torch.bfloat16
    Zd, dYd, Wd = to_dev(Z, dtype), to_dev(dY, dtype), to_dev(Wm, dtype)
    guard = torch.full((M, f), 7.0, dtype=tdt, device="cuda:0")
    rc = L().stage_kernel_gemm_act_bwd(DT[dtype], kind, M, f, K, P(dYd), K, P(Wd), K, P(Zd), fin, P(guard), kernel_set, None)
    assert rc == 0
    torch.cuda.synchronize()
    assert so.max_rel_err(to_np(Zd), dz_ref) <= KTOL[dtype]
    if dtype == "bf16" and kernel_set != 1:
        assert bool((guard == 7.0).all())                  # the tuned kernel stores no da
        dz_once = synth.round_bf16(dz_ref.astype(np.float32)).astype(np.float64)
        assert np.mean(to_np(Zd) == dz_once) > 0.97        # one rounding: from the fp32 product, not from a rounded da
    assert L().stage_kernel_gemm_act_bwd(DT[dtype], 3, M, f, K, P(Zd), K, P(Zd), K, P(Zd), fin, P(guard), kernel_set, None) == -1
    assert L().stage_kernel_gemm_act_bwd(DT[dtype], kind, M, f, K, P(Zd), K, P(Zd), K, None, fin, P(guard), kernel_set, None) == -1


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("kernel_set", [0, 1])
def test_wgrad_group(dtype, kernel_set):
    """Several weight-gradient products C_p += A_p^T.B_p in one call (the W block of Appendix B for several linear
    maps): against the definition, and bit for bit against one stage_kernel_gemm call per product.  The shapes give
    about 300 tiles of 256 x 256 with ragged edges, so the persistent workgroups of the tuned kernel each take more
    than one tile and cross from one product to the next."""
    import torch
    shapes = [(520, 1088, 328), (256, 256, 64), (1536, 2304, 200), (768, 3080, 136), (264, 72, 512), (2560, 5120, 72)]
    n = len(shapes)
    As, Bs, Cs, C1, refs = [], [], [], [], []
    for p, (M, N, K) in enumerate(shapes):
        A = rnd(synth.normal(5, 3 * p, (K, M)), dtype); Bm = rnd(synth.normal(5, 3 * p + 1, (K, N)), dtype)
        C0 = synth.normal(5, 3 * p + 2, (M, N))
        As.append(to_dev(A, dtype)); Bs.append(to_dev(Bm, dtype))
        Cs.append(to_dev(C0, "fp32")); C1.append(to_dev(C0, "fp32"))
        refs.append(C0.astype(np.float64) + A.astype(np.float64).T @ Bm.astype(np.float64))
    ia = lambda v: (C.c_int * n)(*v)
    la = lambda v: (C.c_int64 * n)(*v)
    pa = lambda ts: (C.c_void_p * n)(*[t.data_ptr() for t in ts])
    Ms, Ns, Ks = zip(*shapes)
    rc = L().stage_kernel_wgrad_group(DT[dtype], n, ia(Ms), ia(Ns), ia(Ks), pa(As), la(Ms), pa(Bs), la(Ns), pa(Cs), la(Ns),
                                      kernel_set, None)
    assert rc == 0
    for p, (M, N, K) in enumerate(shapes):
        assert L().stage_kernel_gemm(DT[dtype], 2, M, N, K, P(As[p]), M, P(Bs[p]), N, P(C1[p]), N, None, 0, 1, kernel_set, None) == 0
    torch.cuda.synchronize()
    for p, (M, N, K) in enumerate(shapes):
        assert so.max_rel_err(to_np(Cs[p]), refs[p]) <= (2e-5 if dtype == "fp32" else 1e-5 * math.sqrt(K)), p
        assert torch.equal(Cs[p], C1[p]), p
    assert L().stage_kernel_wgrad_group(DT[dtype], 0, None, None, None, None, None, None, None, None, None, kernel_set, None) == 0
    assert L().stage_kernel_wgrad_group(DT[dtype], -1, ia(Ms), ia(Ns), ia(Ks), pa(As), la(Ms), pa(Bs), la(Ns), pa(Cs), la(Ns), 0, None) == -1
    assert L().stage_kernel_wgrad_group(DT[dtype], n, ia(Ms), ia(Ns), ia(Ks), None, la(Ms), pa(Bs), la(Ns), pa(Cs), la(Ns), 0, None) == -1


def test_gemm_rejects_bad_arguments():
    import torch
    t = torch.zeros(64, 64, device="cuda:0")
    assert L().stage_kernel_gemm(0, 2, 64, 64, 64, P(t), 64, P(t), 64, P(t), 64, None, 0, 0, 0, None) == -1   # wgrad needs acc
    assert L().stage_kernel_gemm(0, 0, 64, 64, 64, None, 64, P(t), 64, P(t), 64, None, 0, 0, 0, None) == -1
    assert L().stage_kernel_gemm(7, 0, 64, 64, 64, P(t), 64, P(t), 64, P(t), 64, None, 0, 0, 0, None) == -1


ATT_SHAPES = [(1, 128, 4, 4, 64), (2, 200, 5, 5, 128), (1, 392, 8, 1, 128), (1, 448, 4, 2, 128), (1, 1, 2, 1, 64), (1, 640, 2, 2, 64),
              (3, 300, 2, 1, 128)]


@pytest.mark.parametrize("dtype,kernel_set", [("fp32", 0), ("fp32", 1), ("bf16", 0), ("bf16", 1), ("bf16", 2), ("bf16", 3), ("bf16", 4)])
@pytest.mark.parametrize("causal", [1, 0])
@pytest.mark.parametrize("b,s,h,hkv,hd", ATT_SHAPES)
def test_attention(dtype, kernel_set, causal, b, s, h, hkv, hd):
    """kernel_set 2 / 3 / 4: the tuned kernels with one workgroup shape forced (0 picks by shape): forward and dQ with 8
    wavefronts, with 4, or with 4 that split each query block's keys in two; dK/dV with 128 keys per workgroup (2, 3) or
    64 (4)."""
    import torch
    d, dkv = h * hd, hkv * hd
    qkv = rnd(synth.normal(2, 1, (b, s, d + 2 * dkv)), dtype)
    do = rnd(synth.normal(2, 2, (b, s, d)), dtype)
    sh = so.Shape(1, d, h, hkv, 64, s, b, causal=bool(causal))
    q = qkv[..., :d].astype(np.float64).reshape(b, s, h, hd)
    k = qkv[..., d:d + dkv].astype(np.float64).reshape(b, s, hkv, hd)
    v = qkv[..., d + dkv:].astype(np.float64).reshape(b, s, hkv, hd)
    o_ref = so.attention_forward(sh, q, k, v)
    qd = to_dev(qkv, dtype)
    od = torch.zeros((b, s, d), dtype=qd.dtype, device="cuda:0")
    lse = torch.zeros((b, h, s), dtype=torch.float32, device="cuda:0")
    assert L().stage_kernel_attention_fwd(DT[dtype], b, s, h, hkv, hd, causal, P(qd), P(od), P(lse), kernel_set, None) == 0
    torch.cuda.synchronize()
    tol = KTOL[dtype] if dtype == "bf16" else 5e-5
    assert so.max_rel_err(to_np(od), o_ref.reshape(b, s, d)) <= tol
    # log-sum-exp of the scaled masked scores, from its definition
    j = h - 1
    S = q[0, :, j] @ k[0, :, j // (h // hkv)].T / math.sqrt(hd)
    if causal:
        S = np.where(np.tril(np.ones((s, s), bool)), S, -np.inf)
    lse_ref = np.log(np.exp(S - S.max(-1, keepdims=True)).sum(-1)) + S.max(-1)
    assert np.abs(to_np(lse[0, j]) - lse_ref).max() <= (1e-4 if dtype == "fp32" else 2e-2)
    # backward consumes the device's own o / lse, like the stage does
    dod = to_dev(do, dtype)
    dqkv = torch.zeros_like(qd)
    delta = torch.zeros((b, h, s), dtype=torch.float32, device="cuda:0")
    assert L().stage_kernel_attention_bwd(DT[dtype], b, s, h, hkv, hd, causal, P(qd), P(od), P(lse), P(dod), P(dqkv),
                                          P(delta), kernel_set, None) == 0
    torch.cuda.synchronize()
    dq, dk, dv = so.attention_backward(sh, q, k, v, do.astype(np.float64).reshape(b, s, h, hd))
    got = to_np(dqkv)
    assert so.max_rel_err(got[..., :d], dq.reshape(b, s, d)) <= tol
    assert so.max_rel_err(got[..., d:d + dkv], dk.reshape(b, s, dkv)) <= tol
    assert so.max_rel_err(got[..., d + dkv:], dv.reshape(b, s, dkv)) <= tol


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("b,s,h,hkv,hd,theta", [(2, 200, 5, 1, 128, 10000.0), (1, 333, 4, 4, 64, 500000.0), (1, 4096, 2, 1, 128, 10000.0)])
def test_rope(dtype, b, s, h, hkv, hd, theta):
    """Rotary embedding of the q and k heads of a qkv buffer in place (v untouched), and its transpose, against the
    oracle's definition; forward then transpose gives back the input up to rounding."""
    import torch
    nh, ld = h + hkv, (h + 2 * hkv) * hd
    x = rnd(synth.normal(7, 1, (b, s, ld)), dtype)
    sh = so.Shape(1, h * hd, h, hkv, 64, s, b, rope_theta=theta)
    table = torch.zeros((s, hd // 2, 2), dtype=torch.float32, device="cuda:0")
    assert L().stage_kernel_rope_table(s, hd, theta, P(table), None) == 0
    torch.cuda.synchronize()
    ang = np.arange(s)[:, None] * theta ** (-2.0 * np.arange(hd // 2) / hd)[None, :]
    assert np.abs(table.cpu().numpy()[..., 0] - np.cos(ang)).max() <= 1e-7 and np.abs(table.cpu().numpy()[..., 1] - np.sin(ang)).max() <= 1e-7
    for inverse in (0, 1):
        xd = to_dev(x, dtype)
        assert L().stage_kernel_rope(DT[dtype], b, s, nh, hd, inverse, P(xd), ld, P(table), None) == 0
        torch.cuda.synchronize()
        got = to_np(xd)
        ref = x.astype(np.float64).copy()
        ref[..., :nh * hd] = so.rope(sh, ref[..., :nh * hd].reshape(b, s, nh, hd), inverse=bool(inverse)).reshape(b, s, nh * hd)
        assert np.array_equal(got[..., nh * hd:], x[..., nh * hd:].astype(got.dtype))
        assert so.max_rel_err(got, ref) <= (1e-6 if dtype == "fp32" else 4e-3)
    assert L().stage_kernel_rope(DT[dtype], b, s, nh, hd, 0, P(xd), nh * hd - 8, P(table), None) == -1
    assert L().stage_kernel_rope_table(s, 96, theta, P(table), None) == -1


@pytest.mark.parametrize("kernel_set", [0, 3, 4])
@pytest.mark.parametrize("causal", [1, 0])
@pytest.mark.parametrize("b,s,h,hkv,hd", [(1, 392, 8, 1, 128), (2, 300, 12, 2, 64), (1, 448, 4, 2, 128)])
def test_attention_bwd_with_split_query_heads(kernel_set, causal, b, s, h, hkv, hd):
    """Grouped-query dK/dV with each KV head's query heads split over several workgroups (fp32 partials in caller
    scratch, summed in a fixed order): against the oracle, and equal to the unsplit pass up to the one extra bf16
    rounding order.  kernel_set 3 / 4: 128 / 64 keys per workgroup (0 picks by shape)."""
    import torch
    d, dkv = h * hd, hkv * hd
    qkv = rnd(synth.normal(6, 1, (b, s, d + 2 * dkv)), "bf16")
    do = rnd(synth.normal(6, 2, (b, s, d)), "bf16")
    sh = so.Shape(1, d, h, hkv, 64, s, b, causal=bool(causal))
    q = qkv[..., :d].astype(np.float64).reshape(b, s, h, hd)
    k = qkv[..., d:d + dkv].astype(np.float64).reshape(b, s, hkv, hd)
    v = qkv[..., d + dkv:].astype(np.float64).reshape(b, s, hkv, hd)
    qd, dod = to_dev(qkv, "bf16"), to_dev(do, "bf16")
    od = torch.zeros((b, s, d), dtype=qd.dtype, device="cuda:0")
    lse = torch.zeros((b, h, s), dtype=torch.float32, device="cuda:0")
    assert L().stage_kernel_attention_fwd(1, b, s, h, hkv, hd, causal, P(qd), P(od), P(lse), 0, None) == 0
    nbytes = L().stage_kernel_attention_bwd_scratch_bytes(b, s, h, hkv, hd)
    assert nbytes > 0 and nbytes % (b * s * 2 * dkv * 4) == 0
    scratch = torch.zeros(nbytes, dtype=torch.uint8, device="cuda:0")
    delta = torch.zeros((b, h, s), dtype=torch.float32, device="cuda:0")
    outs = []
    for use in (True, False):
        dqkv = torch.zeros_like(qd)
        rc = L().stage_kernel_attention_bwd_ws(1, b, s, h, hkv, hd, causal, P(qd), P(od), P(lse), P(dod), P(dqkv), P(delta),
                                               P(scratch) if use else None, nbytes if use else 0, kernel_set, None)
        assert rc == 0
        torch.cuda.synchronize()
        outs.append(to_np(dqkv))
    dq, dk, dv = so.attention_backward(sh, q, k, v, do.astype(np.float64).reshape(b, s, h, hd))
    ref = np.concatenate([dq.reshape(b, s, d), dk.reshape(b, s, dkv), dv.reshape(b, s, dkv)], axis=-1)
    for got in outs:
        for lo, hi in ((0, d), (d, d + dkv), (d + dkv, d + 2 * dkv)):
            assert so.max_rel_err(got[..., lo:hi], ref[..., lo:hi]) <= KTOL["bf16"]
    assert np.array_equal(outs[0][..., :d], outs[1][..., :d])              # dQ does not depend on the split
    assert L().stage_kernel_attention_bwd_ws(1, b, s, h, hkv, hd, causal, P(qd), P(od), P(lse), P(dod), P(dqkv), P(delta),
                                             P(scratch), nbytes - 16, 0, None) == -1


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("norm", ["layernorm", "rmsnorm"])
@pytest.mark.parametrize("rows,d", [(128, 256), (333, 1024), (64, 4096), (1000, 640), (3, 8192)])
def test_norm(dtype, norm, rows, d):
    import torch
    kind = {"layernorm": 0, "rmsnorm": 1}[norm]
    if dtype == "fp32" and d > 4096:
        # a row must fit a workgroup's registers (1024 16-byte pieces): wider fp32 rows are refused, nothing is launched
        t = torch.zeros(rows * d, dtype=torch.float32, device="cuda:0")
        assert L().stage_kernel_norm_fwd(DT[dtype], kind, rows, d, 1e-5, P(t), P(t), P(t), P(t), P(t), None) == -1
        return
    x = rnd(synth.normal(3, 1, (rows, d), mean=0.3, std=2.0), dtype)
    gamma = rnd(synth.normal(3, 2, (d,), mean=1.0, std=0.1), dtype); beta = rnd(synth.normal(3, 3, (d,), std=0.1), dtype)
    dout = rnd(synth.normal(3, 4, (rows, d)), dtype); resid = rnd(synth.normal(3, 5, (rows, d)), dtype)
    out_ref, stats = so.norm_forward(norm, x.astype(np.float64), gamma.astype(np.float64), beta.astype(np.float64), 1e-5)
    dx_ref, dg_ref, db_ref = so.norm_backward(norm, stats, gamma.astype(np.float64), dout.astype(np.float64))
    xd, gd, bd = to_dev(x, dtype), to_dev(gamma, dtype), to_dev(beta, dtype)
    outd = torch.zeros_like(xd); st = torch.zeros((rows, 2), dtype=torch.float32, device="cuda:0")
    assert L().stage_kernel_norm_fwd(DT[dtype], kind, rows, d, 1e-5, P(xd), P(gd), P(bd), P(outd), P(st), None) == 0
    torch.cuda.synchronize()
    assert so.max_rel_err(to_np(outd), out_ref) <= KTOL[dtype]
    assert so.max_rel_err(to_np(st[:, 1]), stats[1][:, 0]) <= 1e-5
    dg0 = synth.normal(3, 6, (d,)); db0 = synth.normal(3, 7, (d,))
    dgd, dbd = to_dev(dg0, "fp32"), to_dev(db0, "fp32")
    part = torch.zeros(L().stage_kernel_norm_partial_bytes(d) // 4, dtype=torch.float32, device="cuda:0")
    dxd = xd.clone()     # in place over x, as the stage uses it
    doutd, residd = to_dev(dout, dtype), to_dev(resid, dtype)      # named: the buffers must outlive the launch
    assert L().stage_kernel_norm_bwd(DT[dtype], kind, rows, d, P(dxd), P(st), P(gd), P(doutd),
                                     P(residd), P(dxd), P(dgd), P(dbd), P(part), None) == 0
    torch.cuda.synchronize()
    assert so.max_rel_err(to_np(dxd), dx_ref + resid) <= KTOL[dtype]
    assert so.max_rel_err(to_np(dgd) - dg0, dg_ref) <= (1e-5 if dtype == "fp32" else 2e-3)
    if norm == "layernorm":
        assert so.max_rel_err(to_np(dbd) - db0, db_ref) <= 1e-5
    else:
        assert np.array_equal(to_np(dbd), db0.astype(np.float64))


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("act", ["gelu", "swiglu"])
@pytest.mark.parametrize("rows,f", [(128, 1024), (77, 1408), (5, 64)])
def test_activation(dtype, act, rows, f):
    import torch
    kind = {"gelu": 0, "swiglu": 1}[act]
    fin = 2 * f if act == "swiglu" else f
    z = rnd(synth.normal(4, 1, (rows, fin), std=2.0), dtype); da = rnd(synth.normal(4, 2, (rows, f)), dtype)
    sh = so.Shape(1, 64, 1, 1, f, 1, 1, act=act)
    z64 = z.astype(np.float64)
    a_ref = so.gelu(z64) if act == "gelu" else z64[:, :f] * so.sigmoid(z64[:, :f]) * z64[:, f:]
    dz_ref = so.act_backward(sh, z64, da.astype(np.float64))
    zd = to_dev(z, dtype); ad = torch.zeros((rows, f), dtype=zd.dtype, device="cuda:0")
    assert L().stage_kernel_act_fwd(DT[dtype], kind, rows, f, P(zd), P(ad), None) == 0
    dad = to_dev(da, dtype)
    assert L().stage_kernel_act_bwd(DT[dtype], kind, rows, f, P(zd), P(dad), None) == 0
    torch.cuda.synchronize()
    assert so.max_rel_err(to_np(ad), a_ref) <= KTOL[dtype]
    assert so.max_rel_err(to_np(zd), dz_ref) <= KTOL[dtype]


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("rows,n,ld", [(128, 256, 256), (333, 1088, 1088), (1000, 64, 192), (5, 2816, 2816), (4096, 520, 1040)])
def test_bias_gradient(dtype, rows, n, ld):
    """dbias += column sums of dZ (the oracle's _bias_grads), strided rows, two calls accumulate, same bits each time."""
    import torch
    dz = rnd(synth.normal(8, 1, (rows, ld)), dtype)
    d0 = synth.normal(8, 2, (n,))
    ref = so._bias_grads({"bo": 0}, {"wo": dz[:, :n].astype(np.float64)})["bo"]
    dzd = to_dev(dz, dtype)
    scr = torch.zeros(L().stage_kernel_bias_grad_scratch_bytes(n) // 4, dtype=torch.float32, device="cuda:0")
    outs = []
    for _ in range(2):
        db = to_dev(d0, "fp32")
        assert L().stage_kernel_bias_grad(DT[dtype], rows, n, P(dzd), ld, P(db), P(scr), None) == 0
        assert L().stage_kernel_bias_grad(DT[dtype], rows, n, P(dzd), ld, P(db), P(scr), None) == 0
        torch.cuda.synchronize()
        outs.append(db.clone())
    assert torch.equal(outs[0], outs[1])
    assert so.max_rel_err(to_np(outs[0]) - d0, 2 * ref) <= 1e-5
    assert L().stage_kernel_bias_grad(DT[dtype], rows, n, None, ld, P(db), P(scr), None) == -1
    assert L().stage_kernel_bias_grad(DT[dtype], rows, n, P(dzd), n - 8, P(db), P(scr), None) == -1


def test_mfma_ceiling_probe():
    """The measurement aid returns sane figures: the rate and the clock it reports agree (an MFMA of 16384 flops every 16
    cycles on each SIMD), random operands do not beat constant ones, and bad arguments are refused."""
    import torch
    from paper_2507_00217_amd import stage as S
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    tf_c, mhz_c = S.probe_mfma_ceiling(False, 20000)
    tf_r, mhz_r = S.probe_mfma_ceiling(True, 20000)
    assert 0.0 < tf_r <= tf_c * 1.05 and 0.0 < mhz_r <= mhz_c * 1.05, (tf_r, tf_c, mhz_r, mhz_c)
    for tf, mhz in ((tf_c, mhz_c), (tf_r, mhz_r)):
        implied_mhz = tf * 1e12 / (cus * 4 * 32768 / 32.0) / 1e6
        assert abs(implied_mhz - mhz) / mhz < 0.1, (tf, mhz, implied_mhz)
    out = C.c_double()
    scr = torch.empty(1 << 20, dtype=torch.uint8, device="cuda:0")
    assert S.lib().stage_probe_mfma_ceiling(1, 0, scr.data_ptr(), scr.numel(), C.byref(out), C.byref(out), None) == -1
    assert S.lib().stage_probe_mfma_ceiling(1, 100, scr.data_ptr(), scr.numel(), None, C.byref(out), None) == -1
    assert S.lib().stage_probe_mfma_ceiling(1, 100, None, scr.numel(), C.byref(out), C.byref(out), None) == -1       # no scratch
    assert S.lib().stage_probe_mfma_ceiling(1, 100, scr.data_ptr(), 4096, C.byref(out), C.byref(out), None) == -1    # too small
