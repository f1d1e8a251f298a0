"""Pins for the CPU oracle: things the mathematics fixes, independent of the
oracle's own code (finite differences, invariants the paper's F/B/W split must
satisfy, closed forms, and PyTorch CPU autograd as a second opinion)."""
import math

import numpy as np
import pytest

from oracle import stage_oracle as so
from paper_2507_00217_amd import synth

F, B, W = so.F, so.B, so.W


def tiny_cfg(norm="layernorm", act="gelu", n_kv=2, causal=True, L=2, b=1, n_mb=3, head_dim=0, rope_theta=0.0, bias=0):
    return dict(n_layers=L, hidden=16, n_heads=2, n_kv_heads=n_kv, ffn=32, seq=8, mb_size=b,
                n_microbatches=n_mb, norm=norm, act=act, dtype="fp32", causal=causal, head_dim=head_dim,
                rope_theta=rope_theta, bias=bias)


def shape_of(cfg, operand_bits=0):
    return so.Shape(cfg["n_layers"], cfg["hidden"], cfg["n_heads"], cfg["n_kv_heads"], cfg["ffn"],
                    cfg["seq"], cfg["mb_size"], cfg["norm"], cfg["act"], cfg.get("causal", True), hd=cfg.get("head_dim", 0) or 0, rope_theta=float(cfg.get("rope_theta", 0.0) or 0.0),
                    operand_bits=operand_bits)


def setup(cfg, seed=11, wstd_boost=10.0, operand_bits=0):
    params = synth.make_weights(cfg, seed)
    # larger linear weights (and biases) than N(0,0.02) so every path carries signal in fp64 checks
    for lp in params:
        for k in ("wqkv", "wo", "win", "wout") + synth.BIAS_NAMES:
            if k in lp:
                lp[k] = lp[k].astype(np.float64) * wstd_boost
    X = synth.make_boundary(cfg, seed + 1).astype(np.float64)
    G = synth.make_boundary(cfg, seed + 2).astype(np.float64)
    return shape_of(cfg, operand_bits), params, X, G


VARIANTS = [("layernorm", "gelu", 2, True), ("rmsnorm", "swiglu", 1, True),
            ("rmsnorm", "swiglu", 2, False), ("layernorm", "swiglu", 1, True), ("rmsnorm", "gelu", 2, True)]


def loss(sh, params, X, G):
    st = so.OracleStage(sh, params)
    return sum(float((st.forward(m, X[m]) * G[m]).sum()) for m in range(X.shape[0]))


@pytest.mark.parametrize("norm,act,n_kv,causal,rope_theta,bias",
                         [v + (0.0, 0) for v in VARIANTS] + [("rmsnorm", "swiglu", 1, True, 10000.0, 0), ("layernorm", "gelu", 2, False, 30.0, 0),
                                                             ("layernorm", "gelu", 2, True, 0.0, 1), ("rmsnorm", "swiglu", 1, True, 10000.0, 1)])
def test_finite_differences(norm, act, n_kv, causal, rope_theta, bias):
    cfg = tiny_cfg(norm, act, n_kv, causal, n_mb=2, rope_theta=rope_theta, bias=bias)
    sh, params, X, G = setup(cfg)
    st = so.OracleStage(sh, params)
    ops = synth.schedule_1f1b(2, 1)
    _, dX, _ = st.run_schedule(ops, X, G)
    rng = np.random.default_rng(5)
    h = 1e-5
    # every parameter tensor of every layer, a few random entries each
    for li in range(sh.n_layers):
        for name, w in params[li].items():
            for _ in range(3):
                idx = tuple(rng.integers(0, n) for n in w.shape)
                orig = float(w[idx])
                pp = [{k: v.astype(np.float64).copy() for k, v in lp.items()} for lp in params]
                pp[li][name][idx] = orig + h
                lp_ = loss(sh, pp, X, G)
                pp[li][name][idx] = orig - h
                lm_ = loss(sh, pp, X, G)
                fd = (lp_ - lm_) / (2 * h)
                an = st.grads[li][name][idx]
                assert abs(fd - an) <= 1e-6 * max(1.0, abs(fd)), (li, name, idx, fd, an)
    for _ in range(8):
        idx = tuple(rng.integers(0, n) for n in X.shape)
        Xp = X.copy(); Xp[idx] += h
        Xm = X.copy(); Xm[idx] -= h
        fd = (loss(sh, params, Xp, G) - loss(sh, params, Xm, G)) / (2 * h)
        assert abs(fd - dX[idx]) <= 1e-6 * max(1.0, abs(fd)), (idx, fd, dX[idx])


@pytest.mark.parametrize("operand_bits,bias", [(0, 0), (8, 0), (0, 1), (8, 1)])
@pytest.mark.parametrize("norm,act,n_kv,causal", VARIANTS)
def test_b_then_w_equals_fused_backward(norm, act, n_kv, causal, operand_bits, bias):
    cfg = tiny_cfg(norm, act, n_kv, causal, bias=bias)
    sh, params, X, G = setup(cfg, operand_bits=operand_bits)
    a = so.OracleStage(sh, params)
    b = so.OracleStage(sh, params)
    for m in range(X.shape[0]):
        a.forward(m, X[m]); b.forward(m, X[m])
        dxa = a.backward_input(m, G[m]); a.backward_weight(m)
        dxb = b.backward_full(m, G[m])
        assert so.max_rel_err(dxa, dxb) <= 1e-12
    for la, lb in zip(a.grads, b.grads):
        for k in la:
            assert np.abs(la[k]).max() > 0
            assert so.max_rel_err(la[k], lb[k]) <= 1e-12, k


@pytest.mark.parametrize("operand_bits", [0, 8])
def test_schedule_order_invariance(operand_bits):
    cfg = tiny_cfg("rmsnorm", "swiglu", 1, n_mb=6)
    sh, params, X, G = setup(cfg, operand_bits=operand_bits)
    res = []
    for ops in (synth.schedule_1f1b(6, 2), synth.schedule_w_deferred(6, 2, 3), synth.schedule_w_lag1(6, 2),
                synth.schedule_greedy(6, 2), synth.schedule_random(6, 3, 42)):
        st = so.OracleStage(sh, params)
        Y, dX, _ = st.run_schedule(ops, X, G)
        assert st.live == 0
        res.append((ops, Y, dX, st.grads))
    ops0, Y0, dX0, g0 = res[0]
    for ops, Y, dX, g in res[1:]:
        assert np.array_equal(Y, Y0) and np.array_equal(dX, dX0)
        w_sorted = [m for k, m in ops if k == W] == sorted(m for k, m in ops if k == W)
        b_sorted = [m for k, m in ops if k == B] == sorted(m for k, m in ops if k == B)
        for la, lb in zip(g, g0):
            for k in la:
                if w_sorted and b_sorted:
                    assert np.array_equal(la[k], lb[k]), k      # same summation order: bitwise
                else:
                    assert so.max_rel_err(la[k], lb[k]) <= 1e-12, k


@pytest.mark.parametrize("operand_bits,bias", [(0, 0), (8, 0), (0, 1)])
def test_sum_over_microbatches_equals_full_batch(operand_bits, bias):
    cfg = tiny_cfg("layernorm", "gelu", 2, n_mb=4, bias=bias)
    sh, params, X, G = setup(cfg, operand_bits=operand_bits)
    st = so.OracleStage(sh, params)
    st.run_schedule(synth.schedule_1f1b(4, 2), X, G)
    big = so.Shape(sh.n_layers, sh.hidden, sh.n_heads, sh.n_kv_heads, sh.ffn, sh.seq, 4 * sh.mb_size,
                   sh.norm, sh.act, sh.causal, operand_bits=operand_bits)
    sb = so.OracleStage(big, params)
    Yb = sb.forward(0, X.reshape(4, sh.seq, sh.hidden))
    sb.backward_input(0, G.reshape(4, sh.seq, sh.hidden)); sb.backward_weight(0)
    for la, lb in zip(st.grads, sb.grads):
        for k in la:
            assert so.max_rel_err(la[k], lb[k]) <= 1e-12, k


@pytest.mark.parametrize("bias", [0, 1])
@pytest.mark.parametrize("norm,act,n_kv,causal,head_dim,rope_theta",
                         [v + (0, 0.0) for v in VARIANTS] + [("rmsnorm", "swiglu", 1, True, 4, 0.0), ("layernorm", "gelu", 2, True, 12, 0.0),
                                                             ("rmsnorm", "swiglu", 1, True, 0, 10000.0), ("layernorm", "gelu", 2, False, 4, 50.0)])
def test_against_torch_autograd(norm, act, n_kv, causal, head_dim, rope_theta, bias):
    """Second opinion from a library: the same layer stack composed from
    PyTorch CPU primitives, differentiated by autograd, in fp64.  The last two cases have heads that do not tile the
    hidden width (n_heads * head_dim = 8 and 24 against hidden 16), as a tensor-parallel share of a layer has."""
    torch = pytest.importorskip("torch")
    cfg = tiny_cfg(norm, act, n_kv, causal, b=2, n_mb=2, head_dim=head_dim, rope_theta=rope_theta, bias=bias)
    sh, params, X, G = setup(cfg)
    st = so.OracleStage(sh, params)
    Y, dX, _ = st.run_schedule(synth.schedule_1f1b(2, 1), X, G)
    lin = lambda t, p, w, b_: torch.nn.functional.linear(t, p[w].T, p.get(b_))      # t W (+ b): the library's linear layer

    tp = [{k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in lp.items()} for lp in params]
    tX = torch.tensor(X, requires_grad=True)
    d, h, hkv, hd, f = sh.hidden, sh.n_heads, sh.n_kv_heads, sh.head_dim, sh.ffn

    def tnorm(x, g, b_):
        if norm == "layernorm":
            return torch.nn.functional.layer_norm(x, (d,), g, b_, 1e-5)
        return x * torch.rsqrt((x * x).mean(-1, keepdim=True) + 1e-5) * g

    def tlayer(x, p):
        bsz, s, _ = x.shape
        qkv = lin(tnorm(x, p["g1"], p.get("b1")), p, "wqkv", "bqkv")
        q = qkv[..., :h * hd].reshape(bsz, s, h, hd).transpose(1, 2)
        k = qkv[..., h * hd:(h + hkv) * hd].reshape(bsz, s, hkv, hd).transpose(1, 2).repeat_interleave(h // hkv, dim=1)
        v = qkv[..., (h + hkv) * hd:].reshape(bsz, s, hkv, hd).transpose(1, 2).repeat_interleave(h // hkv, dim=1)
        if rope_theta:      # the same rotation written as a complex multiplication: (x_2p + i x_2p+1) * exp(i pos theta_p)
            ang = torch.arange(s, dtype=torch.float64)[:, None] * rope_theta ** (-torch.arange(0, hd, 2, dtype=torch.float64) / hd)
            rot = torch.polar(torch.ones_like(ang), ang)
            turn = lambda t: torch.view_as_real(torch.view_as_complex(t.reshape(*t.shape[:-1], hd // 2, 2).contiguous()) * rot).flatten(-2)
            q, k = turn(q), turn(k)
        o = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=causal)
        x1 = x + lin(o.transpose(1, 2).reshape(bsz, s, h * hd), p, "wo", "bo")
        z = lin(tnorm(x1, p["g2"], p.get("b2")), p, "win", "bin")
        a = torch.nn.functional.gelu(z) if act == "gelu" else torch.nn.functional.silu(z[..., :f]) * z[..., f:]
        return x1 + lin(a, p, "wout", "bout")

    total = 0
    for m in range(2):
        y = tX[m]
        for p in tp:
            y = tlayer(y, p)
        assert so.max_rel_err(Y[m], y.detach().numpy()) <= 1e-12
        total = total + (y * torch.tensor(G[m])).sum()
    total.backward()
    assert so.max_rel_err(dX, tX.grad.numpy()) <= 1e-11
    for li in range(sh.n_layers):
        for k in params[li]:
            assert so.max_rel_err(st.grads[li][k], tp[li][k].grad.numpy()) <= 1e-11, (li, k)


def test_closed_forms():
    cfg = tiny_cfg("layernorm", "gelu", 2)
    sh, params, X, G = setup(cfg)
    # zero output projections: the layer is the identity; upstream weights get zero gradient
    pz = [{k: (np.zeros_like(v) if k in ("wo", "wout") else v) for k, v in lp.items()} for lp in params]
    st = so.OracleStage(sh, pz)
    Y, dX, _ = st.run_schedule(synth.schedule_1f1b(3, 1), X, G)
    assert np.array_equal(Y, X) and np.array_equal(dX, G)
    for lg in st.grads:
        assert not lg["wqkv"].any() and not lg["win"].any() and lg["wo"].any() and lg["wout"].any()
    # LayerNorm rows with unit scale: mean 0, variance var/(var+eps)
    x = X[0, 0]
    out, _ = so.norm_forward("layernorm", x, 1.0, 0.0, 1e-5)
    var = x.var(axis=-1)
    assert np.allclose(out.mean(-1), 0, atol=1e-14) and np.allclose(out.var(-1), var / (var + 1e-5), rtol=1e-12)
    out, _ = so.norm_forward("rmsnorm", x, 1.0, 0.0, 0.0)
    assert np.allclose((out * out).mean(-1), 1.0, rtol=1e-12)
    # softmax rows sum to one; causal rows see only the past; s = 1 returns v
    q = X[0, 0].reshape(8, 2, 8)[:, 0]; k = X[1, 0].reshape(8, 2, 8)[:, 1]
    p = so.head_probs(sh, q, k)
    assert np.allclose(p.sum(-1), 1.0, rtol=1e-14) and not np.triu(p, 1).any()
    assert p[0, 0] == 1.0
    s1 = so.Shape(1, 16, 2, 1, 32, 1, 1)
    q1 = X[0, 0, :1].reshape(1, 1, 2, 8); kv1 = X[1, 0, :1, :8].reshape(1, 1, 1, 8)
    o1 = so.attention_forward(s1, q1, kv1, kv1 * 3)
    assert np.allclose(o1[0, 0, 0], kv1[0, 0, 0] * 3) and np.allclose(o1[0, 0, 1], kv1[0, 0, 0] * 3)
    # gelu at known points; swiglu with unit "up" half is silu
    assert so.gelu(np.array(0.0)) == 0.0 and abs(so.gelu(np.array(1.0)) - 0.8413447460685429) < 1e-15
    assert abs(so.gelu_grad(np.array(0.0)) - 0.5) < 1e-15


def test_causality_and_linearity():
    cfg = tiny_cfg("rmsnorm", "swiglu", 1)
    sh, params, X, G = setup(cfg)
    st = so.OracleStage(sh, params)
    y0 = st.forward(0, X[0])
    Xp = X[0].copy(); Xp[0, 5] += 1.0
    y1 = so.OracleStage(sh, params).forward(0, Xp)
    assert np.array_equal(y0[0, :5], y1[0, :5]) and not np.array_equal(y0[0, 5:], y1[0, 5:])
    # dX and grads are linear in the output gradient
    a = so.OracleStage(sh, params); b = so.OracleStage(sh, params)
    a.forward(0, X[0]); b.forward(0, X[0])
    da = a.backward_input(0, G[0]); a.backward_weight(0)
    db = b.backward_input(0, 3.0 * G[0]); b.backward_weight(0)
    assert so.max_rel_err(db, 3.0 * da) <= 1e-13
    for la, lb in zip(a.grads, b.grads):
        for k in la:
            assert so.max_rel_err(lb[k], 3.0 * la[k]) <= 1e-13


def test_gqa_with_all_kv_heads_is_mha():
    """n_kv_heads == n_heads through the grouped path equals plain per-head attention."""
    rng = np.random.default_rng(0)
    sh = so.Shape(1, 16, 4, 4, 32, 6, 1)
    q = rng.standard_normal((1, 6, 4, 4)); k = rng.standard_normal((1, 6, 4, 4)); v = rng.standard_normal((1, 6, 4, 4))
    o = so.attention_forward(sh, q, k, v)
    for j in range(4):
        S = q[0, :, j] @ k[0, :, j].T / 2.0
        S[np.triu_indices(6, 1)] = -np.inf
        P = np.exp(S - S.max(-1, keepdims=True)); P /= P.sum(-1, keepdims=True)
        assert np.allclose(o[0, :, j], P @ v[0, :, j], rtol=1e-13)
    # grouped: 2 kv heads shared by 4 query heads == MHA with the kv heads repeated
    sg = so.Shape(1, 16, 4, 2, 32, 6, 1)
    og = so.attention_forward(sg, q, k[:, :, :2], v[:, :, :2])
    om = so.attention_forward(sh, q, np.repeat(k[:, :, :2], 2, axis=2), np.repeat(v[:, :, :2], 2, axis=2))
    assert np.array_equal(og, om)
    do = rng.standard_normal(q.shape)
    dqg, dkg, dvg = so.attention_backward(sg, q, k[:, :, :2], v[:, :, :2], do)
    dqm, dkm, dvm = so.attention_backward(sh, q, np.repeat(k[:, :, :2], 2, axis=2), np.repeat(v[:, :, :2], 2, axis=2), do)
    assert np.allclose(dqg, dqm, rtol=1e-13)
    assert np.allclose(dkg, dkm.reshape(1, 6, 2, 2, 4).sum(3), rtol=1e-12)
    assert np.allclose(dvg, dvm.reshape(1, 6, 2, 2, 4).sum(3), rtol=1e-12)


@pytest.mark.parametrize("n_sub", [2, 4])
def test_sub_blocks_in_order_equal_whole_ops(n_sub):
    """Sub-block ops (n_sub groups of layers per F/B/W op): back to back they are the whole op, bit for bit; in any
    legal interleaving across microbatches they give the same outputs and (microbatch-ordered) the same gradients."""
    cfg = tiny_cfg("rmsnorm", "swiglu", 1, L=4, n_mb=4)
    sh, params, X, G = setup(cfg)
    whole = so.OracleStage(sh, params)
    ops = synth.schedule_1f1b(4, 2)
    Y0, dX0, _ = whole.run_schedule(ops, X, G)
    a = so.OracleStage(sh, params)
    Y1, dX1, pk = a.run_subschedule(synth.expand_to_subops(ops, n_sub), n_sub, X, G)
    assert np.array_equal(Y0, Y1) and np.array_equal(dX0, dX1) and a.live == 0 and pk == 3
    for la, lb in zip(whole.grads, a.grads):
        for k in la:
            assert np.array_equal(la[k], lb[k]), k
    for seed in range(3):
        sub_ops = synth.subschedule_interleaved(4, n_sub, 3, seed)
        assert sub_ops != synth.expand_to_subops(ops, n_sub)
        b = so.OracleStage(sh, params)
        Y2, dX2, pk = b.run_subschedule(sub_ops, n_sub, X, G)
        assert np.array_equal(Y0, Y2) and np.array_equal(dX0, dX2) and b.live == 0 and pk <= 3
        for la, lb in zip(whole.grads, b.grads):
            for k in la:
                assert np.array_equal(la[k], lb[k]), k


@pytest.mark.parametrize("norm,act,n_kv,causal", VARIANTS[:3])
def test_recomputation_changes_memory_not_results(norm, act, n_kv, causal):
    """Layer-wise activation recomputation (section 7.2, Case 2): between F and B only each layer's input is held
    (L * tokens * hidden elements); B rebuilds the rest; outputs and gradients are bit-identical to the plain path,
    for whole ops, fused backward and interleaved sub-blocks.  Also against torch autograd through the plain path's
    own pin (equality carries it over)."""
    cfg = tiny_cfg(norm, act, n_kv, causal, L=4, n_mb=4)
    sh, params, X, G = setup(cfg)
    plain, rec = so.OracleStage(sh, params), so.OracleStage(sh, params, recompute=True)
    tokens = cfg["mb_size"] * cfg["seq"]
    for st in (plain, rec):
        st.forward(0, X[0])
    assert rec.stash_elems(0) == cfg["n_layers"] * tokens * cfg["hidden"]
    assert plain.stash_elems(0) > 8 * rec.stash_elems(0)
    d0, d1 = plain.backward_input(0, G[0]), rec.backward_input(0, G[0])
    assert np.array_equal(d0, d1)
    assert rec.stash_elems(0) == plain.stash_elems(0)          # rebuilt caches live from B to W
    plain.backward_weight(0); rec.backward_weight(0)
    assert rec.live == 0 and rec.stash_elems(0) == 0
    ops = synth.schedule_1f1b(4, 2)
    plain, rec = so.OracleStage(sh, params), so.OracleStage(sh, params, recompute=True)
    Y0, dX0, _ = plain.run_schedule(ops, X, G)
    Y1, dX1, _ = rec.run_schedule(ops, X, G)
    sub = so.OracleStage(sh, params, recompute=True)
    Y2, dX2, _ = sub.run_subschedule(synth.subschedule_interleaved(4, 2, 3, 5), 2, X, G)
    fused = so.OracleStage(sh, params, recompute=True)
    for m in range(4):
        fused.forward(m, X[m])
    dX3 = np.stack([fused.backward_full(m, G[m]) for m in range(4)])
    assert np.array_equal(Y0, Y1) and np.array_equal(dX0, dX1) and np.array_equal(Y0, Y2) and np.array_equal(dX0, dX2)
    assert np.array_equal(dX0.reshape(dX3.shape), dX3)
    for la, lb, lc, ld in zip(plain.grads, rec.grads, sub.grads, fused.grads):
        for k in la:
            assert np.array_equal(la[k], lb[k]) and np.array_equal(la[k], lc[k]), k
            np.testing.assert_allclose(ld[k], la[k], rtol=1e-12, atol=1e-12)


def test_rope_properties():
    """Rotary embedding: a rotation (norms kept, inverse = transpose), identity at position 0, and the attention scores of
    rotated q, k depend on the two positions only through their difference."""
    sh = so.Shape(1, 16, 2, 2, 32, 12, 1, rope_theta=100.0)
    t = synth.normal(9, 1, (1, 12, 2, 8)).astype(np.float64)
    r = so.rope(sh, t)
    assert np.allclose(np.linalg.norm(r, axis=-1), np.linalg.norm(t, axis=-1), rtol=1e-13)
    assert np.array_equal(r[:, 0], t[:, 0]) and not np.allclose(r[:, 1:], t[:, 1:])
    assert np.allclose(so.rope(sh, r, inverse=True), t, atol=1e-14)
    u = synth.normal(9, 2, (1, 12, 2, 8)).astype(np.float64)
    assert abs((so.rope(sh, t) * u).sum() - (t * so.rope(sh, u, inverse=True)).sum()) < 1e-12      # <R t, u> = <t, R^T u>
    q = np.broadcast_to(t[:, :1], t.shape)          # the same vector at every position
    k = np.broadcast_to(u[:, :1], u.shape)
    S = np.einsum("bmhd,bnhd->bhmn", so.rope(sh, q), so.rope(sh, k))
    for off in range(-5, 6):
        dgl = np.diagonal(S, offset=off, axis1=-2, axis2=-1)
        assert np.allclose(dgl, dgl[..., :1], atol=1e-12), off
    # hand value: pair 0 at position 3 turns by 3 rad (theta^0 = 1)
    one = np.zeros((1, 4, 1, 8)); one[..., 0] = 1.0
    got = so.rope(sh, one)[0, 3, 0]
    assert np.allclose(got[:2], [math.cos(3.0), math.sin(3.0)]) and np.allclose(got[2:], 0.0)


def test_max_rel_err_hand_values():
    """The metric every parity verdict passes through, on values worked by hand: largest absolute difference over the
    largest absolute reference value of the whole tensor; a zero reference falls back to the largest absolute value."""
    assert so.max_rel_err([1.0, 2.0, 3.5], [1.0, 2.0, 4.0]) == 0.125            # 0.5 / 4
    assert so.max_rel_err([[-8.0, 2.0]], [[-8.0, 1.0]]) == 0.125                # the denominator is max |ref| = 8, not 1
    assert so.max_rel_err([0.25, -0.5], [0.0, 0.0]) == 0.5                      # zero reference: max |got|
    assert so.max_rel_err([3.0, -4.0], [3.0, -4.0]) == 0.0
    assert so.max_rel_err(np.float32([1.0, 100.0]), np.float64([2.0, 100.0])) == 0.01   # mixed dtypes compare in fp64


# ---------------------------------------------------------------------------
# the bf16-compute reading (Shape.operand_bits): both operands of every matrix product rounded, exact accumulation
# ---------------------------------------------------------------------------

def round_sig_by_definition(t, bits):
    """x = m 2^e with 0.5 <= |m| < 1  ->  rint(m 2^bits) 2^(e - bits), halves to even: the definition, via frexp."""
    m, e = np.frexp(np.asarray(t, dtype=np.float64))
    return np.ldexp(np.rint(np.ldexp(m, bits)), e - bits)


def test_round_sig_hand_values_definition_and_library():
    r = lambda x: float(so.round_sig(np.array([x]), 8)[0])
    assert r(1.0) == 1.0 and r(0.0) == 0.0 and r(-3.0) == -3.0
    assert r(1 + 2.0 ** -8) == 1.0                       # half-way, kept digit even: down
    assert r(1 + 3 * 2.0 ** -8) == 1 + 2.0 ** -6         # half-way, kept digit odd: up
    assert r(1 + 2.0 ** -8 + 2.0 ** -30) == 1 + 2.0 ** -7    # just above half-way: up
    assert r(255.5) == 256.0 and r(-255.5) == -256.0     # the carry moves into the exponent
    assert r(0.1) == 0.10009765625                       # bf16(0.1) = 0x3DCD
    rng = np.random.default_rng(3)
    x = rng.standard_normal(20000) * np.exp2(rng.integers(-40, 40, 20000))
    for bits in (8, 11, 24):
        assert np.array_equal(so.round_sig(x, bits), round_sig_by_definition(x, bits))
    assert np.array_equal(so.round_sig(so.round_sig(x, 8), 8), so.round_sig(x, 8))      # idempotent
    x0 = x.copy(); so.round_sig(x, 8); assert np.array_equal(x, x0)                      # input untouched
    torch = pytest.importorskip("torch")                 # a library's float32 -> bfloat16 conversion on float32 values
    x32 = x.astype(np.float32)
    want = torch.from_numpy(x32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(so.round_sig(x32.astype(np.float64), 8), want)


def test_operand_rounding_attention_brute_force():
    """Attention forward and backward under the bf16-compute reading against scalar loops that round every product's
    operands one by one (one sequence, GQA, causal)."""
    s, h, hkv, hd = 5, 2, 1, 4
    sh = so.Shape(1, h * hd, h, hkv, 8, s, 1, operand_bits=8)
    rng = np.random.default_rng(9)
    q, k, v, do = (rng.standard_normal((1, s, n, hd)) * 1.7 for n in (h, hkv, hkv, h))
    r = lambda x: float(round_sig_by_definition(np.array([x]), 8)[0])
    o = np.zeros((s, h, hd)); dq = np.zeros((s, h, hd)); dk = np.zeros((s, hkv, hd)); dv = np.zeros((s, hkv, hd))
    for j in range(h):
        P = np.zeros((s, s))
        for i in range(s):
            sc = [sum(r(q[0, i, j, t]) * r(k[0, u, 0, t]) for t in range(hd)) / math.sqrt(hd) for u in range(i + 1)]
            e = [math.exp(x - max(sc)) for x in sc]
            for u in range(i + 1):
                P[i, u] = e[u] / sum(e)
        for i in range(s):
            for t in range(hd):
                o[i, j, t] = sum(r(P[i, u]) * r(v[0, u, 0, t]) for u in range(s))
        dP = np.array([[sum(r(do[0, i, j, t]) * r(v[0, u, 0, t]) for t in range(hd)) for u in range(s)] for i in range(s)])
        dS = P * (dP - (dP * P).sum(axis=1, keepdims=True))
        for u in range(s):
            for t in range(hd):
                dv[u, 0, t] += sum(r(P[i, u]) * r(do[0, i, j, t]) for i in range(s))
                dk[u, 0, t] += sum(r(dS[i, u]) * r(q[0, i, j, t]) for i in range(s)) / math.sqrt(hd)
        for i in range(s):
            for t in range(hd):
                dq[i, j, t] = sum(r(dS[i, u]) * r(k[0, u, 0, t]) for u in range(s)) / math.sqrt(hd)
    assert so.max_rel_err(so.attention_forward(sh, q, k, v)[0], o) <= 1e-13
    gq, gk, gv = so.attention_backward(sh, q, k, v, do)
    assert so.max_rel_err(gq[0], dq) <= 1e-13 and so.max_rel_err(gk[0], dk) <= 1e-13 and so.max_rel_err(gv[0], dv) <= 1e-13
    # and the rounding matters at this size: the exact reading gives something else
    assert so.max_rel_err(so.attention_forward(so.Shape(1, h * hd, h, hkv, 8, s, 1), q, k, v)[0], o) > 1e-4


def test_operand_rounding_linear_maps_brute_force():
    """_linear and the two gradient products of a linear map under the bf16-compute reading: every operand element
    rounded, sums exact -- against scalar loops."""
    rng = np.random.default_rng(4)
    sh = so.Shape(1, 8, 1, 1, 8, 3, 1, operand_bits=8)
    a, w, b, dz = rng.standard_normal((3, 5)), rng.standard_normal((5, 4)), rng.standard_normal(4), rng.standard_normal((3, 4))
    r = lambda x: float(round_sig_by_definition(np.array([x]), 8)[0])
    y = np.array([[sum(r(a[i, t]) * r(w[t, n]) for t in range(5)) + b[n] for n in range(4)] for i in range(3)])
    assert so.max_rel_err(so._linear(sh, {"wo": w, "bo": b}, "wo", a), y) <= 1e-15
    da = np.array([[sum(r(dz[i, n]) * r(w[t, n]) for n in range(4)) for t in range(5)] for i in range(3)])
    dw = np.array([[sum(r(a[i, t]) * r(dz[i, n]) for i in range(3)) for n in range(4)] for t in range(5)])
    assert so.max_rel_err(so._mm(sh, dz, w.T), da) <= 1e-15 and so.max_rel_err(so._mm(sh, a.T, dz), dw) <= 1e-15


@pytest.mark.parametrize("norm,act,n_kv", [("layernorm", "gelu", 2), ("rmsnorm", "swiglu", 1)])
def test_operand_rounding_error_scales_with_the_digits_kept(norm, act, n_kv):
    """The stage under the operand-rounding reading differs from the exact one by an amount that shrinks like
    2^-bits (8 -> 12 digits: a factor 16, here within [5, 50]); with 52 digits kept the two agree to rounding error."""
    cfg = tiny_cfg(norm, act, n_kv, n_mb=2, bias=1)
    ops = synth.schedule_1f1b(2, 1)
    sh, params, X, G = setup(cfg, wstd_boost=4.0)
    ref = so.OracleStage(sh, params); Y0, dX0, _ = ref.run_schedule(ops, X, G)
    dev = {}
    for bits in (8, 12, 52):
        st = so.OracleStage(shape_of(cfg, bits), params)
        Y, dX, _ = st.run_schedule(ops, X, G)
        dev[bits] = max([so.max_rel_err(Y, Y0), so.max_rel_err(dX, dX0)] +
                        [so.max_rel_err(st.grads[l][k], ref.grads[l][k]) for l in range(sh.n_layers) for k in ref.grads[l]])
    assert 1e-4 < dev[8] < 5e-2 and 5.0 < dev[8] / dev[12] < 50.0 and dev[52] < 1e-12, dev
