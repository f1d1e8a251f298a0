"""Parity of the HIP stage (through the C ABI) against the CPU oracle, element
by element, on seeded inputs; plus the invariants the F/B/W split must keep."""
import numpy as np
import pytest

from oracle import stage_oracle as so
from paper_2507_00217_amd import synth
from tests.gpu_util import SMALL, TOL, shape_of, to_dev, to_np

pytestmark = pytest.mark.gpu
F, B, W = 0, 1, 2


def run_gpu(cfg, params, X, G, ops, kernel_set=0, pieces=1):
    import torch
    from paper_2507_00217_amd import stage as S
    st = S.Stage(cfg)
    st.set_kernel_set(kernel_set)
    st.load_weights(params)
    Xd, Gd = to_dev(X, cfg["dtype"]), to_dev(G, cfg["dtype"])
    Y, dX = torch.zeros_like(Xd), torch.zeros_like(Xd)
    step = (len(ops) + pieces - 1) // pieces
    for i in range(0, len(ops), step):
        st.run_schedule(ops[i:i + step], Xd, Gd, Y, dX)
    torch.cuda.synchronize()
    out = to_np(Y), to_np(dX), st.grads(), st.stats()
    st.close()
    return out


def run_oracle(cfg, params, X, G, ops):
    st = so.OracleStage(shape_of(cfg), params)
    Y, dX, peak = st.run_schedule(ops, X.astype(np.float64), G.astype(np.float64))
    return Y, dX, st.grads, peak


def compare(cfg, got, ref, tol):
    Yg, dXg, gg, stats = got
    Yr, dXr, gr, peak = ref
    errs = {"Y": so.max_rel_err(Yg, Yr), "dX": so.max_rel_err(dXg, dXr)}
    for li, (lg, lr) in enumerate(zip(gg, gr)):
        assert set(lg) == set(lr)
        for k in lr:
            errs[f"L{li}.{k}"] = so.max_rel_err(lg[k], lr[k])
    worst = max(errs, key=errs.get)
    print(f"worst {worst} = {errs[worst]:.3e} (tol {tol:g})", flush=True)
    assert errs[worst] <= tol, errs
    assert stats["peak_live"] == peak and stats["live"] == 0
    return errs


def inputs(cfg, base_seed):
    return (synth.make_weights(cfg, base_seed), synth.make_boundary(cfg, base_seed + 1), synth.make_boundary(cfg, base_seed + 2))


@pytest.mark.parametrize("kernel_set", [0, 1])
def test_cfg1_full_fp32(kernel_set):
    cfg = synth.CONFIGS["cfg1"]
    params, X, G = inputs(cfg, 1000)
    ops = synth.make_schedule(cfg)
    compare(cfg, run_gpu(cfg, params, X, G, ops, kernel_set), run_oracle(cfg, params, X, G, ops), TOL["fp32"])


@pytest.mark.parametrize("name", list(SMALL))
@pytest.mark.parametrize("kernel_set", [0, 1])
def test_small_variants_bf16(name, kernel_set):
    cfg = SMALL[name]
    params, X, G = inputs(cfg, 2000 + int(name[3]))
    ops = synth.make_schedule(cfg)
    compare(cfg, run_gpu(cfg, params, X, G, ops, kernel_set), run_oracle(cfg, params, X, G, ops), TOL["bf16"])


@pytest.mark.parametrize("variant", ["cfg1_fp32", "cfg2s", "cfg3s", "cfg5s_recompute", "cfg4s_sub"])
@pytest.mark.parametrize("kernel_set", [0, 1])
def test_linear_biases(variant, kernel_set):
    """GPT-style layers: every linear map carries a bias (added in the product's epilogue, before the residual / the
    activation); the bias gradients, column sums of the dZ tensors, are accumulated by B.  Also under recomputation and
    with sub-block ops."""
    if variant == "cfg1_fp32":
        cfg = dict(synth.CONFIGS["cfg1"], bias=1)
    elif variant == "cfg5s_recompute":
        cfg = dict(SMALL["cfg5s"], bias=1, recompute=1)
    elif variant == "cfg4s_sub":
        cfg = dict(SMALL["cfg4s"], bias=1, n_sub=2)
    else:
        cfg = dict(SMALL[variant], bias=1)
    params, X, G = inputs(cfg, 2900 + len(variant))
    assert set(synth.BIAS_NAMES) <= set(params[0])
    ops = synth.make_schedule(cfg)
    cfg["stash_cap"] = synth.peak_live(ops)
    got = run_gpu(cfg, params, X, G, ops, kernel_set)
    ref = so.OracleStage(shape_of(cfg), params, recompute=bool(cfg.get("recompute")))
    Yr, dXr, peak = ref.run_schedule(ops, X.astype(np.float64), G.astype(np.float64))
    errs = compare(cfg, got, (Yr, dXr, ref.grads, peak), TOL[cfg["dtype"]])
    assert all(f"L0.{b}" in errs for b in synth.BIAS_NAMES)
    # the biases matter on these inputs, and schedule order does not (bitwise, microbatch-ordered ops)
    nob = [{k: v for k, v in lp.items() if k not in synth.BIAS_NAMES} for lp in params]
    assert so.max_rel_err(run_oracle(dict(cfg, bias=0), nob, X, G, ops)[0], Yr) > 1e-3
    if variant == "cfg2s":
        n = cfg["n_microbatches"]
        alt = run_gpu(cfg, params, X, G, synth.schedule_w_deferred(n, 2, 2), kernel_set)
        for la, lb in zip(got[2], alt[2]):
            for k in la:
                assert np.array_equal(la[k], lb[k]), k


@pytest.mark.parametrize("kernel_set", [0, 1])
@pytest.mark.parametrize("heads,kv,hidden", [(2, 1, 512), (6, 2, 512), (3, 3, 256)])
def test_head_width_independent_of_hidden(heads, kv, hidden, kernel_set):
    """Tensor-parallel shares of a layer (the paper's per-GPU shapes at TP > 1): n_heads * head_dim is smaller or
    larger than hidden, so the attention block is rectangular (WQKV [d, (h + 2 h_kv) 128], WO [128 h, d])."""
    cfg = dict(SMALL["cfg3s"], hidden=hidden, n_heads=heads, n_kv_heads=kv, head_dim=128, ffn=704, seq=328,
               n_microbatches=4, stash_cap=3, warmup=2)
    params, X, G = inputs(cfg, 2700 + heads)
    assert params[0]["wo"].shape == (heads * 128, hidden)
    ops = synth.schedule_1f1b(4, 2)
    compare(cfg, run_gpu(cfg, params, X, G, ops, kernel_set), run_oracle(cfg, params, X, G, ops), TOL["bf16"])


@pytest.mark.parametrize("variant", ["cfg1_fp32", "cfg3s", "cfg5s_recompute", "tp_share"])
def test_rotary_position_embedding(variant):
    """Llama-style layers: q and k rotated by position after the QKV product, the transposed rotation on dq and dk
    in B; also under recomputation (the rebuilt stash must hold the rotated q, k again) and with a rectangular
    attention block."""
    if variant == "cfg1_fp32":
        cfg = dict(synth.CONFIGS["cfg1"], rope_theta=10000.0)
    elif variant == "cfg3s":
        cfg = dict(SMALL["cfg3s"], rope_theta=500000.0)
    elif variant == "cfg5s_recompute":
        cfg = dict(SMALL["cfg5s"], rope_theta=10000.0, recompute=1)
    else:
        cfg = dict(SMALL["cfg3s"], hidden=512, n_heads=2, n_kv_heads=1, head_dim=128, ffn=704, rope_theta=10000.0)
    params, X, G = inputs(cfg, 2800 + len(variant))
    ops = synth.make_schedule(cfg)
    cfg["stash_cap"] = synth.peak_live(ops)
    got = run_gpu(cfg, params, X, G, ops)
    ref = so.OracleStage(shape_of(cfg), params, recompute=bool(cfg.get("recompute")))
    Yr, dXr, peak = ref.run_schedule(ops, X.astype(np.float64), G.astype(np.float64))
    compare(cfg, got, (Yr, dXr, ref.grads, peak), TOL[cfg["dtype"]])
    plain = run_oracle(dict(cfg, rope_theta=0.0), params, X, G, ops)
    assert so.max_rel_err(plain[0], Yr) > 1e-3          # the embedding is not a no-op on these inputs


@pytest.mark.parametrize("name", ["cfg3s", "cfg4s"])
def test_small_variants_fp32_storage(name):
    """Same shapes in fp32: isolates arithmetic from bf16 storage rounding."""
    cfg = dict(SMALL[name], dtype="fp32")
    params, X, G = inputs(cfg, 2100)
    ops = synth.make_schedule(cfg)
    compare(cfg, run_gpu(cfg, params, X, G, ops), run_oracle(cfg, params, X, G, ops), TOL["fp32"])


def test_order_invariance_bitwise_and_pieces():
    """Accumulated gradients do not depend on the schedule: bitwise when every
    kind of op comes in microbatch order, to 1e-5 for a random legal order; an
    iteration fed in pieces equals one call."""
    cfg = dict(SMALL["cfg5s"], enforce_mb_order=0)
    params, X, G = inputs(cfg, 2205)
    n = cfg["n_microbatches"]
    base = run_gpu(cfg, params, X, G, synth.schedule_1f1b(n, 3))
    for ops, pieces in ((synth.schedule_w_deferred(n, 3, 3), 1), (synth.schedule_greedy(n, 3), 4)):
        other = run_gpu(cfg, params, X, G, ops, pieces=pieces)
        assert np.array_equal(base[0], other[0]) and np.array_equal(base[1], other[1])
        for la, lb in zip(base[2], other[2]):
            for k in la:
                assert np.array_equal(la[k], lb[k]), k
    rnd_ops = synth.schedule_random(n, 4, 5003)
    other = run_gpu(cfg, params, X, G, rnd_ops)
    assert np.array_equal(base[0], other[0]) and np.array_equal(base[1], other[1])
    for la, lb in zip(base[2], other[2]):
        for k in la:
            assert so.max_rel_err(lb[k], la[k]) <= 1e-5, k


def test_error_paths_leave_state_untouched():
    import torch
    from paper_2507_00217_amd import stage as S
    cfg = dict(synth.CONFIGS["cfg1"], stash_cap=2, enforce_mb_order=1)
    params, X, G = inputs(cfg, 1000)
    st = S.Stage(cfg)
    st.load_weights(params)
    Xd, Gd = to_dev(X, "fp32"), to_dev(G, "fp32")
    Y, dX = torch.zeros_like(Xd), torch.zeros_like(Xd)

    def code(fn, *a):
        with pytest.raises(S.StageError) as e:
            fn(*a)
        return e.value.code

    assert code(st.backward_input, 0, Gd[0], dX[0]) == S.E_ORDER
    assert code(st.backward_weight, 0) == S.E_ORDER
    assert code(st.forward, 4, Xd[0], Y[0]) == S.E_INVAL
    st.forward(0, Xd[0], Y[0])
    assert code(st.forward, 0, Xd[0], Y[0]) == S.E_ORDER
    st.forward(1, Xd[1], Y[1])
    assert code(st.forward, 2, Xd[2], Y[2]) == S.E_STASH_FULL
    assert code(st.backward_input, 1, Gd[1], dX[1]) in (S.E_ORDER,)          # microbatch order enforced: B0 first
    # a list that fails at its last op enqueues nothing
    assert code(st.run_schedule, [(B, 0), (W, 0), (F, 2), (F, 3)], Xd, Gd, Y, dX) == S.E_STASH_FULL
    assert st.stats()["live"] == 2
    st.run_schedule([(B, 0), (W, 0), (F, 2), (B, 1), (W, 1), (F, 3), (B, 2), (W, 2), (B, 3), (W, 3)], Xd, Gd, Y, dX)
    torch.cuda.synchronize()
    assert st.stats() == {"live": 0, "peak_live": 2, "peak_stash_bytes": 2 * (st.sizes["stash"] // 2)}
    ref = run_oracle(cfg, params, X, G, synth.schedule_1f1b(4, 2))
    compare(cfg, (to_np(Y), to_np(dX), st.grads(), dict(st.stats(), peak_live=ref[3])), ref, TOL["fp32"])
    # zero_grads, then a second iteration gives the same gradients again (slots are reused cleanly)
    g1 = st.grads()
    st.zero_grads()
    st.run_schedule(synth.schedule_1f1b(4, 1), Xd, Gd, Y, dX)
    g2 = st.grads()
    for la, lb in zip(g1, g2):
        for k in la:
            assert np.array_equal(la[k], lb[k])
    st.close()


@pytest.mark.parametrize("n_sub", [2, 4])
def test_sub_block_ops(n_sub):
    """Sub-block ops on the GPU: a seeded interleaving at sub-block grain matches the oracle running the same list,
    and is bit-identical to the whole-op run of the same stage (same kernels in the same per-tensor order)."""
    import torch
    from paper_2507_00217_amd import stage as S
    cfg = dict(SMALL["cfg3s"], n_layers=4, n_sub=n_sub, stash_cap=3, n_microbatches=4, enforce_mb_order=1)
    params, X, G = inputs(cfg, 2300)
    sub_ops = synth.subschedule_interleaved(4, n_sub, 3, 11)
    st = S.Stage(cfg)
    st.load_weights(params)
    Xd, Gd = to_dev(X, "bf16"), to_dev(G, "bf16")
    Y, dX = torch.zeros_like(Xd), torch.zeros_like(Xd)
    st.run_subschedule(sub_ops, Xd, Gd, Y, dX)
    torch.cuda.synchronize()
    assert st.stats()["live"] == 0 and st.stats()["peak_live"] <= 3
    got = (to_np(Y), to_np(dX), st.grads(), st.stats())
    ref = so.OracleStage(shape_of(cfg), params)
    Yr, dXr, peak = ref.run_subschedule(sub_ops, n_sub, X.astype(np.float64), G.astype(np.float64))
    compare(cfg, got, (Yr, dXr, ref.grads, peak), TOL["bf16"])
    g_sub = st.grads_tensor().clone(); Y_sub, dX_sub = Y.clone(), dX.clone()
    # whole ops on the same stage, and the single-call sub-block entry points
    st.zero_grads(); Y.zero_(); dX.zero_()
    st.run_schedule(synth.schedule_1f1b(4, 2), Xd, Gd, Y, dX)
    torch.cuda.synchronize()
    assert torch.equal(Y, Y_sub) and torch.equal(dX, dX_sub) and torch.equal(st.grads_tensor(), g_sub)
    st.zero_grads(); Y.zero_(); dX.zero_()
    for k, m, sb in synth.expand_to_subops(synth.schedule_1f1b(4, 2), n_sub):
        if k == F:
            st.forward_sub(m, sb, Xd[m] if sb == 0 else None, Y[m] if sb == n_sub - 1 else None)
        elif k == B:
            st.backward_input_sub(m, sb, Gd[m] if sb == n_sub - 1 else None, dX[m] if sb == 0 else None)
        else:
            st.backward_weight_sub(m, sb)
    torch.cuda.synchronize()
    assert torch.equal(Y, Y_sub) and torch.equal(dX, dX_sub) and torch.equal(st.grads_tensor(), g_sub)
    with pytest.raises(S.StageError) as e:
        st.backward_input_sub(0, 0, None, dX[0])          # B before F
    assert e.value.code == S.E_ORDER
    with pytest.raises(S.StageError) as e:
        st.forward_sub(0, 0, None, None)                  # sub-block 0 needs x
    assert e.value.code == S.E_INVAL
    st.close()


def test_generated_schedule_runs_on_the_stage():
    """Close the loop: the greedy generator's list for one stage of a delayed 4-stage pipeline (sub-blocks, memory
    limit) runs through the engine and gives the same bits as plain whole-op 1F1B."""
    import torch
    from paper_2507_00217_amd import sched as L
    from paper_2507_00217_amd import stage as S
    n_pp, n_mb, n_sub = 4, 8, 2
    a, b = synth.delay_matrices(n_pp, 2, 2.0, 2.0)
    pl, keep = L.make_params(n_pp, n_mb, n_sub, [1.0] * n_pp, [1.2] * n_pp, [0.9] * n_pp, m_limit=float(n_pp),
                             alpha=a, beta=b, msg_bytes=1.0)
    slots, mk = L.crosspipe_greedy(pl)
    cfg = dict(SMALL["cfg3s"], n_layers=2, n_sub=n_sub, stash_cap=n_pp, n_microbatches=n_mb, enforce_mb_order=1)
    params, X, G = inputs(cfg, 2400)
    Xd, Gd = to_dev(X, "bf16"), to_dev(G, "bf16")
    outs = []
    for stage_idx in (0, 2):
        ops = L.crosspipe_stage_ops(slots, stage_idx)
        assert len(ops) == 3 * n_mb * n_sub
        st = S.Stage(cfg)
        st.load_weights(params)
        Y, dX = torch.zeros_like(Xd), torch.zeros_like(Xd)
        st.run_subschedule(ops, Xd, Gd, Y, dX)
        torch.cuda.synchronize()
        assert st.stats()["live"] == 0 and st.stats()["peak_live"] <= n_pp
        outs.append((Y.clone(), dX.clone(), st.grads_tensor().clone()))
        st.close()
    st = S.Stage(cfg)
    st.load_weights(params)
    Y, dX = torch.zeros_like(Xd), torch.zeros_like(Xd)
    st.run_schedule(synth.schedule_1f1b(n_mb, 3), Xd, Gd, Y, dX)
    torch.cuda.synchronize()
    for (y, dx, g) in outs:
        assert torch.equal(y, Y) and torch.equal(dx, dX) and torch.equal(g, st.grads_tensor())
    st.close()


def peak_rebuilt(ops):
    """Largest number of microbatches between their (first) B and their last W in an op list of pairs or triples."""
    started, left, cur, peak = set(), {}, 0, 0
    n_w = {}
    for op in ops:
        if op[0] == W:
            n_w[op[1]] = n_w.get(op[1], 0) + 1
    for op in ops:
        k, m = op[0], op[1]
        if k == B and m not in started:
            started.add(m); left[m] = n_w[m]; cur += 1; peak = max(peak, cur)
        elif k == W:
            left[m] -= 1
            if left[m] == 0:
                started.discard(m); cur -= 1
    return peak


@pytest.mark.parametrize("name", ["cfg1", "cfg3s", "cfg4s", "cfg5s", "cfg2s"])
def test_recomputation_is_bitwise_the_plain_path(name):
    """Layer-wise activation recomputation (section 7.2, Case 2): same bits as the plain path for Y, dX and every
    gradient, within tolerance of the oracle that recomputes, with the smaller stash the sizes promise."""
    import torch
    from paper_2507_00217_amd import stage as S
    base = dict(synth.CONFIGS["cfg1"]) if name == "cfg1" else dict(SMALL[name])
    ops = synth.make_schedule(base)
    cap = synth.peak_live(ops)
    base["stash_cap"] = cap
    rcap = peak_rebuilt(ops)
    params, X, G = inputs(base, 2500)
    plain = run_gpu(base, params, X, G, ops)
    cfg = dict(base, recompute=1, recompute_cap=rcap)
    got = run_gpu(cfg, params, X, G, ops)
    assert np.array_equal(plain[0], got[0]) and np.array_equal(plain[1], got[1])
    for la, lb in zip(plain[2], got[2]):
        for k in la:
            assert np.array_equal(la[k], lb[k]), k
    ref = so.OracleStage(shape_of(cfg), params, recompute=True)
    Yr, dXr, peak = ref.run_schedule(ops, X.astype(np.float64), G.astype(np.float64))
    compare(cfg, got, (Yr, dXr, ref.grads, peak), TOL[cfg["dtype"]])
    sz_plain, sz = S.stage_query_sizes(base), S.stage_query_sizes(cfg)
    assert got[3]["peak_stash_bytes"] <= sz["stash"] and plain[3]["peak_stash_bytes"] == sz_plain["stash"]
    assert rcap == cap or sz["stash"] < sz_plain["stash"]
    print(f"{name}: cap {cap}, rebuilt cap {rcap}, stash {sz_plain['stash'] >> 20} -> {sz['stash'] >> 20} MiB", flush=True)


def test_recomputation_with_sub_blocks_and_cap():
    """Recomputation under interleaved sub-block ops, and the cap on rebuilt stashes refusing a B without touching
    the state."""
    import torch
    from paper_2507_00217_amd import stage as S
    n_sub = 2
    base = dict(SMALL["cfg3s"], n_layers=4, n_sub=n_sub, stash_cap=3, n_microbatches=4, enforce_mb_order=1)
    params, X, G = inputs(base, 2600)
    sub_ops = synth.subschedule_interleaved(4, n_sub, 3, 7)
    rcap = peak_rebuilt(sub_ops)
    Xd, Gd = to_dev(X, "bf16"), to_dev(G, "bf16")
    res = []
    for cfg in (base, dict(base, recompute=1, recompute_cap=rcap)):
        st = S.Stage(cfg)
        st.load_weights(params)
        Y, dX = torch.zeros_like(Xd), torch.zeros_like(Xd)
        st.run_subschedule(sub_ops, Xd, Gd, Y, dX)
        torch.cuda.synchronize()
        assert st.stats()["live"] == 0
        res.append((Y.clone(), dX.clone(), st.grads_tensor().clone()))
        st.close()
    for a, b in zip(*res):
        assert torch.equal(a, b)
    # cap of one rebuilt stash: the second B is refused, nothing changes, and it goes through after W(0)
    cfg = dict(base, n_sub=0, recompute=1, recompute_cap=1)
    st = S.Stage(cfg)
    st.load_weights(params)
    Y, dX = torch.zeros_like(Xd), torch.zeros_like(Xd)
    st.forward(0, Xd[0], Y[0]); st.forward(1, Xd[1], Y[1])
    st.backward_input(0, Gd[0], dX[0])
    with pytest.raises(S.StageError) as e:
        st.backward_input(1, Gd[1], dX[1])
    assert e.value.code == S.E_STASH_FULL and st.stats()["live"] == 2
    with pytest.raises(S.StageError) as e:
        st.run_schedule([(W, 0), (B, 1), (F, 2), (B, 2)], Xd, Gd, Y, dX)       # refused as a whole: B(2) while 1 is rebuilt
    assert e.value.code == S.E_STASH_FULL and st.stats()["live"] == 2
    st.run_schedule([(W, 0), (B, 1), (W, 1), (F, 2), (F, 3), (B, 2), (W, 2), (B, 3), (W, 3)], Xd, Gd, Y, dX)
    torch.cuda.synchronize()
    assert st.stats()["live"] == 0
    assert torch.equal(Y, res[0][0]) and torch.equal(dX, res[0][1]) and torch.equal(st.grads_tensor(), res[0][2])
    st.close()


@pytest.mark.parametrize("defer_w", [False, True])
def test_two_chunks_share_one_stash(defer_w):
    """Two model chunks on one device (paper section 3.1; looped / V-shaped placements): separate weights and
    gradients, one stash and one cap.  A two-chunk order runs through stage_run_chunk_schedule; every chunk matches its
    own oracle and, bit for bit, the same chunk run alone; the shared cap refuses an F on either chunk when the pool
    is empty and leaves everything untouched."""
    import torch
    from paper_2507_00217_amd import stage as S
    n_mb, cap = 5, 3
    cfg = dict(SMALL["cfg3s"], n_microbatches=n_mb, stash_cap=cap, enforce_mb_order=1)
    ops = synth.schedule_two_chunks(n_mb, cap, defer_w)
    assert S.stage_validate_chunk_schedule(cfg, 2, ops)[:2] == (0, -1)
    data = [inputs(cfg, 2900 + 10 * c) for c in range(2)]
    c0 = S.Stage(cfg)
    c1 = S.Stage(cfg, share_with=c0)
    chunks = [c0, c1]
    Xd, Gd, Y, dX = [], [], [], []
    for c, (params, X, G) in enumerate(data):
        chunks[c].load_weights(params)
        Xd.append(to_dev(X, "bf16")); Gd.append(to_dev(G, "bf16"))
        Y.append(torch.zeros_like(Xd[c])); dX.append(torch.zeros_like(Xd[c]))
    S.run_chunk_schedule(chunks, ops, Xd, Gd, Y, dX)
    torch.cuda.synchronize()
    assert c0.stats()["live"] == 0 and c1.stats()["live"] == 0 and c0.stats()["peak_live"] == cap == c1.stats()["peak_live"]
    for c, (params, X, G) in enumerate(data):
        own = [(k, m) for k, m, _, cc in ops if cc == c]
        ref = so.OracleStage(shape_of(cfg), params)
        Yr, dXr, _ = ref.run_schedule(own, X.astype(np.float64), G.astype(np.float64))
        got = (to_np(Y[c]), to_np(dX[c]), chunks[c].grads(), {"peak_live": 0, "live": 0})
        compare(cfg, got, (Yr, dXr, ref.grads, 0), TOL["bf16"])
        alone = S.Stage(dict(cfg, stash_cap=n_mb))
        alone.load_weights(params)
        Ya, dXa = torch.zeros_like(Xd[c]), torch.zeros_like(Xd[c])
        alone.run_schedule(own, Xd[c], Gd[c], Ya, dXa)
        torch.cuda.synchronize()
        assert torch.equal(Ya, Y[c]) and torch.equal(dXa, dX[c]) and torch.equal(alone.grads_tensor(), chunks[c].grads_tensor())
        alone.close()
    # shared cap: three live microbatches spread over both chunks fill the pool
    c0.forward(0, Xd[0][0], Y[0][0]); c1.forward(0, Xd[1][0], Y[1][0]); c0.forward(1, Xd[0][1], Y[0][1])
    for st, m in ((c1, 1), (c0, 2)):
        with pytest.raises(S.StageError) as e:
            st.forward(m, Xd[0][m], Y[0][m])
        assert e.value.code == S.E_STASH_FULL
    assert (c0.stats()["live"], c1.stats()["live"]) == (2, 1)
    with pytest.raises(S.StageError) as e:          # a list that would overflow the shared cap is refused as a whole
        S.run_chunk_schedule(chunks, [(B, 0, -1, 1), (F, 1, -1, 1)], Xd, Gd, Y, dX)
    assert e.value.code == S.E_STASH_FULL and (c0.stats()["live"], c1.stats()["live"]) == (2, 1)
    S.run_chunk_schedule(chunks, [(B, 0, -1, 1), (W, 0, -1, 1), (F, 1, -1, 1), (B, 1, -1, 1), (W, 1, -1, 1),
                                  (B, 0, -1, 0), (W, 0, -1, 0), (B, 1, -1, 0), (W, 1, -1, 0)], Xd, Gd, Y, dX)
    torch.cuda.synchronize()
    assert (c0.stats()["live"], c1.stats()["live"]) == (0, 0)
    # a chunk that needs another workspace than the first one's (here: a rotary table, which the first has none of) may not
    # be given the first one's buffer; with a workspace of its own it is accepted
    import ctypes as C
    rcfg = dict(cfg, rope_theta=10000.0)
    assert S.stage_query_sizes(rcfg)["stash"] == S.stage_query_sizes(cfg)["stash"]
    h = C.c_void_p()
    wts = torch.zeros(S.stage_query_sizes(rcfg)["weights"], dtype=torch.uint8, device="cuda:0")
    grd = torch.zeros(S.stage_query_sizes(rcfg)["grads"], dtype=torch.uint8, device="cuda:0")
    rc = S.lib().stage_init_chunk(C.byref(S.make_config(rcfg)), wts.data_ptr(), grd.data_ptr(), c0._ws.data_ptr(), c0.h, C.byref(h))
    assert rc == S.E_INVAL and not h.value
    c2 = S.Stage(rcfg, share_with=c0)
    assert c2._ws.data_ptr() != c0._ws.data_ptr()
    c2.close(); c1.close(); c0.close()


@pytest.mark.parametrize("name", ["cfg3s", "cfg5s"])
def test_schedule_replays_from_a_hip_graph(name):
    """A whole schedule iteration (gradient clearing included) captured into a HIP graph on a side stream replays to
    the eager result, bit for bit, on every replay -- with eager work and synchronisations between the replays.  The
    path launches kernels only (no memset or memcpy nodes), and the slot assignment made at capture time is the
    one every replay uses, because the tracker is back to empty at the end of an iteration."""
    import torch
    from paper_2507_00217_amd import stage as S
    cfg = SMALL[name]
    params, X, G = inputs(cfg, 9100)
    ops = synth.make_schedule(cfg)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        st = S.Stage(cfg, stream=side)
        st.load_weights(params)
        Xd, Gd = to_dev(X, cfg["dtype"]), to_dev(G, cfg["dtype"])
        Y, dX = torch.zeros_like(Xd), torch.zeros_like(Xd)
        st.zero_grads()
        st.run_schedule(ops, Xd, Gd, Y, dX)            # eager: the reference, and the first launch of every kernel
        side.synchronize()
        Yr, dXr, gr = Y.clone(), dX.clone(), st.grads_tensor().clone()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            st.zero_grads()
            st.run_schedule(ops, Xd, Gd, Y, dX)
        for rep in range(3):
            Y.fill_(7.0)
            dX.fill_(7.0)
            st.grads_tensor().fill_(3.0)
            noise = torch.randn(1 << 18, device="cuda").sum().item()      # eager work and a synchronisation in between
            assert noise == noise
            graph.replay()
            side.synchronize()
            assert torch.equal(Y, Yr) and torch.equal(dX, dXr), rep
            assert torch.equal(st.grads_tensor(), gr), rep
        assert st.stats()["live"] == 0
        st.close()
