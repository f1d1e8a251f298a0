"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
headers declare, and its host logic (sizes, layout, schedule validator with the
stash cap) agrees with brute force.  No compute entry point is called."""
import ctypes
import itertools
import os
import re

import numpy as np
import pytest

from paper_2507_00217_amd import stage as S
from paper_2507_00217_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
F, B, W = 0, 1, 2


def declared_symbols():
    names = set()
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if fn.endswith(".h"):
            txt = open(os.path.join(ROOT, "include", fn)).read()
            txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
            names |= set(re.findall(r"\b((?:stage|crosspipe)_\w+)\s*\(", txt))
    return names


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(S.LIB_PATH)
    names = declared_symbols()
    assert {"stage_init", "stage_forward", "stage_backward_input", "stage_backward_weight", "stage_run_schedule",
            "stage_grads", "stage_kernel_gemm", "crosspipe_greedy", "crosspipe_simulate", "crosspipe_stage_ops"} <= names
    for n in names:
        assert hasattr(lib, n), n


def test_strerror_and_invalid_configs():
    assert S.strerror(0) == "ok" and "stash_cap" in S.strerror(S.E_STASH_FULL)
    good = synth.CONFIGS["cfg1"]
    S.stage_query_sizes(good)
    for key, val in [("hidden", 250), ("n_heads", 3), ("n_kv_heads", 3), ("ffn", 1000), ("seq", 0), ("stash_cap", 5),
                     ("n_heads", 1)]:
        bad = dict(good); bad[key] = val
        with pytest.raises(S.StageError) as e:
            S.stage_query_sizes(bad)
        assert e.value.code == S.E_INVAL
    # null out-pointer
    assert S.lib().stage_query_sizes(ctypes.byref(S.make_config(good)), None) == S.E_INVAL
    assert S.lib().stage_forward(None, 0, None, None) == S.E_INVAL


@pytest.mark.parametrize("name", list(synth.CONFIGS))
def test_layout_and_sizes(name):
    cfg = synth.CONFIGS[name]
    es = 4 if cfg["dtype"] == "fp32" else 2
    expect = 0
    for li in range(cfg["n_layers"]):
        for pname in S.PARAM_IDS:
            off, r, c = S.stage_param_layout(cfg, li, pname)
            if pname in synth.param_names(cfg):
                shp = synth.param_shape(cfg, pname)
                assert r * c == int.__mul__(*shp) if len(shp) == 2 else c == shp[0]
            else:
                assert r == 0 and c == 0
            assert off == expect and off % 8 == 0
            expect += r * c
    sz = S.stage_query_sizes(cfg)
    assert sz["weights"] >= expect * es and sz["grads"] >= expect * 4
    # the stash must at least hold what B and W read back (section 3.2): per layer-microbatch
    d, f, T = cfg["hidden"], cfg["ffn"], cfg["seq"] * cfg["mb_size"]
    dkv = cfg["n_kv_heads"] * (d // cfg["n_heads"])
    fin = 2 * f if cfg["act"] == "swiglu" else f
    need = (6 * d + 2 * dkv + fin + f) * T * es * cfg["n_layers"]
    cap = cfg["stash_cap"] or cfg["n_microbatches"]
    assert sz["stash"] % cap == 0 and need <= sz["stash"] // cap <= 1.6 * need
    assert sz["stash"] + sz["weights"] + sz["grads"] + sz["workspace"] < 200 * 2 ** 30


def ref_validate(ops, n_mb, cap, enforce):
    """Ten-line reference for the validator."""
    state, live, peak, last = [0] * n_mb, 0, 0, [-1, -1, -1]
    for i, (k, m) in enumerate(ops):
        if not (0 <= k <= 2 and 0 <= m < n_mb):
            return S.E_INVAL, i, peak
        if state[m] != k or (enforce and (m <= last[k] or (k != F and k in state[:m]))):
            return S.E_ORDER, i, peak
        if k == F and live >= cap:
            return S.E_STASH_FULL, i, peak
        state[m] = (k + 1) % 3; last[k] = m
        live += (k == F) - (k == W); peak = max(peak, live)
        if live == 0:
            last = [-1, -1, -1]
    return 0, -1, peak


@pytest.mark.parametrize("enforce", [0, 1])
@pytest.mark.parametrize("cap", [1, 2, 3])
def test_validator_brute_force(cap, enforce):
    n_mb = 3
    cfg = dict(synth.CONFIGS["cfg1"], n_microbatches=n_mb, stash_cap=cap, enforce_mb_order=enforce)
    alphabet = [(k, m) for k in range(3) for m in range(n_mb)]
    n_ok = 0
    for length in range(0, 5):
        for ops in itertools.product(alphabet, repeat=length):
            got = S.stage_validate_schedule(cfg, list(ops))
            assert got == ref_validate(ops, n_mb, cap, enforce), ops
            n_ok += got[0] == 0
    assert n_ok > 10
    # all complete interleavings of 2 microbatches' F,B,W chains, extended to full length 9 for 3
    for perm in set(itertools.permutations([0, 0, 0, 1, 1, 1, 2, 2, 2])):
        nxt = [0, 0, 0]
        ops = []
        for m in perm:
            ops.append((nxt[m], m)); nxt[m] += 1
        assert S.stage_validate_schedule(cfg, ops) == ref_validate(ops, n_mb, cap, enforce), ops
    assert S.stage_validate_schedule(cfg, [(3, 0)])[0] == S.E_INVAL
    assert S.stage_validate_schedule(cfg, [(0, 3)])[0] == S.E_INVAL


@pytest.mark.parametrize("name,peak", [("cfg1", 2), ("cfg2", 4), ("cfg3", 8), ("cfg4", 6), ("cfg5", 6)])
def test_config_schedules_validate(name, peak):
    cfg = dict(synth.CONFIGS[name], enforce_mb_order=1)
    ops = synth.make_schedule(cfg)
    assert S.stage_validate_schedule(cfg, ops) == (0, -1, peak)
    # one slot fewer than the schedule's peak: the F that would exceed it is refused
    tight = dict(cfg, stash_cap=peak - 1)
    rc, bad, pk = S.stage_validate_schedule(tight, ops)
    assert rc == S.E_STASH_FULL and ops[bad][0] == F and pk == peak - 1
    # reordering W later keeps the peak under the same cap (same peak activation memory)
    plain = synth.schedule_1f1b(cfg["n_microbatches"], peak - 1)
    assert S.stage_validate_schedule(cfg, plain)[2] == peak


def test_random_order_violates_mb_order_only():
    cfg = dict(synth.CONFIGS["cfg5"])
    ops = synth.schedule_random(32, 8, 5003)
    assert S.stage_validate_schedule(cfg, ops)[0] == 0
    ws = [m for k, m in ops if k == W]
    assert ws != sorted(ws)
    assert S.stage_validate_schedule(dict(cfg, enforce_mb_order=1), ops)[0] == S.E_ORDER


def ref_validate_sub(ops, n_mb, n_sub, cap, enforce):
    """Reference for the sub-block validator."""
    nf, nb, wd = [0] * n_mb, [0] * n_mb, [set() for _ in range(n_mb)]
    live = peak = 0
    last = {}
    def waits(m, k, s):
        if k == B:
            return nf[m] == n_sub and s == n_sub - 1 - nb[m]
        if k == W:
            return s >= n_sub - nb[m] and s not in wd[m]
        return False
    for i, (k, m, s) in enumerate(ops):
        if not (0 <= k <= 2 and 0 <= m < n_mb and 0 <= s < n_sub):
            return S.E_INVAL, i, peak
        ok = (s == nf[m] and nb[m] == 0 and not wd[m]) if k == F else waits(m, k, s)
        if not ok:
            return S.E_ORDER, i, peak
        if enforce and (m <= last.get((k, s), -1) or (k != F and any(waits(x, k, s) for x in range(m)))):
            return S.E_ORDER, i, peak
        if k == F and s == 0 and live >= cap:
            return S.E_STASH_FULL, i, peak
        last[(k, s)] = m
        if k == F:
            if s == 0:
                live += 1; peak = max(peak, live)
            nf[m] += 1
        elif k == B:
            nb[m] += 1
        else:
            wd[m].add(s)
            if len(wd[m]) == n_sub:
                nf[m] = nb[m] = 0; wd[m] = set(); live -= 1
                if live == 0:
                    last = {}
    return 0, -1, peak


@pytest.mark.parametrize("enforce", [0, 1])
def test_sub_block_validator_brute_force(enforce):
    n_mb, n_sub, cap = 2, 2, 1
    cfg = dict(synth.CONFIGS["cfg1"], n_microbatches=n_mb, stash_cap=cap, enforce_mb_order=enforce, n_sub=n_sub)
    alphabet = [(k, m, s) for k in range(3) for m in range(n_mb) for s in range(n_sub)]
    n_ok = 0
    for length in range(0, 5):
        for ops in itertools.product(alphabet, repeat=length):
            got = S.stage_validate_subschedule(cfg, list(ops))
            assert got == ref_validate_sub(ops, n_mb, n_sub, cap, enforce), ops
            n_ok += got[0] == 0
    assert n_ok > 5
    cfg = dict(cfg, n_microbatches=4, stash_cap=3, n_sub=2)
    for seed in range(4):
        ops = synth.subschedule_interleaved(4, 2, 3, seed)
        got = S.stage_validate_subschedule(cfg, ops)
        assert got == ref_validate_sub(ops, 4, 2, 3, enforce) and got[0] == 0
        assert S.stage_validate_subschedule(dict(cfg, stash_cap=1), ops)[0] in (S.E_STASH_FULL, 0)
    assert S.stage_validate_subschedule(cfg, [(0, 0, 2)])[0] == S.E_INVAL
    with pytest.raises(S.StageError):
        S.stage_query_sizes(dict(cfg, n_sub=3))          # must divide n_layers


def test_recomputation_sizes_and_validator():
    """Layer-wise recomputation (section 7.2, Case 2): the F-to-W slot shrinks to the layer inputs, the full-size
    record is only held from B to W and is capped separately; the validator refuses the B that would exceed it."""
    base = dict(synth.CONFIGS["cfg3"])
    plain = S.stage_query_sizes(base)
    cap = base["stash_cap"]
    T, d, L = base["seq"] * base["mb_size"], base["hidden"], base["n_layers"]
    small = L * T * d * 4
    for rcap in (1, 2, cap):
        cfg = dict(base, recompute=1, recompute_cap=rcap)
        sz = S.stage_query_sizes(cfg)
        full = plain["stash"] // cap - small               # a full record has no x of its own
        assert sz["stash"] == cap * small + rcap * full
        assert sz["workspace"] == plain["workspace"] + full // L
    assert S.stage_query_sizes(dict(base, recompute=1))["stash"] == S.stage_query_sizes(dict(base, recompute=1, recompute_cap=cap))["stash"]
    for bad in (dict(recompute=0, recompute_cap=1), dict(recompute=2), dict(recompute=1, recompute_cap=cap + 1),
                dict(recompute=1, recompute_cap=-1)):
        with pytest.raises(S.StageError):
            S.stage_query_sizes(dict(base, **bad))
    cfg = dict(base, n_microbatches=4, stash_cap=4, recompute=1, recompute_cap=1)
    f4 = [(F, m) for m in range(4)]
    rc, bad, peak = S.stage_validate_schedule(cfg, f4 + [(B, 0), (B, 1)])
    assert (rc, bad, peak) == (S.E_STASH_FULL, 5, 4)
    rc, bad, peak = S.stage_validate_schedule(cfg, f4 + [(B, 0), (W, 0), (B, 1), (W, 1), (B, 2), (W, 2), (B, 3), (W, 3)])
    assert (rc, bad, peak) == (0, -1, 4)
    rc, bad, _ = S.stage_validate_schedule(dict(cfg, recompute_cap=2), f4 + [(B, 0), (B, 1), (W, 0), (B, 2), (B, 3)])
    assert (rc, bad) == (S.E_STASH_FULL, 8)
    sub = dict(cfg, n_sub=2)
    rc, bad, _ = S.stage_validate_subschedule(sub, [(F, 0, 0), (F, 0, 1), (F, 1, 0), (F, 1, 1), (B, 0, 1), (B, 1, 1)])
    assert (rc, bad) == (S.E_STASH_FULL, 5)
    rc, bad, _ = S.stage_validate_subschedule(sub, [(F, 0, 0), (F, 0, 1), (F, 1, 0), (F, 1, 1), (B, 0, 1), (B, 0, 0), (W, 0, 1),
                                                    (W, 0, 0), (B, 1, 1)])
    assert (rc, bad) == (0, -1)


def ref_validate_chunks(ops, n_chunks, n_mb, cap, enforce):
    """Reference for the chunk validator: per-chunk microbatch state machines, one cap over all chunks."""
    state = [[0] * n_mb for _ in range(n_chunks)]
    last = [[-1, -1, -1] for _ in range(n_chunks)]
    own = [0] * n_chunks
    live = peak = 0
    for i, (k, m, sub, c) in enumerate(ops):
        if not (0 <= c < n_chunks and 0 <= k <= 2 and 0 <= m < n_mb and sub == -1):
            return S.E_INVAL, i, peak
        if state[c][m] != k or (enforce and (m <= last[c][k] or (k != F and k in state[c][:m]))):
            return S.E_ORDER, i, peak
        if k == F and live >= cap:
            return S.E_STASH_FULL, i, peak
        state[c][m] = (k + 1) % 3; last[c][k] = m
        d = (k == F) - (k == W)
        live += d; own[c] += d; peak = max(peak, live)
        if own[c] == 0 and k == W:
            last[c] = [-1, -1, -1]
    return 0, -1, peak


@pytest.mark.parametrize("enforce", [0, 1])
@pytest.mark.parametrize("cap", [2, 3])
def test_chunk_validator(cap, enforce):
    """Two model chunks on one stash (paper section 3.1: ops carry a chunk index): generated two-chunk orders are
    legal at their cap and not below it; random op sequences agree with the reference, error code, position and peak."""
    cfg = dict(synth.CONFIGS["cfg1"], n_microbatches=3, stash_cap=cap, enforce_mb_order=enforce)
    ops = synth.schedule_two_chunks(3, cap, defer_w=bool(enforce))
    rc, bad, peak = S.stage_validate_chunk_schedule(cfg, 2, ops)
    assert (rc, bad) == (0, -1) and peak == cap
    if cap > 2:
        rc, bad, _ = S.stage_validate_chunk_schedule(dict(cfg, stash_cap=cap - 1), 2, ops)
        assert rc == S.E_STASH_FULL and ops[bad][0] == F
    assert S.stage_validate_chunk_schedule(cfg, 1, ops)[0] == S.E_INVAL            # chunk index out of range
    rng = np.random.default_rng(100 * cap + enforce)
    seen = set()
    for _ in range(3000):
        n = int(rng.integers(1, 12))
        seq = [(int(rng.integers(0, 3)), int(rng.integers(0, 3)), -1, int(rng.integers(0, 2))) for _ in range(n)]
        got = S.stage_validate_chunk_schedule(cfg, 2, seq)
        want = ref_validate_chunks(seq, 2, 3, cap, enforce)
        assert got == want, (seq, got, want)
        seen.add(want[0])
    assert seen >= {S.E_ORDER, S.E_STASH_FULL} or cap > 2
