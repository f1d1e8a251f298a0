"""Seeded input generators: determinism, distribution, bf16 rounding, and that
every generated op list is legal with the stated peak of live microbatches."""
import numpy as np
import pytest

from paper_2507_00217_amd import synth

F, B, W = synth.F, synth.B, synth.W


def test_normal_is_counter_based_and_standard():
    a = synth.normal(3, 1, (5, 1 << 20), threads=4)
    b = synth.normal(3, 1, (5 << 20,), threads=1)
    assert np.array_equal(a.ravel(), b)
    assert np.array_equal(synth.normal(3, 1, (1001,)), b[:1001])
    assert not np.array_equal(synth.normal(4, 1, (1001,)), b[:1001])
    assert not np.array_equal(synth.normal(3, 2, (1001,)), b[:1001])
    assert abs(b.mean()) < 2e-3 and abs(b.std() - 1) < 2e-3
    assert abs((b ** 3).mean()) < 1e-2 and abs((b ** 4).mean() - 3) < 3e-2
    assert abs(np.corrcoef(b[0::2], b[1::2])[0, 1]) < 2e-3


def test_round_bf16_ties_to_even():
    x = np.array([1.0, 1.00390625, 1.01171875, 1.0 + 2 ** -9, -3.1415927, 0.0], dtype=np.float32)
    r = synth.round_bf16(x)
    # 1+2^-8 is a tie between 1 and 1+2^-7 -> even (1.0); 1+3*2^-8 ties to 1+2^-6
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.015625 and r[3] == 1.0 and r[5] == 0.0
    assert abs(r[4] + 3.140625) < 1e-7
    assert np.array_equal(synth.from_bf16_bits(synth.to_bf16_bits(r)), r)


def check_legal(ops, n_mb, cap):
    state = [0] * n_mb
    live = peak = 0
    for k, m in ops:
        assert state[m] == k, (k, m)
        state[m] = (k + 1) % 3
        live += (k == F) - (k == W)
        peak = max(peak, live)
        assert live <= cap
    assert all(s == 0 for s in state) and len(ops) == 3 * n_mb
    return peak


@pytest.mark.parametrize("name,peak", [("cfg1", 2), ("cfg2", 4), ("cfg3", 8), ("cfg4", 6), ("cfg5", 6)])
def test_config_schedules(name, peak):
    cfg = synth.CONFIGS[name]
    ops = synth.make_schedule(cfg)
    cap = cfg["stash_cap"] or cfg["n_microbatches"]
    assert check_legal(ops, cfg["n_microbatches"], cap) == peak == synth.peak_live(ops)
    for kind in (F, B, W):                      # same-kind ops in microbatch order
        mbs = [m for k, m in ops if k == kind]
        assert mbs == sorted(mbs)


def test_cfg3_is_w_deferred():
    ops = synth.make_schedule(synth.CONFIGS["cfg3"])
    assert ops[-8:] == [(B, 12), (B, 13), (B, 14), (B, 15), (W, 12), (W, 13), (W, 14), (W, 15)]
    assert ops[:8] == [(F, i) for i in range(7)] + [(F, 7)]


def test_cfg5_w_postponed_at_most_3_slots():
    ops = synth.make_schedule(synth.CONFIGS["cfg5"])
    base = [op for op in ops if op[0] != W]
    for i in range(32):
        pb = base.index((B, i))
        n_base_before_w = len([op for op in ops[:ops.index((W, i))] if op[0] != W])
        assert 0 <= n_base_before_w - 1 - pb <= 3


@pytest.mark.parametrize("seed", range(5))
def test_random_schedule_is_legal(seed):
    ops = synth.schedule_random(10, 3, seed)
    assert check_legal(ops, 10, 3) <= 3
    assert ops != synth.schedule_random(10, 3, seed + 100)
