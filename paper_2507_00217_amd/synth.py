"""Seeded synthetic inputs for the pipeline-stage engine: workload shapes,
weights, boundary tensors and per-stage op lists.

This module holds none of the method's arithmetic.  It is the one module that
both the HIP path's tests/benchmark and the CPU oracle's tests draw inputs
from, so that the two sides see identical numbers.

Random numbers come from a counter-based generator defined here (splitmix64 on
(seed, tensor id, index) followed by Box-Muller), never from a library RNG, so
values do not depend on library version, thread count or chunking.

Workloads stand in for the paper's evaluation models (section 7, table of
Llama-style layer hyper-parameters; microbatch size 1 and sequence length 4096
by default there): a stage only ever sees activations and gradients at its
boundary, so i.i.d. N(0,1) boundary tensors and N(0, 0.02^2) weights of the
same shapes replace the training corpus and trained weights.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List, Tuple

import numpy as np

F, B, W = 0, 1, 2

# name -> shape of one stage.  "m70" is the paper's M70 layer (section 7, table
# of model hyper-parameters); the others are the parity/benchmark workloads.
CONFIGS: Dict[str, dict] = {
    "cfg1": dict(n_layers=2, hidden=256, n_heads=4, n_kv_heads=4, ffn=1024, seq=128, mb_size=1,
                 n_microbatches=4, norm="layernorm", act="gelu", dtype="fp32", stash_cap=0, schedule="1f1b", warmup=1),
    "cfg2": dict(n_layers=6, hidden=2048, n_heads=16, n_kv_heads=16, ffn=8192, seq=2048, mb_size=1,
                 n_microbatches=8, norm="layernorm", act="gelu", dtype="bf16", stash_cap=0, schedule="1f1b", warmup=3),
    "cfg3": dict(n_layers=4, hidden=4096, n_heads=32, n_kv_heads=32, ffn=11008, seq=4096, mb_size=1,
                 n_microbatches=16, norm="rmsnorm", act="swiglu", dtype="bf16", stash_cap=8, schedule="w_deferred", warmup=7),
    "cfg4": dict(n_layers=8, hidden=5120, n_heads=40, n_kv_heads=40, ffn=13824, seq=2048, mb_size=2,
                 n_microbatches=12, norm="layernorm", act="gelu", dtype="bf16", stash_cap=6, schedule="w_lag1", warmup=4),
    "cfg5": dict(n_layers=2, hidden=8192, n_heads=64, n_kv_heads=8, ffn=28672, seq=4096, mb_size=1,
                 n_microbatches=32, norm="rmsnorm", act="swiglu", dtype="bf16", stash_cap=8, schedule="greedy", warmup=4),
    # the GPT-style stage with linear biases (GPT-style layers carry them; the paper's Llama-style ones do not)
    "cfg2_bias": dict(n_layers=6, hidden=2048, n_heads=16, n_kv_heads=16, ffn=8192, seq=2048, mb_size=1, bias=1,
                      n_microbatches=8, norm="layernorm", act="gelu", dtype="bf16", stash_cap=0, schedule="1f1b", warmup=3),
    # further shapes of the paper's models (section 7): the M8 layer, and the share of an M70 / M8 layer that one GPU
    # holds under 4-way tensor parallelism (a quarter of the heads and of the ffn against the full hidden width); these
    # are Llama-style layers, so they carry the rotary position embedding
    "m8": dict(n_layers=4, hidden=4096, n_heads=32, n_kv_heads=8, ffn=14336, seq=4096, mb_size=1, rope_theta=10000.0,
               n_microbatches=16, norm="rmsnorm", act="swiglu", dtype="bf16", stash_cap=8, schedule="w_deferred", warmup=7),
    "m70_tp4": dict(n_layers=4, hidden=8192, n_heads=16, n_kv_heads=2, head_dim=128, ffn=7168, seq=4096, mb_size=1,
                    rope_theta=10000.0, n_microbatches=16, norm="rmsnorm", act="swiglu", dtype="bf16", stash_cap=8, schedule="w_deferred", warmup=7),
    "m8_tp4": dict(n_layers=4, hidden=4096, n_heads=8, n_kv_heads=2, head_dim=128, ffn=3584, seq=4096, mb_size=1,
                   rope_theta=10000.0, n_microbatches=16, norm="rmsnorm", act="swiglu", dtype="bf16", stash_cap=8, schedule="w_deferred", warmup=7),
}

_MASK = np.uint64(0xFFFFFFFFFFFFFFFF)
_GOLD = np.uint64(0x9E3779B97F4A7C15)


def _splitmix64(z: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        z = (z + _GOLD)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def _key(seed: int, tensor_id: int) -> np.uint64:
    k = _splitmix64(np.array([seed & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64))
    k = _splitmix64(k ^ np.uint64(tensor_id & 0xFFFFFFFFFFFFFFFF))
    return k[0]


def _normal_chunk(key: np.uint64, start_pair: int, n_pairs: int) -> np.ndarray:
    with np.errstate(over="ignore"):
        ctr = (np.arange(start_pair, start_pair + n_pairs, dtype=np.uint64) * np.uint64(2))
        a = _splitmix64(key + ctr * _GOLD)
        b = _splitmix64(key + (ctr + np.uint64(1)) * _GOLD)
    u1 = 1.0 - (a >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)   # (0, 1]
    u2 = (b >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)         # [0, 1)
    r = np.sqrt(-2.0 * np.log(u1))
    t = (2.0 * np.pi) * u2
    out = np.empty(2 * n_pairs, dtype=np.float32)
    out[0::2] = r * np.cos(t)
    out[1::2] = r * np.sin(t)
    return out


def normal(seed: int, tensor_id: int, shape, mean: float = 0.0, std: float = 1.0, threads: int = 8) -> np.ndarray:
    """float32 array of i.i.d. N(mean, std^2); element i depends only on (seed, tensor_id, i)."""
    n = int(np.prod(shape))
    n_pairs = (n + 1) // 2
    key = _key(seed, tensor_id)
    chunk = 1 << 20
    starts = list(range(0, n_pairs, chunk))
    out = np.empty(2 * n_pairs, dtype=np.float32)

    def work(s):
        c = min(chunk, n_pairs - s)
        out[2 * s:2 * (s + c)] = _normal_chunk(key, s, c)

    if len(starts) > 1 and threads > 1:
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(work, starts))
    else:
        for s in starts:
            work(s)
    out = out[:n]
    if std != 1.0:
        out *= np.float32(std)
    if mean != 0.0:
        out += np.float32(mean)
    return out.reshape(shape)


def round_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bfloat16 (ties to even); returned as float32."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    u = (u + r) & np.uint32(0xFFFF0000)
    return u.view(np.float32)


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 values that are exactly representable in bf16 -> uint16 bit patterns."""
    return (np.ascontiguousarray(a, dtype=np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


PARAM_NAMES_LN = ("g1", "b1", "wqkv", "wo", "g2", "b2", "win", "wout")
PARAM_NAMES_RMS = ("g1", "wqkv", "wo", "g2", "win", "wout")
BIAS_NAMES = ("bqkv", "bo", "bin", "bout")      # linear biases, present when cfg["bias"] is set (GPT-style layers)


def param_names(cfg: dict) -> Tuple[str, ...]:
    base = PARAM_NAMES_LN if cfg["norm"] == "layernorm" else PARAM_NAMES_RMS
    return base + BIAS_NAMES if cfg.get("bias") else base


def param_shape(cfg: dict, name: str) -> Tuple[int, ...]:
    d, f = cfg["hidden"], cfg["ffn"]
    hd = cfg.get("head_dim") or d // cfg["n_heads"]          # a tensor-parallel share keeps hidden but has fewer heads
    da, dkv = cfg["n_heads"] * hd, cfg["n_kv_heads"] * hd
    fin = 2 * f if cfg["act"] == "swiglu" else f
    return {"g1": (d,), "b1": (d,), "g2": (d,), "b2": (d,),
            "wqkv": (d, da + 2 * dkv), "wo": (da, d), "win": (d, fin), "wout": (f, d),
            "bqkv": (da + 2 * dkv,), "bo": (d,), "bin": (fin,), "bout": (d,)}[name]


def make_weights(cfg: dict, seed: int) -> List[Dict[str, np.ndarray]]:
    """Linear weights N(0, 0.02^2); norm scales 1 + N(0, 0.02^2); norm shifts and linear biases
    N(0, 0.02^2).  Rounded once to bf16 when cfg['dtype'] == 'bf16'."""
    out = []
    for li in range(cfg["n_layers"]):
        lp = {}
        for pi, name in enumerate(PARAM_NAMES_LN + BIAS_NAMES):
            if name not in param_names(cfg):
                continue
            w = normal(seed, 100 * li + pi, param_shape(cfg, name), mean=1.0 if name in ("g1", "g2") else 0.0, std=0.02)
            lp[name] = round_bf16(w) if cfg["dtype"] == "bf16" else w
        out.append(lp)
    return out


def make_boundary(cfg: dict, seed: int, n_microbatches: int | None = None) -> np.ndarray:
    """N(0,1) stage-boundary tensor [n_mb, mb_size, seq, hidden] (stage input
    activations, or output gradients, depending on the seed passed)."""
    n = cfg["n_microbatches"] if n_microbatches is None else n_microbatches
    x = normal(seed, 7, (n, cfg["mb_size"], cfg["seq"], cfg["hidden"]))
    return round_bf16(x) if cfg["dtype"] == "bf16" else x


# ---------------------------------------------------------------------------
# per-stage ordered op lists (the consumer side of the paper's "per-stage
# schedule S_d", Alg. 1): lists of (kind, microbatch)
# ---------------------------------------------------------------------------

def schedule_1f1b(n_mb: int, warmup: int) -> List[Tuple[int, int]]:
    """1F1B with W immediately after its B (undivided backward order)."""
    warmup = min(warmup, n_mb)
    ops = [(F, i) for i in range(warmup)]
    for i in range(n_mb):
        if i + warmup < n_mb:
            ops.append((F, i + warmup))
        ops += [(B, i), (W, i)]
    return ops


def schedule_two_chunks(n_mb: int, cap: int, defer_w: bool = False) -> List[Tuple[int, int, int, int]]:
    """Per-device op list (kind, mb, sub=-1, chunk) for a device that holds two model chunks of a looped placement (the
    situation of interleaved 1F1B / ZB-V in the paper's table of schedules): microbatch m runs F on chunk 0, later F on
    chunk 1, B on chunk 1, then B on chunk 0.  A list scheduler: backward work first when there is any (deepest chunk
    first), else the forward that is furthest along, while at most `cap` (chunk, microbatch) stashes are live;
    W follows its B at once, or (defer_w) as late as the cap allows."""
    assert cap >= 2
    ops: List[Tuple[int, int, int, int]] = []
    f_done = [0, 0]                  # forwards issued per chunk (microbatches go in order)
    b_done = [0, 0]
    w_pending: List[Tuple[int, int]] = []
    live = 0
    while b_done[0] < n_mb or w_pending:
        # backward available?  chunk 1 needs its own F; chunk 0 needs chunk 1's B of the same microbatch
        if b_done[1] < f_done[1] and (b_done[1] <= b_done[0] or True):
            c = 1
        elif b_done[0] < b_done[1]:
            c = 0
        else:
            c = -1
        can_f1 = f_done[1] < f_done[0] and f_done[1] < n_mb
        can_f0 = f_done[0] < n_mb and live <= cap - 2      # keep a slot for that microbatch's chunk-1 forward
        if live >= cap and w_pending:
            cc, m = w_pending.pop(0); ops.append((W, m, -1, cc)); live -= 1
            continue
        if c >= 0 and (live >= cap or not (can_f0 or can_f1) or f_done[0] - b_done[0] >= cap // 2 + 1):
            m = b_done[c]; ops.append((B, m, -1, c)); b_done[c] += 1
            if defer_w:
                w_pending.append((c, m))
            else:
                ops.append((W, m, -1, c)); live -= 1
            continue
        if live < cap and can_f1 and (f_done[0] - f_done[1] >= 2 or not can_f0):
            ops.append((F, f_done[1], -1, 1)); f_done[1] += 1; live += 1
            continue
        if live < cap and can_f0:
            ops.append((F, f_done[0], -1, 0)); f_done[0] += 1; live += 1
            continue
        if live < cap and can_f1:
            ops.append((F, f_done[1], -1, 1)); f_done[1] += 1; live += 1
            continue
        if c >= 0:
            m = b_done[c]; ops.append((B, m, -1, c)); b_done[c] += 1
            if defer_w:
                w_pending.append((c, m))
            else:
                ops.append((W, m, -1, c)); live -= 1
            continue
        cc, m = w_pending.pop(0); ops.append((W, m, -1, cc)); live -= 1
    return ops


def schedule_w_deferred(n_mb: int, warmup: int, tail: int) -> List[Tuple[int, int]]:
    """1F1B body, but the last `tail` microbatches run all their B first and
    their W afterwards (W fills what would be the tear-down bubbles)."""
    warmup = min(warmup, n_mb)
    ops = [(F, i) for i in range(warmup)]
    for i in range(n_mb - tail):
        if i + warmup < n_mb:
            ops.append((F, i + warmup))
        ops += [(B, i), (W, i)]
    for i in range(n_mb - tail, n_mb):
        if i + warmup < n_mb:
            ops.append((F, i + warmup))
        ops.append((B, i))
    ops += [(W, i) for i in range(n_mb - tail, n_mb)]
    return ops


def schedule_w_lag1(n_mb: int, warmup: int) -> List[Tuple[int, int]]:
    """W interleaved between F and B, each W one slot behind its B."""
    ops = [(F, i) for i in range(warmup)]
    for i in range(n_mb):
        ops.append((B, i))
        if i + warmup < n_mb:
            ops.append((F, i + warmup))
        if i >= 1:
            ops.append((W, i - 1))
    ops.append((W, n_mb - 1))
    return ops


def schedule_greedy(n_mb: int, warmup: int) -> List[Tuple[int, int]]:
    """Alternating B/F base order; W_i postponed d_i in {0,1,2,3,2,1,...} base
    slots after B_i, clamped to the end, emitted in microbatch order."""
    base = [(F, i) for i in range(warmup)]
    for i in range(n_mb):
        base.append((B, i))
        if i + warmup < n_mb:
            base.append((F, i + warmup))
    pos_b = {mb: j for j, (k, mb) in enumerate(base) if k == B}
    after: Dict[int, List[int]] = {}
    nxt = 0
    for i in range(n_mb):
        delay = 3 - abs(3 - (i % 6))
        slot = min(pos_b[i] + delay, len(base) - 1)
        slot = max(slot, nxt)          # keep W in microbatch order
        nxt = slot
        after.setdefault(slot, []).append(i)
    ops = []
    for j, op in enumerate(base):
        ops.append(op)
        ops += [(W, i) for i in after.get(j, [])]
    return ops


def schedule_random(n_mb: int, cap: int, seed: int) -> List[Tuple[int, int]]:
    """Seeded uniform choice among legal next ops: F in microbatch order while
    fewer than `cap` microbatches are live; any B whose F ran; any W whose B ran."""
    cap = cap or n_mb
    rng_vals = _splitmix64(_key(seed, 3) + np.arange(4 * n_mb, dtype=np.uint64) * _GOLD)
    nf, fwd, bwd, ops = 0, [], [], []
    for step in range(3 * n_mb):
        cand = []
        if nf < n_mb and len(fwd) + len(bwd) < cap:
            cand.append((F, nf))
        cand += [(B, m) for m in fwd] + [(W, m) for m in bwd]
        kind, mb = cand[int(rng_vals[step] % np.uint64(len(cand)))]
        if kind == F:
            fwd.append(mb); nf += 1
        elif kind == B:
            fwd.remove(mb); bwd.append(mb)
        else:
            bwd.remove(mb)
        ops.append((kind, mb))
    return ops


def expand_to_subops(ops, n_sub: int) -> List[Tuple[int, int, int]]:
    """Every whole op replaced by its sub-blocks back to back (F, W ascending; B descending)."""
    out = []
    for k, m in ops:
        subs = range(n_sub - 1, -1, -1) if k == B else range(n_sub)
        out += [(k, m, sb) for sb in subs]
    return out


def subschedule_interleaved(n_mb: int, n_sub: int, cap: int, seed: int) -> List[Tuple[int, int, int]]:
    """Seeded random legal order at sub-block grain: F sub-blocks of a microbatch ascending, B descending after all
    its F, W(mb, sub) any time after B(mb, sub); at most `cap` microbatches live; same (kind, sub) in microbatch order."""
    rng_vals = _splitmix64(_key(seed, 4) + np.arange(4 * 3 * n_mb * n_sub, dtype=np.uint64) * _GOLD)
    nf = [0] * n_mb; nb = [0] * n_mb; wdone = [set() for _ in range(n_mb)]
    nxt = {}
    ops, step = [], 0
    live = lambda: sum(1 for m in range(n_mb) if nf[m] > 0 and len(wdone[m]) < n_sub)
    while len(ops) < 3 * n_mb * n_sub:
        cand = []
        for m in range(n_mb):
            if len(wdone[m]) == n_sub:
                continue
            if nf[m] < n_sub and (nf[m] > 0 or live() < cap):
                cand.append((F, m, nf[m]))
            if nf[m] == n_sub and nb[m] < n_sub:
                cand.append((B, m, n_sub - 1 - nb[m]))
            for sb in range(n_sub - nb[m], n_sub):
                if sb not in wdone[m]:
                    cand.append((W, m, sb))
        cand = [c for c in cand if nxt.get((c[0], c[2]), 0) == c[1]]     # each (kind, sub) visits microbatches in order
        k, m, sb = cand[int(rng_vals[step] % np.uint64(len(cand)))]
        step += 1
        nxt[(k, sb)] = m + 1
        if k == F:
            nf[m] += 1
        elif k == B:
            nb[m] += 1
        else:
            wdone[m].add(sb)
        ops.append((k, m, sb))
    return ops


def make_schedule(cfg: dict, n_mb: int | None = None) -> List[Tuple[int, int]]:
    n = cfg["n_microbatches"] if n_mb is None else n_mb
    kind = cfg["schedule"]
    wu = min(cfg["warmup"], n)
    if kind == "1f1b":
        return schedule_1f1b(n, wu)
    if kind == "w_deferred":
        return schedule_w_deferred(n, wu, min(4, n))
    if kind == "w_lag1":
        return schedule_w_lag1(n, wu)
    if kind == "greedy":
        return schedule_greedy(n, wu)
    raise ValueError(kind)


def peak_live(ops) -> int:
    live, peak = 0, 0
    for k, _ in ops:
        if k == F:
            live += 1
        elif k == W:
            live -= 1
        peak = max(peak, live)
    return peak


# ---------------------------------------------------------------------------
# whole-pipeline inputs for the schedule generator / performance model:
# static per-stage orders (paper section 5.1, table of static schedules) as
# (kind, mb, sub) lists per stage, kind 1 = the input-gradient block D
# ---------------------------------------------------------------------------

def pipeline_1f1b(n_pp: int, n_mb: int, n_sub: int = 1) -> List[List[Tuple[int, int, int]]]:
    """1F1B with the weight gradient combined: stage s warms up with n_pp - s - 1 forwards, then alternates one
    forward and one backward (D immediately followed by its W)."""
    out = []
    for s in range(n_pp):
        warm = min(n_pp - s - 1, n_mb)
        ops = [(F, i) for i in range(warm)]
        for i in range(n_mb):
            if i + warm < n_mb:
                ops.append((F, i + warm))
            ops += [(B, i), (W, i)]
        out.append(expand_to_subops(ops, n_sub))
    return out


def delay_matrices(n_pp: int, n_dc: int, lat: float, inv_bw: float):
    """alpha / beta matrices for n_pp stages spread evenly over n_dc datacenters in order: only links that cross a
    datacenter boundary have latency `lat` and inverse bandwidth `inv_bw`; links inside one are free."""
    per = n_pp // n_dc
    dc = [min(i // per, n_dc - 1) for i in range(n_pp)]
    alpha = [[lat if dc[i] != dc[j] else 0.0 for j in range(n_pp)] for i in range(n_pp)]
    beta = [[inv_bw if dc[i] != dc[j] else 0.0 for j in range(n_pp)] for i in range(n_pp)]
    return alpha, beta
