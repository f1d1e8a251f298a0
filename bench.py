#!/usr/bin/env python3
"""Benchmark of the pipeline-stage F/B/W engine on one MI355X.

A "step" is one full schedule iteration of the workload: every F, B and W op of
all its microbatches, in the workload's op order, through stage_run_schedule.
Inputs (weights, boundary activations and gradients) are resident in HBM before
the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config cfg3]

FLOP convention (algorithmic work only): GEMM 2*M*N*K; causal attention forward
2*b*s^2*d (half the dense 4*b*s^2*d), backward 2.5x forward; norm / activation
arithmetic not counted.  F = GEMMs + attention forward, B = GEMMs + attention
backward, W = GEMMs.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA, published
PEAK_FP32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0


def measured_gemm_traffic(config):
    """HBM-side bytes per GEMM launch (average over the forward, input-gradient and grouped weight-gradient launches of
    one iteration of the workload's default schedule), taken from the rocprofv3 --pmc summary
    profiles/<config>_schedule_pmc.md (FETCH_SIZE and WRITE_SIZE, each scaled by the same counter's reading for a plain
    copy kernel of known size).  That file records which GEMM source it was measured with; when the source in the tree
    is another one the figure is stale and None is returned."""
    import hashlib
    import re
    path = os.path.join(ROOT, "profiles", f"{config}_schedule_pmc.md")
    src = os.path.join(ROOT, "paper_2507_00217_amd", "csrc", "gemm_mfma.hip")
    try:
        text = open(path).read()
        sha = hashlib.sha256(open(src, "rb").read()).hexdigest()[:16]
    except OSError:
        return None
    m = re.search(r"gemm_traffic_bytes_per_launch\s*=\s*([0-9.eE+]+)\s*;\s*gemm_mfma\.hip sha256/16\s*=\s*([0-9a-f]{16})", text)
    return float(m.group(1)) if m and m.group(2) == sha else None


def flops_per_layer_mb(cfg):
    d, f, h = cfg["hidden"], cfg["ffn"], cfg["n_heads"]
    hd = cfg.get("head_dim") or d // h
    da, dkv = h * hd, cfg["n_kv_heads"] * hd
    T = cfg["seq"] * cfg["mb_size"]
    fin = 2 * f if cfg["act"] == "swiglu" else f
    gemm = 2.0 * T * (d * (da + 2 * dkv) + da * d + d * fin + f * d)
    attn = (2.0 if cfg.get("causal", True) else 4.0) * cfg["mb_size"] * cfg["seq"] ** 2 * da
    return {"F": gemm + attn, "B": gemm + 2.5 * attn, "W": gemm, "gemm": gemm, "attn_fwd": attn}


def cpu_baseline(cfg, budget_s=30.0):
    """Times the CPU oracle (as it stands) on one layer / one microbatch of the
    same shapes: F, B and W, fp64."""
    import numpy as np
    from oracle import stage_oracle as so
    from paper_2507_00217_amd import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    one = dict(cfg, n_layers=1, n_microbatches=1)
    fl = flops_per_layer_mb(one)
    # bound the sample: shorten the sequence until the estimate fits the budget (assume ~25 GFLOP/s/core fp64)
    est = lambda c: sum(flops_per_layer_mb(c)[k] for k in "FBW") / (25e9 * cores)
    while est(one) > budget_s and one["seq"] > 256:
        one["seq"] //= 2
    fl = flops_per_layer_mb(one)
    params = synth.make_weights(one, 1)
    X = synth.make_boundary(one, 2).astype(np.float64)
    G = synth.make_boundary(one, 3).astype(np.float64)
    sh = so.Shape(1, one["hidden"], one["n_heads"], one["n_kv_heads"], one["ffn"], one["seq"], one["mb_size"],
                  one["norm"], one["act"], True, hd=one.get("head_dim", 0) or 0)
    st = so.OracleStage(sh, params)
    t0 = time.perf_counter(); st.forward(0, X[0]); t1 = time.perf_counter()
    st.backward_input(0, G[0]); t2 = time.perf_counter()
    st.backward_weight(0); t3 = time.perf_counter()
    total = fl["F"] + fl["B"] + fl["W"]
    return {"value": total / (t3 - t0) / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"1 layer x 1 microbatch of the workload's shapes at seq {one['seq']} (F {t1 - t0:.1f}s, B {t2 - t1:.1f}s, "
                      f"W {t3 - t2:.1f}s, fp64 NumPy)",
            "seconds": t3 - t0}


def gemm_table(cfg, name, rounds=20):
    """Every matrix product of one layer of the workload (forward, input gradient, weight gradient) through
    stage_kernel_gemm, and the same product through torch.matmul (hipBLASLt / rocBLAS) on the same operands, timed
    alternately after a common warm-up so that both run at the clock the chip settles to under load.  Prints a
    markdown table; the weight-gradient rows include the library's fp32 read-modify-write of C (torch.matmul writes a
    bf16 C and accumulates nothing)."""
    import ctypes as C
    import torch
    from paper_2507_00217_amd import stage as S
    lib = S.lib()
    vp, i, i64 = C.c_void_p, C.c_int, C.c_int64
    lib.stage_kernel_gemm.argtypes = [i, i, i, i, i, vp, i64, vp, i64, vp, i64, vp, i64, i, i, vp]
    d, f, h = cfg["hidden"], cfg["ffn"], cfg["n_heads"]
    hd = cfg.get("head_dim") or d // h
    da, dq = h * hd, (h + 2 * cfg["n_kv_heads"]) * hd
    T = cfg["seq"] * cfg["mb_size"]
    fin = 2 * f if cfg["act"] == "swiglu" else f
    lin = (("qkv", d, dq), ("wo", da, d), ("win", d, fin), ("wout", f, d))           # name, in, out
    shapes = [(0, T, o, k, "F " + n) for n, k, o in lin] + [(1, T, k, o, "B " + n) for n, k, o in lin] + \
             [(2, k, o, T, "W " + n) for n, k, o in lin]
    stream = torch.cuda.current_stream().cuda_stream
    cases = []
    for mode, M, N, K, label in shapes:
        a_shape = (K, M) if mode == 2 else (M, K)
        b_shape = (N, K) if mode == 1 else (K, N)
        A = torch.randn(a_shape, device="cuda", dtype=torch.bfloat16)
        B = (torch.randn(b_shape, device="cuda", dtype=torch.bfloat16) * 0.02)
        Cm = torch.zeros((M, N), device="cuda", dtype=torch.float32 if mode == 2 else torch.bfloat16)
        At, Bt = (A.t() if mode == 2 else A), (B.t() if mode == 1 else B)
        out_t = torch.empty((M, N), device="cuda", dtype=torch.bfloat16)

        def ours(A=A, B=B, Cm=Cm, mode=mode, M=M, N=N, K=K, a_shape=a_shape, b_shape=b_shape):
            rc = lib.stage_kernel_gemm(1, mode, M, N, K, A.data_ptr(), a_shape[1], B.data_ptr(), b_shape[1], Cm.data_ptr(), N,
                                       None, 0, int(mode == 2), 0, stream)
            assert rc == 0

        def theirs(At=At, Bt=Bt, out_t=out_t):
            torch.matmul(At, Bt, out=out_t)
        cases.append((label, mode, M, N, K, ours, theirs))
    t_end = time.perf_counter() + 2.0                      # common warm-up: the clock settles under sustained load
    while time.perf_counter() < t_end:
        for c in cases:
            c[5](); c[6]()
        torch.cuda.synchronize()
    rows = []
    for label, mode, M, N, K, ours, theirs in cases:
        ms = []
        for fn in (ours, theirs):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            for _ in range(3):
                fn()
            e0.record()
            for _ in range(rounds):
                fn()
            e1.record()
            torch.cuda.synchronize()
            ms.append(e0.elapsed_time(e1) / rounds)
        fl = 2.0 * M * N * K
        rows.append((label, M, N, K, ms[0], fl / ms[0] / 1e9, ms[1], fl / ms[1] / 1e9))
    print(f"| product ({name}) | M | N | K | this library ms | TFLOP/s | torch.matmul ms | TFLOP/s | ratio |")
    print("|---|---|---|---|---|---|---|---|---|")
    for label, M, N, K, m0, t0, m1, t1 in rows:
        print(f"| {label} | {M} | {N} | {K} | {m0:.3f} | {t0:.0f} | {m1:.3f} | {t1:.0f} | {t0 / t1:.2f} |")
    s0, s1 = sum(r[4] for r in rows), sum(r[6] for r in rows)
    fl = sum(2.0 * r[1] * r[2] * r[3] for r in rows)
    print(f"| all twelve | | | | {s0:.3f} | {fl / s0 / 1e9:.0f} | {s1:.3f} | {fl / s1 / 1e9:.0f} | {s1 / s0:.2f} |")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="cfg3")
    ap.add_argument("--kernel-set", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--gemm-table", action="store_true",
                    help="instead of the benchmark: time every matrix product of one layer against torch.matmul, print markdown")
    ap.add_argument("--schedule", default=None, help="override the config's schedule (1f1b, w_deferred, w_lag1, greedy)")
    ap.add_argument("--recompute", type=int, default=0, metavar="CAP",
                    help="layer-wise activation recomputation with at most CAP rebuilt stashes (0 = off); the reported "
                         "TFLOP/s still counts each layer's forward once, so the tax shows as lower throughput")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2507_00217_amd import stage as S
    from paper_2507_00217_amd import synth

    cfg = dict(synth.CONFIGS[args.config], enforce_mb_order=1)
    if args.gemm_table:
        gemm_table(cfg, args.config)
        return
    if args.schedule:
        cfg["schedule"] = args.schedule
    if args.recompute:
        cfg.update(recompute=1, recompute_cap=args.recompute)
    ops = synth.make_schedule(cfg)
    n_mb, L = cfg["n_microbatches"], cfg["n_layers"]
    tdt = torch.float32 if cfg["dtype"] == "fp32" else torch.bfloat16
    seed = 1000 * int(args.config[3]) if args.config[3:].isdigit() else 9000
    st = S.Stage(cfg)
    st.set_kernel_set(args.kernel_set)
    st.load_weights(synth.make_weights(cfg, seed))
    X = torch.from_numpy(synth.make_boundary(cfg, seed + 1)).to("cuda:0", tdt)
    dY = torch.from_numpy(synth.make_boundary(cfg, seed + 2)).to("cuda:0", tdt)
    Y, dX = torch.empty_like(X), torch.empty_like(X)
    ops_c = S.make_ops(ops)
    fl = flops_per_layer_mb(cfg)
    iter_flops = n_mb * L * (fl["F"] + fl["B"] + fl["W"])

    for _ in range(args.warmup):
        st.run_schedule(ops, X, dY, Y, dX, ops_c)
    st.zero_grads()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        st.run_schedule(ops, X, dY, Y, dX, ops_c)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    tflops = iter_flops / (dt / args.steps) / 1e12

    # per-op timing (events on the stage's stream) over one more iteration, op by op
    op_ms = {S.F: 0.0, S.B: 0.0, S.W: 0.0}
    evs = []
    for kind, mb in ops:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        if kind == S.F:
            st.forward(mb, X[mb], Y[mb])
        elif kind == S.B:
            st.backward_input(mb, dY[mb], dX[mb])
        else:
            st.backward_weight(mb)
        e1.record()
        evs.append((kind, e0, e1))
    torch.cuda.synchronize()
    for kind, e0, e1 in evs:
        op_ms[kind] += e0.elapsed_time(e1)
    per_op = {}
    for kind, name in ((S.F, "F"), (S.B, "B"), (S.W, "W")):
        ms = op_ms[kind] / n_mb
        per_op[name] = {"ms": round(ms, 4), "tflops": round(L * fl[name] / ms / 1e9, 1),
                        "frac_peak": round(L * fl[name] / ms / 1e9 / PEAK_BF16_TFLOPS, 4)}

    # per-kernel-class timing, live, with HIP events around every launch of one more iteration
    st.profile(True)
    st.run_schedule(ops, X, dY, Y, dX, ops_c)
    prof = st.profile_read()
    st.profile(False)
    kernels = {}
    for name, r in prof.items():
        if not r["launches"]:
            continue
        rate = r["work"] / (r["ms"] * 1e-3)
        is_flop = name.startswith(("gemm", "attn"))
        kernels[name] = {"launches": r["launches"], "avg_ms": round(r["ms"] / r["launches"], 5),
                         ("tflops" if is_flop else "gbs"): round(rate / (1e12 if is_flop else 1e9), 1)}
    gemm_ms = sum(prof[k]["ms"] for k in ("gemm_nn", "gemm_nt", "gemm_tn"))
    gemm_work = sum(prof[k]["work"] for k in ("gemm_nn", "gemm_nt", "gemm_tn"))
    gemm_n = sum(prof[k]["launches"] for k in ("gemm_nn", "gemm_nt", "gemm_tn"))
    peak = PEAK_BF16_TFLOPS if cfg["dtype"] == "bf16" else PEAK_FP32_TFLOPS
    achieved = gemm_work / (gemm_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma" if cfg["dtype"] == "bf16" else "alu", "kernel": "GEMM family: gemm_mfma_kernel (forward, input gradients) + gemm_wgrad_group_kernel (weight gradients), all launches of one iteration",
                "achieved": round(achieved, 1), "peak": peak, "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                "flops_per_launch": gemm_work / gemm_n, "avg_launch_ms": round(gemm_ms / gemm_n, 5),
                "traffic": measured_gemm_traffic(args.config) if args.kernel_set == 0 and not args.schedule and not args.recompute else None}
    stats = st.stats()
    # what the measured block times mean for a pipeline (the paper's performance model, host code): this stage's
    # T_F/T_D/T_W replicated over 8 stages in 2 datacenters, 2 x n_PP microbatches, memory of 1F1B, with latency and
    # bandwidth delays of 2 T_F on the cross-datacenter hop (the paper's hardest setting); seconds per microbatch
    from paper_2507_00217_amd import sched as SC
    tf, td, tw = (op_ms[k] / n_mb * 1e-3 for k in (S.F, S.B, S.W))
    n_pp = 8
    model = {}
    for name, (lat, bw) in (("no_delay", (0.0, 0.0)), ("delay_2_2", (2.0 * tf, 2.0 * tf))):
        a, b = synth.delay_matrices(n_pp, 2, lat, bw)
        pl, keep = SC.make_params(n_pp, 2 * n_pp, 4, [tf] * n_pp, [td] * n_pp, [tw] * n_pp, m_limit=float(n_pp),
                                  alpha=a, beta=b, msg_bytes=1.0)
        _, mk = SC.crosspipe_greedy(pl)
        rc, _, mk_1f1b = SC.crosspipe_simulate(pl, synth.pipeline_1f1b(n_pp, 2 * n_pp, 4))
        model[name] = {"greedy_s_per_mb": round(mk / (2 * n_pp), 5), "onef1b_s_per_mb": round(mk_1f1b / (2 * n_pp), 5)}
    out = {
        "metric": "stage TFLOP/s per schedule iteration (F+B+W of all microbatches; % of bf16 MFMA peak in frac_peak)",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": f"{args.config}: {L} layers, hidden {cfg['hidden']}, heads {cfg['n_heads']}/{cfg['n_kv_heads']}, "
                               f"ffn {cfg['ffn']}, {cfg['norm']}+{cfg['act']}, seq {cfg['seq']}, mb_size {cfg['mb_size']}, "
                               f"{n_mb} microbatches, schedule {cfg['schedule']}, stash cap {cfg['stash_cap'] or n_mb}"
                               + (f", recomputation with {args.recompute} rebuilt stashes" if args.recompute else ""),
                   "ops": len(ops), "peak_live": stats["peak_live"], "peak_stash_GiB": round(stats["peak_stash_bytes"] / 2 ** 30, 2),
                   "kernel_set": args.kernel_set},
        "frac_peak": round(tflops / PEAK_BF16_TFLOPS, 4),
        "iter_tflop": round(iter_flops / 1e12, 2),
        "per_op": per_op, "kernels": kernels, "roofline": roofline,
        "pipeline_model": dict(model, note="8 stages x this stage's measured T_F/T_D/T_W, 16 microbatches, n_sub 4, memory of "
                               "1F1B; paper context: -33.6 % vs static at T_bw/T_F = 2 on 8-32 GH200 (M70, TP4 PP8)"),
    }
    st.close()
    del st
    torch.cuda.empty_cache()
    if cfg["dtype"] == "bf16":
        # what the matrix cores alone sustain on this GPU (no memory or LDS traffic): with random operands the shader
        # clock settles well below its nominal value, so a kernel on real data cannot reach the published peak
        torch.cuda.synchronize()
        rnd, rnd_mhz = S.probe_mfma_ceiling(True, 200000)      # ~0.25 s: long enough for the clock to settle
        cst, cst_mhz = S.probe_mfma_ceiling(False, 50000)
        out["mfma_ceiling"] = {"random_operands": {"tflops": round(rnd, 1), "shader_mhz": round(rnd_mhz)},
                               "constant_operands": {"tflops": round(cst, 1), "shader_mhz": round(cst_mhz)},
                               "roofline_achieved_over_random_ceiling": round(achieved / rnd, 4),
                               "note": "back-to-back v_mfma_f32_16x16x32_bf16 (the GEMM's instruction) on every CU, 2 wavefronts per SIMD, operands in "
                                       "registers; measured after the timed region"}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
