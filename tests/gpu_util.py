"""Helpers shared by the GPU parity tests (marshalling only)."""
import numpy as np

from oracle import stage_oracle as so
from paper_2507_00217_amd import synth

TOL = {"fp32": 1e-4, "bf16": 2e-2}      # max_i |gpu - ref| / max_j |ref|, per tensor


def shape_of(cfg, operand_bits=0):
    """operand_bits = 8: the oracle's bf16-compute reading (both operands of every matrix product rounded to bf16)."""
    return so.Shape(cfg["n_layers"], cfg["hidden"], cfg["n_heads"], cfg["n_kv_heads"], cfg["ffn"],
                    cfg["seq"], cfg["mb_size"], cfg["norm"], cfg["act"], bool(cfg.get("causal", True)), hd=cfg.get("head_dim", 0) or 0, rope_theta=float(cfg.get("rope_theta", 0.0) or 0.0),
                    operand_bits=operand_bits)


def to_dev(a, dtype, device="cuda:0"):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(device=device, dtype=torch.float32 if dtype == "fp32" else torch.bfloat16)


def to_np(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def rnd(a, dtype):
    return synth.round_bf16(a.astype(np.float32)) if dtype == "bf16" else a.astype(np.float32)


# reduced-size variants of the five workloads: same structure (norm, activation,
# head_dim, GQA ratio, microbatch size, schedule kind), sizes the oracle finishes
# in seconds, several tiles per dimension and ragged tails
SMALL = {
    "cfg2s": dict(synth.CONFIGS["cfg2"], n_layers=2, hidden=512, n_heads=4, n_kv_heads=4, ffn=1088, seq=328, n_microbatches=4, warmup=2),
    "cfg3s": dict(synth.CONFIGS["cfg3"], n_layers=2, hidden=512, n_heads=4, n_kv_heads=4, ffn=1408, seq=448, n_microbatches=6, stash_cap=3, warmup=2),
    "cfg4s": dict(synth.CONFIGS["cfg4"], n_layers=2, hidden=640, n_heads=5, n_kv_heads=5, ffn=1728, seq=200, n_microbatches=5, stash_cap=3, warmup=2),
    "cfg5s": dict(synth.CONFIGS["cfg5"], n_layers=2, hidden=1024, n_heads=8, n_kv_heads=1, ffn=1792, seq=392, n_microbatches=6, stash_cap=4, warmup=3),
}
for _c in SMALL.values():          # cap = the schedule's own peak of live microbatches
    _c["stash_cap"] = synth.peak_live(synth.make_schedule(_c))
