"""ctypes binding of libstage.so: same names as the C ABI (include/stage.h),
argument marshalling only.  PyTorch is used for device memory and the stream;
every step of F / B / W runs in the library's HIP kernels.

The library must have been built (python -m paper_2507_00217_amd.build);
loading fails loudly otherwise -- there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libstage.so")

F, B, W = 0, 1, 2
NORM = {"layernorm": 0, "rmsnorm": 1}
ACT = {"gelu": 0, "swiglu": 1}
DTYPE = {"fp32": 0, "bf16": 1}
PARAM_IDS = {"g1": 0, "b1": 1, "wqkv": 2, "wo": 3, "g2": 4, "b2": 5, "win": 6, "wout": 7,
             "bqkv": 8, "bo": 9, "bin": 10, "bout": 11}
KERNEL_CLASSES = ("gemm_nn", "gemm_nt", "gemm_tn", "attn_fwd", "attn_bwd", "norm_fwd", "norm_bwd", "act_fwd", "act_bwd", "copy", "rope")
OK, E_INVAL, E_ORDER, E_STASH_FULL, E_HIP = 0, -1, -2, -3, -4


class StageConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_layers", "hidden", "n_heads", "n_kv_heads", "ffn", "seq", "mb_size", "n_microbatches",
        "norm", "act", "causal", "dtype", "stash_cap", "enforce_mb_order")] + [("norm_eps", C.c_float), ("n_sub", C.c_int32), ("recompute", C.c_int32), ("recompute_cap", C.c_int32), ("head_dim", C.c_int32), ("rope_theta", C.c_float), ("bias", C.c_int32)]


class StageSubOp(C.Structure):
    _fields_ = [("kind", C.c_int32), ("mb", C.c_int32), ("sub", C.c_int32)]


class StageChunkOp(C.Structure):
    _fields_ = [("kind", C.c_int32), ("mb", C.c_int32), ("sub", C.c_int32), ("chunk", C.c_int32)]


class StageOp(C.Structure):
    _fields_ = [("kind", C.c_int32), ("mb", C.c_int32)]


class StageSizes(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("weights", "grads", "stash", "workspace")]


class StageError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {strerror(code)} ({code})")


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2507_00217_amd.build`")
        # PyTorch ships its own HIP runtime; it must be the one already loaded when libstage.so resolves
        # libamdhip64, or the process ends up with two runtimes and launches on torch's streams fail.
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        vp, ip = C.c_void_p, C.POINTER(C.c_int)
        cfgp, opp, sopp = C.POINTER(StageConfig), C.POINTER(StageOp), C.POINTER(StageSubOp)
        sig = {
            "stage_query_sizes": (C.c_int, [cfgp, C.POINTER(StageSizes)]),
            "stage_validate_schedule": (C.c_int, [cfgp, opp, C.c_int, ip, ip]),
            "stage_param_layout": (C.c_int, [cfgp, C.c_int, C.c_int, C.POINTER(C.c_size_t),
                                             C.POINTER(C.c_int64), C.POINTER(C.c_int64)]),
            "stage_init": (C.c_int, [cfgp, vp, vp, vp, vp, vp, C.POINTER(vp)]),
            "stage_forward": (C.c_int, [vp, C.c_int, vp, vp]),
            "stage_backward_input": (C.c_int, [vp, C.c_int, vp, vp]),
            "stage_backward_weight": (C.c_int, [vp, C.c_int]),
            "stage_run_schedule": (C.c_int, [vp, opp, C.c_int, vp, vp, vp, vp]),
            "stage_validate_subschedule": (C.c_int, [cfgp, sopp, C.c_int, ip, ip]),
            "stage_forward_sub": (C.c_int, [vp, C.c_int, C.c_int, vp, vp]),
            "stage_backward_input_sub": (C.c_int, [vp, C.c_int, C.c_int, vp, vp]),
            "stage_backward_weight_sub": (C.c_int, [vp, C.c_int, C.c_int]),
            "stage_run_subschedule": (C.c_int, [vp, sopp, C.c_int, vp, vp, vp, vp]),
            "stage_init_chunk": (C.c_int, [cfgp, vp, vp, vp, vp, C.POINTER(vp)]),
            "stage_validate_chunk_schedule": (C.c_int, [cfgp, C.c_int, C.POINTER(StageChunkOp), C.c_int, ip, ip]),
            "stage_run_chunk_schedule": (C.c_int, [C.POINTER(vp), C.c_int, C.POINTER(StageChunkOp), C.c_int,
                                                   C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp)]),
            "stage_grads": (C.c_int, [vp, C.POINTER(vp), C.POINTER(C.c_size_t)]),
            "stage_zero_grads": (C.c_int, [vp]),
            "stage_stats": (C.c_int, [vp, ip, ip, C.POINTER(C.c_size_t)]),
            "stage_set_kernel_set": (C.c_int, [vp, C.c_int]),
            "stage_profile": (C.c_int, [vp, C.c_int]),
            "stage_profile_read": (C.c_int, [vp, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int64), C.POINTER(C.c_double)]),
            "stage_destroy": (None, [vp]),
            "stage_strerror": (C.c_char_p, [C.c_int]),
            "stage_probe_mfma_ceiling": (C.c_int, [C.c_int, C.c_int, vp, C.c_size_t, C.POINTER(C.c_double), C.POINTER(C.c_double), vp]),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def probe_mfma_ceiling(random_operands: bool, iters: int = 100000, stream=None) -> Tuple[float, float]:
    """(TFLOP/s, shader MHz) of back-to-back bf16 MFMAs on every compute unit: the rate this GPU sustains on the
    matrix cores alone, which with random operands is well below the published peak."""
    import torch
    tf, mhz = C.c_double(), C.c_double()
    scratch = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    rc = lib().stage_probe_mfma_ceiling(int(bool(random_operands)), iters, scratch.data_ptr(), scratch.numel(), C.byref(tf),
                                        C.byref(mhz), stream.cuda_stream if stream is not None else None)
    if rc:
        raise StageError(rc, "stage_probe_mfma_ceiling")
    return tf.value, mhz.value


def strerror(code: int) -> str:
    return lib().stage_strerror(code).decode()


def make_config(cfg: dict) -> StageConfig:
    return StageConfig(
        n_layers=cfg["n_layers"], hidden=cfg["hidden"], n_heads=cfg["n_heads"], n_kv_heads=cfg["n_kv_heads"],
        ffn=cfg["ffn"], seq=cfg["seq"], mb_size=cfg["mb_size"], n_microbatches=cfg["n_microbatches"],
        norm=NORM[cfg["norm"]], act=ACT[cfg["act"]], causal=int(cfg.get("causal", True)), dtype=DTYPE[cfg["dtype"]],
        stash_cap=cfg.get("stash_cap", 0), enforce_mb_order=int(cfg.get("enforce_mb_order", 0)),
        norm_eps=cfg.get("norm_eps", 1e-5), n_sub=cfg.get("n_sub", 0),
        recompute=int(cfg.get("recompute", 0)), recompute_cap=cfg.get("recompute_cap", 0),
        head_dim=cfg.get("head_dim", 0) or 0, rope_theta=float(cfg.get("rope_theta", 0.0) or 0.0),
        bias=int(cfg.get("bias", 0) or 0))


def make_ops(ops: Sequence[Tuple[int, int]]):
    arr = (StageOp * max(1, len(ops)))()
    for i, (k, m) in enumerate(ops):
        arr[i].kind, arr[i].mb = k, m
    return arr


def make_subops(ops: Sequence[Tuple[int, int, int]]):
    arr = (StageSubOp * max(1, len(ops)))()
    for i, (k, m, sb) in enumerate(ops):
        arr[i].kind, arr[i].mb, arr[i].sub = k, m, sb
    return arr


def stage_validate_subschedule(cfg: dict, ops) -> Tuple[int, int, int]:
    """Returns (code, first_bad_index, peak_live)."""
    bad, peak = C.c_int(-1), C.c_int(0)
    rc = lib().stage_validate_subschedule(C.byref(make_config(cfg)), make_subops(ops), len(ops), C.byref(bad), C.byref(peak))
    return rc, bad.value, peak.value


def make_chunkops(ops: Sequence[Tuple[int, int, int, int]]):
    """ops: (kind, mb, sub, chunk), sub = -1 for a whole op."""
    arr = (StageChunkOp * max(1, len(ops)))()
    for i, (k, m, sb, c) in enumerate(ops):
        arr[i].kind, arr[i].mb, arr[i].sub, arr[i].chunk = k, m, sb, c
    return arr


def stage_validate_chunk_schedule(cfg: dict, n_chunks: int, ops) -> Tuple[int, int, int]:
    """Host only. Returns (rc, first_bad_index, peak_live over all chunks)."""
    bad, peak = C.c_int(-1), C.c_int(0)
    rc = lib().stage_validate_chunk_schedule(C.byref(make_config(cfg)), n_chunks, make_chunkops(ops), len(ops), C.byref(bad), C.byref(peak))
    return rc, bad.value, peak.value


def run_chunk_schedule(chunks: "List[Stage]", ops, Xs, dYs, Ys, dXs):
    """Runs (kind, mb, sub, chunk) ops over stages that share one stash; Xs[c] ... dXs[c] are chunk c's boundary tensors."""
    n = len(chunks)
    ptrs = lambda ts: (C.c_void_p * n)(*[(t.data_ptr() if t is not None else None) for t in ts])
    hs = (C.c_void_p * n)(*[st.h for st in chunks])
    rc = lib().stage_run_chunk_schedule(hs, n, make_chunkops(ops), len(ops), ptrs(Xs), ptrs(dYs), ptrs(Ys), ptrs(dXs))
    if rc:
        raise StageError(rc, "stage_run_chunk_schedule")


def stage_query_sizes(cfg: dict) -> Dict[str, int]:
    out = StageSizes()
    rc = lib().stage_query_sizes(C.byref(make_config(cfg)), C.byref(out))
    if rc:
        raise StageError(rc, "stage_query_sizes")
    return {n: getattr(out, n) for n in ("weights", "grads", "stash", "workspace")}


def stage_validate_schedule(cfg: dict, ops) -> Tuple[int, int, int]:
    """Returns (code, first_bad_index, peak_live)."""
    bad, peak = C.c_int(-1), C.c_int(0)
    rc = lib().stage_validate_schedule(C.byref(make_config(cfg)), make_ops(ops), len(ops), C.byref(bad), C.byref(peak))
    return rc, bad.value, peak.value


def stage_param_layout(cfg: dict, layer: int, name: str) -> Tuple[int, int, int]:
    """Returns (offset_elems, rows, cols)."""
    off, r, c = C.c_size_t(), C.c_int64(), C.c_int64()
    rc = lib().stage_param_layout(C.byref(make_config(cfg)), layer, PARAM_IDS[name], C.byref(off), C.byref(r), C.byref(c))
    if rc:
        raise StageError(rc, "stage_param_layout")
    return off.value, r.value, c.value


class Stage:
    """Owns the device buffers (torch tensors) and the stage_t handle."""

    def __init__(self, cfg: dict, device: str = "cuda:0", stream=None, share_with: "Stage" = None):
        """share_with: make this stage a further model chunk on share_with's stash (and stream): slots and caps are
        then common to both."""
        import torch
        self.torch = torch
        self.cfg = dict(cfg)
        self.ccfg = make_config(cfg)
        self.device = torch.device(device)
        self.tdtype = torch.float32 if cfg["dtype"] == "fp32" else torch.bfloat16
        sz = stage_query_sizes(cfg)
        self.sizes = sz
        with torch.cuda.device(self.device):
            self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
            self._weights = torch.zeros(sz["weights"], dtype=torch.uint8, device=self.device)
            self._grads = torch.zeros(sz["grads"], dtype=torch.uint8, device=self.device)
            h = C.c_void_p()
            if share_with is None:
                self._stash = torch.empty(sz["stash"], dtype=torch.uint8, device=self.device)
                self._ws = torch.empty(sz["workspace"], dtype=torch.uint8, device=self.device)
                rc = lib().stage_init(C.byref(self.ccfg), self._weights.data_ptr(), self._grads.data_ptr(),
                                      self._stash.data_ptr(), self._ws.data_ptr(), self.stream.cuda_stream, C.byref(h))
            else:
                self.stream = share_with.stream
                self._stash = share_with._stash                                  # keeps it alive
                self._ws = torch.empty(sz["workspace"], dtype=torch.uint8, device=self.device)    # the chunk's own
                rc = lib().stage_init_chunk(C.byref(self.ccfg), self._weights.data_ptr(), self._grads.data_ptr(),
                                            self._ws.data_ptr(), share_with.h, C.byref(h))
        if rc:
            raise StageError(rc, "stage_init" if share_with is None else "stage_init_chunk")
        self.h = h

    # -- weights / grads marshalling ------------------------------------------
    def load_weights(self, params: List[Dict[str, np.ndarray]]):
        torch = self.torch
        flat = self._weights.view(self.tdtype)
        for li, lp in enumerate(params):
            for name, w in lp.items():
                off, r, c = stage_param_layout(self.cfg, li, name)
                assert r * c == w.size, (name, r, c, w.shape)
                t = torch.from_numpy(np.ascontiguousarray(w, dtype=np.float32).reshape(-1))
                flat[off:off + r * c].copy_(t.to(self.tdtype))

    def grads_tensor(self):
        p, n = C.c_void_p(), C.c_size_t()
        rc = lib().stage_grads(self.h, C.byref(p), C.byref(n))
        if rc:
            raise StageError(rc, "stage_grads")
        assert p.value == self._grads.data_ptr()
        return self._grads.view(self.torch.float32)[:n.value]

    def grads(self) -> List[Dict[str, np.ndarray]]:
        self.stream.synchronize()
        g = self.grads_tensor().cpu().numpy()
        out = []
        for li in range(self.cfg["n_layers"]):
            lp = {}
            for name in PARAM_IDS:
                off, r, c = stage_param_layout(self.cfg, li, name)
                if r * c:
                    lp[name] = g[off:off + r * c].reshape((c,) if r == 1 and name[0] in "gb" else (r, c)).copy()
            out.append(lp)
        return out

    # -- the ops -----------------------------------------------------------------
    def _chk(self, rc, what):
        if rc:
            raise StageError(rc, what)

    def forward(self, mb: int, x, y):
        self._chk(lib().stage_forward(self.h, mb, x.data_ptr(), y.data_ptr()), "stage_forward")

    def backward_input(self, mb: int, dy, dx):
        self._chk(lib().stage_backward_input(self.h, mb, dy.data_ptr(), dx.data_ptr()), "stage_backward_input")

    def backward_weight(self, mb: int):
        self._chk(lib().stage_backward_weight(self.h, mb), "stage_backward_weight")

    def run_schedule(self, ops, X, dY, Y, dX, ops_c=None):
        arr = ops_c if ops_c is not None else make_ops(ops)
        p = lambda t: t.data_ptr() if t is not None else None
        self._chk(lib().stage_run_schedule(self.h, arr, len(ops), p(X), p(dY), p(Y), p(dX)), "stage_run_schedule")

    def forward_sub(self, mb: int, sub: int, x, y):
        p = lambda t: t.data_ptr() if t is not None else None
        self._chk(lib().stage_forward_sub(self.h, mb, sub, p(x), p(y)), "stage_forward_sub")

    def backward_input_sub(self, mb: int, sub: int, dy, dx):
        p = lambda t: t.data_ptr() if t is not None else None
        self._chk(lib().stage_backward_input_sub(self.h, mb, sub, p(dy), p(dx)), "stage_backward_input_sub")

    def backward_weight_sub(self, mb: int, sub: int):
        self._chk(lib().stage_backward_weight_sub(self.h, mb, sub), "stage_backward_weight_sub")

    def run_subschedule(self, ops, X, dY, Y, dX):
        p = lambda t: t.data_ptr() if t is not None else None
        self._chk(lib().stage_run_subschedule(self.h, make_subops(ops), len(ops), p(X), p(dY), p(Y), p(dX)),
                  "stage_run_subschedule")

    def zero_grads(self):
        self._chk(lib().stage_zero_grads(self.h), "stage_zero_grads")

    def stats(self) -> Dict[str, int]:
        a, b, c = C.c_int(), C.c_int(), C.c_size_t()
        self._chk(lib().stage_stats(self.h, C.byref(a), C.byref(b), C.byref(c)), "stage_stats")
        return {"live": a.value, "peak_live": b.value, "peak_stash_bytes": c.value}

    def set_kernel_set(self, which: int):
        self._chk(lib().stage_set_kernel_set(self.h, which), "stage_set_kernel_set")

    def profile(self, enable: bool):
        self._chk(lib().stage_profile(self.h, int(enable)), "stage_profile")

    def profile_read(self) -> Dict[str, Dict[str, float]]:
        out = {}
        for cls, name in enumerate(KERNEL_CLASSES):
            ms, n, w = C.c_double(), C.c_int64(), C.c_double()
            self._chk(lib().stage_profile_read(self.h, cls, C.byref(ms), C.byref(n), C.byref(w)), "stage_profile_read")
            out[name] = {"ms": ms.value, "launches": n.value, "work": w.value}
        return out

    def close(self):
        if getattr(self, "h", None):
            self.stream.synchronize()
            lib().stage_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
