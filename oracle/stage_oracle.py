"""CPU oracle for one pipeline stage's F / B / W compute.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, obviously-correct
definition that the HIP path is checked against.  Only tests, the smoke check
and the benchmark's cpu_baseline leg may import it; the product path never
does, and this file imports nothing from the product package.

What it defines (paper section 3.1, "Computation Blocks", and Appendix B,
"Weight Gradient Separation"): the backward of a model chunk is split into an
input-gradient block (the paper's D; called B here) and a weight-gradient block
(W), so that a schedule may run F, B and W of every microbatch as separate ops
in any legal order.  For a linear map Y = X W this means B computes
dX = dY W^T and W computes dW = X^T dY.  Section 3.2 fixes the activation
lifetime: cached in F, released after B and W.  The split is a re-bracketing
of ordinary backpropagation, so the oracle is the textbook definition written
out in NumPy, in fp64 unless a dtype is passed, with the full s-by-s attention
matrix materialised and no blocking or fusion.

The paper does not itemise the layer ("Llama-style Transformer layers",
section 7).  The reading used here: pre-norm decoder layer, no dropout,
exact-erf GELU, eps = 1e-5, biased variance, gradients summed (not averaged)
over microbatches, norm-parameter gradients produced by B.  Linear biases and
the rotary embedding are optional (Llama-style layers have no biases; GPT-style
ones do): a layer has the biases whose keys (bqkv, bo, bin, bout) its parameter
dict holds, and their gradients -- column sums of the dZ tensors, which B
produces -- are accumulated by B, like the norm parameters'.

Precision.  The paper trains in bf16 (section 7; Appendix E counts two bytes
per element).  Two readings of that are implemented, selected by
Shape.operand_bits:
  0   exact: every tensor stays in the working dtype (fp64).  This is the plain
      definition and the reference for fp32 workloads, for every pin below and
      for bf16 workloads wherever the stated tolerance can be met against it.
  8   bf16 compute: BOTH OPERANDS OF EVERY MATRIX PRODUCT (the linear maps and
      their two gradient products, Q K^T, P V and the four products of the
      attention backward) are rounded to 8 significant bits (bf16, nearest
      even) and the product is accumulated exactly; everything else -- norms,
      softmax, activations, residual adds, reductions -- stays exact.  That is
      the least any engine whose matrix units take bf16 operands must round,
      and it says nothing about where an implementation stores what.  The
      softmax exponent multiplies a score's rounding error by the score's
      magnitude, so for wide layers (logit standard deviation 2-3 with the
      synthetic N(0, 0.02^2) weights at hidden 4096-8192) this reading and
      the exact one differ by more than the 2e-2 tolerance at depth; parity of
      a bf16 engine at such sizes is therefore stated against this reading,
      and the exact one is reported beside it.

    n1 = Norm1(x);  [q|k|v] = n1 Wqkv;  o = Attention(q, k, v)
    x1 = x + o Wo;  n2 = Norm2(x1)
    GELU:   u = n2 Win;        a = gelu(u)
    SwiGLU: [g|u] = n2 Win;    a = silu(g) * u
    y  = x1 + a Wout

Parity pins (tests/test_oracle_*.py): central finite differences in fp64,
B-then-W == fused backward, schedule-order invariance, sum over microbatches
== full-batch gradient, closed-form special cases, and PyTorch CPU autograd as
a second opinion.  No function here is "parity unpinned".
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, List, Sequence, Tuple

import numpy as np
from scipy.special import erf

F, B, W = 0, 1, 2  # op kinds of a per-stage ordered schedule (paper Alg. 1, "S_d")


@dataclass(frozen=True)
class Shape:
    n_layers: int
    hidden: int
    n_heads: int
    n_kv_heads: int
    ffn: int
    seq: int
    mb_size: int
    norm: str = "layernorm"   # "layernorm" | "rmsnorm"
    act: str = "gelu"         # "gelu" | "swiglu"
    causal: bool = True
    eps: float = 1e-5
    rope_theta: float = 0.0   # > 0: rotary position embedding on q and k with this base (Llama-style layers); 0 = none
    hd: int = 0               # width of one head; 0 = hidden / n_heads.  A tensor-parallel share of a layer (the paper's
                              # per-GPU shapes at TP > 1) keeps hidden but has fewer heads, so n_heads * hd < hidden.
    operand_bits: int = 0     # 0: exact.  n > 0: both operands of every matrix product are rounded to n significant bits
                              # (8 = bf16) before the product, which is then accumulated exactly (see "Precision" above)

    @property
    def head_dim(self) -> int:
        return self.hd if self.hd else self.hidden // self.n_heads

    @property
    def q_dim(self) -> int:
        return self.n_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim


def round_sig(t, bits: int):
    """t (fp64) rounded to `bits` significant binary digits, ties to even; the exponent range stays fp64's (values of
    a stage are far from bf16's under- and overflow).  Done on the bit patterns: an fp64 significand has 53 digits,
    so the low 53 - bits are dropped after adding half of the last kept place (one less when that place is even);
    a carry out of the significand moves into the exponent field, which is what rounding up to a power of two is."""
    drop = 53 - bits
    u = np.array(t, dtype=np.float64).view(np.uint64)             # a copy: the input is left alone
    u += ((u >> np.uint64(drop)) & np.uint64(1)) + np.uint64((1 << (drop - 1)) - 1)
    u &= np.uint64(~((1 << drop) - 1) & 0xFFFFFFFFFFFFFFFF)
    return u.view(np.float64)


def _op(sh: "Shape", t):
    """A matrix-product operand in the precision the reading fixes."""
    return round_sig(t, sh.operand_bits) if sh.operand_bits else t


def _mm(sh: "Shape", a, b):
    """a @ b with both operands in operand precision, accumulated in the working dtype."""
    return _op(sh, a) @ _op(sh, b)


Params = List[Dict[str, np.ndarray]]
# per layer: g1, (b1), wqkv [d, d+2*dkv], wo [d, d], g2, (b2),
#            win [d, f] or [d, 2f] (gate | up), wout [f, d],
#            optional linear biases bqkv [d+2*dkv], bo [d], bin [f] or [2f], bout [d]
BIAS_OF = {"wqkv": "bqkv", "wo": "bo", "win": "bin", "wout": "bout"}


def _linear(sh: "Shape", p, w: str, a):
    """a W (+ b when the layer has that bias)."""
    y = _mm(sh, a, p[w])
    return y + p[BIAS_OF[w]] if BIAS_OF[w] in p else y


def _bias_grads(p, dz: Dict[str, np.ndarray]) -> Dict[str, np.ndarray]:
    """db = column sums of the dZ of each linear map that has a bias (dz: weight name -> dZ)."""
    return {BIAS_OF[w]: _flat(t).sum(axis=0) for w, t in dz.items() if BIAS_OF[w] in p}


# --------------------------------------------------------------------------
# building blocks, forward
# --------------------------------------------------------------------------

def norm_forward(kind: str, x, gamma, beta, eps):
    """Row-wise normalisation over the last axis.  Returns (out, stats)."""
    if kind == "layernorm":
        mu = x.mean(axis=-1, keepdims=True)
        var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)      # biased
        rstd = 1.0 / np.sqrt(var + eps)
        xhat = (x - mu) * rstd
        return xhat * gamma + beta, (xhat, rstd)
    if kind == "rmsnorm":
        ms = (x * x).mean(axis=-1, keepdims=True)
        rstd = 1.0 / np.sqrt(ms + eps)
        xhat = x * rstd
        return xhat * gamma, (xhat, rstd)
    raise ValueError(kind)


def head_probs(sh: Shape, qh, kh):
    """softmax_rows(qh kh^T / sqrt(hd) + causal mask) for one head: [s,s]."""
    s, hd = qh.shape
    S = _mm(sh, qh, kh.T) * (1.0 / math.sqrt(hd))
    if sh.causal:
        S = np.where(np.tril(np.ones((s, s), dtype=bool)), S, -np.inf)
    S = S - S.max(axis=-1, keepdims=True)
    e = np.exp(S)
    return e / e.sum(axis=-1, keepdims=True)


def attention_forward(sh: Shape, q, k, v):
    """q [b,s,h,hd], k,v [b,s,hkv,hd] -> o [b,s,h,hd].  Query head j reads
    KV head j // (h / hkv).  Sequences of a microbatch do not interact."""
    b, s, h, hd = q.shape
    group = h // sh.n_kv_heads
    o = np.zeros_like(q)
    for ib in range(b):
        for j in range(h):
            g = j // group
            o[ib, :, j, :] = _mm(sh, head_probs(sh, q[ib, :, j, :], k[ib, :, g, :]), v[ib, :, g, :])
    return o


def gelu(u):
    return 0.5 * u * (1.0 + erf(u / math.sqrt(2.0)))


def gelu_grad(u):
    return 0.5 * (1.0 + erf(u / math.sqrt(2.0))) + u * np.exp(-0.5 * u * u) / math.sqrt(2.0 * math.pi)


def sigmoid(g):
    return 1.0 / (1.0 + np.exp(-g))


def rope(sh: Shape, t, inverse: bool = False):
    """Rotary position embedding of t [b, s, heads, head_dim] (RoFormer, section 3.4.2 there; the paper's layers are
    Llama-style): consecutive pairs (2p, 2p+1) of a head are rotated by the angle pos * theta^(-2p / head_dim), pos =
    position in the sequence.  The inverse rotation is its transpose, which is what the backward pass applies."""
    if not sh.rope_theta:
        return t
    b, s, nh, hd = t.shape
    ang = np.arange(s, dtype=np.float64)[:, None] * sh.rope_theta ** (-2.0 * np.arange(hd // 2, dtype=np.float64) / hd)[None, :]
    cos, sin = np.cos(ang)[None, :, None, :], np.sin(ang)[None, :, None, :]
    if inverse:
        sin = -sin
    te, to = t[..., 0::2], t[..., 1::2]
    out = np.empty_like(t)
    out[..., 0::2] = te * cos - to * sin
    out[..., 1::2] = te * sin + to * cos
    return out


def layer_forward(sh: Shape, p: Dict[str, np.ndarray], x):
    """x [b,s,d] -> (y [b,s,d], cache)."""
    b, s, d = x.shape
    h, hkv, hd, dkv, f = sh.n_heads, sh.n_kv_heads, sh.head_dim, sh.kv_dim, sh.ffn
    c = {"x": x}
    n1, c["norm1"] = norm_forward(sh.norm, x, p["g1"], p.get("b1", 0.0), sh.eps)
    c["n1"] = n1
    qkv = _linear(sh, p, "wqkv", n1)
    dq_ = sh.q_dim
    q = rope(sh, qkv[..., :dq_].reshape(b, s, h, hd))
    k = rope(sh, qkv[..., dq_:dq_ + dkv].reshape(b, s, hkv, hd))
    v = qkv[..., dq_ + dkv:].reshape(b, s, hkv, hd)
    c["q"], c["k"], c["v"] = q, k, v
    o = attention_forward(sh, q, k, v)
    o = o.reshape(b, s, dq_)
    c["o"] = o
    x1 = x + _linear(sh, p, "wo", o)
    c["x1"] = x1
    n2, c["norm2"] = norm_forward(sh.norm, x1, p["g2"], p.get("b2", 0.0), sh.eps)
    c["n2"] = n2
    z = _linear(sh, p, "win", n2)
    c["z"] = z
    if sh.act == "gelu":
        a = gelu(z)
    elif sh.act == "swiglu":
        g, u = z[..., :f], z[..., f:]
        a = g * sigmoid(g) * u
    else:
        raise ValueError(sh.act)
    c["a"] = a
    y = x1 + _linear(sh, p, "wout", a)
    return y, c


# --------------------------------------------------------------------------
# building blocks, backward
# --------------------------------------------------------------------------

def norm_backward(kind: str, stats, gamma, dout):
    """Returns (dx, dgamma, dbeta-or-None) for out = xhat*gamma (+beta)."""
    xhat, rstd = stats
    dxhat = dout * gamma
    red = tuple(range(dout.ndim - 1))
    dgamma = (dout * xhat).sum(axis=red)
    if kind == "layernorm":
        dbeta = dout.sum(axis=red)
        m1 = dxhat.mean(axis=-1, keepdims=True)
        m2 = (dxhat * xhat).mean(axis=-1, keepdims=True)
        dx = (dxhat - m1 - xhat * m2) * rstd
        return dx, dgamma, dbeta
    m2 = (dxhat * xhat).mean(axis=-1, keepdims=True)
    dx = (dxhat - xhat * m2) * rstd
    return dx, dgamma, None


def attention_backward(sh: Shape, q, k, v, do):
    """Gradients of o = softmax(q k^T / sqrt(hd) + mask) v.  do [b,s,h,hd].
    The probabilities are recomputed from q, k (same definition as forward)
    instead of being cached, to keep the s-by-s matrices transient."""
    b, s, h, hd = q.shape
    group = h // sh.n_kv_heads
    scale = 1.0 / math.sqrt(hd)
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    for ib in range(b):
        for j in range(h):
            g = j // group
            p = head_probs(sh, q[ib, :, j, :], k[ib, :, g, :])
            doj = _op(sh, do[ib, :, j, :])
            dv[ib, :, g, :] += _op(sh, p).T @ doj
            dp = doj @ _op(sh, v[ib, :, g, :]).T
            ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
            ds_op = _op(sh, ds)                      # operand of both remaining products
            dq[ib, :, j, :] = (ds_op @ _op(sh, k[ib, :, g, :])) * scale
            dk[ib, :, g, :] += (ds_op.T @ _op(sh, q[ib, :, j, :])) * scale
    return dq, dk, dv


def act_backward(sh: Shape, z, da):
    if sh.act == "gelu":
        return da * gelu_grad(z)
    f = sh.ffn
    g, u = z[..., :f], z[..., f:]
    sg = sigmoid(g)
    dg = da * u * (sg + g * sg * (1.0 - sg))
    du = da * g * sg
    return np.concatenate([dg, du], axis=-1)


def _flat(t):
    return t.reshape(-1, t.shape[-1])


def layer_backward_input(sh: Shape, p, c, dy):
    """The B op of one layer: dx, the dZ tensors W will need, and norm grads."""
    b, s, d = dy.shape
    dkv = sh.kv_dim
    saved = {"dz_out": dy}
    da = _mm(sh, dy, p["wout"].T)
    dz_in = act_backward(sh, c["z"], da)
    saved["dz_in"] = dz_in
    dn2 = _mm(sh, dz_in, p["win"].T)
    dx1_n, dg2, db2 = norm_backward(sh.norm, c["norm2"], p["g2"], dn2)
    dx1 = dy + dx1_n
    saved["dz_o"] = dx1
    do = _mm(sh, dx1, p["wo"].T)
    dq, dk, dv = attention_backward(sh, c["q"], c["k"], c["v"],
                                    do.reshape(b, s, sh.n_heads, sh.head_dim))
    dq, dk = rope(sh, dq, inverse=True), rope(sh, dk, inverse=True)
    dz_qkv = np.concatenate([dq.reshape(b, s, sh.q_dim), dk.reshape(b, s, dkv), dv.reshape(b, s, dkv)], axis=-1)
    saved["dz_qkv"] = dz_qkv
    dn1 = _mm(sh, dz_qkv, p["wqkv"].T)
    dx_n, dg1, db1 = norm_backward(sh.norm, c["norm1"], p["g1"], dn1)
    dx = dx1 + dx_n
    ng = {"g1": dg1, "g2": dg2}
    if sh.norm == "layernorm":
        ng["b1"], ng["b2"] = db1, db2
    ng.update(_bias_grads(p, {"wout": dy, "win": dz_in, "wo": dx1, "wqkv": dz_qkv}))
    return dx, saved, ng


def layer_backward_weight(sh: Shape, c, saved):
    """The W op of one layer: dW = A^T dZ for the four linear maps."""
    return {
        "wout": _mm(sh, _flat(c["a"]).T, _flat(saved["dz_out"])),
        "win": _mm(sh, _flat(c["n2"]).T, _flat(saved["dz_in"])),
        "wo": _mm(sh, _flat(c["o"]).T, _flat(saved["dz_o"])),
        "wqkv": _mm(sh, _flat(c["n1"]).T, _flat(saved["dz_qkv"])),
    }


def layer_backward_full(sh: Shape, p, c, dy):
    """Classic fused backward: every linear yields its input and weight
    gradient at the same point of the reverse sweep.  Written separately from
    the split pair above so that comparing them is a real check."""
    b, s, d = dy.shape
    dkv = sh.kv_dim
    gr = {}
    A = _flat(c["a"]); G = _flat(dy)
    gr["wout"] = _mm(sh, A.T, G)
    if "bout" in p:
        gr["bout"] = G.sum(axis=0)
    da = _mm(sh, G, p["wout"].T).reshape(c["a"].shape)
    dz = act_backward(sh, c["z"], da)
    gr["win"] = _mm(sh, _flat(c["n2"]).T, _flat(dz))
    if "bin" in p:
        gr["bin"] = _flat(dz).sum(axis=0)
    dn2 = _mm(sh, dz, p["win"].T)
    t, gr["g2"], db2 = norm_backward(sh.norm, c["norm2"], p["g2"], dn2)
    dx1 = dy + t
    gr["wo"] = _mm(sh, _flat(c["o"]).T, _flat(dx1))
    if "bo" in p:
        gr["bo"] = _flat(dx1).sum(axis=0)
    do = _mm(sh, dx1, p["wo"].T)
    dq, dk, dv = attention_backward(sh, c["q"], c["k"], c["v"],
                                    do.reshape(b, s, sh.n_heads, sh.head_dim))
    dq, dk = rope(sh, dq, inverse=True), rope(sh, dk, inverse=True)
    dqkv = np.concatenate([dq.reshape(b, s, sh.q_dim), dk.reshape(b, s, dkv), dv.reshape(b, s, dkv)], axis=-1)
    gr["wqkv"] = _mm(sh, _flat(c["n1"]).T, _flat(dqkv))
    if "bqkv" in p:
        gr["bqkv"] = _flat(dqkv).sum(axis=0)
    dn1 = _mm(sh, dqkv, p["wqkv"].T)
    t, gr["g1"], db1 = norm_backward(sh.norm, c["norm1"], p["g1"], dn1)
    if sh.norm == "layernorm":
        gr["b1"], gr["b2"] = db1, db2
    return dx1 + t, gr


# --------------------------------------------------------------------------
# the stage: F / B / W ops per microbatch, run in schedule order
# --------------------------------------------------------------------------

class OracleStage:
    """State: params, accumulated grads, and per-microbatch caches that live
    from F(m) to W(m) (section 3.2).  Gradients are *summed* over microbatches."""

    def __init__(self, sh: Shape, params: Params, dtype=np.float64, recompute: bool = False):
        """recompute: layer-wise activation recomputation (the memory/batch-size trade-off's Case 2, section 7.2):
        F keeps only every layer's input; B rebuilds a layer's cache by running its forward again just before
        that layer's backward, and the rebuilt cache then lives until W."""
        self.sh = sh
        self.dtype = dtype
        self.recompute = recompute
        self.params = [{k: np.asarray(v, dtype=dtype) for k, v in lp.items()} for lp in params]
        self.zero_grads()
        self._cache: Dict[int, list] = {}
        self._saved: Dict[int, list] = {}

    def zero_grads(self):
        self.grads = [{k: np.zeros_like(v) for k, v in lp.items()} for lp in self.params]

    def _x(self, t):
        sh = self.sh
        return np.asarray(t, dtype=self.dtype).reshape(sh.mb_size, sh.seq, sh.hidden)

    def forward(self, mb: int, x):
        assert mb not in self._cache, "F twice"
        caches = []
        y = self._x(x)
        for lp in self.params:
            y, c = layer_forward(self.sh, lp, y)
            caches.append(self._keep(c))
        self._cache[mb] = caches
        return y

    def _keep(self, c):
        """What F leaves in the stash for one layer."""
        return {"x": c["x"]} if self.recompute else c

    def _full(self, mb: int, li: int):
        """The layer's complete cache, rebuilt from its stashed input when only that was kept."""
        c = self._cache[mb][li]
        if len(c) == 1:
            _, c = layer_forward(self.sh, self.params[li], c["x"])
            self._cache[mb][li] = c
        return c

    def stash_elems(self, mb: int) -> int:
        """Array elements held for a microbatch right now (stash footprint in elements)."""
        def count(v):
            if isinstance(v, np.ndarray):
                return v.size
            if isinstance(v, (tuple, list)):
                return sum(count(e) for e in v)
            return 0
        return sum(count(v) for c in self._cache.get(mb, []) for v in c.values())

    def backward_input(self, mb: int, dy):
        assert mb in self._cache and mb not in self._saved, "B needs F once"
        d = self._x(dy)
        saved = [None] * len(self.params)
        for li in reversed(range(len(self.params))):
            d, saved[li], ng = layer_backward_input(self.sh, self.params[li], self._full(mb, li), d)
            for k, v in ng.items():
                self.grads[li][k] += v
        self._saved[mb] = saved
        return d

    def backward_weight(self, mb: int):
        assert mb in self._saved, "W needs B"
        for li in range(len(self.params)):
            for k, v in layer_backward_weight(self.sh, self._cache[mb][li], self._saved[mb][li]).items():
                self.grads[li][k] += v
        del self._cache[mb], self._saved[mb]

    # -- sub-block ops (paper section 4.2.1): sub-block `sub` of n_sub covers layers [sub, sub+1) * L / n_sub ----
    def _layers(self, sub: int, n_sub: int):
        per = len(self.params) // n_sub
        assert per * n_sub == len(self.params)
        return range(sub * per, (sub + 1) * per)

    def forward_sub(self, mb: int, sub: int, n_sub: int, x=None):
        """F of one sub-block; x is given for sub 0, later sub-blocks continue from the previous one's output.
        Returns the sub-block's output (the stage output for the last sub-block)."""
        if sub == 0:
            assert mb not in self._cache
            self._cache[mb] = []
            y = self._x(x)
        else:
            assert len(self._cache[mb]) == self._layers(sub, n_sub)[0]
            y = self._carry[mb]
        for li in self._layers(sub, n_sub):
            y, c = layer_forward(self.sh, self.params[li], y)
            self._cache[mb].append(self._keep(c))
        if not hasattr(self, "_carry"):
            self._carry = {}
        self._carry[mb] = y
        return y

    def backward_input_sub(self, mb: int, sub: int, n_sub: int, dy=None):
        """B of one sub-block, from the last sub-block down to 0; dy is given for the last one."""
        L = len(self.params)
        if sub == n_sub - 1:
            assert len(self._cache[mb]) == L and mb not in self._saved
            self._saved[mb] = [None] * L
            d = self._x(dy)
        else:
            assert self._saved[mb][self._layers(sub, n_sub)[-1] + 1] is not None
            d = self._carry[mb]
        for li in reversed(self._layers(sub, n_sub)):
            d, self._saved[mb][li], ng = layer_backward_input(self.sh, self.params[li], self._full(mb, li), d)
            for k, v in ng.items():
                self.grads[li][k] += v
        self._carry[mb] = d
        return d

    def backward_weight_sub(self, mb: int, sub: int, n_sub: int):
        """W of one sub-block (any order after its B); the microbatch's cache is dropped after the last one."""
        for li in self._layers(sub, n_sub):
            assert self._saved[mb][li] is not None and self._saved[mb][li] != "done"
            for k, v in layer_backward_weight(self.sh, self._cache[mb][li], self._saved[mb][li]).items():
                self.grads[li][k] += v
            self._saved[mb][li] = "done"
        if all(sv == "done" for sv in self._saved[mb]):
            del self._cache[mb], self._saved[mb], self._carry[mb]

    def run_subschedule(self, ops, n_sub: int, X, dY):
        """ops: (kind, mb, sub) triples. Returns (Y, dX, peak_live)."""
        Y = np.zeros(np.shape(X), dtype=self.dtype)
        dX = np.zeros(np.shape(X), dtype=self.dtype)
        peak = self.live
        for kind, mb, sub in ops:
            if kind == F:
                y = self.forward_sub(mb, sub, n_sub, X[mb] if sub == 0 else None)
                if sub == n_sub - 1:
                    Y[mb] = y
            elif kind == B:
                d = self.backward_input_sub(mb, sub, n_sub, dY[mb] if sub == n_sub - 1 else None)
                if sub == 0:
                    dX[mb] = d
            elif kind == W:
                self.backward_weight_sub(mb, sub, n_sub)
            else:
                raise ValueError(kind)
            peak = max(peak, self.live)
        return Y, dX, peak

    def backward_full(self, mb: int, dy):
        """Fused B+W (the paper's undivided backward block)."""
        assert mb in self._cache and mb not in self._saved
        d = self._x(dy)
        for li in reversed(range(len(self.params))):
            d, gr = layer_backward_full(self.sh, self.params[li], self._full(mb, li), d)
            for k, v in gr.items():
                self.grads[li][k] += v
        del self._cache[mb]
        return d

    @property
    def live(self) -> int:
        return len(self._cache)

    def run_schedule(self, ops: Sequence[Tuple[int, int]], X, dY):
        """ops: (kind, mb) pairs.  X, dY: [n_mb, b, s, d].  Returns (Y, dX, peak_live)."""
        Y = np.zeros(np.shape(X), dtype=self.dtype)
        dX = np.zeros(np.shape(X), dtype=self.dtype)
        peak = self.live
        for kind, mb in ops:
            if kind == F:
                Y[mb] = self.forward(mb, X[mb])
            elif kind == B:
                dX[mb] = self.backward_input(mb, dY[mb])
            elif kind == W:
                self.backward_weight(mb)
            else:
                raise ValueError(kind)
            peak = max(peak, self.live)
        return Y, dX, peak


def max_rel_err(got, ref) -> float:
    """max_i |got_i - ref_i| / max_j |ref_j|  (the per-tensor reading of
    "max relative error"; element-wise relative error is unbounded near 0)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.abs(ref).max()
    if den == 0.0:
        return float(np.abs(got).max())
    return float(np.abs(got - ref).max() / den)
