"""Oracle stage: a stack of LLaMa-like decoder layers with forward / backward-p1 / backward-p2.

Test infrastructure.  Mirrors the module structure of the paper's Section 3.2: every module has
`forward` and `backward_p1`; modules that own parameters also have `backward_p2`.  Stash rule of
Section 4.2: a parametrised module keeps its input activation and its output derivative from p1
until p2 consumes them; a functional module drops its activations inside p1.

Layer wiring (the paper names the ingredients only; this is the standard pre-norm arrangement):
    x1 = x0 + Wo-linear( attention( rope(q), rope(k), v ) ),  [q,k,v] = RMSNorm(x0; g1) Wqkv
    x2 = x1 + Wd-linear( silu(g) * u ),                        [g,u]   = RMSNorm(x1; g2) Wgu
An MLP-only block (n_heads == 0) is the second line alone.
"""
from __future__ import annotations

import numpy as np

from . import ops


class _Linear:
    def __init__(self, w):
        self.w = w
        self.grad = np.zeros_like(w)
        self.x, self.dy = {}, {}

    def forward(self, mb, x):
        self.x[mb] = x
        return ops.linear_fwd(x, self.w)

    def backward_p1(self, mb, dy):
        self.dy[mb] = dy
        return ops.linear_p1(dy, self.w)

    def backward_p2(self, mbs, concat):
        if concat:   # Section 3.2 / Figure 2: concatenate over the batch dimension, one call
            x = np.concatenate([self.x[m] for m in mbs], axis=0)
            dy = np.concatenate([self.dy[m] for m in mbs], axis=0)
            self.grad += ops.linear_p2(x, dy)
        else:        # one call per micro-batch, accumulated
            for m in mbs:
                self.grad += ops.linear_p2(self.x[m], self.dy[m])
        for m in mbs:
            del self.x[m], self.dy[m]


class _RMSNorm:
    def __init__(self, g, eps):
        self.g, self.eps = g, eps
        self.grad = np.zeros_like(g)
        self.x, self.dy = {}, {}

    def forward(self, mb, x):
        self.x[mb] = x
        return ops.rmsnorm_fwd(x, self.g, self.eps)

    def backward_p1(self, mb, dy):
        self.dy[mb] = dy
        return ops.rmsnorm_p1(dy, self.x[mb], self.g, self.eps)

    def backward_p2(self, mbs, concat):
        if concat:
            x = np.concatenate([self.x[m] for m in mbs], axis=0)
            dy = np.concatenate([self.dy[m] for m in mbs], axis=0)
            self.grad += ops.rmsnorm_p2(dy, x, self.eps)
        else:
            for m in mbs:
                self.grad += ops.rmsnorm_p2(self.dy[m], self.x[m], self.eps)
        for m in mbs:
            del self.x[m], self.dy[m]


class _SwiGLU:                      # functional: no p2, activations released in p1
    def __init__(self):
        self.ab = {}

    def forward(self, mb, a, b):
        self.ab[mb] = (a, b)
        return ops.swiglu_fwd(a, b)

    def backward_p1(self, mb, dm):
        a, b = self.ab.pop(mb)
        return ops.swiglu_p1(dm, a, b)


class _Attention:                   # rope on q,k + scaled dot-product attention; functional
    def __init__(self, seq, n_heads, head_dim, base, causal):
        self.cfg = (seq, n_heads, head_dim)
        self.base, self.causal = base, causal
        self.saved = {}

    def forward(self, mb, q, k, v):
        seq, nh, dh = self.cfg
        q = ops.rope_fwd(q, seq, nh, dh, self.base)
        k = ops.rope_fwd(k, seq, nh, dh, self.base)
        o, p = ops.attention_fwd(q, k, v, seq, nh, dh, self.causal)
        self.saved[mb] = (q, k, v, p)
        return o

    def backward_p1(self, mb, do):
        seq, nh, dh = self.cfg
        q, k, v, p = self.saved.pop(mb)
        dq, dk, dv = ops.attention_p1(do, q, k, v, p, seq, nh, dh)
        dq = ops.rope_p1(dq, seq, nh, dh, self.base)
        dk = ops.rope_p1(dk, seq, nh, dh, self.base)
        return dq, dk, dv


class _Layer:
    def __init__(self, shape, p, l, dtype):
        cast = lambda a: np.asarray(a, dtype=dtype)
        self.attn = shape.n_heads > 0
        self.d, self.f = shape.d_model, shape.d_ffn
        if self.attn:
            self.norm1 = _RMSNorm(cast(p["g1"][l]), shape.rms_eps)
            self.qkv = _Linear(cast(p["w_qkv"][l]))
            self.sdpa = _Attention(shape.seq, shape.n_heads, shape.head_dim, shape.rope_base, shape.causal)
            self.out = _Linear(cast(p["w_o"][l]))
        self.norm2 = _RMSNorm(cast(p["g2"][l]), shape.rms_eps)
        self.gu = _Linear(cast(p["w_gu"][l]))
        self.act = _SwiGLU()
        self.down = _Linear(cast(p["w_d"][l]))

    def parametrised(self):
        mods = [self.norm2, self.gu, self.down]
        if self.attn:
            mods += [self.norm1, self.qkv, self.out]
        return mods

    def forward(self, mb, x0):
        d, f = self.d, self.f
        x1 = x0
        if self.attn:
            qkv = self.qkv.forward(mb, self.norm1.forward(mb, x0))
            a = self.sdpa.forward(mb, qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:])
            x1 = x0 + self.out.forward(mb, a)
        gu = self.gu.forward(mb, self.norm2.forward(mb, x1))
        m = self.act.forward(mb, gu[:, :f], gu[:, f:])
        return x1 + self.down.forward(mb, m)

    def backward_p1(self, mb, dx2):
        dm = self.down.backward_p1(mb, dx2)
        dg, du = self.act.backward_p1(mb, dm)
        dh2 = self.gu.backward_p1(mb, np.concatenate([dg, du], axis=1))
        dx1 = dx2 + self.norm2.backward_p1(mb, dh2)
        if not self.attn:
            return dx1
        da = self.out.backward_p1(mb, dx1)
        dq, dk, dv = self.sdpa.backward_p1(mb, da)
        dh1 = self.qkv.backward_p1(mb, np.concatenate([dq, dk, dv], axis=1))
        return dx1 + self.norm1.backward_p1(mb, dh1)


class OracleStage:
    """One pipeline stage.  `params` is the dict of per-layer lists made by the input generator."""

    def __init__(self, shape, params, dtype=np.float64):
        self.shape, self.dtype = shape, dtype
        self.layers = [_Layer(shape, params, l, dtype) for l in range(shape.n_layers)]

    def forward(self, mb, x):
        x = np.asarray(x, dtype=self.dtype)
        for layer in self.layers:
            x = layer.forward(mb, x)
        return x

    def backward_p1(self, mb, dy):
        """Input gradient of the stage for micro-batch mb (Section 3.1, backward-p1 of every layer)."""
        g = np.asarray(dy, dtype=self.dtype)
        for layer in reversed(self.layers):
            g = layer.backward_p1(mb, g)
        return g

    def backward_p2(self, mbs, concat=False):
        """Deferred parameter gradients for the given micro-batches, accumulated into the grads."""
        for layer in self.layers:
            for mod in layer.parametrised():
                mod.backward_p2(list(mbs), concat)

    def grads(self):
        """Accumulated parameter gradients, same keys and layouts as the parameter dict."""
        g = {k: [] for k in ("w_qkv", "w_o", "g1", "w_gu", "w_d", "g2")}
        for layer in self.layers:
            if layer.attn:
                g["w_qkv"].append(layer.qkv.grad)
                g["w_o"].append(layer.out.grad)
                g["g1"].append(layer.norm1.grad)
            g["w_gu"].append(layer.gu.grad)
            g["w_d"].append(layer.down.grad)
            g["g2"].append(layer.norm2.grad)
        return g
