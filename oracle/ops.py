"""Oracle operations: forward / backward-p1 / backward-p2 of each module (test infrastructure).

Conventions: activations are token-major [T, width]; a micro-batch of B sequences of length S has
T = B*S rows, sequence b occupying rows b*S .. (b+1)*S-1.  Weights are [in, out] so Y = X @ W.
Heads are column blocks: head h = columns h*dh .. (h+1)*dh-1.  All functions are pure.
"""
from __future__ import annotations

import numpy as np


# ----------------------------------------------------------------------------------------------
# Linear without bias (Section 3.2 "no linear bias"; stash rule of Section 4.2)
# ----------------------------------------------------------------------------------------------
def linear_fwd(x, w):
    """Y = X W."""
    return x @ w


def linear_p1(dy, w):
    """backward-p1 of a linear layer (Section 3.1): dL/dX = dL/dY W^T."""
    return dy @ w.T


def linear_p2(x, dy):
    """backward-p2 of a linear layer (Section 3.1): dL/dW = X^T dL/dY, from the stashed X and dY."""
    return x.T @ dy


# ----------------------------------------------------------------------------------------------
# RMSNorm with gain g:  y_t = g * x_t * r_t,  r_t = (mean_i x_ti^2 + eps)^(-1/2)
# ----------------------------------------------------------------------------------------------
def _rstd(x, eps):
    return 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + x.dtype.type(eps))


def rmsnorm_fwd(x, g, eps):
    return x * _rstd(x, eps) * g


def rmsnorm_p1(dy, x, g, eps):
    """dL/dx.  With yhat = dy*g:  dx_t = r_t*yhat_t - x_t * r_t^3 * (1/d) * sum_i yhat_ti x_ti."""
    r = _rstd(x, eps)
    yhat = dy * g
    d = x.shape[-1]
    proj = np.sum(yhat * x, axis=-1, keepdims=True) / d
    return r * yhat - x * (r ** 3) * proj


def rmsnorm_p2(dy, x, eps):
    """dL/dg_i = sum_t dy_ti * x_ti * r_t."""
    return np.sum(dy * x * _rstd(x, eps), axis=0)


# ----------------------------------------------------------------------------------------------
# SwiGLU:  m = silu(a) * b,  silu(a) = a * sigmoid(a)
# ----------------------------------------------------------------------------------------------
def _sigmoid(a):
    return 1.0 / (1.0 + np.exp(-a))


def swiglu_fwd(a, b):
    return a * _sigmoid(a) * b


def swiglu_p1(dm, a, b):
    """(dL/da, dL/db):  silu'(a) = sigmoid(a) * (1 + a*(1 - sigmoid(a)))."""
    s = _sigmoid(a)
    da = dm * b * s * (1.0 + a * (1.0 - s))
    db = dm * a * s
    return da, db


# ----------------------------------------------------------------------------------------------
# Rotary embedding, half-split pairing: within each head vector of length dh, element i (< dh/2)
# is paired with element i + dh/2 and the pair is rotated by the angle p * base^(-2i/dh), where p
# is the token's position inside its own sequence.
# ----------------------------------------------------------------------------------------------
def _rope_angles(n_tokens, seq, head_dim, base, dtype):
    pos = (np.arange(n_tokens) % seq).astype(np.float64)
    i = np.arange(head_dim // 2, dtype=np.float64)
    theta = np.power(float(base), -2.0 * i / head_dim)
    ang = pos[:, None] * theta[None, :]                       # [T, dh/2]
    return np.cos(ang).astype(dtype), np.sin(ang).astype(dtype)


def _rope_apply(x, seq, n_heads, head_dim, base, sign):
    t = x.shape[0]
    c, s = _rope_angles(t, seq, head_dim, base, x.dtype)
    s = s * sign
    xh = x.reshape(t, n_heads, head_dim)
    half = head_dim // 2
    xa, xb = xh[:, :, :half], xh[:, :, half:]
    out = np.empty_like(xh)
    out[:, :, :half] = xa * c[:, None, :] - xb * s[:, None, :]
    out[:, :, half:] = xa * s[:, None, :] + xb * c[:, None, :]
    return out.reshape(t, n_heads * head_dim)


def rope_fwd(x, seq, n_heads, head_dim, base):
    return _rope_apply(x, seq, n_heads, head_dim, base, +1.0)


def rope_p1(dy, seq, n_heads, head_dim, base):
    """The rotation is orthogonal, so its backward is the rotation by the negated angle."""
    return _rope_apply(dy, seq, n_heads, head_dim, base, -1.0)


# ----------------------------------------------------------------------------------------------
# Row softmax with an optional causal mask, and its backward-p1 (Section 3.2 names the softmax
# backward-p1 as one of the operations worth compiling).  Functional: no backward-p2.
# ----------------------------------------------------------------------------------------------
def softmax_fwd(s, causal=False):
    """P = softmax over the last axis of s [..., S, S]; causal: entry (i, j) with j > i is masked (P = 0 exactly)."""
    if causal:
        n = s.shape[-1]
        s = np.where(np.triu(np.ones((n, n), dtype=bool), k=1), -np.inf, s)
    e = np.exp(s - np.max(s, axis=-1, keepdims=True))
    return e / np.sum(e, axis=-1, keepdims=True)


def softmax_p1(p, dp):
    """dL/dS from dL/dP and the forward's P:  dS = P * (dP - rowsum(dP * P)).  Masked entries have P = 0, so dS = 0."""
    return p * (dp - np.sum(dp * p, axis=-1, keepdims=True))


# ----------------------------------------------------------------------------------------------
# Scaled dot-product attention per (sequence, head), scores scaled by 1/sqrt(dh), optional causal
# mask (query i sees keys j <= i).  A functional module: backward-p1 only (Section 4.1).
# ----------------------------------------------------------------------------------------------
def attention_fwd(q, k, v, seq, n_heads, head_dim, causal=True):
    """Returns (o [T, H*dh], P [B, H, S, S])."""
    t = q.shape[0]
    nb = t // seq
    scale = 1.0 / np.sqrt(float(head_dim))
    o = np.empty_like(q)
    p_all = np.zeros((nb, n_heads, seq, seq), dtype=q.dtype)
    for b in range(nb):
        rows = slice(b * seq, (b + 1) * seq)
        for h in range(n_heads):
            cols = slice(h * head_dim, (h + 1) * head_dim)
            s = (q[rows, cols] @ k[rows, cols].T) * q.dtype.type(scale)
            p = softmax_fwd(s, causal)
            p_all[b, h] = p
            o[rows, cols] = p @ v[rows, cols]
    return o, p_all


def attention_p1(do, q, k, v, p_all, seq, n_heads, head_dim):
    """(dq, dk, dv) from the upstream do and the forward's probabilities P.

    dv = P^T do;  dP = do v^T;  dS = softmax_p1(P, dP);  dq = dS k / sqrt(dh);
    dk = dS^T q / sqrt(dh).  Masked entries have P = 0 and therefore dS = 0.
    """
    t = q.shape[0]
    nb = t // seq
    scale = q.dtype.type(1.0 / np.sqrt(float(head_dim)))
    dq, dk, dv = np.empty_like(q), np.empty_like(k), np.empty_like(v)
    for b in range(nb):
        rows = slice(b * seq, (b + 1) * seq)
        for h in range(n_heads):
            cols = slice(h * head_dim, (h + 1) * head_dim)
            p = p_all[b, h]
            dv[rows, cols] = p.T @ do[rows, cols]
            dp = do[rows, cols] @ v[rows, cols].T
            ds = softmax_p1(p, dp)
            dq[rows, cols] = (ds @ k[rows, cols]) * scale
            dk[rows, cols] = (ds.T @ q[rows, cols]) * scale
    return dq, dk, dv
