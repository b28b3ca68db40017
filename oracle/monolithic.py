"""Monolithic (unsplit) backward of the same stage, written independently of `stage.py`.

Test infrastructure.  Section 3.2 of the paper states that calling backward-p2 directly after
backward-p1 reproduces ordinary reverse-mode differentiation; this file is that ordinary backward:
all micro-batches are stacked into one batch [N, S, d], each layer's input gradient and parameter
gradients are produced together in one reverse sweep, and nothing is stashed per module.  The
formulas are deliberately arranged differently from `ops.py` (complex-number rotary embedding,
normalised-vector form of the RMSNorm Jacobian, batched einsum attention) so that agreement of the
two is evidence for both.
"""
from __future__ import annotations

import numpy as np


def _rope_complex(x, n_heads, head_dim, base, conj):
    # x: [N, S, H*dh]; pair (i, i+dh/2) viewed as a complex number times exp(+-i p theta_i)
    n, s, _ = x.shape
    half = head_dim // 2
    xh = x.reshape(n, s, n_heads, head_dim)
    z = xh[..., :half] + 1j * xh[..., half:]
    theta = float(base) ** (-np.arange(half, dtype=np.float64) / half)
    phase = np.exp((-1j if conj else 1j) * np.arange(s, dtype=np.float64)[:, None] * theta[None, :])
    z = z * phase[None, :, None, :]
    return np.concatenate([z.real, z.imag], axis=-1).reshape(n, s, n_heads * head_dim)


def _norm_fwd(x, g, eps):
    r = (np.mean(x ** 2, axis=-1, keepdims=True) + eps) ** -0.5
    xhat = x * r
    return xhat * g, xhat, r


def _norm_bwd(dy, xhat, r, g):
    yhat = dy * g
    dx = r * (yhat - xhat * np.mean(yhat * xhat, axis=-1, keepdims=True))
    dg = np.einsum("nsd,nsd->d", dy, xhat)
    return dx, dg


def monolithic_backward(shape, params, xs, dys):
    """xs, dys: lists (one per micro-batch) of [T, d] arrays.  Returns (dx list, grads dict, x_out list)."""
    S, B, d, f = shape.seq, shape.micro_batch, shape.d_model, shape.d_ffn
    H, dh, eps = shape.n_heads, shape.head_dim, shape.rms_eps
    attn = H > 0
    x = np.concatenate([np.asarray(a, np.float64).reshape(B, S, d) for a in xs], axis=0)
    dy = np.concatenate([np.asarray(a, np.float64).reshape(B, S, d) for a in dys], axis=0)
    N = x.shape[0]
    W = {k: [np.asarray(w, np.float64) for w in v] for k, v in params.items()}

    tape = []
    for l in range(shape.n_layers):
        rec = {"x0": x}
        if attn:
            h1, rec["xh1"], rec["r1"] = _norm_fwd(x, W["g1"][l], eps)
            qkv = h1 @ W["w_qkv"][l]
            q = _rope_complex(qkv[..., :d], H, dh, shape.rope_base, False).reshape(N, S, H, dh)
            k = _rope_complex(qkv[..., d:2 * d], H, dh, shape.rope_base, False).reshape(N, S, H, dh)
            v = qkv[..., 2 * d:].reshape(N, S, H, dh)
            sc = np.einsum("nihe,njhe->nhij", q, k) / np.sqrt(dh)
            if shape.causal:
                i, j = np.indices((S, S))
                sc = np.where(j > i, -np.inf, sc)
            sc = sc - sc.max(axis=-1, keepdims=True)
            P = np.exp(sc)
            P /= P.sum(axis=-1, keepdims=True)
            a = np.einsum("nhij,njhe->nihe", P, v).reshape(N, S, d)
            x = x + a @ W["w_o"][l]
            rec.update(h1=h1, q=q, k=k, v=v, P=P, a=a)
        rec["x1"] = x
        h2, rec["xh2"], rec["r2"] = _norm_fwd(x, W["g2"][l], eps)
        gu = h2 @ W["w_gu"][l]
        ga, up = gu[..., :f], gu[..., f:]
        sig = 1.0 / (1.0 + np.exp(-ga))
        m = ga * sig * up
        x = x + m @ W["w_d"][l]
        rec.update(h2=h2, ga=ga, up=up, sig=sig, m=m)
        tape.append(rec)
    x_out = x

    G = {k: [None] * shape.n_layers for k in W}
    g = dy
    for l in reversed(range(shape.n_layers)):
        rec = tape[l]
        # MLP half: gradient w.r.t. parameters and inputs together
        G["w_d"][l] = np.einsum("nsf,nsd->fd", rec["m"], g)
        dm = g @ W["w_d"][l].T
        dsilu = rec["sig"] + rec["ga"] * rec["sig"] * (1.0 - rec["sig"])
        dgu = np.concatenate([dm * rec["up"] * dsilu, dm * rec["ga"] * rec["sig"]], axis=-1)
        G["w_gu"][l] = np.einsum("nsd,nsf->df", rec["h2"], dgu)
        dh2 = dgu @ W["w_gu"][l].T
        dx, G["g2"][l] = _norm_bwd(dh2, rec["xh2"], rec["r2"], W["g2"][l])
        g = g + dx
        if not attn:
            continue
        G["w_o"][l] = np.einsum("nsa,nsd->ad", rec["a"], g)
        da = (g @ W["w_o"][l].T).reshape(N, S, H, dh)
        P, q, k, v = rec["P"], rec["q"], rec["k"], rec["v"]
        dv = np.einsum("nhij,nihe->njhe", P, da)
        dP = np.einsum("nihe,njhe->nhij", da, v)
        dS = P * dP - P * np.einsum("nhij,nhij->nhi", P, dP)[..., None]
        dq = np.einsum("nhij,njhe->nihe", dS, k) / np.sqrt(dh)
        dk = np.einsum("nhij,nihe->njhe", dS, q) / np.sqrt(dh)
        dq = _rope_complex(dq.reshape(N, S, d), H, dh, shape.rope_base, True)
        dk = _rope_complex(dk.reshape(N, S, d), H, dh, shape.rope_base, True)
        dqkv = np.concatenate([dq, dk, dv.reshape(N, S, d)], axis=-1)
        G["w_qkv"][l] = np.einsum("nsd,nse->de", rec["h1"], dqkv)
        dh1 = dqkv @ W["w_qkv"][l].T
        dx, G["g1"][l] = _norm_bwd(dh1, rec["xh1"], rec["r1"], W["g1"][l])
        g = g + dx

    if not attn:
        for key in ("w_qkv", "w_o", "g1"):
            G[key] = []
    T = B * S
    dxs = [g[i * B:(i + 1) * B].reshape(T, d) for i in range(len(xs))]
    outs = [x_out[i * B:(i + 1) * B].reshape(T, d) for i in range(len(xs))]
    return dxs, G, outs
