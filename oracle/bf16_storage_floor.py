"""How much error does bf16 STORAGE alone cause?  (Test infrastructure: an analysis script beside the oracle.)

Runs the oracle's own operations in fp64 on a LLaMa-7B-shaped stage, once as they are (the oracle) and once with
one round-to-nearest-even bf16 rounding at every point where a bf16 implementation with fp32 accumulation has to
store a tensor or form a matrix-core operand: the norm outputs, q / k / v before and after the rotary embedding, the
probabilities P, the attention output, both residual-stream tensors of a layer, gate | up, the SwiGLU output, and in
the backward pass the derivatives of all of those plus dS.  Everything else (every sum, every exponential) stays in
fp64.  The max-norm relative error of the second run against the first is the floor that ANY such implementation sits
on, whatever its kernels; the HIP path's measured error is to be read against it.

    python -m oracle.bf16_storage_floor [n_layers] [seq]        (defaults: 1 layer, seq 1024; one micro-batch)

Imports only numpy, the oracle's operations and the seeded input generators.  About 10 s per layer at seq 1024.
"""
from __future__ import annotations

import sys

import numpy as np

import seeded_inputs as si
from oracle import ops
from oracle.stage import OracleStage


def _max_rel(got, ref):
    return float(np.max(np.abs(got - ref)) / np.max(np.abs(ref)))


def storage_floor(n_layers: int = 1, seq: int = 1024) -> dict:
    shape = si.CONFIGS["llama7b_s1024"].replace(n_layers=n_layers, seq=seq, n_microbatches=1)
    params = si.stage_params(shape)
    x, dy = si.stage_input(shape, 0), si.stage_upstream_grad(shape, 0)
    r = lambda a: si.round_bf16(a).astype(np.float64)
    ref = OracleStage(shape, params)
    o_ref = ref.forward(0, x)
    dx_ref = ref.backward_p1(0, dy)
    ref.backward_p2([0])
    g_ref = ref.grads()
    S, H, dh, d, f = shape.seq, shape.n_heads, shape.head_dim, shape.d_model, shape.d_ffn
    eps, base, B = shape.rms_eps, shape.rope_base, shape.micro_batch
    W = lambda k, l: np.asarray(params[k][l], np.float64)
    heads = [(b, h, slice(b * S, (b + 1) * S), slice(h * dh, (h + 1) * dh)) for b in range(B) for h in range(H)]
    saved, cur = [], np.asarray(x, np.float64)
    for l in range(n_layers):
        x0 = cur
        h1 = r(ops.rmsnorm_fwd(x0, W("g1", l), eps))
        qkv = r(ops.linear_fwd(h1, W("w_qkv", l)))
        q = r(ops.rope_fwd(qkv[:, :d], S, H, dh, base))
        k = r(ops.rope_fwd(qkv[:, d:2 * d], S, H, dh, base))
        v = qkv[:, 2 * d:]
        _, p = ops.attention_fwd(q, k, v, S, H, dh, shape.causal)
        a = np.empty_like(q)
        for b, h, rows, cols in heads:                      # P enters the product with v as a bf16 operand
            a[rows, cols] = r(p[b, h]) @ v[rows, cols]
        a = r(a)
        x1 = r(x0 + ops.linear_fwd(a, W("w_o", l)))
        h2 = r(ops.rmsnorm_fwd(x1, W("g2", l), eps))
        gu = r(ops.linear_fwd(h2, W("w_gu", l)))
        m = r(ops.swiglu_fwd(gu[:, :f], gu[:, f:]))
        cur = r(x1 + ops.linear_fwd(m, W("w_d", l)))
        saved.append((x0, h1, q, k, v, p, a, x1, h2, gu, m))
    err = {"x_out": _max_rel(cur, o_ref)}
    g = np.asarray(dy, np.float64)
    gr = {}
    scale = 1.0 / np.sqrt(dh)
    for l in reversed(range(n_layers)):
        x0, h1, q, k, v, p, a, x1, h2, gu, m = saved[l]
        dx2 = g
        gr[("w_d", l)] = ops.linear_p2(m, dx2)
        dm = r(ops.linear_p1(dx2, W("w_d", l)))
        dgate, dup = ops.swiglu_p1(dm, gu[:, :f], gu[:, f:])
        dgu = r(np.concatenate([dgate, dup], axis=1))
        gr[("w_gu", l)] = ops.linear_p2(h2, dgu)
        dh2 = r(ops.linear_p1(dgu, W("w_gu", l)))
        gr[("g2", l)] = ops.rmsnorm_p2(dh2, x1, eps)
        dx1 = r(dx2 + ops.rmsnorm_p1(dh2, x1, W("g2", l), eps))
        gr[("w_o", l)] = ops.linear_p2(a, dx1)
        da = r(ops.linear_p1(dx1, W("w_o", l)))
        dq, dk, dv = np.empty_like(q), np.empty_like(q), np.empty_like(q)
        for b, h, rows, cols in heads:                      # P and dS enter their products as bf16 operands
            P = p[b, h]
            dS = ops.softmax_p1(P, da[rows, cols] @ v[rows, cols].T)
            dv[rows, cols] = r(P).T @ da[rows, cols]
            dq[rows, cols] = (r(dS) @ k[rows, cols]) * scale
            dk[rows, cols] = (r(dS).T @ q[rows, cols]) * scale
        dq = r(ops.rope_p1(r(dq), S, H, dh, base))
        dk = r(ops.rope_p1(r(dk), S, H, dh, base))
        dqkv = np.concatenate([dq, dk, r(dv)], axis=1)
        gr[("w_qkv", l)] = ops.linear_p2(h1, dqkv)
        dh1 = r(ops.linear_p1(dqkv, W("w_qkv", l)))
        gr[("g1", l)] = ops.rmsnorm_p2(dh1, x0, eps)
        g = r(dx1 + ops.rmsnorm_p1(dh1, x0, W("g1", l), eps))
    err["dx"] = _max_rel(g, dx_ref)
    for (key, l), val in gr.items():
        err[f"d{key}[{l}]"] = _max_rel(val, g_ref[key][l])
    return err


if __name__ == "__main__":
    layers = int(sys.argv[1]) if len(sys.argv) > 1 else 1
    seq = int(sys.argv[2]) if len(sys.argv) > 2 else 1024
    e = storage_floor(layers, seq)
    print(f"bf16 storage floor, LLaMa-7B layer shape, {layers} layer(s), seq {seq}: x_out {e['x_out']:.3e}, dx {e['dx']:.3e}")
    for l in range(layers):
        print(f"  layer {l}: " + ", ".join(f"d{k}={e[f'd{k}[{l}]']:.2e}" for k in ("w_qkv", "w_o", "g1", "w_gu", "w_d", "g2")))
    worst = max(e, key=e.get)
    print(f"  worst tensor {worst} = {e[worst]:.3e}")
