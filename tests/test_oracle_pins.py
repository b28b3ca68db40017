"""Pins for the CPU oracle: things fixed by mathematics or by library routines, not by the oracle itself."""
import copy

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from oracle import ops
import seeded_inputs as si


def _inputs(shape):
    p = si.stage_params(shape)
    p = {k: [np.asarray(w, np.float64) for w in v] for k, v in p.items()}
    xs = [np.asarray(si.stage_input(shape, m), np.float64) for m in range(shape.n_microbatches)]
    dys = [np.asarray(si.stage_upstream_grad(shape, m), np.float64) for m in range(shape.n_microbatches)]
    return p, xs, dys


def _run_split(shape, p, xs, dys, concat=False, order=None):
    st = oracle.OracleStage(shape, p)
    outs = [st.forward(m, xs[m]) for m in range(len(xs))]
    dxs = [None] * len(xs)
    for m in (order or range(len(xs))):
        dxs[m] = st.backward_p1(m, dys[m])
    st.backward_p2(range(len(xs)), concat=concat)
    return outs, dxs, st.grads()


def _relerr(a, b):
    return np.max(np.abs(np.asarray(a) - np.asarray(b))) / max(np.max(np.abs(b)), 1e-300)


# ---------------------------------------------------------------------------------- check 1
def _loss(shape, p, xs, dys):
    st = oracle.OracleStage(shape, p)
    return sum(float(np.sum(st.forward(m, xs[m]) * dys[m])) for m in range(len(xs)))


@pytest.mark.parametrize("attn", [True, False])
def test_finite_differences_every_input_and_parameter(tiny_shape, attn):
    """Central differences of L = sum(x_out * dY) w.r.t. sampled elements of every input and parameter."""
    shape = tiny_shape if attn else tiny_shape.replace(n_heads=0, head_dim=0)
    p, xs, dys = _inputs(shape)
    # weights of the real recipe are tiny (0.02); scale them up so every path carries signal
    for k in ("w_qkv", "w_o", "w_gu", "w_d"):
        p[k] = [w * 10.0 for w in p[k]]
    _, dxs, grads = _run_split(shape, p, xs, dys)
    rng = np.random.default_rng(0)

    def check(target, analytic, label):
        flat = target.reshape(-1)
        for i in rng.choice(flat.size, size=min(flat.size, 24), replace=False):
            old = flat[i]
            h = 1e-6 * max(1.0, abs(old))
            flat[i] = old + h
            lp = _loss(shape, p, xs, dys)
            flat[i] = old - h
            lm = _loss(shape, p, xs, dys)
            flat[i] = old
            fd = (lp - lm) / (2 * h)
            an = analytic.reshape(-1)[i]
            assert abs(fd - an) <= 2e-6 * max(1.0, abs(an)), (label, i, fd, an)

    for m in range(len(xs)):
        check(xs[m], dxs[m], f"x{m}")
    for key, lst in p.items():
        for l, w in enumerate(lst):
            check(w, grads[key][l], f"{key}[{l}]")


# ---------------------------------------------------------------------------------- check 2
@pytest.mark.parametrize("attn", [True, False])
def test_split_equals_monolithic(tiny_shape, attn):
    shape = tiny_shape.replace(n_layers=3, n_microbatches=3, seq=10)
    if not attn:
        shape = shape.replace(n_heads=0, head_dim=0)
    p, xs, dys = _inputs(shape)
    outs, dxs, grads = _run_split(shape, p, xs, dys, order=[2, 0, 1])
    mdx, mgr, mout = oracle.monolithic_backward(shape, p, xs, dys)
    for m in range(len(xs)):
        assert _relerr(outs[m], mout[m]) < 1e-12
        assert _relerr(dxs[m], mdx[m]) < 1e-12
    for key in grads:
        for l in range(len(grads[key])):
            assert _relerr(grads[key][l], mgr[key][l]) < 1e-11, (key, l)


def test_p2_right_after_p1_is_ordinary_backprop(tiny_shape):
    """Calling p2 for a micro-batch immediately after its p1 gives the same totals as deferring."""
    p, xs, dys = _inputs(tiny_shape)
    _, dxs, grads = _run_split(tiny_shape, p, xs, dys)
    st = oracle.OracleStage(tiny_shape, p)
    for m in range(len(xs)):
        st.forward(m, xs[m])
    for m in range(len(xs)):
        assert _relerr(st.backward_p1(m, dys[m]), dxs[m]) == 0.0
        st.backward_p2([m])
    g2 = st.grads()
    for key in grads:
        for l in range(len(grads[key])):
            assert _relerr(g2[key][l], grads[key][l]) < 1e-13


# ---------------------------------------------------------------------------------- check 3
def test_accumulated_equals_concatenated(tiny_shape):
    shape = tiny_shape.replace(n_microbatches=4)
    p, xs, dys = _inputs(shape)
    _, dx_a, g_loop = _run_split(shape, p, xs, dys, concat=False)
    _, dx_b, g_cat = _run_split(shape, p, xs, dys, concat=True)
    for key in g_loop:
        for l in range(len(g_loop[key])):
            assert _relerr(g_loop[key][l], g_cat[key][l]) < 1e-12
    # one micro-batch holding all sequences == the micro-batches stacked
    big = shape.replace(micro_batch=shape.micro_batch * 4, n_microbatches=1)
    xo, dxo, g_big = _run_split(big, p, [np.concatenate(xs)], [np.concatenate(dys)])
    assert _relerr(dxo[0], np.concatenate(dx_a)) < 1e-12
    for key in g_loop:
        for l in range(len(g_loop[key])):
            assert _relerr(g_big[key][l], g_loop[key][l]) < 1e-12


# ---------------------------------------------------------------------------------- check 4
def test_linear_closed_forms():
    rng = np.random.default_rng(1)
    w = rng.standard_normal((5, 7))
    g = rng.standard_normal((5, 7))
    # X = identity: Y = W, so dL/dW = G exactly and dL/dX = G W^T
    assert np.array_equal(ops.linear_p2(np.eye(5), g), g)
    assert np.array_equal(ops.linear_fwd(np.eye(5), w), w)
    # one-hot rows: token t selects input feature c[t]; dW row c collects the dY rows of its tokens
    c = np.array([3, 0, 3, 1])
    x = np.zeros((4, 5)); x[np.arange(4), c] = 1.0
    dy = rng.standard_normal((4, 7))
    dw = ops.linear_p2(x, dy)
    assert np.allclose(dw[3], dy[0] + dy[2], rtol=0, atol=1e-15)
    assert np.allclose(dw[0], dy[1]) and np.allclose(dw[1], dy[3])
    assert np.all(dw[[2, 4]] == 0)
    # dX[t, i] = <dY[t, :], W[i, :]> written out
    dx = ops.linear_p1(dy, w)
    for t in range(4):
        for i in range(5):
            assert abs(dx[t, i] - sum(dy[t, j] * w[i, j] for j in range(7))) < 1e-13


# ---------------------------------------------------------------------------------- library routines
def _t(a):
    return torch.tensor(a, dtype=torch.float64, requires_grad=True)


def test_rmsnorm_against_library_and_autograd():
    rng = np.random.default_rng(2)
    x, g, dy = rng.standard_normal((9, 32)), 1 + 0.1 * rng.standard_normal(32), rng.standard_normal((9, 32))
    eps = 1e-3   # large on purpose: a misplaced eps shows
    tx, tg = _t(x), _t(g)
    ty = F.rms_norm(tx, (32,), tg, eps)
    assert _relerr(ops.rmsnorm_fwd(x, g, eps), ty.detach().numpy()) < 1e-14
    ty.backward(torch.tensor(dy))
    assert _relerr(ops.rmsnorm_p1(dy, x, g, eps), tx.grad.numpy()) < 1e-13
    assert _relerr(ops.rmsnorm_p2(dy, x, eps), tg.grad.numpy()) < 1e-13


def test_rmsnorm_invariants():
    rng = np.random.default_rng(3)
    x, g, dy = rng.standard_normal((4, 64)), rng.standard_normal(64), rng.standard_normal((4, 64))
    eps = 1e-6
    y = ops.rmsnorm_fwd(x, np.ones(64), eps)
    r2 = 1.0 / (np.mean(x * x, axis=1) + eps)
    assert np.allclose(np.mean(y * y, axis=1), 1 - eps * r2, rtol=1e-12)
    dx = ops.rmsnorm_p1(dy, x, g, eps)
    # dx . x = r^3 * (yhat . x) * eps   (exactly orthogonal as eps -> 0)
    r = np.sqrt(r2)
    assert np.allclose(np.sum(dx * x, axis=1), r ** 3 * np.sum(dy * g * x, axis=1) * eps, rtol=1e-6, atol=1e-12)
    # scale invariance of the forward when eps = 0
    assert np.allclose(ops.rmsnorm_fwd(3.0 * x, g, 0.0), ops.rmsnorm_fwd(x, g, 0.0), rtol=1e-13)


def test_swiglu_against_library_and_autograd():
    rng = np.random.default_rng(4)
    a, b, dm = 3 * rng.standard_normal((5, 11)), rng.standard_normal((5, 11)), rng.standard_normal((5, 11))
    ta, tb = _t(a), _t(b)
    tm = F.silu(ta) * tb
    assert _relerr(ops.swiglu_fwd(a, b), tm.detach().numpy()) < 1e-14
    tm.backward(torch.tensor(dm))
    da, db = ops.swiglu_p1(dm, a, b)
    assert _relerr(da, ta.grad.numpy()) < 1e-13 and _relerr(db, tb.grad.numpy()) < 1e-13
    assert ops.swiglu_fwd(np.zeros(3), np.ones(3)).tolist() == [0, 0, 0]
    # silu'(0) = 1/2
    assert np.allclose(ops.swiglu_p1(np.ones(1), np.zeros(1), np.ones(1))[0], 0.5)


def test_rope_properties():
    rng = np.random.default_rng(5)
    S, H, dh = 12, 3, 16
    q, k = rng.standard_normal((2 * S, H * dh)), rng.standard_normal((2 * S, H * dh))
    rq = ops.rope_fwd(q, S, H, dh, 10000.0)
    rk = ops.rope_fwd(k, S, H, dh, 10000.0)
    # position 0 of every sequence is untouched, other positions are not
    assert np.array_equal(rq[[0, S]], q[[0, S]]) and not np.allclose(rq[1], q[1])
    # positions restart for each sequence in the micro-batch
    assert np.allclose(ops.rope_fwd(q[S:], S, H, dh, 10000.0), rq[S:], rtol=0, atol=0)
    # norm of each head vector is preserved
    n0 = np.linalg.norm(q.reshape(-1, H, dh), axis=-1)
    assert np.allclose(np.linalg.norm(rq.reshape(-1, H, dh), axis=-1), n0, rtol=1e-13)
    # backward is the inverse (orthogonal map)
    assert _relerr(ops.rope_p1(rq, S, H, dh, 10000.0), q) < 1e-14
    # relative-position property: <R_i q, R_j k> depends on i - j only
    qv, kv = rng.standard_normal(dh), rng.standard_normal(dh)
    Q = ops.rope_fwd(np.tile(qv, (S, 1)), S, 1, dh, 10000.0)
    K = ops.rope_fwd(np.tile(kv, (S, 1)), S, 1, dh, 10000.0)
    G = Q @ K.T
    for off in range(-3, 4):
        diag = np.diagonal(G, offset=off)
        assert np.allclose(diag, diag[0], rtol=1e-12, atol=1e-12)
    # explicit angle: pair (i, i+dh/2) at position p rotates by p * base^(-2i/dh)
    e = np.zeros((S, dh)); e[:, 2] = 1.0
    r = ops.rope_fwd(e, S, 1, dh, 100.0)
    p = 5; ang = p * 100.0 ** (-2 * 2 / dh)
    assert abs(r[p, 2] - np.cos(ang)) < 1e-14 and abs(r[p, 2 + dh // 2] - np.sin(ang)) < 1e-14
    # autograd of the complex-multiplication form
    tx = _t(q)
    z = torch.complex(tx.view(2 * S, H, dh)[..., :dh // 2], tx.view(2 * S, H, dh)[..., dh // 2:])
    th = 10000.0 ** (-torch.arange(dh // 2, dtype=torch.float64) * 2 / dh)
    pos = (torch.arange(2 * S) % S).to(torch.float64)
    zr = z * torch.polar(torch.ones(2 * S, dh // 2, dtype=torch.float64), pos[:, None] * th)[:, None, :]
    ty = torch.cat([zr.real, zr.imag], dim=-1).reshape(2 * S, H * dh)
    assert _relerr(rq, ty.detach().numpy()) < 1e-13
    ty.backward(torch.tensor(k))
    assert _relerr(ops.rope_p1(k, S, H, dh, 10000.0), tx.grad.numpy()) < 1e-13


@pytest.mark.parametrize("causal", [True, False])
def test_attention_against_library_and_autograd(causal):
    rng = np.random.default_rng(6)
    B, S, H, dh = 2, 9, 3, 8
    q, k, v, do = (rng.standard_normal((B * S, H * dh)) for _ in range(4))
    o, P = ops.attention_fwd(q, k, v, S, H, dh, causal)
    tq, tk, tv = _t(q), _t(k), _t(v)
    heads = lambda t: t.view(B, S, H, dh).transpose(1, 2)
    to = F.scaled_dot_product_attention(heads(tq), heads(tk), heads(tv), is_causal=causal)
    to = to.transpose(1, 2).reshape(B * S, H * dh)
    assert _relerr(o, to.detach().numpy()) < 1e-13
    to.backward(torch.tensor(do))
    dq, dk, dv = ops.attention_p1(do, q, k, v, P, S, H, dh)
    assert _relerr(dq, tq.grad.numpy()) < 1e-12
    assert _relerr(dk, tk.grad.numpy()) < 1e-12
    assert _relerr(dv, tv.grad.numpy()) < 1e-12
    # invariants: rows of P sum to one, masked entries are exactly zero
    assert np.allclose(P.sum(-1), 1.0, rtol=1e-14)
    if causal:
        assert np.all(P[..., np.triu_indices(S, 1)[0], np.triu_indices(S, 1)[1]] == 0)


def test_attention_special_cases():
    rng = np.random.default_rng(7)
    H, dh = 2, 4
    q, k, v, do = (rng.standard_normal((3, H * dh)) for _ in range(4))
    # sequence length 1 (three sequences of one token): o = v, dq = dk = 0, dv = do
    o, P = ops.attention_fwd(q, k, v, 1, H, dh, True)
    assert np.array_equal(o, v) and np.all(P == 1)
    dq, dk, dv = ops.attention_p1(do, q, k, v, P, 1, H, dh)
    assert np.all(dq == 0) and np.all(dk == 0) and np.array_equal(dv, do)
    # causal: changing a later token leaves earlier outputs unchanged
    S = 6
    q, k, v = (rng.standard_normal((S, H * dh)) for _ in range(3))
    o1, _ = ops.attention_fwd(q, k, v, S, H, dh, True)
    k2, v2 = k.copy(), v.copy(); k2[4] += 1.0; v2[4] -= 2.0
    o2, _ = ops.attention_fwd(q, k2, v2, S, H, dh, True)
    assert np.array_equal(o1[:4], o2[:4]) and not np.allclose(o1[4:], o2[4:])
    # equal keys -> uniform probabilities over the visible prefix -> running mean of v
    o3, P3 = ops.attention_fwd(q, np.ones_like(k), v, S, H, dh, True)
    assert np.allclose(o3, np.cumsum(v, 0) / np.arange(1, S + 1)[:, None], rtol=1e-13)
    # softmax backward annihilates constants: rows of dS sum to zero => dq from constant k rows is 0
    dq, _, _ = ops.attention_p1(rng.standard_normal((S, H * dh)), q, np.ones_like(k), v, P3, S, H, dh)
    assert np.max(np.abs(dq)) < 1e-14


@pytest.mark.parametrize("causal", [True, False])
def test_softmax_against_library_and_autograd(causal):
    """Row softmax and its backward-p1 against torch.softmax and autograd, plus the textbook invariants."""
    rng = np.random.default_rng(8)
    S = 11
    s, dp = rng.standard_normal((3, S, S)) * 3.0, rng.standard_normal((3, S, S))
    P = ops.softmax_fwd(s, causal)
    ts = _t(s)
    tm = ts.masked_fill(torch.triu(torch.ones(S, S, dtype=torch.bool), 1), float("-inf")) if causal else ts
    tP = torch.softmax(tm, dim=-1)
    assert _relerr(P, tP.detach().numpy()) < 1e-14
    tP.backward(torch.tensor(dp))
    dS = ops.softmax_p1(P, dp)
    assert _relerr(dS, ts.grad.numpy()) < 1e-13
    assert np.allclose(P.sum(-1), 1.0, rtol=1e-14) and np.max(np.abs(dS.sum(-1))) < 1e-14
    if causal:
        iu = np.triu_indices(S, 1)
        assert np.all(P[:, iu[0], iu[1]] == 0) and np.all(dS[:, iu[0], iu[1]] == 0)
    # shift invariance of the forward; a constant upstream gradient is annihilated by the backward
    assert _relerr(ops.softmax_fwd(s + 5.0, causal), P) < 1e-13
    assert np.max(np.abs(ops.softmax_p1(P, np.full_like(dp, 0.7)))) < 1e-15
    # one live entry per row (first row of a causal matrix): P = 1 there and dS = 0
    if causal:
        assert P[0, 0, 0] == 1.0 and dS[0, 0, 0] == 0.0


def test_whole_stage_against_autograd(tiny_shape):
    """Stage forward rebuilt from library routines; its autograd gradients must match the split backward."""
    shape = tiny_shape.replace(seq=8)
    p, xs, dys = _inputs(shape)
    outs, dxs, grads = _run_split(shape, p, xs, dys)
    S, B, d, f, H, dh = shape.seq, shape.micro_batch, shape.d_model, shape.d_ffn, shape.n_heads, shape.head_dim
    tp = {k: [_t(w) for w in v] for k, v in p.items()}
    th = shape.rope_base ** (-torch.arange(dh // 2, dtype=torch.float64) * 2 / dh)
    ph = torch.polar(torch.ones(S, dh // 2, dtype=torch.float64), torch.arange(S, dtype=torch.float64)[:, None] * th)

    def rope(t):
        t = t.view(B, S, H, dh)
        z = torch.complex(t[..., :dh // 2], t[..., dh // 2:]) * ph[None, :, None, :]
        return torch.cat([z.real, z.imag], -1)

    for m in range(len(xs)):
        tx = _t(xs[m]); x = tx
        for l in range(shape.n_layers):
            qkv = F.rms_norm(x, (d,), tp["g1"][l], shape.rms_eps) @ tp["w_qkv"][l]
            q, k = rope(qkv[:, :d]).transpose(1, 2), rope(qkv[:, d:2 * d]).transpose(1, 2)
            v = qkv[:, 2 * d:].view(B, S, H, dh).transpose(1, 2)
            a = F.scaled_dot_product_attention(q, k, v, is_causal=True).transpose(1, 2).reshape(B * S, d)
            x = x + a @ tp["w_o"][l]
            gu = F.rms_norm(x, (d,), tp["g2"][l], shape.rms_eps) @ tp["w_gu"][l]
            x = x + (F.silu(gu[:, :f]) * gu[:, f:]) @ tp["w_d"][l]
        assert _relerr(outs[m], x.detach().numpy()) < 1e-12
        x.backward(torch.tensor(dys[m]))
        assert _relerr(dxs[m], tx.grad.numpy()) < 1e-11
    for key in grads:
        for l in range(len(grads[key])):
            assert _relerr(grads[key][l], tp[key][l].grad.numpy()) < 1e-11, (key, l)


def test_zero_down_projection_kills_mlp_branch(tiny_shape):
    shape = tiny_shape.replace(n_layers=1, n_heads=0, head_dim=0)
    p, xs, dys = _inputs(shape)
    p["w_d"] = [np.zeros_like(w) for w in p["w_d"]]
    outs, dxs, grads = _run_split(shape, p, xs, dys)
    assert np.array_equal(outs[0], xs[0]) and np.array_equal(dxs[0], dys[0])
    assert np.all(grads["w_gu"][0] == 0) and np.all(grads["g2"][0] == 0)


def test_fp32_switch_close_to_fp64(tiny_shape):
    p, xs, dys = _inputs(tiny_shape)
    st64 = oracle.OracleStage(tiny_shape, p)
    st32 = oracle.OracleStage(tiny_shape, p, dtype=np.float32)
    a = st64.backward_p1(0, dys[0]) if st64.forward(0, xs[0]) is not None else None
    b = st32.backward_p1(0, dys[0]) if st32.forward(0, xs[0]) is not None else None
    assert b.dtype == np.float32 and _relerr(b, a) < 1e-5


# ---------------------------------------------------------------------------------- planted mistakes
@pytest.mark.parametrize("mutation", ["rope_sign", "eps_outside", "softmax_no_rowsum", "silu_grad", "transpose"])
def test_planted_mistakes_are_caught(tiny_shape, monkeypatch, mutation):
    """Each plausible slip in the oracle must break agreement with the independent monolithic backward."""
    if mutation == "rope_sign":
        monkeypatch.setattr(ops, "rope_p1", ops.rope_fwd)
    elif mutation == "eps_outside":
        monkeypatch.setattr(ops, "_rstd", lambda x, eps: 1.0 / (np.sqrt(np.mean(x * x, -1, keepdims=True)) + 1e-2))
    elif mutation == "softmax_no_rowsum":
        monkeypatch.setattr(ops, "softmax_p1", lambda p, dp: p * dp)        # the rowsum(dP * P) term dropped
    elif mutation == "silu_grad":
        monkeypatch.setattr(ops, "swiglu_p1", lambda dm, a, b: (dm * b * ops._sigmoid(a), dm * a * ops._sigmoid(a)))
    elif mutation == "transpose":
        monkeypatch.setattr(ops, "linear_p2", lambda x, dy: (dy.T @ x).T * 1.0 + 1e-3)
    p, xs, dys = _inputs(tiny_shape)
    _, dxs, grads = _run_split(tiny_shape, p, xs, dys)
    mdx, mgr, _ = oracle.monolithic_backward(tiny_shape, p, xs, dys)
    worst = max(_relerr(dxs[m], mdx[m]) for m in range(len(xs)))
    worst = max([worst] + [_relerr(grads[k][l], mgr[k][l]) for k in grads for l in range(len(grads[k]))])
    assert worst > 1e-6


def test_bf16_storage_floor_analysis_runs_and_orders_of_magnitude():
    """The analysis script beside the oracle (fp64 arithmetic, bf16 rounding at the storage points of a bf16
    implementation) at a reduced sequence length: the floor of one 7B-shaped layer is several 1e-3, far above fp64
    noise and below the 2e-2 tolerance that a single layer has to meet."""
    from oracle.bf16_storage_floor import storage_floor
    e = storage_floor(1, 64)
    assert set(e) >= {"x_out", "dx", "dw_qkv[0]", "dw_o[0]", "dg1[0]", "dw_gu[0]", "dw_d[0]", "dg2[0]"}
    assert all(1e-3 < v < 2e-2 for v in e.values()), e
