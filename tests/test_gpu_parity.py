"""GPU parity: every HIP kernel and the whole stage against the CPU oracle on the same seeded inputs.

Bar: max-norm relative error <= 1e-4 (fp32 storage) and <= 2e-2 (bf16 storage against the fp64 oracle)
for stage outputs; single kernels are held to tighter bounds derived from their arithmetic (one bf16
rounding of the output = at most 2^-8 of the element; fp32 accumulation otherwise)."""
import numpy as np
import pytest
import torch

import oracle
from oracle import ops
import paper_2405_18047_amd as tbp
import seeded_inputs as si
from gpu_util import DEV, compare_stage, make_gpu_stage, max_rel, run_oracle, stage_tolerance, to_dev, to_np

pytestmark = pytest.mark.gpu


def _rnd(seed, name, shape, dtype, scale=1.0):
    return si.store_round(scale * si.standard_normal(seed, name, shape), dtype)


def _say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------------------------------- GEMM
GEMM_SHAPES = [  # (M, N, K): several tiles plus ragged tails in every dimension (multiples of 8 for bf16)
    (256, 256, 64), (520, 392, 200), (1000, 136, 72), (136, 1000, 328), (264, 520, 1096), (8, 8, 8),
    (4096, 4344, 72), (4344, 4096, 40),     # 272 large tiles: the output is cut into whole rounds + a small-tile rest
    # long contractions on 192 / 272 large tiles with a ragged last tile in M, N and K (the weight-gradient kernel)
    (4096, 3064, 264), (3064, 4096, 1000), (4096, 4344, 328),
    # outputs that fill the chip badly with 256 x 256 tiles: the storage-type NN / NT products take 256 x 192 tiles
    (2040, 5128, 328), (1024, 11016, 200),
    # 432 large tiles: one whole round + 176, the rest of which runs on 256 x 192 tiles (cut along N, and along M)
    (4096, 6904, 264), (6904, 4096, 136),
    # [2048, 5120]: one full round of 128 x 320 tiles; ragged in M, N and K
    (2048, 5120, 328), (2040, 5112, 264),
]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("layout", [tbp.NN, tbp.NT, tbp.TN])
@pytest.mark.parametrize("mnk", GEMM_SHAPES)
def test_gemm_matches_definition(dtype, layout, mnk):
    M, N, K = mnk
    _say(f"gemm dtype={dtype} layout={layout} M,N,K={mnk}")
    a_shape = (K, M) if layout == tbp.TN else (M, K)
    b_shape = (N, K) if layout == tbp.NT else (K, N)
    A, B = _rnd(11, "A", a_shape, dtype), _rnd(11, "B", b_shape, dtype)
    a64, b64 = A.astype(np.float64), B.astype(np.float64)
    # the three layouts are the three products of a linear layer: forward, backward-p1, backward-p2
    ref = {tbp.NN: ops.linear_fwd, tbp.NT: ops.linear_p1, tbp.TN: ops.linear_p2}[layout](a64, b64)
    dA, dB = to_dev(A, dtype), to_dev(B, dtype)
    got32 = tbp.tbp_gemm(layout, dA, dB, out_f32=True)
    assert max_rel(to_np(got32), ref) < 2e-5
    # accumulate twice on top of a known start, with alpha
    C0 = _rnd(11, "C0", (M, N), "f32")
    acc = to_dev(C0, "f32")
    tbp.tbp_gemm(layout, dA, dB, C_out=acc, accumulate=True, alpha=0.5)
    tbp.tbp_gemm(layout, dA, dB, C_out=acc, accumulate=True, alpha=0.5)
    assert max_rel(to_np(acc), ref + C0) < 2e-5
    if dtype == "bf16":     # storage-type output with a residual, rounded once
        R = _rnd(11, "R", (M, N), dtype, 4.0)
        got = tbp.tbp_gemm(layout, dA, dB, R=to_dev(R, dtype))
        assert max_rel(to_np(got), ref + R) < 4.5e-3


@pytest.mark.parametrize("layout", [tbp.NN, tbp.NT])
@pytest.mark.parametrize("mnk", [(1024, 4096, 32768), (1000, 4040, 32776), (1280, 2304, 49152)])
def test_gemm_with_split_contraction(layout, mnk):
    """bf16 products whose output is too small to fill the chip: given scratch memory, several workgroups share a tile
    and their partial sums meet in the scratch.  Same result as the definition, identical from call to call (the
    partials are added in a fixed order), the scratch is reusable without being cleared by the caller, and a residual
    is still added once."""
    M, N, K = mnk
    dtype = "bf16"
    _say(f"gemm split-K layout={layout} M,N,K={mnk}")
    need = tbp.lib().tbp_gemm_workspace_bytes(tbp.TBP_BF16, layout, M, N, K, 0)
    assert need > 0, "these shapes are meant to take the split path"
    assert tbp.lib().tbp_gemm_workspace_bytes(tbp.TBP_BF16, tbp.TN, M, N, K, 1) == 0
    assert tbp.lib().tbp_gemm_workspace_bytes(tbp.TBP_BF16, layout, 4096, 4096, K, 0) == 0      # 256 tiles: no split
    assert tbp.lib().tbp_gemm_workspace_bytes(tbp.TBP_BF16, layout, M, N, 4096, 0) == 0         # short contraction: no gain
    a_shape = (M, K)
    b_shape = (N, K) if layout == tbp.NT else (K, N)
    A, B = _rnd(13, "A", a_shape, dtype), _rnd(13, "B", b_shape, dtype)
    R = _rnd(13, "R", (M, N), dtype, 4.0)
    a64, b64 = A.astype(np.float64), B.astype(np.float64)
    ref = ops.linear_p1(a64, b64) if layout == tbp.NT else ops.linear_fwd(a64, b64)
    dA, dB, dR = to_dev(A, dtype), to_dev(B, dtype), to_dev(R, dtype)
    ws = torch.empty(need + 4096, dtype=torch.uint8, device=DEV).fill_(0xA5)      # junk, larger than needed
    got1 = tbp.tbp_gemm(layout, dA, dB, workspace=ws)
    assert max_rel(to_np(got1), ref) < 4.5e-3
    got2 = tbp.tbp_gemm(layout, dA, dB, workspace=ws)
    assert torch.equal(got1, got2)
    got3 = tbp.tbp_gemm(layout, dA, dB, R=dR, alpha=0.5, workspace=ws)
    assert max_rel(to_np(got3), 0.5 * ref + R) < 4.5e-3
    # without scratch the same call takes the ordinary path and agrees to rounding
    plain = tbp.tbp_gemm(layout, dA, dB)
    assert max_rel(to_np(plain), to_np(got1).astype(np.float64)) < 8e-3
    # too small a workspace is not used (and not an error)
    small = torch.empty(1024, dtype=torch.uint8, device=DEV)
    assert max_rel(to_np(tbp.tbp_gemm(layout, dA, dB, workspace=small)), ref) < 4.5e-3


def test_gemm_strided_views_and_empty():
    # operands that are column blocks of wider matrices (leading dimension > row length), as the stage uses them
    dtype = "bf16"
    big = _rnd(12, "big", (300, 3 * 128), dtype)
    W = _rnd(12, "w", (128, 200), dtype)
    d_big, d_w = to_dev(big, dtype), to_dev(W, dtype)
    view = d_big[:, 128:256]
    got = tbp.tbp_gemm(tbp.NN, view, d_w, out_f32=True)
    assert max_rel(to_np(got), ops.linear_fwd(big[:, 128:256].astype(np.float64), W.astype(np.float64))) < 2e-5
    got = tbp.tbp_gemm(tbp.TN, view, d_big[:, 256:], out_f32=True)
    assert max_rel(to_np(got), ops.linear_p2(big[:, 128:256].astype(np.float64), big[:, 256:].astype(np.float64))) < 2e-5
    # K = 0 gives zeros (or leaves an accumulated C alone); M = 0 is a no-op
    z = tbp.tbp_gemm(tbp.NN, torch.empty((16, 0), dtype=torch.bfloat16, device=DEV),
                     torch.empty((0, 24), dtype=torch.bfloat16, device=DEV), out_f32=True)
    assert torch.count_nonzero(z).item() == 0
    e = tbp.tbp_gemm(tbp.NN, torch.empty((0, 8), dtype=torch.bfloat16, device=DEV), d_w[:8], out_f32=True)
    assert e.shape == (0, 200)


# ------------------------------------------------------------------------------------------- elementwise
@pytest.mark.parametrize("dtype,rows,d", [("bf16", 37, 4096), ("bf16", 1030, 5120), ("bf16", 5, 264), ("bf16", 3, 8192),
                                          ("f32", 37, 256), ("f32", 515, 1028), ("f32", 2, 4096)])
def test_rmsnorm_fwd_and_p1(dtype, rows, d):
    _say(f"rmsnorm dtype={dtype} rows={rows} d={d}")
    eps = 1e-6
    x, dy, res = (_rnd(13, n, (rows, d), dtype) for n in ("x", "dy", "res"))
    g = _rnd(13, "g", (d,), dtype, 0.1) + si.store_round(np.ones(d), dtype)
    g = si.store_round(g, dtype)
    x64, dy64, g64 = x.astype(np.float64), dy.astype(np.float64), g.astype(np.float64)
    out_tol = 4.5e-3 if dtype == "bf16" else 2e-6
    y = tbp.tbp_rmsnorm_fwd(to_dev(x, dtype), to_dev(g, dtype), eps)
    assert max_rel(to_np(y), ops.rmsnorm_fwd(x64, g64, eps)) < out_tol
    dx, dg = tbp.tbp_rmsnorm_p1(to_dev(dy, dtype), to_dev(x, dtype), to_dev(g, dtype), eps, resid=to_dev(res, dtype))
    assert max_rel(to_np(dx), res.astype(np.float64) + ops.rmsnorm_p1(dy64, x64, g64, eps)) < out_tol
    assert max_rel(to_np(dg), ops.rmsnorm_p2(dy64, x64, eps)) < 2e-5
    dx2, _ = tbp.tbp_rmsnorm_p1(to_dev(dy, dtype), to_dev(x, dtype), to_dev(g, dtype), eps)
    assert max_rel(to_np(dx2), ops.rmsnorm_p1(dy64, x64, g64, eps)) < out_tol


@pytest.mark.parametrize("dtype,rows,d", [("bf16", 4096, 4096), ("bf16", 2051, 5120), ("bf16", 515, 8192), ("bf16", 300, 2048),
                                          ("bf16", 3, 264), ("f32", 130, 1028),
                                          # widths that leave lanes of the 8-wave rows without a vector, one row only
                                          ("bf16", 66, 2056), ("bf16", 9, 4104), ("bf16", 1, 4096)])
def test_rmsnorm_p1_partial_rows_and_their_sum(dtype, rows, d):
    """The two halves of the RMSNorm backward as the stage runs them: backward-p1 leaves dx and the partial rows of the
    gain gradient, backward-p2 adds partial rows up; partial rows of two micro-batches stored one after the other are
    summed by one call."""
    _say(f"rmsnorm partial rows dtype={dtype} rows={rows} d={d}")
    eps = 1e-6
    x, dy, res, x2, dy2 = (_rnd(31, n, (rows, d), dtype) for n in ("x", "dy", "res", "x2", "dy2"))
    g = si.store_round(1.0 + 0.1 * si.standard_normal(31, "g", (d,)), dtype)
    f64 = lambda a: a.astype(np.float64)
    out_tol = 4.5e-3 if dtype == "bf16" else 2e-6
    n_part = tbp.lib().tbp_rmsnorm_partial_rows(tbp.TBP_BF16 if dtype == "bf16" else tbp.TBP_F32, rows, d)
    assert 1 <= n_part <= min(rows, 256)
    dx, parts = tbp.tbp_rmsnorm_p1_partials(to_dev(dy, dtype), to_dev(x, dtype), to_dev(g, dtype), eps, resid=to_dev(res, dtype))
    assert parts.shape == (n_part, d)
    assert max_rel(to_np(dx), f64(res) + ops.rmsnorm_p1(f64(dy), f64(x), f64(g), eps)) < out_tol
    want = ops.rmsnorm_p2(f64(dy), f64(x), eps)
    assert max_rel(to_np(tbp.tbp_gain_partials_sum(parts)), want) < 2e-5
    dx2, parts2 = tbp.tbp_rmsnorm_p1_partials(to_dev(dy2, dtype), to_dev(x2, dtype), to_dev(g, dtype), eps)
    assert max_rel(to_np(dx2), ops.rmsnorm_p1(f64(dy2), f64(x2), f64(g), eps)) < out_tol
    both = torch.cat([parts, parts2], dim=0).contiguous()
    want2 = ops.rmsnorm_p2(np.concatenate([f64(dy), f64(dy2)]), np.concatenate([f64(x), f64(x2)]), eps)
    assert max_rel(to_np(tbp.tbp_gain_partials_sum(both)), want2) < 2e-5
    acc = tbp.tbp_gain_partials_sum(parts)
    tbp.tbp_gain_partials_sum(parts2, dg=acc)
    assert max_rel(to_np(acc), want2) < 2e-5
    # the one-call form agrees bit for bit (same kernels)
    dx1, dg1 = tbp.tbp_rmsnorm_p1(to_dev(dy, dtype), to_dev(x, dtype), to_dev(g, dtype), eps, resid=to_dev(res, dtype))
    assert torch.equal(dx1, dx) and torch.equal(dg1, tbp.tbp_gain_partials_sum(parts))


@pytest.mark.parametrize("dtype,rows,f", [("bf16", 129, 11008), ("bf16", 7, 5504), ("f32", 130, 688), ("f32", 1, 4)])
def test_swiglu_fwd_and_p1(dtype, rows, f):
    _say(f"swiglu dtype={dtype} rows={rows} f={f}")
    gu = _rnd(14, "gu", (rows, 2 * f), dtype, 2.0)
    dm = _rnd(14, "dm", (rows, f), dtype)
    gu64, dm64 = gu.astype(np.float64), dm.astype(np.float64)
    tol = 4.5e-3 if dtype == "bf16" else 2e-6
    m = tbp.tbp_swiglu_fwd(to_dev(gu, dtype))
    assert max_rel(to_np(m), ops.swiglu_fwd(gu64[:, :f], gu64[:, f:])) < tol
    dgu = tbp.tbp_swiglu_p1(to_dev(dm, dtype), to_dev(gu, dtype))
    da, db = ops.swiglu_p1(dm64, gu64[:, :f], gu64[:, f:])
    assert max_rel(to_np(dgu), np.concatenate([da, db], axis=1)) < tol


@pytest.mark.parametrize("dtype,seq,nb,H,dh", [("bf16", 1024, 1, 8, 128), ("bf16", 40, 3, 5, 64), ("f32", 128, 2, 4, 64),
                                               ("f32", 12, 2, 3, 8)])
def test_rope_fwd_and_inverse(dtype, seq, nb, H, dh):
    _say(f"rope dtype={dtype} seq={seq} nb={nb} H={H} dh={dh}")
    rows, ld = seq * nb, H * dh + (dh if dtype == "bf16" else 8)     # a trailing block that must stay untouched
    x = _rnd(15, "x", (rows, ld), dtype)
    x64 = x.astype(np.float64)
    table = tbp.tbp_rope_table(seq, dh, 10000.0)
    tol = 4.5e-3 if dtype == "bf16" else 2e-6
    for inverse in (False, True):
        got = to_np(tbp.tbp_rope(to_dev(x, dtype), seq, H, dh, table, inverse=inverse))
        fn = ops.rope_p1 if inverse else ops.rope_fwd
        assert max_rel(got[:, :H * dh], fn(x64[:, :H * dh], seq, H, dh, 10000.0)) < tol
        assert np.array_equal(got[:, H * dh:], x64[:, H * dh:])


@pytest.mark.parametrize("dtype,n_mat,seq", [("bf16", 3, 1024), ("bf16", 2, 264), ("bf16", 1, 4096), ("f32", 4, 128),
                                             ("f32", 2, 260)])
@pytest.mark.parametrize("causal", [True, False])
def test_softmax_fwd_and_p1(dtype, n_mat, seq, causal):
    _say(f"softmax dtype={dtype} n_mat={n_mat} seq={seq} causal={causal}")
    sc = _rnd(16, "s", (n_mat, seq, seq), "f32", 3.0)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    P = tbp.tbp_softmax_fwd(to_dev(sc, "f32"), causal, tdt)
    ref = ops.softmax_fwd(sc.astype(np.float64), causal)
    got = to_np(P)
    tol = 4.5e-3 if dtype == "bf16" else 2e-6
    assert max_rel(got, ref) < tol
    if causal:
        iu = np.triu_indices(seq, 1)
        assert np.all(got[:, iu[0], iu[1]] == 0)
    # backward on the stored probabilities (what the materialised attention does)
    Pst = si.store_round(ref, dtype)
    dP = _rnd(16, "dp", (n_mat, seq, seq), dtype)
    p64, g64 = Pst.astype(np.float64), dP.astype(np.float64)
    ds_ref = ops.softmax_p1(p64, g64)
    ddP = to_dev(dP, dtype)
    if causal:   # the kernel must not depend on what lies above the diagonal: poison it
        ddP = torch.where(torch.triu(torch.ones(seq, seq, dtype=torch.bool, device=DEV), 1), torch.full_like(ddP, float("nan")), ddP)
    dS = to_np(tbp.tbp_softmax_p1(to_dev(Pst, dtype), ddP, causal))
    if causal:   # compare the lower triangle; the zero-filled band must be exact zeros, the rest is never read
        low = np.tril(np.ones((seq, seq), bool))
        assert max_rel(np.where(low, dS, 0.0), ds_ref) < tol
        i, j = np.indices((seq, seq))
        band = (j > i) & (j < np.minimum(seq, (i // 256 + 1) * 256))
        assert np.all(dS[:, band] == 0)
    else:
        assert max_rel(dS, ds_ref) < tol


@pytest.mark.parametrize("seq,nb,H,dh,causal", [(256, 1, 2, 128, True), (136, 2, 3, 64, True), (520, 1, 2, 128, True),
                                                (200, 1, 2, 64, False), (1024, 1, 4, 128, True), (8, 1, 1, 64, True),
                                                # 8 (sequence, head) pairs: the dq product's XCD-grouped tile map;
                                                # 256 pairs x 3 query tiles: its paired-tile kernel, middle tile alone
                                                (256, 2, 4, 64, True), (384, 4, 64, 64, True),
                                                # 32 pairs x 8 key blocks: several rounds of workgroups per XCD
                                                (1024, 1, 32, 64, True),
                                                # the longest sequence the kernels take
                                                (4096, 1, 1, 128, True)])
@pytest.mark.parametrize("recompute", [False, True])
def test_fused_attention_backward(seq, nb, H, dh, causal, recompute):
    """dq, dk, dv of the fused backward (probabilities rebuilt from the row log-sum-exp) against the oracle's; dq either
    from the product with the dS^T that the first pass writes out, or from the recompute pass."""
    _say(f"attention p1 seq={seq} batch={nb} heads={H} dh={dh} causal={causal} recompute={recompute}")
    d = H * dh
    q, k, v, do = (_rnd(42, n, (nb * seq, d), "bf16") for n in ("q", "k", "v", "do"))
    q64, k64, v64 = q.astype(np.float64), k.astype(np.float64), v.astype(np.float64)
    _, P = ops.attention_fwd(q64, k64, v64, seq, H, dh, causal)
    dq, dk, dv = ops.attention_p1(do.astype(np.float64), q64, k64, v64, P, seq, H, dh)
    qkv = to_dev(np.concatenate([q, k, v], axis=1), "bf16")
    out, lse2 = tbp.tbp_attention_fwd(qkv, seq, H, dh, causal)
    got = to_np(tbp.tbp_attention_p1(qkv, out, to_dev(do, "bf16"), lse2, seq, H, dh, causal, recompute=recompute))
    for name, ref, blk in (("dq", dq, got[:, :d]), ("dk", dk, got[:, d:2 * d]), ("dv", dv, got[:, 2 * d:])):
        err = max_rel(blk, ref)
        _say(f"   {name}: {err:.2e}")
        assert err < 1.5e-2, name


# ------------------------------------------------------------------------------------------- whole stage
@pytest.mark.parametrize("seq,nb,H,dh,causal", [(256, 1, 2, 128, True), (136, 2, 3, 64, True), (520, 1, 2, 128, True),
                                                (200, 1, 2, 64, False), (1024, 1, 4, 128, True), (8, 1, 1, 64, True),
                                                (4096, 1, 1, 128, True)])
def test_fused_attention_forward(seq, nb, H, dh, causal):
    """Fused attention against the oracle's materialised form; the row log-sum-exp against what the oracle's
    probabilities imply (lse_i = s_ii - log P_ii on the diagonal, which is never masked)."""
    _say(f"attention fwd seq={seq} batch={nb} heads={H} dh={dh} causal={causal}")
    d = H * dh
    q, k, v = (_rnd(41, n, (nb * seq, d), "bf16") for n in ("q", "k", "v"))
    o_ref, P = ops.attention_fwd(q.astype(np.float64), k.astype(np.float64), v.astype(np.float64), seq, H, dh, causal)
    qkv = to_dev(np.concatenate([q, k, v], axis=1), "bf16")
    out, lse2 = tbp.tbp_attention_fwd(qkv, seq, H, dh, causal)
    assert max_rel(to_np(out), o_ref) < 1e-2
    got = to_np(lse2) * np.log(2.0)
    for b in range(nb):
        for h in range(H):
            qh = q[b * seq:(b + 1) * seq, h * dh:(h + 1) * dh].astype(np.float64)
            kh = k[b * seq:(b + 1) * seq, h * dh:(h + 1) * dh].astype(np.float64)
            sii = np.sum(qh * kh, axis=1) / np.sqrt(dh)
            ref = sii - np.log(np.diagonal(P[b, h]))
            assert np.max(np.abs(got[b, h] - ref)) < 2e-3 * max(1.0, np.max(np.abs(ref)))


@pytest.mark.parametrize("gain", [6.0, 0.05])
def test_fused_attention_forward_score_range(gain):
    """The forward kernel keeps the reference point of its exponentials within a fixed distance of the running row
    maximum instead of on it.  Large scores (the maximum climbs by many octaves along the row, so the reference point
    moves several times) and tiny ones (it never moves after the first block) must give the oracle's output and row
    log-sum-exp all the same."""
    seq, nb, H, dh = 640, 1, 2, 128
    _say(f"attention fwd score range gain={gain}")
    d = H * dh
    q = _rnd(43, "q", (nb * seq, d), "bf16", scale=gain)
    k, v = (_rnd(43, n, (nb * seq, d), "bf16") for n in ("k", "v"))
    o_ref, P = ops.attention_fwd(q.astype(np.float64), k.astype(np.float64), v.astype(np.float64), seq, H, dh, True)
    qkv = to_dev(np.concatenate([q, k, v], axis=1), "bf16")
    out, lse2 = tbp.tbp_attention_fwd(qkv, seq, H, dh, True)
    assert max_rel(to_np(out), o_ref) < 1e-2
    got = to_np(lse2) * np.log(2.0)
    for h in range(H):
        s = (q[:, h * dh:(h + 1) * dh].astype(np.float64) @ k[:, h * dh:(h + 1) * dh].astype(np.float64).T) / np.sqrt(dh)
        s = np.where(np.tril(np.ones((seq, seq), bool)), s, -np.inf)
        mx = s.max(axis=1)
        ref = mx + np.log(np.exp(s - mx[:, None]).sum(axis=1))
        assert np.max(np.abs(got[0, h] - ref)) < 2e-3 * max(1.0, np.max(np.abs(ref)))


def _stage_inputs(shape):
    params = si.stage_params(shape)
    xs = [si.stage_input(shape, m) for m in range(shape.n_microbatches)]
    dys = [si.stage_upstream_grad(shape, m) for m in range(shape.n_microbatches)]
    return params, xs, dys


def _run_gpu(shape, params, xs, dys, mode=tbp.TBP_P2_LOOP, accumulate=True, p1_order=None, attention=tbp.TBP_ATTN_AUTO,
             gain_grad=tbp.TBP_GAIN_PARTIALS):
    st = make_gpu_stage(shape, params, attention=attention, gain_grad=gain_grad)
    n = len(xs)
    outs = [st.forward(m, to_dev(xs[m], shape.dtype)) for m in range(n)]
    dxs = [None] * n
    for m in (p1_order or range(n)):
        dxs[m] = st.backward_p1(m, to_dev(dys[m], shape.dtype))
    st.backward_p2(range(n), mode=mode, accumulate=accumulate)
    torch.cuda.synchronize()
    return st, outs, dxs


SMALL = {
    "tiny_f32": si.CONFIGS["tiny_f32"],                                   # the benchmark's fp32 configuration, whole
    "ragged_f32": si.StageShape("ragged_f32", 2, 72, 3, 24, 100, 20, 3, 3, "f32", 31),
    "small_bf16": si.StageShape("small_bf16", 2, 256, 4, 64, 688, 136, 2, 3, "bf16", 32),
    "mlp_small_bf16": si.StageShape("mlp_small_bf16", 3, 264, 0, 0, 520, 100, 1, 4, "bf16", 33),
    "mlp_f32": si.StageShape("mlp_f32", 2, 64, 0, 0, 172, 33, 1, 2, "f32", 34),
    "tiles_bf16": si.StageShape("tiles_bf16", 1, 512, 4, 128, 1032, 520, 1, 2, "bf16", 35),   # several 256-tiles + tails
}


# the attention of the bf16 stages with head_dim 64 / 128 runs fused by default; the same stages are also run with the
# materialised form (probabilities stashed)
STAGE_CASES = [(n, tbp.TBP_ATTN_AUTO) for n in SMALL] + [("small_bf16", tbp.TBP_ATTN_MATERIALISED),
                                                        ("tiles_bf16", tbp.TBP_ATTN_MATERIALISED),
                                                        ("small_bf16", tbp.TBP_ATTN_FUSED_RECOMPUTE),
                                                        ("tiles_bf16", tbp.TBP_ATTN_FUSED_RECOMPUTE)]


@pytest.mark.parametrize("name,attention", STAGE_CASES)
@pytest.mark.parametrize("mode", [tbp.TBP_P2_LOOP, tbp.TBP_P2_KCONCAT])
def test_stage_matches_oracle(name, attention, mode):
    shape = SMALL[name]
    _say(f"stage {name} mode={mode} attention={attention} shape={shape}")
    params, xs, dys = _stage_inputs(shape)
    outs, dxs, grads = run_oracle(shape, params, xs, dys)
    st, g_outs, g_dxs = _run_gpu(shape, params, xs, dys, mode=mode, accumulate=False,
                                 p1_order=list(reversed(range(len(xs)))), attention=attention)
    compare_stage(shape, g_outs, g_dxs, st.grads, outs, dxs, grads, stage_tolerance(shape.dtype), f"{name}/{mode}")
    stats = st.stats()
    assert stats["w_live_bytes"] == 0 and stats["a_live_bytes"] == 0 and stats["high_water_bytes"] > 0
    st.close()


@pytest.mark.parametrize("name", ["tiny_f32", "ragged_f32", "small_bf16", "mlp_small_bf16", "tiles_bf16"])
@pytest.mark.parametrize("mode", [tbp.TBP_P2_LOOP, tbp.TBP_P2_KCONCAT])
def test_stage_with_gain_gradients_in_p2_matches_oracle(name, mode):
    """The RMSNorm gain gradients computed in backward-p2 from stashed (x, dy) (Section 3.1 taken literally): same
    outputs and gradients; p1 leaves no gain partials and the norm operands are released by p2."""
    shape = SMALL[name]
    _say(f"stage (literal gain p2) {name} mode={mode} shape={shape}")
    params, xs, dys = _stage_inputs(shape)
    outs, dxs, grads = run_oracle(shape, params, xs, dys)
    st, g_outs, g_dxs = _run_gpu(shape, params, xs, dys, mode=mode, accumulate=False,
                                 p1_order=list(reversed(range(len(xs)))), gain_grad=tbp.TBP_GAIN_LITERAL)
    compare_stage(shape, g_outs, g_dxs, st.grads, outs, dxs, grads, stage_tolerance(shape.dtype), f"{name}/{mode}/literal")
    stats = st.stats()
    assert stats["w_live_bytes"] == 0 and stats["a_live_bytes"] == 0 and stats["high_water_bytes"] > 0
    # a second set on top of the first: accumulation doubles every gradient
    for m in range(len(xs)):
        st.forward(m, to_dev(xs[m], shape.dtype))
    for m in range(len(xs)):
        st.backward_p1(m, to_dev(dys[m], shape.dtype))
    st.backward_p2(range(len(xs)), mode=mode, accumulate=True)
    torch.cuda.synchronize()
    twice = {k: [2.0 * g for g in v] for k, v in grads.items()}
    compare_stage(shape, g_outs, g_dxs, st.grads, outs, dxs, twice, stage_tolerance(shape.dtype), f"{name}/{mode}/literal x2")
    st.close()


@pytest.mark.parametrize("dtype,rows,d", [("f32", 0, 64), ("f32", 1, 4), ("f32", 37, 72), ("f32", 1030, 4096),
                                          ("bf16", 1, 8), ("bf16", 300, 520), ("bf16", 1030, 4096), ("bf16", 64, 8192)])
def test_rmsnorm_gain_p2(dtype, rows, d):
    """dg = sum_t dy x r as its own backward-p2 operation, overwriting and accumulating."""
    _say(f"rmsnorm_gain_p2 {dtype} rows={rows} d={d}")
    x = _rnd(21, "x", (rows, d), dtype, 1.5)
    dy = _rnd(21, "dy", (rows, d), dtype)
    eps = 1e-5
    want = ops.rmsnorm_p2(dy.astype(np.float64), x.astype(np.float64), eps)
    got = tbp.tbp_rmsnorm_gain_p2(to_dev(dy, dtype), to_dev(x, dtype), eps)
    if rows == 0:
        assert float(got.abs().max()) == 0.0
        return
    assert max_rel(to_np(got), want) < 2e-5
    again = tbp.tbp_rmsnorm_gain_p2(to_dev(dy, dtype), to_dev(x, dtype), eps, dg=got.clone())
    assert max_rel(to_np(again), 2.0 * want) < 2e-5


def test_p2_on_a_second_stream_overlapping_the_next_p1():
    """p2({m}) enqueued on a second stream once p1(m) is done, while p1(m+1) runs on the first: the weight-gradient
    products read only what p1(m) has finished writing, so the gradients equal the oracle's."""
    shape = SMALL["tiles_bf16"].replace(n_microbatches=3)
    params, xs, dys = _stage_inputs(shape)
    _, dxs, grads = run_oracle(shape, params, xs, dys)
    tol = stage_tolerance(shape.dtype)
    st = make_gpu_stage(shape, params)
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    for m in range(3):
        st.forward(m, to_dev(xs[m], shape.dtype))
    g_dxs = []
    for m in range(3):
        g_dxs.append(st.backward_p1(m, to_dev(dys[m], shape.dtype)))
        side.wait_stream(main)
        with torch.cuda.stream(side):
            st.backward_p2([m], tbp.TBP_P2_LOOP, accumulate=(m > 0))
    main.wait_stream(side)
    torch.cuda.synchronize()
    for k, v in st.grads.items():
        for l in range(len(v)):
            assert max_rel(to_np(v[l]), grads[k][l]) < tol, (k, l)
    for m in range(3):
        assert max_rel(to_np(g_dxs[m]), dxs[m]) < tol
    st.close()


def test_p2_call_patterns_agree():
    """p2 right after each p1 (ordinary backprop), p2 by subsets, loop and K-concatenated: same gradients."""
    shape = SMALL["small_bf16"].replace(n_microbatches=4)
    params, xs, dys = _stage_inputs(shape)
    _, _, grads = run_oracle(shape, params, xs, dys)
    tol = stage_tolerance(shape.dtype)
    results = []
    # (a) interleaved: p1(m) then p2({m})
    st = make_gpu_stage(shape, params, act_slots=1)       # one activation slot is enough for this order
    for m in range(4):
        st.forward(m, to_dev(xs[m], shape.dtype))
        st.backward_p1(m, to_dev(dys[m], shape.dtype))
        st.backward_p2([m], tbp.TBP_P2_LOOP, accumulate=(m > 0))
    torch.cuda.synchronize()
    results.append({k: [to_np(g) for g in v] for k, v in st.grads.items()})
    st.close()
    # (b) all forwards, all p1, then p2 on {0,1} K-concatenated (overwrite) and {3,2} looped (accumulate)
    st = make_gpu_stage(shape, params)
    for m in range(4):
        st.forward(m, to_dev(xs[m], shape.dtype))
    for m in range(4):
        st.backward_p1(m, to_dev(dys[m], shape.dtype))
    mid = st.stats()
    assert mid["a_live_bytes"] == 0 and mid["w_live_bytes"] > 0
    st.backward_p2([0, 1], tbp.TBP_P2_KCONCAT, accumulate=False)
    assert st.stats()["w_live_bytes"] * 2 == mid["w_live_bytes"]
    st.backward_p2([3, 2], tbp.TBP_P2_LOOP, accumulate=True)
    torch.cuda.synchronize()
    results.append({k: [to_np(g) for g in v] for k, v in st.grads.items()})
    # the stage is reusable: micro-batch indices are EMPTY again
    st.forward(0, to_dev(xs[0], shape.dtype))
    with pytest.raises(tbp.TbpError):
        st.backward_p2([0], tbp.TBP_P2_LOOP)
    with pytest.raises(tbp.TbpError):
        st.backward_p2([1, 3], tbp.TBP_P2_KCONCAT)
    st.close()
    for r in results:
        for k in r:
            for l in range(len(r[k])):
                assert max_rel(r[k][l], grads[k][l]) < tol, (k, l)
    for k in results[0]:
        for l in range(len(results[0][k])):
            assert max_rel(results[0][k][l], results[1][k][l]) < 1e-4     # fp32 summation order only


def test_activation_slots_run_out():
    shape = SMALL["mlp_f32"]
    params, xs, _ = _stage_inputs(shape)
    st = make_gpu_stage(shape, params, act_slots=1)
    st.forward(0, to_dev(xs[0], shape.dtype))
    with pytest.raises(tbp.TbpError) as e:
        st.forward(1, to_dev(xs[1], shape.dtype))
    assert e.value.status == 3
    with pytest.raises(tbp.TbpError) as e:
        st.forward(0, to_dev(xs[0], shape.dtype))
    assert e.value.status == 2
    torch.cuda.synchronize()
    st.close()
