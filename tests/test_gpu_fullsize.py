"""Parity at the benchmark's real layer shapes (LLaMa-7B: d_model 4096, 32 heads x 128, FFN 11008, seq 1024).

The full 8-layer x 4-micro-batch oracle costs about 41 TFLOP in fp64, so:
  * a stage of the real layer shape with fewer layers / micro-batches is compared in full, every tensor;
  * at the full benchmark configuration, with the launch configuration bench.py times, the forward output of
    the first tokens of each sequence is compared with the oracle run on the truncated sequence (causal
    attention: token t depends on tokens <= t only, through every layer), and the weight gradients are checked
    through properties that hold at any size (loop == K-concatenated, subsets accumulate to the whole).
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2405_18047_amd as tbp
import seeded_inputs as si
from gpu_util import compare_stage, make_gpu_stage, max_rel, run_oracle, stage_tolerance, to_dev, to_np

pytestmark = pytest.mark.gpu


_PARAMS = {}


def _params(shape):
    """Parameters are a pure function of (seed, layer, dims): generated once per process for each such key (the
    8-layer 7B set takes a minute of host time and three tests use it)."""
    key = (shape.seed, shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn, shape.dtype)
    if key not in _PARAMS:
        _PARAMS.clear()                      # one set at a time: an 8-layer 7B set is 6.5 GB of float32
        _PARAMS[key] = si.stage_params(shape)
    return _PARAMS[key]


def _inputs(shape):
    return (_params(shape), [si.stage_input(shape, m) for m in range(shape.n_microbatches)],
            [si.stage_upstream_grad(shape, m) for m in range(shape.n_microbatches)])


def _gpu_step(st, xs, dys, p2_calls):
    outs = [st.forward(m, to_dev(xs[m], "bf16")) for m in range(len(xs))]
    dxs = [st.backward_p1(m, to_dev(dys[m], "bf16")) for m in range(len(xs))]
    for mbs, mode, acc in p2_calls:
        st.backward_p2(mbs, mode, accumulate=acc)
    torch.cuda.synchronize()
    return outs, dxs


@pytest.mark.timeout(600)
def test_real_layer_shape_full_compare():
    shape = si.CONFIGS["llama7b_s1024"].replace(n_layers=1, n_microbatches=2)
    print(f"real-shape stage {shape}", flush=True)
    params, xs, dys = _inputs(shape)
    outs, dxs, grads = run_oracle(shape, params, xs, dys)
    print("oracle done", flush=True)
    st = make_gpu_stage(shape, params)
    g_outs = [st.forward(m, to_dev(xs[m], "bf16")) for m in range(2)]
    g_dxs = [st.backward_p1(m, to_dev(dys[m], "bf16")) for m in range(2)]
    st.backward_p2([0, 1], tbp.TBP_P2_KCONCAT, accumulate=False)
    torch.cuda.synchronize()
    compare_stage(shape, g_outs, g_dxs, st.grads, outs, dxs, grads, stage_tolerance("bf16"), "7B layer shape")
    st.close()


@pytest.mark.timeout(600)
def test_mlp_config_real_shape_full_compare():
    shape = si.CONFIGS["mlp_bf16"].replace(n_layers=2, n_microbatches=3)
    print(f"real-shape MLP stage {shape}", flush=True)
    params, xs, dys = _inputs(shape)
    outs, dxs, grads = run_oracle(shape, params, xs, dys)
    st = make_gpu_stage(shape, params)
    g_outs = [st.forward(m, to_dev(xs[m], "bf16")) for m in range(3)]
    g_dxs = [st.backward_p1(m, to_dev(dys[m], "bf16")) for m in range(3)]
    st.backward_p2([0, 1, 2], tbp.TBP_P2_LOOP, accumulate=False)
    torch.cuda.synchronize()
    compare_stage(shape, g_outs, g_dxs, st.grads, outs, dxs, grads, stage_tolerance("bf16"), "MLP real shape")
    st.close()


@pytest.mark.timeout(600)
def test_13b_mlp_block_shape_full_compare():
    """The MLP half of a 13B-shaped layer (d_model 5120, FFN 13824, 2048 tokens per micro-batch): [2048, 5120] outputs
    are 160 tiles of 256 x 256, which the forward and backward-p1 products run on 256 x 192 tiles instead.  Every
    tensor is compared, twice in a row on the same stage."""
    shape = si.StageShape("mlp_13b_block", 1, 5120, 0, 0, 13824, 2048, 1, 2, "bf16", 20240524)
    print(f"13B MLP block {shape}", flush=True)
    params, xs, dys = _inputs(shape)
    outs, dxs, grads = run_oracle(shape, params, xs, dys)
    print("oracle done", flush=True)
    st = make_gpu_stage(shape, params)
    for rep in range(2):
        g_outs = [st.forward(m, to_dev(xs[m], "bf16")) for m in range(2)]
        g_dxs = [st.backward_p1(m, to_dev(dys[m], "bf16")) for m in range(2)]
        st.backward_p2([0, 1], tbp.TBP_P2_KCONCAT, accumulate=False)
        torch.cuda.synchronize()
        compare_stage(shape, g_outs, g_dxs, st.grads, outs, dxs, grads, stage_tolerance("bf16"), f"13B MLP block, pass {rep}")
    st.close()


@pytest.mark.timeout(600)
def test_stage_with_split_contraction():
    """A stage whose backward-p1 product dh2 = [dg, du] Wgu^T has a small output ([1024, 1024]: 16 large tiles) and a
    very long contraction (2 x 24576): the stage runs it with the contraction split over several workgroups per tile,
    using scratch from its own workspace, whose arrival counters are cleared before every such product."""
    shape = si.StageShape("mlp_long_k", 1, 1024, 0, 0, 24576, 1024, 1, 2, "bf16", 20240525)
    assert tbp.lib().tbp_gemm_workspace_bytes(tbp.TBP_BF16, tbp.NT, shape.tokens, shape.d_model, 2 * shape.d_ffn, 0) > 0
    params, xs, dys = _inputs(shape)
    outs, dxs, grads = run_oracle(shape, params, xs, dys)
    print("oracle done", flush=True)
    st = make_gpu_stage(shape, params)
    for rep in range(2):
        g_outs = [st.forward(m, to_dev(xs[m], "bf16")) for m in range(2)]
        g_dxs = [st.backward_p1(m, to_dev(dys[m], "bf16")) for m in range(2)]
        st.backward_p2([0, 1], tbp.TBP_P2_KCONCAT, accumulate=False)
        torch.cuda.synchronize()
        compare_stage(shape, g_outs, g_dxs, st.grads, outs, dxs, grads, stage_tolerance("bf16"), f"long-K MLP, pass {rep}")
    st.close()


@pytest.mark.timeout(900)
def test_full_benchmark_configuration_properties():
    """Full configuration (8 layers x 4 micro-batches), launch configuration of bench.py: properties that hold at
    any size.  (End-to-end agreement with fp64 is not asserted at this depth: every stored bf16 intermediate
    adds about 2^-8 relative noise and the branches dominate the residual at this weight scale, so the error
    grows with the square root of the depth; per-layer parity at depth is test_deep_stage_per_layer_parity.)"""
    shape = si.CONFIGS["llama7b_s1024"]
    print(f"full configuration {shape}", flush=True)
    params = si.stage_params(shape)
    print("parameters generated", flush=True)
    M = shape.n_microbatches
    xs = [si.stage_input(shape, m) for m in range(M)]
    dys = [si.stage_upstream_grad(shape, m) for m in range(M)]
    st = make_gpu_stage(shape, params)

    def run(p2_calls):
        outs = [st.forward(m, to_dev(xs[m], "bf16")) for m in range(M)]
        dxs = [st.backward_p1(m, to_dev(dys[m], "bf16")) for m in range(M)]
        for mbs, mode, acc in p2_calls:
            st.backward_p2(mbs, mode, accumulate=acc)
        torch.cuda.synchronize()
        return outs, dxs, {k: [g.clone() for g in v] for k, v in st.grads.items()}

    outs, dxs, g_cat = run([(range(M), tbp.TBP_P2_KCONCAT, False)])
    for t in outs + dxs:
        assert torch.isfinite(t.float()).all()
    # causality through all 8 layers: the first tokens' outputs equal those of the oracle on the truncated
    # sequence (loose bound: 8 layers of bf16 storage), and do not depend on later tokens at all on the GPU
    cut = 48
    ost = oracle.OracleStage(shape.replace(seq=cut), params)
    err = max_rel(to_np(outs[0][:cut]), ost.forward(0, xs[0][:cut]))
    print(f"forward prefix after 8 layers: {err:.3e}", flush=True)
    assert err < 6e-2
    # same stash contents, different p2 call patterns
    _, dxs2, g_loop = run([(range(M), tbp.TBP_P2_LOOP, False)])
    _, _, g_split = run([([0, 1], tbp.TBP_P2_KCONCAT, False), ([2, 3], tbp.TBP_P2_KCONCAT, True)])
    for a, b in zip(dxs, dxs2):
        assert torch.equal(a, b)                      # the path is deterministic
    for k in g_cat:
        for l in range(len(g_cat[k])):
            ref = to_np(g_cat[k][l])
            assert max_rel(to_np(g_loop[k][l]), ref) < 1e-4, (k, l)
            assert max_rel(to_np(g_split[k][l]), ref) < 1e-4, (k, l)
    st.close()


@pytest.mark.timeout(900)
def test_deep_stage_per_layer_parity():
    """Parity at depth with oracle-supplied layer inputs: the oracle runs one micro-batch through all 8 layers
    (forward and backward-p1); layers 0, 4 and 7 are then run alone on the GPU from the oracle's layer input and
    upstream gradient (rounded once to bf16) and compared with the oracle on exactly those rounded inputs."""
    shape = si.CONFIGS["llama7b_s1024"].replace(n_microbatches=1)
    params = si.stage_params(shape)
    x0, dy = si.stage_input(shape, 0), si.stage_upstream_grad(shape, 0)
    full = oracle.OracleStage(shape, params)
    layer_in = [np.asarray(x0, np.float64)]
    for layer in full.layers:
        layer_in.append(layer.forward(0, layer_in[-1]))
    print("oracle forward done", flush=True)
    layer_dy = [None] * shape.n_layers + [np.asarray(dy, np.float64)]
    for l in reversed(range(shape.n_layers)):
        layer_dy[l] = full.layers[l].backward_p1(0, layer_dy[l + 1])
    print("oracle backward-p1 done", flush=True)
    one = shape.replace(n_layers=1)
    for l in (0, 4, 7):
        p_l = {k: [v[l]] for k, v in params.items()}
        x_l = si.store_round(layer_in[l], "bf16")
        dy_l = si.store_round(layer_dy[l + 1], "bf16")
        outs, dxs, grads = run_oracle(one, p_l, [x_l], [dy_l])
        st = make_gpu_stage(one, p_l)
        g_out = st.forward(0, to_dev(x_l, "bf16"))
        g_dx = st.backward_p1(0, to_dev(dy_l, "bf16"))
        st.backward_p2([0], tbp.TBP_P2_KCONCAT, accumulate=False)
        torch.cuda.synchronize()
        compare_stage(one, [g_out], [g_dx], st.grads, outs, dxs, grads, stage_tolerance("bf16"), f"layer {l} of 8")
        st.close()


@pytest.mark.timeout(600)
def test_headline_layer_shape_full_compare():
    """One layer x two micro-batches of the benchmark's headline workload (seq 2048, micro-batch 2: 4096 tokens per
    micro-batch), in the launch configuration bench.py times: fused attention at (B 2, H 32, S 2048, dh 128), the
    256 x 256 tiles at 4096 rows, the weight-gradient products over 8192 concatenated rows.  Every tensor against the
    oracle, K-concatenated and looped backward-p2."""
    shape = si.CONFIGS["llama7b_s2048"].replace(n_layers=1, n_microbatches=2)
    print(f"headline layer shape {shape}", flush=True)
    params, xs, dys = _inputs(shape)
    outs, dxs, grads = run_oracle(shape, params, xs, dys)
    print("oracle done", flush=True)
    st = make_gpu_stage(shape, params)
    tol = stage_tolerance("bf16")
    g_outs, g_dxs = _gpu_step(st, xs, dys, [([0, 1], tbp.TBP_P2_KCONCAT, False)])
    compare_stage(shape, g_outs, g_dxs, st.grads, outs, dxs, grads, tol, "7B seq 2048 x mb 2, K-concat")
    g_outs, g_dxs = _gpu_step(st, xs, dys, [([0, 1], tbp.TBP_P2_LOOP, False)])
    compare_stage(shape, g_outs, g_dxs, st.grads, outs, dxs, grads, tol, "7B seq 2048 x mb 2, loop")
    st.close()


@pytest.mark.timeout(600)
@pytest.mark.parametrize("n_mb", [1, 2])
def test_13b_layer_shape_full_compare(n_mb):
    """One whole 13B-shaped layer (d_model 5120, 40 heads x 128, FFN 13824, seq 2048, micro-batch 1), attention
    included: 40 (sequence, head) pairs is a multiple of 8 but not of 32, so the XCD-grouped tile maps of the fused
    attention and of the dQ product take their ragged branch.  Every tensor against the oracle."""
    shape = si.CONFIGS["llama13b_s2048"].replace(n_layers=1, n_microbatches=n_mb)
    print(f"13B layer shape {shape}", flush=True)
    params, xs, dys = _inputs(shape)
    outs, dxs, grads = run_oracle(shape, params, xs, dys, concat=(n_mb == 2))
    print("oracle done", flush=True)
    st = make_gpu_stage(shape, params)
    mode = tbp.TBP_P2_KCONCAT if n_mb == 2 else tbp.TBP_P2_LOOP
    g_outs, g_dxs = _gpu_step(st, xs, dys, [(list(range(n_mb)), mode, False)])
    compare_stage(shape, g_outs, g_dxs, st.grads, outs, dxs, grads, stage_tolerance("bf16"), f"13B layer, {n_mb} mb")
    st.close()


def _depth_report(shape, st_grads, g_outs, g_dxs, outs, dxs, grads, label):
    """Per-tensor max-norm relative error of an end-to-end run, printed layer by layer; returns {tensor: error}."""
    err = {}
    for m in range(len(outs)):
        err[f"x_out[{m}]"] = max_rel(to_np(g_outs[m]), outs[m])
        err[f"dx[{m}]"] = max_rel(to_np(g_dxs[m]), dxs[m])
    for k, lst in st_grads.items():
        for l, g in enumerate(lst):
            err[f"d{k}[{l}]"] = max_rel(to_np(g), grads[k][l])
    print(f"[end-to-end {label}] " + ", ".join(f"{k}={v:.2e}" for k, v in err.items() if k.startswith(("x_out", "dx["))),
          flush=True)
    for l in range(shape.n_layers):
        print(f"[end-to-end {label}] layer {l}: " + ", ".join(f"d{k}={err[f'd{k}[{l}]']:.2e}" for k in st_grads), flush=True)
    worst = max(err, key=err.get)
    print(f"[end-to-end {label}] worst tensor {worst} = {err[worst]:.3e}; tensors above 2e-2: "
          f"{sorted(k for k, v in err.items() if v > 2e-2)}", flush=True)
    return err


_DEPTH8 = {}


def _depth8_errors(name, n_mb):
    """8-layer stage against the 8-layer oracle, end to end (the GPU's own bf16 intermediates flow through all
    layers), every tensor.  Computed once per process and shared by the tests below."""
    if (name, n_mb) not in _DEPTH8:
        shape = si.CONFIGS[name].replace(n_microbatches=n_mb)
        print(f"8-layer end-to-end {shape}", flush=True)
        params, xs, dys = _inputs(shape)
        outs, dxs, grads = run_oracle(shape, params, xs, dys, concat=True)
        print("oracle done", flush=True)
        st = make_gpu_stage(shape, params)
        g_outs, g_dxs = _gpu_step(st, xs, dys, [(list(range(n_mb)), tbp.TBP_P2_KCONCAT, False)])
        _DEPTH8[(name, n_mb)] = _depth_report(shape, st.grads, g_outs, g_dxs, outs, dxs, grads, f"{name} x {n_mb} mb")
        st.close()
    return _DEPTH8[(name, n_mb)]


DEPTH8_CASES = [("llama7b_s1024", 2), ("llama7b_s2048", 1)]


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name,n_mb", DEPTH8_CASES)
def test_eight_layer_end_to_end_error_measured(name, n_mb):
    """Measures and prints the end-to-end error of the 8-layer 7B stage, per tensor and per layer.  The bound asserted
    here is a sanity bound (three times the stated tolerance), NOT the target: the target is the next test."""
    err = _depth8_errors(name, n_mb)
    assert all(np.isfinite(v) for v in err.values())
    assert max(err.values()) < 6e-2, max(err, key=err.get)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name,n_mb", DEPTH8_CASES)
@pytest.mark.xfail(strict=True, reason="NOT MET at depth 8: measured worst tensor 3.9e-2 (seq 1024 x 2 micro-batches) and "
                   "4.6e-2 (seq 2048 x micro-batch 2 x 1), x_out 2.0e-2, dx 3.1-3.8e-2, every dW 2.0-3.9e-2, against the "
                   "stated 2e-2; fp64 arithmetic with bf16 rounding at the same storage points shows the same error, "
                   "so it is the storage format's, one layer alone is at 1e-2")
def test_eight_layer_end_to_end_within_stated_tolerance(name, n_mb):
    """The benchmark definition's target: the 8-layer 7B-shaped stage within 2e-2 (max-norm relative, bf16 against
    fp64) end to end."""
    err = _depth8_errors(name, n_mb)
    assert max(err.values()) <= stage_tolerance("bf16"), {k: v for k, v in err.items() if v > stage_tolerance("bf16")}
