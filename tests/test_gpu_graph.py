"""A whole step of the stage (forward, backward-p1 and backward-p2 of every micro-batch) recorded into a HIP graph and
replayed: the library allocates nothing, synchronises nothing and clears memory with kernels only, so its launches can
be captured as they are.  Every replay must reproduce the eager run bit for bit (all kernels are deterministic), also
with eager work and synchronisations between the replays."""
import pytest
import torch

import paper_2405_18047_amd as tbp
import seeded_inputs as si
from gpu_util import make_gpu_stage, to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mode", [tbp.TBP_P2_KCONCAT, tbp.TBP_P2_LOOP])
def test_step_replayed_from_a_graph_equals_the_eager_step(mode):
    shape = si.StageShape("graph_bf16", 2, 256, 4, 64, 688, 136, 2, 3, "bf16", 36)
    print(f"graph replay of a whole step, p2 mode {mode}, shape={shape}", flush=True)
    params = si.stage_params(shape)
    n = shape.n_microbatches
    host = {"a": ([si.stage_input(shape, m) for m in range(n)], [si.stage_upstream_grad(shape, m) for m in range(n)]),
            "b": ([si.stage_input(shape, m + n) for m in range(n)], [si.stage_upstream_grad(shape, m + n) for m in range(n)])}
    dev = {k: ([to_dev(x, shape.dtype) for x in xs], [to_dev(d, shape.dtype) for d in dys]) for k, (xs, dys) in host.items()}
    st = make_gpu_stage(shape, params)
    # static buffers: a graph replays fixed addresses
    x_in = [torch.empty_like(t) for t in dev["a"][0]]
    dy_in = [torch.empty_like(t) for t in dev["a"][1]]
    x_out = [torch.empty_like(t) for t in x_in]
    dx_out = [torch.empty_like(t) for t in x_in]

    def load(which):
        for m in range(n):
            x_in[m].copy_(dev[which][0][m])
            dy_in[m].copy_(dev[which][1][m])

    def step():
        for m in range(n):
            st.forward(m, x_in[m], out=x_out[m])
        for m in range(n):
            st.backward_p1(m, dy_in[m], out=dx_out[m])
        st.backward_p2(range(n), mode, accumulate=False)

    def snapshot():
        torch.cuda.synchronize()
        return ([t.clone() for t in x_out], [t.clone() for t in dx_out],
                {k: [g.clone() for g in v] for k, v in st.grads.items()})

    want = {}
    for which in ("a", "b"):
        load(which)
        step()
        want[which] = snapshot()
    assert not torch.equal(want["a"][1][0], want["b"][1][0])      # the two input sets really differ

    load("a")
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep, which in enumerate(("a", "b", "a", "b")):
        print(f"   replay {rep} on input set {which}", flush=True)
        load(which)
        graph.replay()
        outs, dxs, grads = snapshot()
        for m in range(n):
            assert torch.equal(outs[m], want[which][0][m]), ("x_out", rep, m)
            assert torch.equal(dxs[m], want[which][1][m]), ("dx", rep, m)
        for k, v in grads.items():
            for l, g in enumerate(v):
                assert torch.equal(g, want[which][2][k][l]), (k, l, rep)
        # the program's own eager work between replays: a step on the other input set overwrites every output
        load("b" if which == "a" else "a")
        step()
        torch.cuda.synchronize()
    st.close()


@pytest.mark.parametrize("shape", [
    si.StageShape("graph_first_bf16", 1, 512, 4, 128, 1032, 264, 1, 2, "bf16", 37),       # attention: rotation table
    si.StageShape("graph_first_long_k", 1, 1024, 0, 0, 24576, 1024, 1, 2, "bf16", 38),    # a product with a split contraction
], ids=lambda s: s.name)
def test_graph_recorded_before_any_eager_call(shape):
    """A stage whose very first calls are recorded, not run: nothing the later eager calls rely on (rotation table,
    cleared counters) may have been set up by a launch that so far exists only in the graph."""
    print(f"graph recorded before any eager call, shape={shape}", flush=True)
    params = si.stage_params(shape)
    n = shape.n_microbatches
    xs = [to_dev(si.stage_input(shape, m), shape.dtype) for m in range(n)]
    dys = [to_dev(si.stage_upstream_grad(shape, m), shape.dtype) for m in range(n)]
    x_out = [torch.empty_like(t) for t in xs]
    dx_out = [torch.empty_like(t) for t in xs]
    st = make_gpu_stage(shape, params)

    def step():
        for m in range(n):
            st.forward(m, xs[m], out=x_out[m])
        for m in range(n):
            st.backward_p1(m, dys[m], out=dx_out[m])
        st.backward_p2(range(n), tbp.TBP_P2_KCONCAT, accumulate=False)

    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    step()                                     # eager, before the graph has ever run
    torch.cuda.synchronize()
    want = ([t.clone() for t in x_out], [t.clone() for t in dx_out], {k: [g.clone() for g in v] for k, v in st.grads.items()})
    for t in x_out + dx_out:
        t.zero_()
    st.zero_grads()
    graph.replay()
    torch.cuda.synchronize()
    for m in range(n):
        assert torch.equal(x_out[m], want[0][m]) and torch.equal(dx_out[m], want[1][m]), m
    for k, v in st.grads.items():
        for l, g in enumerate(v):
            assert torch.equal(g, want[2][k][l]), (k, l)
    # and the eager result is the right one: compare with a second stage that never saw a graph
    ref = make_gpu_stage(shape, params)
    outs = [ref.forward(m, xs[m]) for m in range(n)]
    dxs = [ref.backward_p1(m, dys[m]) for m in range(n)]
    ref.backward_p2(range(n), tbp.TBP_P2_KCONCAT, accumulate=False)
    torch.cuda.synchronize()
    for m in range(n):
        assert torch.equal(outs[m], want[0][m]) and torch.equal(dxs[m], want[1][m]), m
    for k, v in ref.grads.items():
        for l, g in enumerate(v):
            assert torch.equal(g, want[2][k][l]), (k, l)
    ref.close()
    st.close()
