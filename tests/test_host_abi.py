"""CPU-only checks of the C ABI: the library loads, exports what the header declares, and its host logic
(configuration checks, stash sizing, state machine) behaves without any GPU work being launched."""
import ctypes as C
import os
import re

import pytest

import paper_2405_18047_amd as tbp
import seeded_inputs as si

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "tbp.h")).read()
    names = set(re.findall(r"\b(tbp_[a-z0-9_]+)\s*\(", header))
    assert {"tbp_stage_forward", "tbp_stage_backward_p1", "tbp_stage_backward_p2", "tbp_stash_query"} <= names
    L = tbp.lib()
    for n in sorted(names):
        assert hasattr(L, n), n
    assert "gfx950" in tbp.tbp_version()


def _sizes(shape, **kw):
    return tbp.tbp_stash_query(tbp.config_from_shape(shape, **kw))


def test_stash_sizes_follow_the_stash_rule():
    """W class = inputs and output derivatives of the four linear layers (+ fp32 gain partials); A class = the rest."""
    for name in ("llama7b_s1024", "llama13b_s2048", "mlp_bf16"):
        s = si.CONFIGS[name]
        T, d, f, L, M = s.tokens, s.d_model, s.d_ffn, s.n_layers, s.n_microbatches
        if s.n_heads:
            w_el = 8 * d + 3 * f
            a_el = 5 * d + s.n_heads * s.seq + 2 * f
        else:
            w_el = 2 * d + 3 * f
            a_el = d + 2 * f
        got = _sizes(s, attention=tbp.TBP_ATTN_MATERIALISED)
        w_expect = L * M * T * w_el * 2
        # + per norm and micro-batch the fp32 partial rows of the gain gradient, as backward-p1's row kernel leaves them
        n_part = tbp.lib().tbp_rmsnorm_partial_rows(tbp.TBP_BF16, T, d)
        assert 1 <= n_part <= 256
        g_expect = L * 2 * M * n_part * d * 4          # (room for both norms of a layer, used or not)
        assert w_expect + g_expect <= got["w_stash_bytes"] <= w_expect * 1.001 + g_expect + 4096 * L
        assert got["a_stash_bytes"] == L * M * T * a_el * 2
        assert got["arena_bytes"] >= got["w_stash_bytes"] + got["a_stash_bytes"] + got["workspace_bytes"]
        if s.n_heads:     # fused attention keeps a row log-sum-exp (fp32 per token and head) instead of the probabilities
            fused = _sizes(s, attention=tbp.TBP_ATTN_FUSED)
            assert fused["a_stash_bytes"] == L * M * T * ((5 * d + 2 * f) * 2 + s.n_heads * 4)
            assert fused["w_stash_bytes"] == got["w_stash_bytes"]
            assert _sizes(s)["a_stash_bytes"] == fused["a_stash_bytes"]       # AUTO picks it for bf16, head_dim 128
            # dq by a recompute pass: the same stash, and the dS^T workspace (batch * heads * seq^2 elements) is gone
            lean = _sizes(s, attention=tbp.TBP_ATTN_FUSED_RECOMPUTE)
            assert lean["a_stash_bytes"] == fused["a_stash_bytes"] and lean["w_stash_bytes"] == fused["w_stash_bytes"]
            assert fused["workspace_bytes"] - lean["workspace_bytes"] == s.micro_batch * s.n_heads * s.seq * s.seq * 2
        # gain gradients computed in p2: each norm's input moves from the forward->p1 slots to slabs kept until p2 and
        # the derivative of its output is kept as well; the fp32 partials disappear
        lit = _sizes(s, gain_grad=tbp.TBP_GAIN_LITERAL)
        n_norms = 2 if s.n_heads else 1
        assert lit["a_stash_bytes"] == _sizes(s)["a_stash_bytes"] - L * M * T * n_norms * d * 2
        w_lit = L * M * T * (w_el + 2 * n_norms * d) * 2
        assert w_lit <= lit["w_stash_bytes"] <= w_lit * 1.001 + 4096 * L
    # fewer activation slots shrink only the forward->p1 part
    s = si.CONFIGS["llama7b_s1024"]
    assert _sizes(s, act_slots=1)["a_stash_bytes"] * 4 == _sizes(s)["a_stash_bytes"]
    assert _sizes(s, act_slots=1)["w_stash_bytes"] == _sizes(s)["w_stash_bytes"]
    # 13B stage: everything fits the 288 GB of one MI355X
    assert _sizes(si.CONFIGS["llama13b_s2048"])["arena_bytes"] < 150 * 2**30


@pytest.mark.parametrize("field,value", [("d_model", 4100), ("d_ffn", 11004), ("seq", 4104), ("head_dim", 120),
                                         ("n_layers", 0), ("dtype", 7), ("d_model", 16384), ("seq", 8192), ("attention", 4),
                                         ("gain_grad", 2)])
def test_bad_configs_are_rejected(field, value):
    cfg = tbp.config_from_shape(si.CONFIGS["llama7b_s1024"])
    setattr(cfg, field, value)
    with pytest.raises(tbp.TbpError) as e:
        tbp.tbp_stash_query(cfg)
    assert e.value.status == 1 and str(e.value)


def test_fused_attention_is_refused_where_it_is_not_built():
    cfg = tbp.config_from_shape(si.CONFIGS["tiny_f32"], attention=tbp.TBP_ATTN_FUSED)       # fp32 storage
    with pytest.raises(tbp.TbpError) as e:
        tbp.tbp_stash_query(cfg)
    assert e.value.status == 1
    cfg = tbp.config_from_shape(si.CONFIGS["llama7b_s1024"], attention=tbp.TBP_ATTN_FUSED)
    cfg.n_heads, cfg.head_dim = 128, 32                                                       # head_dim 32
    with pytest.raises(tbp.TbpError):
        tbp.tbp_stash_query(cfg)
    tbp.tbp_stash_query(tbp.config_from_shape(si.CONFIGS["tiny_f32"]))                       # AUTO falls back


class _FakeStage:
    """A stage over made-up device addresses: valid for every host-side check, never used to launch."""

    def __init__(self, shape, arena_bytes=None, **kw):
        L = tbp.lib()
        self.cfg = tbp.config_from_shape(shape, **kw)
        n = shape.n_layers
        arr = (C.c_void_p * n)(*[0x10000 * (i + 1) for i in range(n)])
        self._keep = arr
        from paper_2405_18047_amd.binding import _tbp_params
        p = _tbp_params()
        for name, _ in p._fields_:
            setattr(p, name, C.cast(arr, C.POINTER(C.c_void_p)))
        need = tbp.tbp_stash_query(self.cfg)["arena_bytes"]
        self.h = C.c_void_p()
        self.status = L.tbp_stage_create(C.byref(self.cfg), C.byref(p), C.c_void_p(0x1000000),
                                         need if arena_bytes is None else arena_bytes, C.byref(self.h))


def test_state_machine_rejects_wrong_order_without_launching():
    L = tbp.lib()
    st = _FakeStage(si.CONFIGS["tiny_f32"])
    assert st.status == 0
    fake = C.c_void_p(0x2000000)
    # p1 before forward, p2 before p1, out-of-range micro-batch, duplicate and non-consecutive sets
    assert L.tbp_stage_backward_p1(st.h, 0, fake, fake, None) == 2
    assert b"forward" in L.tbp_last_error()
    one = (C.c_int * 2)(0, 1)
    assert L.tbp_stage_backward_p2(st.h, one, 1, 0, 1, None) == 2
    assert L.tbp_stage_forward(st.h, 4, fake, fake, None) == 1
    assert L.tbp_stage_forward(st.h, -1, fake, fake, None) == 1
    assert L.tbp_stage_forward(st.h, 0, None, fake, None) == 1
    dup = (C.c_int * 2)(1, 1)
    assert L.tbp_stage_backward_p2(st.h, dup, 2, 0, 1, None) == 1
    assert L.tbp_stage_backward_p2(st.h, one, 0, 0, 1, None) == 1
    assert L.tbp_stage_backward_p2(st.h, one, 2, 5, 1, None) == 1
    from paper_2405_18047_amd.binding import _tbp_stash_stats
    stats = _tbp_stash_stats()
    assert L.tbp_stage_stash_stats(st.h, C.byref(stats)) == 0
    assert (stats.w_live_bytes, stats.a_live_bytes, stats.high_water_bytes) == (0, 0, 0)
    assert L.tbp_stage_reset(st.h) == 0
    L.tbp_stage_destroy(st.h)


def test_create_rejects_small_arena_and_null_pointers():
    L = tbp.lib()
    st = _FakeStage(si.CONFIGS["tiny_f32"], arena_bytes=1024)
    assert st.status == 3 and b"arena" in L.tbp_last_error()
    cfg = tbp.config_from_shape(si.CONFIGS["tiny_f32"])
    h = C.c_void_p()
    assert L.tbp_stage_create(C.byref(cfg), None, C.c_void_p(0x1000), 1 << 40, C.byref(h)) == 1


def test_single_op_argument_checks():
    L = tbp.lib()
    fake = C.c_void_p(0x2000000)
    # bf16 extents must be multiples of 8; accumulate needs fp32 output; unknown layout
    assert L.tbp_gemm(1, 2, 100, 64, 64, 1.0, fake, 100, fake, 64, fake, 64, 1, 0, None, None) == 1
    assert L.tbp_gemm(1, 1, 64, 64, 64, 1.0, fake, 64, fake, 64, fake, 64, 0, 1, None, None) == 1
    assert L.tbp_gemm(1, 3, 64, 64, 64, 1.0, fake, 64, fake, 64, fake, 64, 0, 0, None, None) == 1
    assert L.tbp_gemm(1, 0, 0, 64, 64, 1.0, None, 64, None, 64, None, 64, 0, 0, None, None) == 0   # empty: no-op
    assert L.tbp_rmsnorm_fwd(1, 4, 12, 1e-6, fake, fake, fake, None) == 1
    assert L.tbp_softmax_fwd(1, 1, 8192, 1, fake, fake, None) == 1
    assert L.tbp_rope(1, 4, 8, 2, 24, 48, fake, 0, fake, None) == 1
    assert L.tbp_rmsnorm_p1_scratch_bytes(4096) == 256 * 4096 * 4
    # partial rows of the gain gradient: one per workgroup of the row kernel, never more than 256, none without rows
    assert L.tbp_rmsnorm_partial_rows(1, 4096, 4096) == 256 and L.tbp_rmsnorm_partial_rows(1, 0, 4096) == 0
    assert 1 <= L.tbp_rmsnorm_partial_rows(1, 5, 264) <= 5 and 1 <= L.tbp_rmsnorm_partial_rows(0, 37, 256) <= 37
    assert L.tbp_rmsnorm_p1_partials(1, 4, 12, 1e-6, fake, fake, fake, None, fake, fake, None) == 1
    assert L.tbp_gain_partials_sum(None, 3, 64, 0, fake, None) == 1
    # the variant with the library's static scratch refuses widths its array was not built for, before any device call
    assert L.tbp_rmsnorm_p1_static(1, 4, 8200, 1e-6, fake, fake, fake, None, fake, fake, None) == 1
    assert b"static scratch" in L.tbp_last_error()
    assert L.tbp_rmsnorm_p1_static(0, 4, 4100, 1e-6, fake, fake, fake, None, fake, fake, None) == 1
    assert L.tbp_rmsnorm_p1_static(1, 4, 4096, 1e-6, fake, fake, fake, None, None, fake, None) == 1      # null dx
    # leading dimensions beyond what the kernels' buffer ranges address are refused, not wrapped
    assert L.tbp_gemm(1, 0, 64, 64, 64, 1.0, fake, 1 << 22, fake, 64, fake, 64, 0, 0, None, None) == 1
    assert L.tbp_attention_fwd(1, 1, 2, 4096, 64, 1, fake, 1 << 19, fake, 128, fake, None) == 1
    # dS^T scratch of the fused attention backward: row sums + panels of 128 queries (seq rounded up to 128 on one side)
    assert L.tbp_attention_p1_scratch_bytes(2, 3, 200) == 4864 + 2 * 3 * 2 * 200 * 128 * 2


def test_gemm_workspace_policy_and_checks():
    """tbp_gemm_workspace_bytes is host arithmetic: scratch is asked for only where splitting the contraction pays
    (a bf16 NN / NT product with a storage-type output that neither tile shape can spread over the chip, and a long
    contraction), and it is exactly the arrival counters plus one fp32 tile per slice."""
    L = tbp.lib()
    need = L.tbp_gemm_workspace_bytes(1, tbp.NT, 1024, 4096, 32768, 0)
    assert need == 1024 + 64 * 4 * 256 * 256 * 4                          # 64 tiles, four slices
    assert L.tbp_gemm_workspace_bytes(1, tbp.NN, 1024, 4096, 32768, 0) == need
    for args in [(1, tbp.TN, 1024, 4096, 32768, 0),      # weight-gradient layout: never split
                 (1, tbp.NT, 1024, 4096, 32768, 1),      # fp32 output
                 (0, tbp.NT, 1024, 4096, 32768, 0),      # fp32 storage
                 (1, tbp.NT, 4096, 4096, 32768, 0),      # 256 large tiles already fill the chip
                 (1, tbp.NT, 2048, 5120, 27648, 0),      # 216 tiles of 256 x 192 do
                 (1, tbp.NT, 1024, 4096, 4096, 0),       # short contraction: the exchange would cost more than it saves
                 (1, tbp.NT, 0, 4096, 32768, 0), (1, 7, 1024, 4096, 32768, 0)]:
        assert L.tbp_gemm_workspace_bytes(*args) == 0, args
    fake = C.c_void_p(0x2000000)
    # a misaligned workspace is refused before anything is launched
    assert L.tbp_gemm_ws(1, tbp.NT, 1024, 4096, 32768, 1.0, fake, 32768, fake, 32768, fake, 4096, 0, 0, None,
                         C.c_void_p(0x3000010), need, None) == 1
    assert "aligned" in L.tbp_last_error().decode()
