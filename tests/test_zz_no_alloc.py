"""The entry point that allocates nothing (tbp_rmsnorm_p1_static) against the entry point it is a variant of
(tbp_rmsnorm_p1, which takes its scratch from the caller), through the raw C ABI: two calls in a row on the same GPU,
the second with a smaller input, so that whatever the first call left in the library's static scratch is there when
the second runs.  Same kernels, so the results are compared bit for bit, and against the oracle to the usual bar."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2405_18047_amd as tbp
import seeded_inputs as si
from gpu_util import DEV, max_rel, to_dev, to_np
from oracle import ops

pytestmark = pytest.mark.gpu


def _case(L, dtype, rows, d, seed, use_resid):
    eps = 1e-6
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    code = tbp.TBP_BF16 if dtype == "bf16" else tbp.TBP_F32
    x, dy, res = (si.store_round(si.standard_normal(seed, n, (rows, d)), dtype) for n in ("x", "dy", "res"))
    g = si.store_round(1.0 + 0.1 * si.standard_normal(seed, "g", (d,)), dtype)
    dx_, dy_, dres_, dg_ = to_dev(x, dtype), to_dev(dy, dtype), to_dev(res, dtype), to_dev(g, dtype)
    p = lambda t: C.c_void_p(t.data_ptr())
    rp = p(dres_) if use_resid else None
    # every output buffer exists before the call under test: the call itself gets no chance to allocate through torch
    out_ref = torch.full((rows, d), 7.0, dtype=tdt, device=DEV)
    out_new = torch.full((rows, d), -3.0, dtype=tdt, device=DEV)
    dg_ref = torch.full((d,), 5.0, dtype=torch.float32, device=DEV)
    dg_new = torch.full((d,), -9.0, dtype=torch.float32, device=DEV)
    ws = torch.empty(L.tbp_rmsnorm_p1_scratch_bytes(d), dtype=torch.uint8, device=DEV)
    stream = torch.cuda.current_stream().cuda_stream
    torch.cuda.synchronize()
    n_allocs = lambda: torch.cuda.memory_stats().get("allocation.all.allocated", 0)      # cumulative count: only ever grows
    before = n_allocs()
    assert L.tbp_rmsnorm_p1_static(code, rows, d, eps, p(dy_), p(dx_), p(dg_), rp, p(out_new), p(dg_new), stream) == 0, \
        L.tbp_last_error()
    assert n_allocs() == before
    assert L.tbp_rmsnorm_p1(code, rows, d, eps, p(dy_), p(dx_), p(dg_), rp, p(out_ref), p(dg_ref), p(ws), stream) == 0, \
        L.tbp_last_error()
    torch.cuda.synchronize()
    assert torch.equal(out_new, out_ref), "dx differs from the entry point with a caller's scratch"
    assert torch.equal(dg_new, dg_ref), "dg differs from the entry point with a caller's scratch"
    x64, dy64, g64 = x.astype(np.float64), dy.astype(np.float64), g.astype(np.float64)
    ref = ops.rmsnorm_p1(dy64, x64, g64, eps) + (res.astype(np.float64) if use_resid else 0.0)
    assert max_rel(to_np(out_new), ref) < (4.5e-3 if dtype == "bf16" else 2e-6)
    assert max_rel(to_np(dg_new), ops.rmsnorm_p2(dy64, x64, eps)) < 2e-5


@pytest.mark.parametrize("dtype,first,second", [("bf16", (4099, 4096), (517, 1024)), ("bf16", (300, 8192), (64, 8192)),
                                                ("f32", (1031, 1024), (3, 64))])
def test_static_scratch_entry_point_twice_in_a_row(dtype, first, second):
    L = tbp.lib()
    print(f"rmsnorm_p1_static dtype={dtype} first={first} second={second}", flush=True)
    _case(L, dtype, first[0], first[1], 71, True)
    _case(L, dtype, second[0], second[1], 72, False)        # smaller input right after, stale partial rows beyond it


def test_static_scratch_entry_point_rejects_oversize():
    L = tbp.lib()
    t = torch.zeros(16, dtype=torch.float32, device=DEV)
    p = C.c_void_p(t.data_ptr())
    assert L.tbp_rmsnorm_p1_static(tbp.TBP_BF16, 4, 8200, 1e-6, p, p, p, None, p, p, None) == 1      # TBP_EINVAL
    assert b"static scratch" in L.tbp_last_error()
    assert L.tbp_rmsnorm_p1_static(tbp.TBP_F32, 4, 4100, 1e-6, p, p, p, None, p, p, None) == 1
