"""ctypes binding of libtbp.so: argument marshalling only, every computation runs in the HIP kernels.

Function names mirror the C ABI (include/tbp.h).  Tensors are torch tensors on the GPU (torch supplies
device memory and the current stream, nothing else).  A missing library is an error, never a fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

__all__ = [
    "TBP_F32", "TBP_BF16", "TBP_P2_LOOP", "TBP_P2_KCONCAT", "TBP_ATTN_AUTO", "TBP_ATTN_MATERIALISED", "TBP_ATTN_FUSED", "TBP_ATTN_FUSED_RECOMPUTE", "TBP_GAIN_PARTIALS", "TBP_GAIN_LITERAL", "NN", "NT", "TN", "TbpError", "lib", "library_path",
    "tbp_config", "tbp_stash_query", "Stage", "tbp_gemm", "tbp_rmsnorm_fwd", "tbp_rmsnorm_p1", "tbp_rmsnorm_p1_partials", "tbp_gain_partials_sum", "tbp_rmsnorm_p1_static", "tbp_rmsnorm_gain_p2", "tbp_swiglu_fwd",
    "tbp_swiglu_p1", "tbp_rope_table", "tbp_rope", "tbp_softmax_fwd", "tbp_softmax_p1", "tbp_version",
    "tbp_attention_fwd", "tbp_attention_p1",
    "config_from_shape",
]

TBP_F32, TBP_BF16 = 0, 1
TBP_P2_LOOP, TBP_P2_KCONCAT = 0, 1
TBP_ATTN_AUTO, TBP_ATTN_MATERIALISED, TBP_ATTN_FUSED, TBP_ATTN_FUSED_RECOMPUTE = 0, 1, 2, 3
TBP_GAIN_PARTIALS, TBP_GAIN_LITERAL = 0, 1
NN, NT, TN = 0, 1, 2
_STATUS = {0: "TBP_OK", 1: "TBP_EINVAL", 2: "TBP_ESTATE", 3: "TBP_ENOMEM", 4: "TBP_EDEVICE"}


class TbpError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS.get(status, status)}: {message}")
        self.status = status


class tbp_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "head_dim", "d_ffn", "seq", "micro_batch",
                                        "max_microbatches", "act_slots", "causal", "dtype")] + \
               [("rms_eps", C.c_float), ("rope_base", C.c_float), ("attention", C.c_int32), ("gain_grad", C.c_int32)]


class _tbp_params(C.Structure):
    _fields_ = [(n, C.POINTER(C.c_void_p)) for n in ("w_qkv", "w_o", "g1", "w_gu", "w_d", "g2",
                                                    "dw_qkv", "dw_o", "dg1", "dw_gu", "dw_d", "dg2")]


class _tbp_stash_sizes(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("w_stash_bytes", "a_stash_bytes", "workspace_bytes", "arena_bytes")]


class _tbp_stash_stats(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("w_live_bytes", "a_live_bytes", "high_water_bytes")]


def library_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libtbp.so")


_lib = None


def lib() -> C.CDLL:
    """The loaded HIP library.  Raises if it has not been built (python -m paper_2405_18047_amd.build)."""
    global _lib
    if _lib is None:
        path = library_path()
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: build it with `python -m paper_2405_18047_amd.build`; "
                               "there is no fallback path")
        L = C.CDLL(path)
        L.tbp_last_error.restype = C.c_char_p
        L.tbp_version.restype = C.c_char_p
        L.tbp_rmsnorm_p1_scratch_bytes.restype = C.c_size_t
        L.tbp_rope_table_bytes.restype = C.c_size_t
        L.tbp_stage_destroy.restype = None
        L.tbp_gemm.argtypes = [C.c_int] * 5 + [C.c_float, C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p,
                                                C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        L.tbp_gemm_ws.argtypes = [C.c_int] * 5 + [C.c_float, C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p,
                                                   C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.tbp_gemm_workspace_bytes.argtypes = [C.c_int] * 6
        L.tbp_gemm_workspace_bytes.restype = C.c_size_t
        L.tbp_rmsnorm_fwd.argtypes = [C.c_int, C.c_int, C.c_int, C.c_float] + [C.c_void_p] * 4
        L.tbp_rmsnorm_p1.argtypes = [C.c_int, C.c_int, C.c_int, C.c_float] + [C.c_void_p] * 8
        L.tbp_rmsnorm_partial_rows.argtypes = [C.c_int] * 3
        L.tbp_rmsnorm_p1_partials.argtypes = [C.c_int, C.c_int, C.c_int, C.c_float] + [C.c_void_p] * 7
        L.tbp_gain_partials_sum.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        L.tbp_rmsnorm_p1_static.argtypes = [C.c_int, C.c_int, C.c_int, C.c_float] + [C.c_void_p] * 7
        L.tbp_swiglu_fwd.argtypes = [C.c_int, C.c_int, C.c_int] + [C.c_void_p] * 3
        L.tbp_swiglu_p1.argtypes = [C.c_int, C.c_int, C.c_int] + [C.c_void_p] * 4
        L.tbp_rope_table.argtypes = [C.c_int, C.c_int, C.c_float, C.c_void_p, C.c_void_p]
        L.tbp_rope.argtypes = [C.c_int] * 6 + [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        L.tbp_softmax_fwd.argtypes = [C.c_int] * 4 + [C.c_void_p] * 3
        L.tbp_softmax_p1.argtypes = [C.c_int] * 4 + [C.c_void_p] * 3
        L.tbp_stash_query.argtypes = [C.POINTER(tbp_config), C.POINTER(_tbp_stash_sizes)]
        L.tbp_stage_create.argtypes = [C.POINTER(tbp_config), C.POINTER(_tbp_params), C.c_void_p, C.c_size_t,
                                       C.POINTER(C.c_void_p)]
        L.tbp_stage_destroy.argtypes = [C.c_void_p]
        L.tbp_stage_forward.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
        L.tbp_stage_backward_p1.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
        L.tbp_stage_backward_p2.argtypes = [C.c_void_p, C.POINTER(C.c_int), C.c_int, C.c_int, C.c_int, C.c_void_p]
        L.tbp_stage_stash_stats.argtypes = [C.c_void_p, C.POINTER(_tbp_stash_stats)]
        L.tbp_stage_reset.argtypes = [C.c_void_p]
        L.tbp_mfma_ceiling.argtypes = [C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
        L.tbp_attention_p1_scratch_bytes.argtypes = [C.c_int] * 3
        L.tbp_attention_p1_scratch_bytes.restype = C.c_size_t
        L.tbp_attention_p1.argtypes = [C.c_int] * 6 + [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        L.tbp_attention_p1_recompute.argtypes = L.tbp_attention_p1.argtypes
        L.tbp_attention_p1_recompute_scratch_bytes.argtypes = [C.c_int] * 3
        L.tbp_attention_p1_recompute_scratch_bytes.restype = C.c_size_t
        L.tbp_attention_fwd.argtypes = [C.c_int] * 6 + [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        L.tbp_rmsnorm_p1_scratch_bytes.argtypes = [C.c_int]
        L.tbp_rmsnorm_gain_p2.argtypes = [C.c_int, C.c_int, C.c_int, C.c_float, C.c_void_p, C.c_void_p, C.c_int] + [C.c_void_p] * 3
        L.tbp_rope_table_bytes.argtypes = [C.c_int, C.c_int]
        _lib = L
    return _lib


def _check(status: int):
    if status != 0:
        raise TbpError(status, lib().tbp_last_error().decode())


def tbp_version() -> str:
    return lib().tbp_version().decode()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return TBP_BF16
    if t.dtype == torch.float32:
        return TBP_F32
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _ptr(t):
    return None if (t is None or t.numel() == 0) else C.c_void_p(t.data_ptr())


def config_from_shape(shape, act_slots: int = 0, max_microbatches: int | None = None,
                      attention: int = TBP_ATTN_AUTO, gain_grad: int = TBP_GAIN_PARTIALS) -> tbp_config:
    """tbp_config for a seeded_inputs.StageShape-like object (any object with the same field names)."""
    return tbp_config(n_layers=shape.n_layers, d_model=shape.d_model, n_heads=shape.n_heads, head_dim=shape.head_dim,
                      d_ffn=shape.d_ffn, seq=shape.seq, micro_batch=shape.micro_batch,
                      max_microbatches=max_microbatches or shape.n_microbatches, act_slots=act_slots,
                      causal=1 if shape.causal else 0, dtype=TBP_BF16 if shape.dtype == "bf16" else TBP_F32,
                      rms_eps=shape.rms_eps, rope_base=shape.rope_base, attention=attention, gain_grad=gain_grad)


def tbp_stash_query(cfg: tbp_config) -> dict:
    out = _tbp_stash_sizes()
    _check(lib().tbp_stash_query(C.byref(cfg), C.byref(out)))
    return {n: getattr(out, n) for n, _ in out._fields_}


class Stage:
    """Owns the device tensors a tbp_stage refers to (weights, fp32 gradients, arena) and forwards the calls."""

    KEYS = ("w_qkv", "w_o", "g1", "w_gu", "w_d", "g2")

    def __init__(self, cfg: tbp_config, params: dict, device="cuda:0"):
        self.cfg = cfg
        self.device = torch.device(device)
        self.params = params
        attn = cfg.n_heads > 0
        self.keys = self.KEYS if attn else ("w_gu", "w_d", "g2")
        self.grads = {k: [torch.zeros(t.shape, dtype=torch.float32, device=self.device) for t in params[k]]
                      for k in self.keys}
        self.sizes = tbp_stash_query(cfg)
        self.arena = torch.empty(self.sizes["arena_bytes"] + 256, dtype=torch.uint8, device=self.device)
        base = self.arena.data_ptr()
        self._arena_ptr = (base + 255) // 256 * 256
        n = cfg.n_layers
        arr = C.c_void_p * n
        self._arrays = {}
        p = _tbp_params()
        for k in self.KEYS:
            for prefix, src in (("", params), ("d", self.grads)):
                name = prefix + k if prefix == "" else ("d" + k if k.startswith("w_") else "d" + k)
                if k in self.keys:
                    a = arr(*[t.data_ptr() for t in src[k]])
                    for t in src[k]:
                        assert t.is_contiguous() and t.device == self.device
                    self._arrays[name] = a
                    setattr(p, name, C.cast(a, C.POINTER(C.c_void_p)))
                else:
                    setattr(p, name, None)
        self._p = p
        h = C.c_void_p()
        _check(lib().tbp_stage_create(C.byref(cfg), C.byref(p), C.c_void_p(self._arena_ptr),
                                      self.sizes["arena_bytes"], C.byref(h)))
        self._h = h

    @property
    def tokens(self) -> int:
        return self.cfg.seq * self.cfg.micro_batch

    def _act(self, like=None):
        dt = torch.bfloat16 if self.cfg.dtype == TBP_BF16 else torch.float32
        return torch.empty((self.tokens, self.cfg.d_model), dtype=dt, device=self.device)

    def forward(self, mb: int, x: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
        out = self._act() if out is None else out
        _check(lib().tbp_stage_forward(self._h, mb, _ptr(x), _ptr(out), _stream()))
        return out

    def backward_p1(self, mb: int, dy: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
        out = self._act() if out is None else out
        _check(lib().tbp_stage_backward_p1(self._h, mb, _ptr(dy), _ptr(out), _stream()))
        return out

    def backward_p2(self, mbs, mode: int = TBP_P2_LOOP, accumulate: bool = True):
        mbs = list(mbs)
        arr = (C.c_int * max(len(mbs), 1))(*mbs)
        _check(lib().tbp_stage_backward_p2(self._h, arr, len(mbs), mode, 1 if accumulate else 0, _stream()))

    def stats(self) -> dict:
        out = _tbp_stash_stats()
        _check(lib().tbp_stage_stash_stats(self._h, C.byref(out)))
        return {n: getattr(out, n) for n, _ in out._fields_}

    def reset(self):
        _check(lib().tbp_stage_reset(self._h))

    def zero_grads(self):
        for lst in self.grads.values():
            for g in lst:
                g.zero_()

    def close(self):
        if getattr(self, "_h", None):
            lib().tbp_stage_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ---- single operations ------------------------------------------------------------------------------
def tbp_gemm(layout: int, A: torch.Tensor, B: torch.Tensor, *, out_f32: bool = False, alpha: float = 1.0,
             C_out: torch.Tensor | None = None, accumulate: bool = False, R: torch.Tensor | None = None,
             workspace: torch.Tensor | bool | None = None) -> torch.Tensor:
    """workspace: a uint8 device tensor for tbp_gemm_ws, or True to allocate what tbp_gemm_workspace_bytes asks for."""
    dt = _dt(A)
    if layout == TN:
        K, M = A.shape
    else:
        M, K = A.shape
    N = B.shape[0] if layout == NT else B.shape[1]
    if C_out is None:
        C_out = torch.empty((M, N), dtype=torch.float32 if (out_f32 or dt == TBP_F32) else A.dtype, device=A.device)
    ld = lambda t: t.stride(0) if t.numel() > 0 else max(t.shape[-1], 8)     # empty tensors carry no usable stride
    f32 = 1 if C_out.dtype == torch.float32 else 0
    if workspace is True:
        need = lib().tbp_gemm_workspace_bytes(dt, layout, M, N, K, f32)
        workspace = torch.empty(need, dtype=torch.uint8, device=A.device) if need else None
    if workspace is None or workspace is False:
        _check(lib().tbp_gemm(dt, layout, M, N, K, alpha, _ptr(A), ld(A), _ptr(B), ld(B), _ptr(C_out), ld(C_out),
                              f32, 1 if accumulate else 0, _ptr(R), _stream()))
    else:
        _check(lib().tbp_gemm_ws(dt, layout, M, N, K, alpha, _ptr(A), ld(A), _ptr(B), ld(B), _ptr(C_out), ld(C_out),
                                 f32, 1 if accumulate else 0, _ptr(R), _ptr(workspace), workspace.numel(), _stream()))
    return C_out


def tbp_rmsnorm_fwd(x, g, eps):
    y = torch.empty_like(x)
    _check(lib().tbp_rmsnorm_fwd(_dt(x), x.shape[0], x.shape[1], eps, _ptr(x), _ptr(g), _ptr(y), _stream()))
    return y


def tbp_rmsnorm_p1(dy, x, g, eps, resid=None):
    rows, d = x.shape
    dx = torch.empty_like(x)
    dg = torch.empty(d, dtype=torch.float32, device=x.device)
    scratch = torch.empty(lib().tbp_rmsnorm_p1_scratch_bytes(d), dtype=torch.uint8, device=x.device)
    _check(lib().tbp_rmsnorm_p1(_dt(x), rows, d, eps, _ptr(dy), _ptr(x), _ptr(g), _ptr(resid), _ptr(dx), _ptr(dg),
                                _ptr(scratch), _stream()))
    return dx, dg


def tbp_rmsnorm_p1_partials(dy, x, g, eps, resid=None):
    """-> (dx, partial rows [tbp_rmsnorm_partial_rows, d] fp32 of the gain gradient)."""
    rows, d = x.shape
    dx = torch.empty_like(x)
    parts = torch.empty((lib().tbp_rmsnorm_partial_rows(_dt(x), rows, d), d), dtype=torch.float32, device=x.device)
    _check(lib().tbp_rmsnorm_p1_partials(_dt(x), rows, d, eps, _ptr(dy), _ptr(x), _ptr(g), _ptr(resid), _ptr(dx),
                                         C.c_void_p(parts.data_ptr()), _stream()))
    return dx, parts


def tbp_gain_partials_sum(parts, dg=None):
    """dg (new, or += into the given fp32 vector) = column sums of parts [n_rows, d]."""
    n_rows, d = parts.shape
    accumulate = dg is not None
    if dg is None:
        dg = torch.empty(d, dtype=torch.float32, device=parts.device)
    _check(lib().tbp_gain_partials_sum(_ptr(parts), n_rows, d, 1 if accumulate else 0, C.c_void_p(dg.data_ptr()), _stream()))
    return dg


def tbp_rmsnorm_p1_static(dy, x, g, eps, resid=None, dx=None, dg=None):
    """tbp_rmsnorm_p1 without a scratch argument (the library's own static device array).  Pass dx and dg to make the
    call itself allocation-free."""
    rows, d = x.shape
    dx = torch.empty_like(x) if dx is None else dx
    dg = torch.empty(d, dtype=torch.float32, device=x.device) if dg is None else dg
    _check(lib().tbp_rmsnorm_p1_static(_dt(x), rows, d, eps, _ptr(dy), _ptr(x), _ptr(g), _ptr(resid), _ptr(dx), _ptr(dg),
                                       _stream()))
    return dx, dg


def tbp_rmsnorm_gain_p2(dy, x, eps, dg=None):
    """dg (new, or += into the given fp32 vector) = sum over rows of dy * x * rsqrt(mean(x^2) + eps)."""
    rows, d = x.shape
    accumulate = dg is not None
    if dg is None:
        dg = torch.empty(d, dtype=torch.float32, device=x.device)
    scratch = torch.empty(lib().tbp_rmsnorm_p1_scratch_bytes(d), dtype=torch.uint8, device=x.device)
    _check(lib().tbp_rmsnorm_gain_p2(_dt(x), rows, d, eps, _ptr(dy), _ptr(x), 1 if accumulate else 0, _ptr(dg),
                                     _ptr(scratch), _stream()))
    return dg


def tbp_swiglu_fwd(gu):
    rows, f2 = gu.shape
    m = torch.empty((rows, f2 // 2), dtype=gu.dtype, device=gu.device)
    _check(lib().tbp_swiglu_fwd(_dt(gu), rows, f2 // 2, _ptr(gu), _ptr(m), _stream()))
    return m


def tbp_swiglu_p1(dm, gu):
    dgu = torch.empty_like(gu)
    _check(lib().tbp_swiglu_p1(_dt(gu), gu.shape[0], gu.shape[1] // 2, _ptr(dm), _ptr(gu), _ptr(dgu), _stream()))
    return dgu


def tbp_rope_table(seq, head_dim, base, device="cuda:0"):
    t = torch.empty(lib().tbp_rope_table_bytes(seq, head_dim), dtype=torch.uint8, device=device)
    _check(lib().tbp_rope_table(seq, head_dim, base, _ptr(t), _stream()))
    return t


def tbp_rope(x, seq, n_heads, head_dim, table, inverse=False):
    """In place on the first n_heads*head_dim columns of x [rows, ld]."""
    _check(lib().tbp_rope(_dt(x), x.shape[0], seq, n_heads, head_dim, x.stride(0), _ptr(table), 1 if inverse else 0,
                          _ptr(x), _stream()))
    return x


def tbp_softmax_fwd(scores, causal, dtype):
    n_mat, seq, _ = scores.shape
    P = torch.zeros(scores.shape, dtype=dtype, device=scores.device)
    _check(lib().tbp_softmax_fwd(TBP_BF16 if dtype == torch.bfloat16 else TBP_F32, n_mat, seq, 1 if causal else 0,
                                 _ptr(scores), _ptr(P), _stream()))
    return P


def tbp_attention_fwd(qkv, seq, n_heads, head_dim, causal=True):
    """qkv [batch*seq, 3*n_heads*head_dim] (q | k | v, rotated) -> (out [batch*seq, n_heads*head_dim], lse2 [batch, heads, seq])."""
    rows = qkv.shape[0]
    batch = rows // seq
    out = torch.empty((rows, n_heads * head_dim), dtype=qkv.dtype, device=qkv.device)
    lse = torch.empty((batch, n_heads, seq), dtype=torch.float32, device=qkv.device)
    _check(lib().tbp_attention_fwd(_dt(qkv), batch, n_heads, seq, head_dim, 1 if causal else 0, _ptr(qkv), qkv.stride(0),
                                   _ptr(out), out.stride(0), _ptr(lse), _stream()))
    return out, lse


def tbp_attention_p1(qkv, out, d_out, lse, seq, n_heads, head_dim, causal=True, recompute=False):
    """-> dqkv [batch*seq, 3*n_heads*head_dim] (dq | dk | dv, not rotated back).  recompute: tbp_attention_p1_recompute."""
    rows = qkv.shape[0]
    batch = rows // seq
    dqkv = torch.empty_like(qkv)
    L = lib()
    nbytes = (L.tbp_attention_p1_recompute_scratch_bytes if recompute else L.tbp_attention_p1_scratch_bytes)(batch, n_heads, seq)
    scratch = torch.empty(nbytes + 256, dtype=torch.uint8, device=qkv.device)
    base = (scratch.data_ptr() + 255) // 256 * 256
    _check((L.tbp_attention_p1_recompute if recompute else L.tbp_attention_p1)(_dt(qkv), batch, n_heads, seq, head_dim, 1 if causal else 0, _ptr(qkv), qkv.stride(0),
                                  _ptr(out), _ptr(d_out), out.stride(0), _ptr(lse), _ptr(dqkv), dqkv.stride(0), base,
                                  _stream()))
    return dqkv


def tbp_softmax_p1(P, dP, causal):
    """In place: dP becomes dS."""
    n_mat, seq, _ = P.shape
    _check(lib().tbp_softmax_p1(_dt(P), n_mat, seq, 1 if causal else 0, _ptr(P), _ptr(dP), _stream()))
    return dP
