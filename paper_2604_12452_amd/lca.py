"""Thin ctypes binding of liblca (see include/lca.h): argument marshalling only.

Every step of the path runs inside the library's HIP kernels.  Tensors are torch tensors on the GPU
(torch is used for device memory and streams only); bf16 data may be passed as ``torch.bfloat16`` or
as int16/uint16 bit patterns.  There is no CPU fallback: if ``liblca.so`` has not been built the
first call raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("LCA_LIB_PATH", os.path.join(_PKG, "liblca.so"))   # override: another build of the same library

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP = range(5)
MODE_MLA, MODE_GQA = 0, 1
BF16, F32, F16 = 0, 1, 2
REDUCE_DEFAULT, REDUCE_WEIGHTED, REDUCE_MEAN, REDUCE_MAXSEL, REDUCE_MAXPOOL = range(5)

EXPORTS = ("lca_workspace_size", "lca_cache_bytes", "lca_condense", "lca_prefill_attn", "dense_mla_attn",
           "lca_decode_attn", "lca_decode_attn_cached", "lca_cache_update", "lca_deviation_stats", "lca_quantize_cache",
           "lca_decode_attn_q8", "lca_prefill_attn_up", "lca_last_error")


class LcaError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"liblca status {status}: {message}")
        self.status = status


class _CDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("B", "L", "H", "S", "d_pool", "d_sel", "g", "w", "n_q", "mode", "dtype")] + [
        ("scale", ctypes.c_float), ("rep_logit_bias", ctypes.c_float), ("pool_reduce", ctypes.c_int32), ("sel_reduce", ctypes.c_int32)]


class _CLayout(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("m_cap", "k_cap", "k_start")]


@dataclass
class CacheLayout:
    """Mirror of ``lca_cache_layout``: rows allocated for representatives / raw tail, ring row of the oldest tail token."""
    m_cap: int
    k_cap: int
    k_start: int = 0

    def c(self) -> _CLayout:
        return _CLayout(self.m_cap, self.k_cap, self.k_start)


@dataclass
class Desc:
    """Mirror of ``lca_desc``; names follow the paper (L tokens, group size g, window w)."""
    B: int
    L: int
    H: int
    S: int
    d_pool: int
    d_sel: int
    g: int
    w: int
    n_q: int = 0
    mode: int = MODE_MLA
    dtype: int = BF16
    scale: float = 1.0
    rep_logit_bias: float = 0.0
    pool_reduce: int = 0      # REDUCE_*: 0 = the method's own (weighted pooling / max selection)
    sel_reduce: int = 0

    @property
    def d_qk(self) -> int:
        return self.d_pool + self.d_sel if self.mode == MODE_MLA else self.d_sel

    @property
    def m(self) -> int:
        return (self.L - self.w) // self.g if self.L > self.w else 0

    @property
    def k(self) -> int:
        return self.L - self.m * self.g

    @property
    def kv_heads(self) -> int:
        return 1 if self.mode == MODE_MLA else self.S

    def c(self) -> _CDesc:
        return _CDesc(self.B, self.L, self.H, self.S, self.d_pool, self.d_sel, self.g, self.w, self.n_q, self.mode,
                      self.dtype, float(self.scale), float(self.rep_logit_bias), self.pool_reduce, self.sel_reduce)


_lib = None


def load() -> ctypes.CDLL:
    """Load liblca.so; raises if it has not been built (``python -m paper_2604_12452_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: build it with `python -m paper_2604_12452_amd.build`; "
                                    "there is no fallback path")
        lib = ctypes.CDLL(LIB_PATH)
        for name in EXPORTS:
            getattr(lib, name).restype = ctypes.c_int
        lib.lca_last_error.restype = ctypes.c_char_p
        _lib = lib
    return _lib


def _ptr(t):
    """Device address of a tensor (or None / int passthrough)."""
    if t is None:
        return ctypes.c_void_p(0)
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    if not t.is_contiguous():
        raise ValueError("liblca needs contiguous tensors")
    return ctypes.c_void_p(t.data_ptr())


def _nbytes(t) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def _stream(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def _check(status: int):
    if status != OK:
        raise LcaError(status, load().lca_last_error().decode())


def workspace_size(desc: Desc) -> int:
    n = ctypes.c_size_t(0)
    cd = desc.c()
    _check(load().lca_workspace_size(ctypes.byref(cd), ctypes.byref(n)))
    return int(n.value)


def cache_bytes(desc: Desc):
    a, b = ctypes.c_size_t(0), ctypes.c_size_t(0)
    cd = desc.c()
    _check(load().lca_cache_bytes(ctypes.byref(cd), ctypes.byref(a), ctypes.byref(b)))
    return int(a.value), int(b.value)


def condense(desc: Desc, Q, POOL, SEL, pool_rep, sel_rep, anchor_idx, alpha_dbg, workspace, stream=None):
    cd = desc.c()
    _check(load().lca_condense(ctypes.byref(cd), _ptr(Q), _ptr(POOL), _ptr(SEL), _ptr(pool_rep), _ptr(sel_rep),
                               _ptr(anchor_idx), _ptr(alpha_dbg), _ptr(workspace), ctypes.c_size_t(_nbytes(workspace)),
                               _stream(stream)))


def prefill_attn(desc: Desc, Q, POOL, SEL, pool_rep, sel_rep, O, lse, workspace, stream=None):
    cd = desc.c()
    _check(load().lca_prefill_attn(ctypes.byref(cd), _ptr(Q), _ptr(POOL), _ptr(SEL), _ptr(pool_rep), _ptr(sel_rep),
                                   _ptr(O), _ptr(lse), _ptr(workspace), ctypes.c_size_t(_nbytes(workspace)),
                                   _stream(stream)))


def prefill_attn_up(desc: Desc, Q, POOL, SEL, pool_rep, sel_rep, W_up, O_up, lse, workspace, stream=None):
    cd = desc.c()
    _check(load().lca_prefill_attn_up(ctypes.byref(cd), _ptr(Q), _ptr(POOL), _ptr(SEL), _ptr(pool_rep), _ptr(sel_rep), _ptr(W_up),
                                      _ptr(O_up), _ptr(lse), _ptr(workspace), ctypes.c_size_t(_nbytes(workspace)), _stream(stream)))


def dense_attn(desc: Desc, Q, POOL, SEL, O, lse, workspace, stream=None):
    cd = desc.c()
    _check(load().dense_mla_attn(ctypes.byref(cd), _ptr(Q), _ptr(POOL), _ptr(SEL), _ptr(O), _ptr(lse), _ptr(workspace),
                                 ctypes.c_size_t(_nbytes(workspace)), _stream(stream)))


def decode_attn(desc: Desc, q, pool_rep, sel_rep, pool_tail, sel_tail, O, workspace, stream=None):
    cd = desc.c()
    _check(load().lca_decode_attn(ctypes.byref(cd), _ptr(q), _ptr(pool_rep), _ptr(sel_rep), _ptr(pool_tail),
                                  _ptr(sel_tail), _ptr(O), _ptr(workspace), ctypes.c_size_t(_nbytes(workspace)),
                                  _stream(stream)))


def decode_attn_cached(desc: Desc, layout: CacheLayout, q, pool_rep, sel_rep, pool_tail, sel_tail, O, workspace, stream=None):
    cd, cl = desc.c(), layout.c()
    _check(load().lca_decode_attn_cached(ctypes.byref(cd), ctypes.byref(cl), _ptr(q), _ptr(pool_rep), _ptr(sel_rep), _ptr(pool_tail),
                                         _ptr(sel_tail), _ptr(O), _ptr(workspace), ctypes.c_size_t(_nbytes(workspace)), _stream(stream)))


def cache_update(desc: Desc, layout: CacheLayout, q_recent, pool_tail, sel_tail, pool_rep, sel_rep, anchor_idx, workspace, stream=None):
    cd, cl = desc.c(), layout.c()
    _check(load().lca_cache_update(ctypes.byref(cd), ctypes.byref(cl), _ptr(q_recent), _ptr(pool_tail), _ptr(sel_tail), _ptr(pool_rep),
                                   _ptr(sel_rep), _ptr(anchor_idx), _ptr(workspace), ctypes.c_size_t(_nbytes(workspace)), _stream(stream)))


def quantize_cache(desc: Desc, layout, pool_rep, sel_rep, pool_q8, sel_q8, scales, first_row=0, stream=None):
    cd = desc.c()
    cl = layout.c() if layout is not None else None
    _check(load().lca_quantize_cache(ctypes.byref(cd), ctypes.byref(cl) if cl is not None else None, ctypes.c_int32(first_row), _ptr(pool_rep), _ptr(sel_rep),
                                     _ptr(pool_q8), _ptr(sel_q8), _ptr(scales), _stream(stream)))


def decode_attn_q8(desc: Desc, layout, q, pool_q8, sel_q8, scales, pool_tail, sel_tail, O, workspace, stream=None):
    cd = desc.c()
    cl = layout.c() if layout is not None else None
    _check(load().lca_decode_attn_q8(ctypes.byref(cd), ctypes.byref(cl) if cl is not None else None, _ptr(q), _ptr(pool_q8), _ptr(sel_q8),
                                     _ptr(scales), _ptr(pool_tail), _ptr(sel_tail), _ptr(O), _ptr(workspace),
                                     ctypes.c_size_t(_nbytes(workspace)), _stream(stream)))


def deviation_stats(desc: Desc, POOL, SEL, pool_rep, sel_rep, stats, workspace, stream=None):
    cd = desc.c()
    _check(load().lca_deviation_stats(ctypes.byref(cd), _ptr(POOL), _ptr(SEL), _ptr(pool_rep), _ptr(sel_rep), _ptr(stats), _ptr(workspace),
                                      ctypes.c_size_t(_nbytes(workspace)), _stream(stream)))


# ---------------------------------------------------------------------------------------------
# device-buffer helpers (torch used for memory only)
# ---------------------------------------------------------------------------------------------
def torch_dtype(desc: Desc):
    import torch
    return {BF16: torch.bfloat16, F32: torch.float32, F16: torch.float16}[desc.dtype]


def alloc_workspace(desc: Desc, device="cuda"):
    import torch
    return torch.empty(max(workspace_size(desc), 256), dtype=torch.uint8, device=device)


def alloc_condensed(desc: Desc, device="cuda", alpha: bool = False):
    """Buffers lca_condense writes: (pool_rep, sel_rep, anchor_idx, alpha_dbg or None)."""
    import torch
    dt = torch_dtype(desc)
    m = desc.m
    pool_rep = torch.empty((desc.B, desc.S, m, desc.d_pool), dtype=dt, device=device)
    sel_rep = torch.empty((desc.B, desc.S, m, desc.d_sel), dtype=dt, device=device)
    anchor = torch.empty((desc.B, desc.S, m), dtype=torch.int32, device=device)
    a = torch.empty((desc.B, desc.S, m * desc.g), dtype=torch.float32, device=device) if alpha else None
    return pool_rep, sel_rep, anchor, a
