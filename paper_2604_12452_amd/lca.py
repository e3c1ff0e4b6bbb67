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
LIB_PATH = os.path.join(_PKG, "liblca.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP = range(5)
MODE_MLA, MODE_GQA = 0, 1
BF16, F32, F16 = 0, 1, 2
REDUCE_DEFAULT, REDUCE_WEIGHTED, REDUCE_MEAN, REDUCE_MAXSEL, REDUCE_MAXPOOL = range(5)

EXPORTS = ("lca_workspace_size", "lca_cache_bytes", "lca_condensed_rows", "lca_condense", "lca_condense_noalloc", "lca_prefill_attn", "dense_mla_attn",
           "lca_decode_attn", "lca_decode_attn_cached", "lca_cache_update", "lca_deviation_stats", "lca_quantize_cache",
           "lca_decode_attn_q8", "lca_prefill_attn_up", "lca_probe_hbm_read", "lca_probe_mfma_bf16", "lca_last_error")
PROBE_WORDS = 256                     # LCA_PROBE_WORDS
PROBE_MFMA_FLOATS = 256 * 256 * 4     # LCA_PROBE_MFMA_FLOATS


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
        """Number of groups / representatives per set, as the library derives it (lca_condensed_rows)."""
        return condensed_rows(self)[0]

    @property
    def k(self) -> int:
        """Number of raw tail tokens, as the library derives it (lca_condensed_rows)."""
        return condensed_rows(self)[1]

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
        # PyTorch brings a HIP runtime of its own, with the system runtime's soname.  Opened after torch, this library is served
        # by torch's copy; opened before it, the library maps the system's copy and torch still maps its own afterwards: two
        # runtimes in one process, and the one that initialises second finds no device (every launch then fails with
        # "no ROCm-capable device is detected").  The tensors this binding takes are torch's, so torch goes first.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
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
    if not t.is_cuda:
        raise ValueError(f"a tensor of shape {tuple(t.shape)} is not a device tensor: liblca takes device pointers")
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


# The library receives bare pointers and cannot see how large a buffer is, so the binding compares every tensor with the
# size and element type the header documents for it before anything is launched: a kernel reading or writing past a
# buffer is a GPU memory fault, not an exception.  Only sizes and types are compared (marshalling), no values.
_ELT_NAMES = {BF16: ("torch.bfloat16", "torch.int16", "torch.uint16"), F32: ("torch.float32",), F16: ("torch.float16",)}
_KIND_NAMES = {"i32": ("torch.int32",), "f32": ("torch.float32",), "u8": ("torch.uint8",)}


def _fit(desc: Desc, t, name: str, elems: int, kind: str = "elt", optional: bool = False):
    """Raise ValueError unless tensor `t` has the element type `kind` stands for and holds at least `elems` elements."""
    if t is None:
        if optional or elems == 0:
            return
        raise ValueError(f"{name} is required")
    if isinstance(t, int):          # a raw device address: the caller vouches for it
        return
    names = _ELT_NAMES[desc.dtype] if kind == "elt" else _KIND_NAMES[kind]
    if str(t.dtype) not in names:
        raise ValueError(f"{name} has dtype {t.dtype}, expected {' / '.join(names)}")
    if t.numel() < elems:
        raise ValueError(f"{name} holds {t.numel()} elements, the descriptor needs {elems}")


def _fit_inputs(desc: Desc, Q, POOL, SEL, L=None):
    L = desc.L if L is None else L
    _fit(desc, Q, "Q", desc.B * L * desc.H * desc.d_qk)
    _fit(desc, POOL, "POOL", desc.B * L * desc.kv_heads * desc.d_pool)
    _fit(desc, SEL, "SEL", desc.B * L * desc.kv_heads * desc.d_sel)


def _fit_reps(desc: Desc, pool_rep, sel_rep, rows: int):
    _fit(desc, pool_rep, "pool_rep", desc.B * desc.S * rows * desc.d_pool)
    _fit(desc, sel_rep, "sel_rep", desc.B * desc.S * rows * desc.d_sel)


def _fit_tails(desc: Desc, pool_tail, sel_tail, rows: int):
    _fit(desc, pool_tail, "pool_tail", desc.B * desc.kv_heads * rows * desc.d_pool)
    _fit(desc, sel_tail, "sel_tail", desc.B * desc.kv_heads * rows * desc.d_sel)


def workspace_size(desc: Desc) -> int:
    n = ctypes.c_size_t(0)
    cd = desc.c()
    _check(load().lca_workspace_size(ctypes.byref(cd), ctypes.byref(n)))
    return int(n.value)


def condensed_rows(desc: Desc):
    """(m, k) of section 4.2's partition for this descriptor, from the library."""
    m, k = ctypes.c_int32(0), ctypes.c_int32(0)
    cd = desc.c()
    _check(load().lca_condensed_rows(ctypes.byref(cd), ctypes.byref(m), ctypes.byref(k)))
    return int(m.value), int(k.value)


def cache_bytes(desc: Desc):
    a, b = ctypes.c_size_t(0), ctypes.c_size_t(0)
    cd = desc.c()
    _check(load().lca_cache_bytes(ctypes.byref(cd), ctypes.byref(a), ctypes.byref(b)))
    return int(a.value), int(b.value)


def condense(desc: Desc, Q, POOL, SEL, pool_rep, sel_rep, anchor_idx, alpha_dbg, workspace, stream=None):
    cd = desc.c()
    m, _ = condensed_rows(desc)
    _fit_inputs(desc, Q, POOL, SEL)
    _fit_reps(desc, pool_rep, sel_rep, m)
    _fit(desc, anchor_idx, "anchor_idx", desc.B * desc.S * m, "i32")
    _fit(desc, alpha_dbg, "alpha_dbg", desc.B * desc.S * m * desc.g, "f32", optional=True)
    _check(load().lca_condense(ctypes.byref(cd), _ptr(Q), _ptr(POOL), _ptr(SEL), _ptr(pool_rep), _ptr(sel_rep),
                               _ptr(anchor_idx), _ptr(alpha_dbg), _ptr(workspace), ctypes.c_size_t(_nbytes(workspace)),
                               _stream(stream)))


def condense_noalloc(desc: Desc, Q, POOL, SEL, pool_rep, sel_rep, anchor_idx, alpha_dbg, stream=None):
    cd = desc.c()
    m, _ = condensed_rows(desc)
    _fit_inputs(desc, Q, POOL, SEL)
    _fit_reps(desc, pool_rep, sel_rep, m)
    _fit(desc, anchor_idx, "anchor_idx", desc.B * desc.S * m, "i32")
    _fit(desc, alpha_dbg, "alpha_dbg", desc.B * desc.S * m * desc.g, "f32", optional=True)
    _check(load().lca_condense_noalloc(ctypes.byref(cd), _ptr(Q), _ptr(POOL), _ptr(SEL), _ptr(pool_rep), _ptr(sel_rep),
                                       _ptr(anchor_idx), _ptr(alpha_dbg), _stream(stream)))


def prefill_attn(desc: Desc, Q, POOL, SEL, pool_rep, sel_rep, O, lse, workspace, stream=None):
    cd = desc.c()
    _fit_inputs(desc, Q, POOL, SEL)
    _fit_reps(desc, pool_rep, sel_rep, condensed_rows(desc)[0])
    _fit(desc, O, "O", desc.B * desc.L * desc.H * desc.d_pool)
    _fit(desc, lse, "lse", desc.B * desc.L * desc.H, "f32", optional=True)
    _check(load().lca_prefill_attn(ctypes.byref(cd), _ptr(Q), _ptr(POOL), _ptr(SEL), _ptr(pool_rep), _ptr(sel_rep),
                                   _ptr(O), _ptr(lse), _ptr(workspace), ctypes.c_size_t(_nbytes(workspace)),
                                   _stream(stream)))


def prefill_attn_up(desc: Desc, Q, POOL, SEL, pool_rep, sel_rep, W_up, O_up, lse, workspace, stream=None):
    cd = desc.c()
    _fit_inputs(desc, Q, POOL, SEL)
    _fit_reps(desc, pool_rep, sel_rep, condensed_rows(desc)[0])
    _fit(desc, W_up, "W_up", desc.H * 128 * desc.d_pool)
    _fit(desc, O_up, "O_up", desc.B * desc.L * desc.H * 128)
    _fit(desc, lse, "lse", desc.B * desc.L * desc.H, "f32", optional=True)
    _check(load().lca_prefill_attn_up(ctypes.byref(cd), _ptr(Q), _ptr(POOL), _ptr(SEL), _ptr(pool_rep), _ptr(sel_rep), _ptr(W_up),
                                      _ptr(O_up), _ptr(lse), _ptr(workspace), ctypes.c_size_t(_nbytes(workspace)), _stream(stream)))


def dense_attn(desc: Desc, Q, POOL, SEL, O, lse, workspace, stream=None):
    cd = desc.c()
    _fit_inputs(desc, Q, POOL, SEL)
    _fit(desc, O, "O", desc.B * desc.L * desc.H * desc.d_pool)
    _fit(desc, lse, "lse", desc.B * desc.L * desc.H, "f32", optional=True)
    _check(load().dense_mla_attn(ctypes.byref(cd), _ptr(Q), _ptr(POOL), _ptr(SEL), _ptr(O), _ptr(lse), _ptr(workspace),
                                 ctypes.c_size_t(_nbytes(workspace)), _stream(stream)))


def _fit_decode(desc: Desc, layout, q, pool_rep, sel_rep, pool_tail, sel_tail, O, rep_kind="elt", scales=None):
    m, k = condensed_rows(desc)
    m_cap, k_cap = (layout.m_cap, layout.k_cap) if layout is not None else (m, k)
    _fit(desc, q, "q", desc.B * desc.H * desc.d_qk)
    _fit(desc, pool_rep, "pool_rep", desc.B * desc.S * m_cap * desc.d_pool if m > 0 else 0, rep_kind)
    _fit(desc, sel_rep, "sel_rep", desc.B * desc.S * m_cap * desc.d_sel if m > 0 else 0, rep_kind)
    if rep_kind == "u8":
        _fit(desc, scales, "scales", desc.B * desc.S * m_cap * 2 if m > 0 else 0, "f32")
    _fit_tails(desc, pool_tail, sel_tail, k_cap)
    _fit(desc, O, "O", desc.B * desc.H * desc.d_pool)


def decode_attn(desc: Desc, q, pool_rep, sel_rep, pool_tail, sel_tail, O, workspace, stream=None):
    cd = desc.c()
    _fit_decode(desc, None, q, pool_rep, sel_rep, pool_tail, sel_tail, O)
    _check(load().lca_decode_attn(ctypes.byref(cd), _ptr(q), _ptr(pool_rep), _ptr(sel_rep), _ptr(pool_tail),
                                  _ptr(sel_tail), _ptr(O), _ptr(workspace), ctypes.c_size_t(_nbytes(workspace)),
                                  _stream(stream)))


def decode_attn_cached(desc: Desc, layout: CacheLayout, q, pool_rep, sel_rep, pool_tail, sel_tail, O, workspace, stream=None):
    cd, cl = desc.c(), layout.c()
    _fit_decode(desc, layout, q, pool_rep, sel_rep, pool_tail, sel_tail, O)
    _check(load().lca_decode_attn_cached(ctypes.byref(cd), ctypes.byref(cl), _ptr(q), _ptr(pool_rep), _ptr(sel_rep), _ptr(pool_tail),
                                         _ptr(sel_tail), _ptr(O), _ptr(workspace), ctypes.c_size_t(_nbytes(workspace)), _stream(stream)))


def cache_update(desc: Desc, layout: CacheLayout, q_recent, pool_tail, sel_tail, pool_rep, sel_rep, anchor_idx, workspace, stream=None):
    cd, cl = desc.c(), layout.c()
    _fit(desc, q_recent, "q_recent", desc.B * (desc.n_q or desc.g) * desc.H * desc.d_qk)
    _fit_tails(desc, pool_tail, sel_tail, layout.k_cap)
    _fit_reps(desc, pool_rep, sel_rep, layout.m_cap)
    _fit(desc, anchor_idx, "anchor_idx", desc.B * desc.S * layout.m_cap, "i32", optional=True)
    _check(load().lca_cache_update(ctypes.byref(cd), ctypes.byref(cl), _ptr(q_recent), _ptr(pool_tail), _ptr(sel_tail), _ptr(pool_rep),
                                   _ptr(sel_rep), _ptr(anchor_idx), _ptr(workspace), ctypes.c_size_t(_nbytes(workspace)), _stream(stream)))


def quantize_cache(desc: Desc, layout, pool_rep, sel_rep, pool_q8, sel_q8, scales, first_row=0, stream=None):
    cd = desc.c()
    cl = layout.c() if layout is not None else None
    m, _ = condensed_rows(desc)
    rows = layout.m_cap if layout is not None else m
    if 0 <= first_row < m:          # (otherwise the library rejects first_row or has nothing to do, and reads nothing)
        _fit_reps(desc, pool_rep, sel_rep, rows)
        _fit(desc, pool_q8, "pool_q8", desc.B * desc.S * rows * desc.d_pool, "u8")
        _fit(desc, sel_q8, "sel_q8", desc.B * desc.S * rows * desc.d_sel, "u8")
        _fit(desc, scales, "scales", desc.B * desc.S * rows * 2, "f32")
    _check(load().lca_quantize_cache(ctypes.byref(cd), ctypes.byref(cl) if cl is not None else None, ctypes.c_int32(first_row), _ptr(pool_rep), _ptr(sel_rep),
                                     _ptr(pool_q8), _ptr(sel_q8), _ptr(scales), _stream(stream)))


def decode_attn_q8(desc: Desc, layout, q, pool_q8, sel_q8, scales, pool_tail, sel_tail, O, workspace, stream=None):
    cd = desc.c()
    cl = layout.c() if layout is not None else None
    _fit_decode(desc, layout, q, pool_q8, sel_q8, pool_tail, sel_tail, O, rep_kind="u8", scales=scales)
    _check(load().lca_decode_attn_q8(ctypes.byref(cd), ctypes.byref(cl) if cl is not None else None, _ptr(q), _ptr(pool_q8), _ptr(sel_q8),
                                     _ptr(scales), _ptr(pool_tail), _ptr(sel_tail), _ptr(O), _ptr(workspace),
                                     ctypes.c_size_t(_nbytes(workspace)), _stream(stream)))


def deviation_stats(desc: Desc, POOL, SEL, pool_rep, sel_rep, stats, workspace, stream=None):
    cd = desc.c()
    _fit(desc, POOL, "POOL", desc.B * desc.L * desc.kv_heads * desc.d_pool)
    _fit(desc, SEL, "SEL", desc.B * desc.L * desc.kv_heads * desc.d_sel)
    _fit_reps(desc, pool_rep, sel_rep, condensed_rows(desc)[0])
    _fit(desc, stats, "stats", desc.B * desc.S * 6, "f32")
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


def probe_hbm_read(buf, wg_sums, stream=None):
    """Stream `buf` out of HBM once (measurement aid); `wg_sums` (PROBE_WORDS int32 / uint32) receives per-workgroup word sums."""
    if _nbytes(wg_sums) < PROBE_WORDS * 4 or wg_sums.element_size() != 4:
        raise ValueError(f"wg_sums must hold {PROBE_WORDS} 32-bit words")
    _check(load().lca_probe_hbm_read(_ptr(buf), ctypes.c_size_t(_nbytes(buf)), _ptr(wg_sums), _stream(stream)))


def probe_mfma_bf16(iters: int, out, pattern: int = 0, stream=None) -> int:
    """Back-to-back bf16 matrix-core products on every SIMD (measurement aid; pattern 0: small integers with a closed form,
    1: hashed full-mantissa operands); returns the number of wavefronts that ran."""
    if _nbytes(out) < PROBE_MFMA_FLOATS * 4 or str(out.dtype) != "torch.float32":
        raise ValueError(f"out must hold {PROBE_MFMA_FLOATS} float32")
    waves = ctypes.c_int32(0)
    _check(load().lca_probe_mfma_bf16(ctypes.c_int32(iters), ctypes.c_int32(pattern), _ptr(out), ctypes.byref(waves), _stream(stream)))
    return int(waves.value)
