"""fp64 CPU oracle for Latent-Condensed Attention — TEST INFRASTRUCTURE ONLY.

Only the tests, ``__graft_entry__.smoke()`` and the CPU-baseline leg of ``bench.py`` may import
this package.  The GPU library never does, and nothing here imports the GPU package.

The arithmetic lives in ``lca_oracle.c`` (plain C, doubles, OpenMP over independent outputs); this
module only compiles it with gcc on first use and marshals numpy arrays into it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lca_oracle.c")
_LIB = os.path.join(_HERE, "liblca_oracle.so")

MODE_MLA = 0
MODE_GQA = 1
RED_DEFAULT, RED_WEIGHTED, RED_MEAN, RED_MAXSEL, RED_MAXPOOL = range(5)


def build(force: bool = False) -> str:
    """Compile lca_oracle.c into liblca_oracle.so (gcc, host only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".{os.getpid()}.tmp"
        subprocess.run(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"],
            check=True,
        )
        os.replace(tmp, _LIB)
    return _LIB


class _Desc(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("L", ctypes.c_int32), ("H", ctypes.c_int32), ("S", ctypes.c_int32),
        ("d_pool", ctypes.c_int32), ("d_sel", ctypes.c_int32),
        ("g", ctypes.c_int32), ("w", ctypes.c_int32), ("n_q", ctypes.c_int32),
        ("mode", ctypes.c_int32),
        ("scale", ctypes.c_double), ("rep_logit_bias", ctypes.c_double),
        ("pool_reduce", ctypes.c_int32), ("sel_reduce", ctypes.c_int32),
    ]


@dataclass
class Desc:
    """Problem description in the paper's notation (section 4.2): L tokens, group size g, window w."""
    B: int
    L: int
    H: int
    S: int
    d_pool: int
    d_sel: int
    g: int
    w: int
    n_q: int = 0  # 0 -> g (Algorithm 1 averages the last g queries)
    mode: int = MODE_MLA
    scale: float = 1.0
    rep_logit_bias: float = 0.0
    pool_reduce: int = 0   # 0 = the method (weighted pooling); 1 weighted, 2 mean, 3 max selection, 4 max pooling (Table 5)
    sel_reduce: int = 0    # 0 = the method (max selection)

    @property
    def d_qk(self) -> int:
        return self.d_pool + self.d_sel if self.mode == MODE_MLA else self.d_sel

    @property
    def d_v(self) -> int:
        return self.d_pool

    @property
    def m(self) -> int:
        return (self.L - self.w) // self.g if self.L > self.w else 0

    @property
    def k(self) -> int:
        return self.L - self.m * self.g

    @property
    def kv_heads(self) -> int:
        return 1 if self.mode == MODE_MLA else self.S

    @property
    def nq(self) -> int:
        return self.n_q if self.n_q > 0 else self.g

    def c(self) -> _Desc:
        return _Desc(self.B, self.L, self.H, self.S, self.d_pool, self.d_sel, self.g, self.w, self.nq,
                     self.mode, float(self.scale), float(self.rep_logit_bias), self.pool_reduce, self.sel_reduce)


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        for name in ("oracle_num_groups", "oracle_summary_query", "oracle_condense", "oracle_lca_attn_rows",
                     "oracle_dense_attn_rows", "oracle_decode_attn", "oracle_cache_bytes"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def _f64(a, shape=None) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float64)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"{what}: oracle rejected the arguments (code {rc})")


def _kv_shape(d: Desc, width: int):
    return (d.B, d.L, width) if d.mode == MODE_MLA else (d.B, d.L, d.S, width)


def summary_query(d: Desc, q_tail) -> np.ndarray:
    """Mean of the last n_q queries (and of the set's heads): q_tail [B,n_q,H,d_qk] -> [B,S,d_qk]."""
    q_tail = _f64(q_tail, (d.B, d.nq, d.H, d.d_qk))
    qbar = np.empty((d.B, d.S, d.d_qk), dtype=np.float64)
    cd = d.c()
    _check(_load().oracle_summary_query(ctypes.byref(cd), _p(q_tail), _p(qbar)), "summary_query")
    return qbar


def condense(d: Desc, qbar, POOL, SEL):
    """Eq. 6-8 for every group. Returns dict(pool_rep, sel_rep, anchor, alpha, margin)."""
    qbar = _f64(qbar, (d.B, d.S, d.d_qk))
    POOL = _f64(POOL, _kv_shape(d, d.d_pool))
    SEL = _f64(SEL, _kv_shape(d, d.d_sel))
    m = d.m
    out = dict(
        pool_rep=np.zeros((d.B, d.S, m, d.d_pool), dtype=np.float64),
        sel_rep=np.zeros((d.B, d.S, m, d.d_sel), dtype=np.float64),
        anchor=np.zeros((d.B, d.S, m), dtype=np.int32),
        alpha=np.zeros((d.B, d.S, m * d.g), dtype=np.float64),
        margin=np.zeros((d.B, d.S, m), dtype=np.float64),
    )
    cd = d.c()
    _check(_load().oracle_condense(ctypes.byref(cd), _p(qbar), _p(POOL), _p(SEL), _p(out["pool_rep"]),
                                   _p(out["sel_rep"]), _p(out["anchor"]), _p(out["alpha"]), _p(out["margin"])),
           "condense")
    return out


def lca_attn_rows(d: Desc, rows, q_rows, POOL, SEL, pool_rep, sel_rep, want_lse: bool = False):
    """Eq. 10 with per-row visibility for the listed query rows. q_rows [B,n_rows,H,d_qk] -> O [B,n_rows,H,d_v]."""
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    n = int(rows.shape[0])
    q_rows = _f64(q_rows, (d.B, n, d.H, d.d_qk))
    POOL = _f64(POOL, _kv_shape(d, d.d_pool))
    SEL = _f64(SEL, _kv_shape(d, d.d_sel))
    pool_rep = _f64(pool_rep, (d.B, d.S, d.m, d.d_pool))
    sel_rep = _f64(sel_rep, (d.B, d.S, d.m, d.d_sel))
    O = np.empty((d.B, n, d.H, d.d_v), dtype=np.float64)
    lse = np.empty((d.B, n, d.H), dtype=np.float64) if want_lse else None
    cd = d.c()
    _check(_load().oracle_lca_attn_rows(ctypes.byref(cd), ctypes.c_int(n), _p(rows), _p(q_rows), _p(POOL), _p(SEL),
                                        _p(pool_rep), _p(sel_rep), _p(O), _p(lse)), "lca_attn_rows")
    return (O, lse) if want_lse else O


def dense_attn_rows(d: Desc, rows, q_rows, POOL, SEL, want_lse: bool = False):
    """Eq. 5 (absorbed form for MLA), causal, for the listed query rows."""
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    n = int(rows.shape[0])
    q_rows = _f64(q_rows, (d.B, n, d.H, d.d_qk))
    POOL = _f64(POOL, _kv_shape(d, d.d_pool))
    SEL = _f64(SEL, _kv_shape(d, d.d_sel))
    O = np.empty((d.B, n, d.H, d.d_v), dtype=np.float64)
    lse = np.empty((d.B, n, d.H), dtype=np.float64) if want_lse else None
    cd = d.c()
    _check(_load().oracle_dense_attn_rows(ctypes.byref(cd), ctypes.c_int(n), _p(rows), _p(q_rows), _p(POOL), _p(SEL),
                                          _p(O), _p(lse)), "dense_attn_rows")
    return (O, lse) if want_lse else O


def decode_attn(d: Desc, q, pool_rep, sel_rep, pool_tail, sel_tail) -> np.ndarray:
    """One decode step over the condensed cache; d.L counts the newest token (last row of the tail)."""
    P = d.kv_heads
    q = _f64(q, (d.B, d.H, d.d_qk))
    pool_rep = _f64(pool_rep, (d.B, d.S, d.m, d.d_pool))
    sel_rep = _f64(sel_rep, (d.B, d.S, d.m, d.d_sel))
    pool_tail = _f64(pool_tail, (d.B, P, d.k, d.d_pool))
    sel_tail = _f64(sel_tail, (d.B, P, d.k, d.d_sel))
    O = np.empty((d.B, d.H, d.d_v), dtype=np.float64)
    cd = d.c()
    _check(_load().oracle_decode_attn(ctypes.byref(cd), _p(q), _p(pool_rep), _p(sel_rep), _p(pool_tail),
                                      _p(sel_tail), _p(O)), "decode_attn")
    return O


def cache_update(d: Desc, q_recent, pool_old, sel_old):
    """Online cache update during decoding (section 4.3, "Decoding and Online Cache Update"): the g oldest raw
    tokens of the tail become one representative, scored with the mean of the last n_q queries (Eq. 6) and
    reduced by Eq. 7 and Eq. 8 — i.e. the condensation of a one-group problem.

    q_recent [B,n_q,H,d_qk] (oldest first); pool_old [B,P,g,d_pool], sel_old [B,P,g,d_sel] as the tail stores
    them (P = 1 for MLA, S for GQA).  Returns dict(pool_rep [B,S,d_pool], sel_rep [B,S,d_sel],
    anchor [B,S] (0..g-1 inside the g tokens), alpha [B,S,g], margin [B,S])."""
    P = d.kv_heads
    q_recent = _f64(q_recent, (d.B, d.nq, d.H, d.d_qk))
    pool_old = _f64(pool_old, (d.B, P, d.g, d.d_pool))
    sel_old = _f64(sel_old, (d.B, P, d.g, d.d_sel))
    common = dict(B=d.B, H=d.H, S=d.S, d_pool=d.d_pool, d_sel=d.d_sel, g=d.g, mode=d.mode, scale=d.scale)
    qbar = summary_query(Desc(L=d.nq, w=0, n_q=d.nq, **common), q_recent)
    # the one-group problem in the prefill layout: tokens first, then KV heads
    if d.mode == MODE_MLA:
        POOL, SEL = pool_old[:, 0], sel_old[:, 0]
    else:
        POOL, SEL = pool_old.transpose(0, 2, 1, 3), sel_old.transpose(0, 2, 1, 3)
    c = condense(Desc(L=d.g, w=0, n_q=d.g, **common), qbar, np.ascontiguousarray(POOL), np.ascontiguousarray(SEL))
    return dict(pool_rep=c["pool_rep"][:, :, 0], sel_rep=c["sel_rep"][:, :, 0], anchor=c["anchor"][:, :, 0],
                alpha=c["alpha"], margin=c["margin"][:, :, 0])


def deviation_stats(d: Desc, POOL, SEL, pool_rep, sel_rep) -> np.ndarray:
    """Theorem 1's per-token deviations (appendix, Tables 9-10): [B,S,6] = mean dk, mean dk/||k||, max dk, mean dv,
    mean dv/||v||, max dv over the condensed tokens, keys and values in the space attention works in."""
    POOL = _f64(POOL, _kv_shape(d, d.d_pool))
    SEL = _f64(SEL, _kv_shape(d, d.d_sel))
    pool_rep = _f64(pool_rep, (d.B, d.S, d.m, d.d_pool))
    sel_rep = _f64(sel_rep, (d.B, d.S, d.m, d.d_sel))
    stats = np.zeros((d.B, d.S, 6), dtype=np.float64)
    cd = d.c()
    _check(_load().oracle_deviation_stats(ctypes.byref(cd), _p(POOL), _p(SEL), _p(pool_rep), _p(sel_rep), _p(stats)), "deviation_stats")
    return stats


def up_project(O, W_up) -> np.ndarray:
    """Value up-projection of a latent-space output (section 3, Eq. 5: o = (sum_i p_i c_i) W^UV_h): O [B, n, H, d_v] and
    W_up [H, d_up, d_v] (row u of head h = column u of W^UV_h) -> [B, n, H, d_up].  A plain contraction."""
    return np.einsum("bnhd,hud->bnhu", np.asarray(O, dtype=np.float64), np.asarray(W_up, dtype=np.float64))


def cache_bytes(d: Desc, elt_bytes: int):
    """(dense_bytes, condensed_bytes) of the KV cache for one attention layer."""
    a, b = ctypes.c_uint64(0), ctypes.c_uint64(0)
    cd = d.c()
    _check(_load().oracle_cache_bytes(ctypes.byref(cd), ctypes.c_int(elt_bytes), ctypes.byref(a), ctypes.byref(b)),
           "cache_bytes")
    return int(a.value), int(b.value)


def num_threads() -> int:
    """Threads the OpenMP loops will use (OMP_NUM_THREADS, else the CPUs this process may run on)."""
    env = os.environ.get("OMP_NUM_THREADS", "")
    if env.isdigit() and int(env) > 0:
        return int(env)
    return len(os.sched_getaffinity(0))


