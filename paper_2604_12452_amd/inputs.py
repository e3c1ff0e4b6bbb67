"""Seeded synthetic inputs for the LCA hot path (numpy only, no method arithmetic).

The paper measures on real activations of long prompts (DeepSeek-V2-Lite on LongBench-E / RULER);
neither weights nor prompts are available here, so these generators stand in for them with the
shapes of an MLA layer (d_c = 512, d_R = 64, 16 heads) or a Llama-3-8B-shaped GQA layer, and with
sequences that are locally redundant the way the method assumes (section 4.1): AR(1) latents,
optionally with topic shifts.

Everything is drawn in floating point from ``numpy.random.Generator(PCG64)``, rounded ONCE to the
storage type (bf16 or fp32) and handed out in storage form; the same arrays feed the CPU oracle
(after exact widening with :func:`to_f64`) and the GPU library.  bf16 arrays are ``uint16`` bit
patterns.  RoPE here is part of the input recipe (the method receives keys and queries with the
rotation already applied), not of the method.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace

import numpy as np
from scipy.signal import lfilter

MODE_MLA = 0
MODE_GQA = 1


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    L: int
    H: int
    S: int
    d_pool: int
    d_sel: int
    g: int
    w: int
    dtype: str            # "bf16" | "f16" | "f32"
    mode: int = MODE_MLA
    n_q: int = 0          # 0 -> g
    theta: float = 10000.0
    rho: float = 0.9
    segments: int = 0     # >0: concatenate this many equal segments with independent random means
    segment_sigma: float = 2.0
    q_var_dim: int = 0    # queries ~ N(0, 1/q_var_dim) per component; 0 -> d_qk
    seed: int = 0
    scale: float = 1.0

    @property
    def d_qk(self) -> int:
        return self.d_pool + self.d_sel if self.mode == MODE_MLA else self.d_sel

    @property
    def d_v(self) -> int:
        return self.d_pool

    @property
    def nq(self) -> int:
        return self.n_q if self.n_q > 0 else self.g

    @property
    def kv_heads(self) -> int:
        return 1 if self.mode == MODE_MLA else self.S

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


def configs() -> dict:
    """The five benchmark configurations (window 1024 = the paper's default, section 5.1; the tiny
    case uses 128 so that it has groups at L = 1024)."""
    mla = dict(H=16, S=1, d_pool=512, d_sel=64, g=16, w=1024, dtype="bf16")
    return {
        "cfg1": Workload("cfg1_tiny_f32", B=1, L=1024, H=4, S=1, d_pool=128, d_sel=32, g=16, w=128, dtype="f32",
                         q_var_dim=128, seed=1001),
        "cfg2": Workload("cfg2_mla_8k", B=1, L=8192, seed=1002, **mla),
        "cfg3": Workload("cfg3_mla_32k_topics", B=2, L=32768, segments=64, seed=1003, **mla),
        "cfg4": Workload("cfg4_mla_128k", B=1, L=131072, seed=1004, **mla),
        "cfg5": Workload("cfg5_gqa_64k", B=1, L=65536, H=32, S=8, d_pool=128, d_sel=128, g=16, w=1024, dtype="bf16",
                         mode=MODE_GQA, theta=500000.0, seed=1005),
    }


# ---------------------------------------------------------------------------------------------
# storage types
# ---------------------------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even), returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return f32_to_bf16_bits(x.astype(np.float32))
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f16":
        return np.ascontiguousarray(x, dtype=np.float16)      # one rounding to nearest even, also from float64
    raise ValueError(dtype)


def to_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of a storage-form array to float64."""
    if dtype == "bf16":
        return bf16_bits_to_f32(a).astype(np.float64)
    return np.asarray(a, dtype=np.float32).astype(np.float64)


# ---------------------------------------------------------------------------------------------
# pieces of the recipe
# ---------------------------------------------------------------------------------------------
def _rng(seed: int, stream: int, b: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([int(seed), int(stream), int(b)]))


def rope(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding on the last axis: pairs (2u, 2u+1) rotated by pos * theta^(-2u/d).
    x is [n, ..., d]; pos [n] gives the position of each index of axis 0."""
    d = x.shape[-1]
    inv = theta ** (-np.arange(0, d, 2, dtype=np.float64) / d)           # [d/2]
    ang = pos.astype(np.float64)[:, None] * inv[None, :]                  # [n, d/2]
    shape = (x.shape[0],) + (1,) * (x.ndim - 2) + (d // 2,)
    c, s = np.cos(ang).reshape(shape), np.sin(ang).reshape(shape)
    xe, xo = x[..., 0::2], x[..., 1::2]
    out = np.empty_like(x)
    out[..., 0::2] = xe * c - xo * s
    out[..., 1::2] = xe * s + xo * c
    return out


def ar1(rng: np.random.Generator, n: int, width, rho: float) -> np.ndarray:
    """Stationary AR(1) along axis 0 with unit-variance Gaussian innovations: x_t = rho x_{t-1} + e_t."""
    wshape = tuple(int(x) for x in np.atleast_1d(width))
    e = rng.standard_normal((int(np.prod(wshape)), n))        # time along the contiguous axis: fast filtering
    e[:, 0] /= np.sqrt(1.0 - rho * rho)
    x = lfilter([1.0], [1.0, -rho], e, axis=-1)
    return np.ascontiguousarray(x.T).reshape((n,) + wshape)


def gen_kv(wl: Workload, b: int):
    """(POOL, SEL) of sequence b in storage form. MLA: C^KV [L,d_c], K^R [L,d_R]; GQA: V, K [L,S,d]."""
    pos = np.arange(wl.L)
    if wl.mode == MODE_MLA:
        c = ar1(_rng(wl.seed, 1, b), wl.L, wl.d_pool, wl.rho)
        if wl.segments > 0:
            seg_len = -(-wl.L // wl.segments)
            mu = wl.segment_sigma * _rng(wl.seed, 2, b).standard_normal((wl.segments, wl.d_pool))
            c += np.repeat(mu, seg_len, axis=0)[: wl.L]
        kr = rope(_rng(wl.seed, 3, b).standard_normal((wl.L, wl.d_sel)), pos, wl.theta)
        return to_storage(c, wl.dtype), to_storage(kr, wl.dtype)
    v = ar1(_rng(wl.seed, 1, b), wl.L, (wl.S, wl.d_pool), wl.rho)
    k = rope(ar1(_rng(wl.seed, 3, b), wl.L, (wl.S, wl.d_sel), wl.rho), pos, wl.theta)
    return to_storage(v, wl.dtype), to_storage(k, wl.dtype)


def gen_kv_all(wl: Workload):
    """gen_kv of every sequence, [(POOL_b, SEL_b)]: the sequences have random streams of their own, so they are drawn side by side
    (the data does not depend on the order)."""
    with ThreadPoolExecutor(max_workers=min(16, len(os.sched_getaffinity(0)), wl.B)) as ex:
        return list(ex.map(lambda b: gen_kv(wl, b), range(wl.B)))


def gen_q_rows(wl: Workload, b: int, t0: int, t1: int) -> np.ndarray:
    """Queries of tokens [t0, t1) of sequence b, storage form, [t1-t0, H, d_qk].

    Drawn chunk-wise from a counter-style stream keyed by (seed, b, chunk) so that any row range can
    be regenerated without the rest: chunk c covers tokens [c*CH, (c+1)*CH)."""
    CH = 1024
    out = []
    std = 1.0 / np.sqrt(wl.q_var_dim or wl.d_qk)
    d_rope = wl.d_sel
    for c in range(t0 // CH, (t1 - 1) // CH + 1):
        lo, hi = c * CH, min((c + 1) * CH, wl.L)
        x = _rng(wl.seed, 1000 + c, b).standard_normal((hi - lo, wl.H, wl.d_qk), dtype=np.float32) * np.float32(std)
        x[..., wl.d_qk - d_rope:] = rope(x[..., wl.d_qk - d_rope:].astype(np.float64), np.arange(lo, hi), wl.theta)
        a, z = max(t0, lo) - lo, min(t1, hi) - lo
        out.append(to_storage(x[a:z], wl.dtype))
    return np.concatenate(out, axis=0)


def gen_all(wl: Workload):
    """Full inputs in storage form: Q [B,L,H,d_qk], POOL, SEL ([B,L,d] MLA or [B,L,S,d] GQA)."""
    CH = 1024
    jobs = [(b, t0, min(t0 + CH, wl.L)) for b in range(wl.B) for t0 in range(0, wl.L, CH)]
    with ThreadPoolExecutor(max_workers=min(16, len(os.sched_getaffinity(0)))) as ex:
        parts = list(ex.map(lambda j: gen_q_rows(wl, *j), jobs))
    per_b = len(jobs) // wl.B
    Q = np.stack([np.concatenate(parts[b * per_b:(b + 1) * per_b], axis=0) for b in range(wl.B)])
    kv = gen_kv_all(wl)
    return Q, np.stack([p for p, _ in kv]), np.stack([s for _, s in kv])


def sample_rows(wl: Workload, n: int, tile: int = 128, seed: int = 7) -> np.ndarray:
    """Query rows for sampled parity at large L: the mask's edge rows, both sides of a few query-tile
    boundaries, and seeded random rows; sorted, unique, within [0, L)."""
    w, g, L = wl.w, wl.g, wl.L
    must = [0, 1, g - 1, g, w - 1, w, w + 1, w + g - 2, w + g - 1, w + g, w + 2 * g - 1, L - g - 1, L - 2, L - 1,
            tile - 1, tile, L // 2 - 1, L // 2, L - tile - 1, L - tile]
    rows = {int(r) for r in must if 0 <= r < L}
    rng = np.random.Generator(np.random.PCG64([wl.seed, seed]))
    while len(rows) < min(n, L):
        rows.add(int(rng.integers(0, L)))
    return np.array(sorted(rows), dtype=np.int32)
