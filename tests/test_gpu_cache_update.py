"""GPU parity of the online cache update and of the decode step over a growing cache (ring tail, spare rows),
through the C ABI (lca_cache_update, lca_decode_attn_cached), against the oracle (section 4.3, "Decoding and
Online Cache Update").  The decode shapes are the ones the decode kernels are built for."""
import numpy as np
import pytest

from tests import helpers as hp
from paper_2604_12452_amd import inputs  # noqa: I001

pytestmark = pytest.mark.gpu

SHAPES = [
    (inputs.MODE_GQA, 128, 128, 8, 2, "bf16"),
    (inputs.MODE_GQA, 128, 128, 4, 4, "bf16"),
    (inputs.MODE_MLA, 512, 64, 16, 1, "bf16"),
    (inputs.MODE_MLA, 512, 64, 16, 4, "bf16"),
    (inputs.MODE_MLA, 512, 64, 8, 8, "bf16"),
    (inputs.MODE_MLA, 128, 32, 4, 1, "f32"),
    (inputs.MODE_GQA, 128, 128, 8, 2, "f16"),
    (inputs.MODE_MLA, 512, 64, 16, 1, "f16"),
]


def _storage(rng, shape, dtype, sigma=1.0):
    return inputs.to_storage(rng.standard_normal(shape) * sigma, dtype)


class Cache:
    """A decoding batch's cache on the device, in the layout lca_cache_layout describes, plus an exact float64
    mirror of the rows in use on the host (representatives as the GPU wrote them)."""

    def __init__(self, wl, m_cap, k_cap, k_start, rng):
        import torch
        from paper_2604_12452_amd import lca
        self.wl, self.lca, self.torch = wl, lca, torch
        self.m_cap, self.k_cap, self.k_start = m_cap, k_cap, k_start
        P = wl.kv_heads
        dt = lca.torch_dtype(hp.lca_desc(wl))
        nan = float("nan")
        self.pool_rep = torch.full((wl.B, wl.S, m_cap, wl.d_pool), nan, dtype=dt, device="cuda")
        self.sel_rep = torch.full((wl.B, wl.S, m_cap, wl.d_sel), nan, dtype=dt, device="cuda")
        self.anchor = torch.full((wl.B, wl.S, m_cap), -7, dtype=torch.int32, device="cuda")
        self.pool_tail = torch.full((wl.B, P, k_cap, wl.d_pool), nan, dtype=dt, device="cuda")
        self.sel_tail = torch.full((wl.B, P, k_cap, wl.d_sel), nan, dtype=dt, device="cuda")
        self.k = 0
        self.rng = rng

    def layout(self):
        return self.lca.CacheLayout(self.m_cap, self.k_cap, self.k_start)

    def push(self, n=1):
        """append n random raw tokens at the ring's end"""
        wl = self.wl
        P = wl.kv_heads
        for _ in range(n):
            assert self.k < self.k_cap
            r = (self.k_start + self.k) % self.k_cap
            self.pool_tail[:, :, r] = hp.to_dev(_storage(self.rng, (wl.B, P, wl.d_pool), wl.dtype), wl.dtype)
            self.sel_tail[:, :, r] = hp.to_dev(_storage(self.rng, (wl.B, P, wl.d_sel), wl.dtype), wl.dtype)
            self.k += 1

    def tail_rows(self, lo, hi):
        """tail tokens [lo, hi) (0 = oldest) as float64 [B,P,n,width] x 2, in order"""
        idx = [(self.k_start + i) % self.k_cap for i in range(lo, hi)]
        return hp.from_dev(self.pool_tail[:, :, idx], self.wl.dtype), hp.from_dev(self.sel_tail[:, :, idx], self.wl.dtype)


def _update_and_check(oracle, cache, L, q_recent_store, m_before):
    """lca_cache_update at length L and its comparison with the oracle fed the same ring rows and queries."""
    wl = cache.wl.with_(L=L)
    desc = hp.lca_desc(wl)
    od = hp.oracle_desc(oracle, wl)
    m = od.m
    assert m == m_before + 1
    pool_old, sel_old = cache.tail_rows(0, wl.g)
    before = [x.clone() for x in (cache.pool_rep, cache.sel_rep, cache.anchor, cache.pool_tail, cache.sel_tail)]
    ws = cache.lca.alloc_workspace(desc)
    cache.lca.cache_update(desc, cache.layout(), hp.to_dev(q_recent_store, wl.dtype), cache.pool_tail, cache.sel_tail, cache.pool_rep,
                           cache.sel_rep, cache.anchor, ws)
    cache.torch.cuda.synchronize()
    ref = oracle.cache_update(od, inputs.to_f64(q_recent_store, wl.dtype), pool_old, sel_old)
    got_pool = hp.from_dev(cache.pool_rep[:, :, m - 1], wl.dtype)
    got_sel = hp.from_dev(cache.sel_rep[:, :, m - 1], wl.dtype)
    anchor = cache.anchor[:, :, m - 1].cpu().numpy()
    differ = anchor - (m - 1) * wl.g != ref["anchor"]
    assert not (differ & (ref["margin"] > hp.ANCHOR_MARGIN)).any(), "anchor mismatch above the score margin"
    assert not (differ & (ref["margin"] == 0.0)).any(), "an exact tie did not go to the lowest index"
    assert ((anchor >= (m - 1) * wl.g) & (anchor < m * wl.g)).all()
    if differ.any():      # a near-tie may take another token only if it scores within the margin of the maximum
        a_gpu = np.take_along_axis(ref["alpha"], (anchor - (m - 1) * wl.g)[..., None].astype(np.int64), axis=-1)[..., 0]
        gap = np.log(ref["alpha"].max(axis=-1)[differ]) - np.log(a_gpu[differ])
        assert (gap <= hp.ANCHOR_MARGIN).all(), f"a GPU anchor scores {gap.max():.3e} below the maximum"
    for b in range(wl.B):
        for s in range(wl.S):                                      # the selected component is a bit-exact copy of the anchor's row
            p = 0 if wl.mode == inputs.MODE_MLA else s
            np.testing.assert_array_equal(got_sel[b, s], sel_old[b, p, anchor[b, s] - (m - 1) * wl.g])
    same = ~differ
    err = hp.vec_rel_err(got_pool[same], ref["pool_rep"][same])
    assert err <= hp.TOL[wl.dtype], f"pooled representative rel err {err:.3e}"
    # nothing else was touched: other representative rows, the anchors of other rows, the ring
    keep = [i for i in range(cache.m_cap) if i != m - 1]
    for new, old in zip((cache.pool_rep, cache.sel_rep, cache.anchor), before[:3]):
        assert cache.torch.equal(new[:, :, keep].view(cache.torch.uint8 if new.dtype != cache.torch.int32 else cache.torch.int32),
                                 old[:, :, keep].view(cache.torch.uint8 if old.dtype != cache.torch.int32 else cache.torch.int32))
    for new, old in zip((cache.pool_tail, cache.sel_tail), before[3:]):
        assert cache.torch.equal(new.view(cache.torch.uint8), old.view(cache.torch.uint8))
    # the g condensed ring rows are free now
    cache.k_start = (cache.k_start + wl.g) % cache.k_cap
    cache.k -= wl.g
    return err


def _decode_and_check(oracle, cache, L, q_store):
    """lca_decode_attn_cached at length L vs the oracle's decode step over the same cache, linearised."""
    import torch
    wl = cache.wl.with_(L=L)
    desc = hp.lca_desc(wl)
    od = hp.oracle_desc(oracle, wl)
    assert od.k == cache.k, (od.k, cache.k)
    O = torch.full((wl.B, wl.H, wl.d_pool), float("nan"), dtype=cache.lca.torch_dtype(desc), device="cuda")
    ws = cache.lca.alloc_workspace(desc)
    cache.lca.decode_attn_cached(desc, cache.layout(), hp.to_dev(q_store, wl.dtype), cache.pool_rep, cache.sel_rep, cache.pool_tail,
                                 cache.sel_tail, O, ws)
    torch.cuda.synchronize()
    pool_tail, sel_tail = cache.tail_rows(0, cache.k)
    ref = oracle.decode_attn(od, inputs.to_f64(q_store, wl.dtype), hp.from_dev(cache.pool_rep[:, :, :od.m], wl.dtype),
                             hp.from_dev(cache.sel_rep[:, :, :od.m], wl.dtype), pool_tail, sel_tail)
    err = hp.vec_rel_err(hp.from_dev(O, wl.dtype), ref)
    assert err <= hp.TOL[wl.dtype], f"decode rel err {err:.3e} at L = {L}"
    return err


@pytest.mark.parametrize("mode,d_pool,d_sel,H,S,dtype", SHAPES)
@pytest.mark.parametrize("g,w,m_before,slack,k_start", [(16, 100, 5, 0, 0), (4, 9, 0, 3, 11), (16, 64, 12, 40, 100), (8, 0, 2, 1, 7)])
def test_cache_update_matches_oracle(oracle, mode, d_pool, d_sel, H, S, dtype, g, w, m_before, slack, k_start):
    B = 3
    k_cap = w + g + slack
    k_start %= k_cap                                               # some cases wrap around the ring's end
    L = w + (m_before + 1) * g                                     # the update that makes representative m_before is due
    wl = inputs.Workload("update", B=B, L=L, H=H, S=S, d_pool=d_pool, d_sel=d_sel, g=g, w=w, dtype=dtype, mode=mode, seed=0,
                         scale=1.0 / np.sqrt(d_pool + d_sel if mode == inputs.MODE_MLA else d_sel))
    print(f"[case] {wl} k_cap={k_cap} k_start={k_start}", flush=True)
    rng = np.random.default_rng(1000 + g + w + m_before)
    cache = Cache(wl, m_cap=m_before + 1 + slack, k_cap=k_cap, k_start=k_start, rng=rng)
    cache.push(w + g)
    q_recent = _storage(rng, (B, g, H, wl.d_qk), dtype, sigma=2.0)
    err = _update_and_check(oracle, cache, L, q_recent, m_before)
    print(f"  pooled err {err:.2e}", flush=True)


@pytest.mark.parametrize("mode,d_pool,d_sel,H,S,dtype", SHAPES)
@pytest.mark.parametrize("g", [4, 16, 32])
def test_cache_update_exact_tie_takes_the_lowest_index(oracle, mode, d_pool, d_sel, H, S, dtype, g):
    """The top-scoring token among the g oldest ring rows (for set 0) is copied over another of them: two equal rows hold the
    largest score exactly, and the update must name the older one (Eq. 8, lowest index on ties); the ring wraps inside the g rows."""
    B, w = 3, 20
    k_cap = w + g + 3
    k_start = k_cap - g // 2
    L = w + 2 * g
    wl = inputs.Workload("update_tie", B=B, L=L, H=H, S=S, d_pool=d_pool, d_sel=d_sel, g=g, w=w, dtype=dtype, mode=mode, seed=0,
                         scale=1.0 / np.sqrt(d_pool + d_sel if mode == inputs.MODE_MLA else d_sel))
    print(f"[case] {wl}", flush=True)
    rng = np.random.default_rng(2000 + g)
    cache = Cache(wl, m_cap=3, k_cap=k_cap, k_start=k_start, rng=rng)
    cache.push(w + g)
    q_recent = _storage(rng, (B, g, H, wl.d_qk), dtype, sigma=2.0)
    od = hp.oracle_desc(oracle, wl)
    pool_old, sel_old = cache.tail_rows(0, g)
    first = oracle.cache_update(od, inputs.to_f64(q_recent, dtype), pool_old, sel_old)
    expect = np.zeros(B, dtype=np.int64)
    for b in range(B):
        top = int(first["anchor"][b, 0])
        other = (top + 1 + b) % g
        for T in (cache.pool_tail, cache.sel_tail):
            T[b, :, (k_start + other) % k_cap] = T[b, :, (k_start + top) % k_cap]
        expect[b] = min(top, other)
    pool_old, sel_old = cache.tail_rows(0, g)
    ref = oracle.cache_update(od, inputs.to_f64(q_recent, dtype), pool_old, sel_old)
    assert (ref["margin"][:, 0] == 0.0).all() and np.array_equal(ref["anchor"][:, 0], expect)
    _update_and_check(oracle, cache, L, q_recent, 1)
    assert np.array_equal(cache.anchor[:, 0, 1].cpu().numpy() - g, expect)


@pytest.mark.parametrize("mode,d_pool,d_sel,H,S,dtype", SHAPES)
def test_decode_loop_with_online_updates(oracle, mode, d_pool, d_sel, H, S, dtype):
    """A decoding batch from an empty cache: every step appends a token to the ring and decodes; every g-th step
    (once the window is full) condenses the g oldest tokens first.  Each update and each decode step is checked
    against the oracle on the cache the GPU holds at that moment; the ring wraps several times."""
    B, g, w = 2, 8, 21
    steps = w + 5 * g + 3
    wl = inputs.Workload("loop", B=B, L=1, H=H, S=S, d_pool=d_pool, d_sel=d_sel, g=g, w=w, dtype=dtype, mode=mode, seed=0,
                         scale=1.0 / np.sqrt(d_pool + d_sel if mode == inputs.MODE_MLA else d_sel))
    print(f"[case] {wl}", flush=True)
    rng = np.random.default_rng(77)
    cache = Cache(wl, m_cap=6, k_cap=w + g + 2, k_start=5, rng=rng)
    q_hist = []
    m = 0
    worst_u = worst_d = 0.0
    for L in range(1, steps + 1):
        cache.push()
        q_hist.append(_storage(rng, (B, H, wl.d_qk), dtype, sigma=2.0))
        if L >= w + g and (L - w) % g == 0:
            worst_u = max(worst_u, _update_and_check(oracle, cache, L, np.stack(q_hist[-g:], axis=1), m))
            m += 1
        worst_d = max(worst_d, _decode_and_check(oracle, cache, L, q_hist[-1]))
    assert m == 5
    print(f"  {steps} steps, {m} updates: worst update err {worst_u:.2e}, worst decode err {worst_d:.2e}", flush=True)


def test_cache_calls_reject_bad_arguments(oracle):
    import torch
    from paper_2604_12452_amd import lca
    wl = inputs.Workload("bad", B=1, L=64 + 16, H=8, S=2, d_pool=128, d_sel=128, g=16, w=64, dtype="bf16", mode=inputs.MODE_GQA, seed=0)
    desc = hp.lca_desc(wl)
    buf = torch.zeros(1 << 20, dtype=torch.bfloat16, device="cuda")
    idx = torch.zeros(64, dtype=torch.int32, device="cuda")
    ws = lca.alloc_workspace(desc)
    ok = lca.CacheLayout(m_cap=4, k_cap=80, k_start=0)
    lca.cache_update(desc, ok, buf, buf, buf, buf, buf, idx, ws)                       # the valid call
    for bad_desc, layout in ((hp.lca_desc(wl.with_(L=64 + 17)), ok),                   # no update due at this length
                             (hp.lca_desc(wl.with_(L=70)), ok),                        # window not yet full
                             (desc, lca.CacheLayout(0, 80, 0)),                        # no room for the representative
                             (desc, lca.CacheLayout(4, 79, 0)),                        # ring smaller than w + g
                             (desc, lca.CacheLayout(4, 80, 80))):                      # ring start outside the ring
        with pytest.raises(lca.LcaError) as e:
            lca.cache_update(bad_desc, layout, buf, buf, buf, buf, buf, idx, ws)
        assert e.value.status == lca.ERR_INVALID_ARG
    with pytest.raises(lca.LcaError):
        lca.decode_attn_cached(desc, lca.CacheLayout(0, 80, 0), buf, buf, buf, buf, buf, buf, ws)
    torch.cuda.synchronize()
