"""GPU parity of the 8-bit representative cache: lca_quantize_cache against the oracle's format (codes and scales
bit-exact: the scale is a power of two, so the only rounding is the one to the code), and the decode step over
the quantised cache against the oracle's decode step fed the dequantised values."""
import numpy as np
import pytest

from paper_2604_12452_amd import inputs
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def _quantize_on_gpu(lca, torch, desc, layout, pool_rep, sel_rep):
    pq = torch.full(pool_rep.shape, 0x55, dtype=torch.uint8, device="cuda")
    sq = torch.full(sel_rep.shape, 0x55, dtype=torch.uint8, device="cuda")
    sc = torch.full(pool_rep.shape[:3] + (2,), float("nan"), dtype=torch.float32, device="cuda")
    lca.quantize_cache(desc, layout, pool_rep, sel_rep, pq, sq, sc)
    torch.cuda.synchronize()
    return pq, sq, sc


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("d_pool,d_sel,mode", [(512, 64, inputs.MODE_MLA), (128, 128, inputs.MODE_GQA), (24, 16, inputs.MODE_MLA)])
def test_quantize_cache_codes_and_scales_bit_exact(dtype, d_pool, d_sel, mode):
    import torch
    from oracle import q8
    from paper_2604_12452_amd import lca
    B, S, m, spare = 2, 2, 37, 3
    wl = inputs.Workload("q8", B=B, L=16 * m + 8, H=2 * S, S=S, d_pool=d_pool, d_sel=d_sel, g=16, w=8, dtype=dtype, mode=mode)
    assert hp.lca_desc(wl).m == m
    rng = np.random.default_rng(17)
    # rows of very different magnitudes, values that hit code midpoints (multiples of 2^-k), an all-zero row, a row of tiny values
    def rows(d):
        x = rng.standard_normal((B, S, m + spare, d)) * np.exp(rng.uniform(-12, 6, (B, S, m + spare, 1)))
        x[0, 0, 1] = 0.0
        x[0, 1, 2] = np.round(rng.standard_normal(d) * 16) / 16 * 7.0
        x[1, 0, 3] = rng.standard_normal(d) * 1e-30
        x[1, 1, 4, ::2] = -0.0
        return inputs.to_storage(x, dtype)
    P, Sl = rows(d_pool), rows(d_sel)
    desc = hp.lca_desc(wl)
    layout = lca.CacheLayout(m_cap=m + spare, k_cap=desc.k, k_start=0)
    pq, sq, sc = _quantize_on_gpu(lca, torch, desc, layout, hp.to_dev(P, dtype), hp.to_dev(Sl, dtype))
    for name, src, got in (("pool", P, pq), ("sel", Sl, sq)):
        ref_codes, ref_scale = q8.quantize_rows(inputs.to_f64(src, dtype)[:, :, :m])
        g = got.cpu().numpy()
        bad = g[:, :, :m] != ref_codes
        assert not bad.any(), f"{name}: {int(bad.sum())} codes differ, first at {np.argwhere(bad)[0]}"
        assert (g[:, :, m:] == 0x55).all(), f"{name}: rows past m were written"
        col = 0 if name == "pool" else 1
        assert np.array_equal(sc.cpu().numpy()[:, :, :m, col].astype(np.float64), ref_scale)
    assert torch.isnan(sc[:, :, m:]).all()


MLA, GQA = inputs.MODE_MLA, inputs.MODE_GQA


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("mode,H,S", [(MLA, 16, 1), (MLA, 16, 4), (MLA, 8, 8), (MLA, 5, 1), (GQA, 8, 2), (GQA, 14, 2), (GQA, 4, 4), (GQA, 16, 1)])
@pytest.mark.parametrize("L,g,w,ring", [(1000, 16, 100, False), (2100, 16, 64, True), (77, 4, 9, False), (50, 16, 64, False), (333, 8, 0, True)])
def test_decode_over_the_quantized_cache(oracle, dtype, mode, H, S, L, g, w, ring):
    """Condense on the GPU, quantise the representatives, decode the newest token over (codes, scales, raw tail) and
    compare with the oracle's decode step over the dequantised representatives (exact in the 16-bit type) and the
    same tail.  `ring`: spare representative rows and a tail ring that wraps."""
    import torch
    from oracle import q8
    from paper_2604_12452_amd import lca
    B = 3
    d_pool, d_sel = (512, 64) if mode == MLA else (128, 128)
    wl = inputs.Workload("decode_q8", B=B, L=L, H=H, S=S, d_pool=d_pool, d_sel=d_sel, g=g, w=w, dtype=dtype, mode=mode, seed=31 + L,
                         theta=10000.0 if mode == MLA else 500000.0)
    print(f"[case] {wl} ring={ring}", flush=True)
    Q, POOL, SEL = inputs.gen_all(wl)
    run = hp.GpuRun(wl, Q, POOL, SEL).condense(alpha=False)
    m, k, P = run.desc.m, run.desc.k, wl.kv_heads
    tdt = lca.torch_dtype(run.desc)
    m_cap, k_cap, k_start = (m + 5, k + 7, k + 3) if ring else (m, k, 0)
    layout = lca.CacheLayout(m_cap=m_cap, k_cap=k_cap, k_start=k_start) if ring else None
    pool_rep = torch.full((B, S, m_cap, d_pool), float("nan"), dtype=tdt, device="cuda")
    sel_rep = torch.full((B, S, m_cap, d_sel), float("nan"), dtype=tdt, device="cuda")
    pool_rep[:, :, :m], sel_rep[:, :, :m] = run.pool_rep, run.sel_rep
    pool_tail = torch.full((B, P, k_cap, d_pool), float("nan"), dtype=tdt, device="cuda")
    sel_tail = torch.full((B, P, k_cap, d_sel), float("nan"), dtype=tdt, device="cuda")
    idx = (k_start + torch.arange(k, device="cuda")) % k_cap
    if mode == MLA:
        raw_pool, raw_sel = run.POOL[:, None, m * g:], run.SEL[:, None, m * g:]
    else:
        raw_pool, raw_sel = run.POOL[:, m * g:].permute(0, 2, 1, 3), run.SEL[:, m * g:].permute(0, 2, 1, 3)
    pool_tail[:, :, idx], sel_tail[:, :, idx] = raw_pool, raw_sel
    pq, sq, sc = _quantize_on_gpu(lca, torch, run.desc, layout, pool_rep, sel_rep)
    q = run.Q[:, L - 1].contiguous()
    O = torch.full((B, H, d_pool), float("nan"), dtype=tdt, device="cuda")
    lca.decode_attn_q8(run.desc, layout, q, pq, sq, sc, pool_tail, sel_tail, O, run.ws)
    torch.cuda.synchronize()
    scn = sc.cpu().numpy().astype(np.float64)
    pr = q8.dequantize_rows(pq.cpu().numpy()[:, :, :m], scn[:, :, :m, 0])
    sr = q8.dequantize_rows(sq.cpu().numpy()[:, :, :m], scn[:, :, :m, 1])
    od = hp.oracle_desc(oracle, wl)
    tails = (hp.from_dev(raw_pool.contiguous(), dtype), hp.from_dev(raw_sel.contiguous(), dtype))
    ref = oracle.decode_attn(od, hp.from_dev(q, dtype), pr, sr, *tails)
    err = hp.vec_rel_err(hp.from_dev(O, dtype), ref)
    # what 8 bits cost against the 16-bit cache (reported, not gated: it is the format's error, not the kernel's)
    ref16 = oracle.decode_attn(od, hp.from_dev(q, dtype), hp.from_dev(run.pool_rep, dtype), hp.from_dev(run.sel_rep, dtype), *tails)
    print(f"  decode over 8-bit cache: err {err:.2e} against the oracle on the same codes; the codes cost {hp.vec_rel_err(ref, ref16):.2e}", flush=True)
    assert err <= hp.TOL[dtype]


def test_decode_loop_over_the_quantized_cache(oracle):
    """A decoding batch from an empty cache, as in the 16-bit loop test, with an 8-bit mirror of the representatives:
    every online update writes its 16-bit row, lca_quantize_cache(first_row = m - 1) adds that row's codes (and must
    leave every other row alone), and every step decodes over (codes, scales, ring) and is checked against the oracle."""
    import torch
    from oracle import q8
    from paper_2604_12452_amd import lca
    from tests.test_gpu_cache_update import Cache, _storage, _update_and_check
    B, g, w, H, S = 2, 8, 21, 16, 1
    steps = w + 5 * g + 3
    wl = inputs.Workload("loop_q8", B=B, L=1, H=H, S=S, d_pool=512, d_sel=64, g=g, w=w, dtype="bf16", seed=0, scale=1.0 / np.sqrt(576.0))
    rng = np.random.default_rng(78)
    cache = Cache(wl, m_cap=6, k_cap=w + g + 2, k_start=5, rng=rng)
    pq = torch.full((B, S, cache.m_cap, 512), 0x55, dtype=torch.uint8, device="cuda")
    sq = torch.full((B, S, cache.m_cap, 64), 0x55, dtype=torch.uint8, device="cuda")
    sc = torch.full((B, S, cache.m_cap, 2), float("nan"), dtype=torch.float32, device="cuda")
    q_hist, m, worst = [], 0, 0.0
    for L in range(1, steps + 1):
        cache.push()
        q_hist.append(_storage(rng, (B, H, wl.d_qk), "bf16", sigma=2.0))
        wlL = wl.with_(L=L)
        desc = hp.lca_desc(wlL)
        if L >= w + g and (L - w) % g == 0:
            _update_and_check(oracle, cache, L, np.stack(q_hist[-g:], axis=1), m)
            m += 1
            before = (pq.clone(), sq.clone(), sc.clone())
            lca.quantize_cache(desc, cache.layout(), cache.pool_rep, cache.sel_rep, pq, sq, sc, first_row=m - 1)
            torch.cuda.synchronize()
            keep = [i for i in range(cache.m_cap) if i != m - 1]
            for new, old in zip((pq, sq, sc), before):
                assert torch.equal(new[:, :, keep].view(torch.uint8), old[:, :, keep].view(torch.uint8)), "a row other than m - 1 was touched"
            for codes, src, col in ((pq, cache.pool_rep, 0), (sq, cache.sel_rep, 1)):
                rc, rs = q8.quantize_rows(hp.from_dev(src[:, :, m - 1], "bf16"))
                assert np.array_equal(codes[:, :, m - 1].cpu().numpy(), rc)
                assert np.array_equal(sc[:, :, m - 1, col].cpu().numpy().astype(np.float64), rs)
        od = hp.oracle_desc(oracle, wlL)
        assert od.m == m and od.k == cache.k
        O = torch.full((B, H, 512), float("nan"), dtype=torch.bfloat16, device="cuda")
        ws = lca.alloc_workspace(desc)
        lca.decode_attn_q8(desc, cache.layout(), hp.to_dev(q_hist[-1], "bf16"), pq, sq, sc, cache.pool_tail, cache.sel_tail, O, ws)
        torch.cuda.synchronize()
        scn = sc.cpu().numpy().astype(np.float64)
        pr = q8.dequantize_rows(pq.cpu().numpy()[:, :, :m], scn[:, :, :m, 0])
        sr = q8.dequantize_rows(sq.cpu().numpy()[:, :, :m], scn[:, :, :m, 1])
        pool_tail, sel_tail = cache.tail_rows(0, cache.k)
        ref = oracle.decode_attn(od, inputs.to_f64(q_hist[-1], "bf16"), pr, sr, pool_tail, sel_tail)
        err = hp.vec_rel_err(hp.from_dev(O, "bf16"), ref)
        assert err <= hp.TOL["bf16"], f"decode rel err {err:.3e} at L = {L}"
        worst = max(worst, err)
    assert m == 5
    print(f"  {steps} steps, {m} updates, worst decode err over the 8-bit cache {worst:.2e}", flush=True)


def test_quantize_and_q8_decode_reject_bad_arguments():
    import ctypes
    import torch
    from paper_2604_12452_amd import lca
    wl = inputs.Workload("bad", B=1, L=200, H=16, S=1, d_pool=512, d_sel=64, g=16, w=40, dtype="bf16")
    desc = hp.lca_desc(wl)
    # buffers large enough for every call below, of the element types the binding checks before it calls the library
    buf = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    b16, f32 = torch.zeros(1 << 20, dtype=torch.bfloat16, device="cuda"), torch.zeros(1 << 20, dtype=torch.float32, device="cuda")
    with pytest.raises(lca.LcaError):
        lca.quantize_cache(desc, None, b16, b16, buf, buf, f32, first_row=desc.m + 1)
    with pytest.raises(lca.LcaError):
        lca.quantize_cache(hp.lca_desc(wl.with_(dtype="f32", d_pool=128, d_sel=32)), None, f32, f32, buf, buf, f32)
    odd = inputs.Workload("bad", B=1, L=200, H=4, S=1, d_pool=128, d_sel=32, g=16, w=40, dtype="bf16")      # widths without an 8-bit decode kernel
    with pytest.raises(lca.LcaError) as e:
        lca.decode_attn_q8(hp.lca_desc(odd), None, b16, buf, buf, f32, b16, b16, b16, buf)
    assert e.value.status == lca.ERR_UNSUPPORTED
    lca.quantize_cache(desc, None, b16, b16, buf, buf, f32, first_row=desc.m)      # nothing to do: valid
    torch.cuda.synchronize()


def _random_decode_cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        mode = int(rng.integers(0, 2))
        if mode == MLA:
            H, S = [(16, 1), (16, 4), (8, 8), (7, 1), (12, 3)][int(rng.integers(0, 5))]
        else:
            H, S = [(8, 2), (14, 2), (4, 4), (16, 1), (6, 2), (5, 1), (3, 3)][int(rng.integers(0, 7))]
        L = int(rng.choice([rng.integers(1, 40), rng.integers(30, 200), rng.integers(150, 700), rng.integers(600, 2500)]))
        g = int(rng.choice([1, 2, 4, 8, 16, 32]))
        w = int(rng.choice([0, rng.integers(0, 30), rng.integers(20, 300)]))
        if L > w and (L - w) % g == 0:
            w += 1                      # keep at least the new token in the raw tail (k >= 1), as the decode convention has it
        out.append((mode, H, S, L, g, w, int(rng.integers(0, 2)), ["bf16", "f16"][int(rng.integers(0, 2))], int(rng.integers(0, 2)),
                    int(rng.integers(1, 5))))
    return out


@pytest.mark.parametrize("mode,H,S,L,g,w,ring,dtype,use_q8,B", _random_decode_cases(32, 4711))
def test_decode_random_shapes(oracle, mode, H, S, L, g, w, ring, dtype, use_q8, B):
    """Seeded random decode steps over both cache kinds: lengths from a single token to a few thousand (one tile, ragged
    tiles, several workgroups per sequence or one), every group size, both widths and head ratios, rings that wrap."""
    import torch
    from oracle import q8
    from paper_2604_12452_amd import lca
    d_pool, d_sel = (512, 64) if mode == MLA else (128, 128)
    wl = inputs.Workload("decode_rand", B=B, L=L, H=H, S=S, d_pool=d_pool, d_sel=d_sel, g=g, w=w, dtype=dtype, mode=mode, seed=900 + L + g,
                         n_q=min(g, L), theta=10000.0 if mode == MLA else 500000.0)
    print(f"[case] {wl} ring={ring} q8={use_q8}", flush=True)
    Q, POOL, SEL = inputs.gen_all(wl)
    run = hp.GpuRun(wl, Q, POOL, SEL).condense(alpha=False)
    m, k, P = run.desc.m, run.desc.k, wl.kv_heads
    tdt = lca.torch_dtype(run.desc)
    m_cap, k_cap, k_start = (m + 3, k + 5, (k + 2) % (k + 5)) if ring else (m, k, 0)
    layout = lca.CacheLayout(m_cap=m_cap, k_cap=k_cap, k_start=k_start)
    pool_rep = torch.full((B, S, max(m_cap, 1), d_pool), float("nan"), dtype=tdt, device="cuda")
    sel_rep = torch.full((B, S, max(m_cap, 1), d_sel), float("nan"), dtype=tdt, device="cuda")
    if m:
        pool_rep[:, :, :m], sel_rep[:, :, :m] = run.pool_rep, run.sel_rep
    pool_tail = torch.full((B, P, k_cap, d_pool), float("nan"), dtype=tdt, device="cuda")
    sel_tail = torch.full((B, P, k_cap, d_sel), float("nan"), dtype=tdt, device="cuda")
    idx = (k_start + torch.arange(k, device="cuda")) % k_cap
    if mode == MLA:
        raw_pool, raw_sel = run.POOL[:, None, m * g:], run.SEL[:, None, m * g:]
    else:
        raw_pool, raw_sel = run.POOL[:, m * g:].permute(0, 2, 1, 3), run.SEL[:, m * g:].permute(0, 2, 1, 3)
    pool_tail[:, :, idx], sel_tail[:, :, idx] = raw_pool, raw_sel
    q = run.Q[:, L - 1].contiguous()
    O = torch.full((B, H, d_pool), float("nan"), dtype=tdt, device="cuda")
    if use_q8:
        pq, sq, sc = _quantize_on_gpu(lca, torch, run.desc, layout, pool_rep, sel_rep)
        lca.decode_attn_q8(run.desc, layout, q, pq, sq, sc, pool_tail, sel_tail, O, run.ws)
        scn = sc.cpu().numpy().astype(np.float64)
        pr = q8.dequantize_rows(pq.cpu().numpy()[:, :, :m], scn[:, :, :m, 0])
        sr = q8.dequantize_rows(sq.cpu().numpy()[:, :, :m], scn[:, :, :m, 1])
    else:
        lca.decode_attn_cached(run.desc, layout, q, pool_rep, sel_rep, pool_tail, sel_tail, O, run.ws)
        pr, sr = hp.from_dev(pool_rep[:, :, :m], dtype), hp.from_dev(sel_rep[:, :, :m], dtype)
    torch.cuda.synchronize()
    ref = oracle.decode_attn(hp.oracle_desc(oracle, wl), hp.from_dev(q, dtype), pr, sr, hp.from_dev(raw_pool.contiguous(), dtype),
                             hp.from_dev(raw_sel.contiguous(), dtype))
    err = hp.vec_rel_err(hp.from_dev(O, dtype), ref)
    print(f"  err {err:.2e}", flush=True)
    assert err <= hp.TOL[dtype]
