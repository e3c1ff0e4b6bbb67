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
    assert wl.m == m
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
    layout = lca.CacheLayout(m_cap=m + spare, k_cap=wl.k, k_start=0)
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
