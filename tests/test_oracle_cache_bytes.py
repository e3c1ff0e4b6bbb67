"""Pins for the KV-cache size formula (section 4.3 decoding paragraph, appendix B) — CPU only."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "kv_cache_gb.txt")


def _golden():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            label, dense, lca = line.split()[:3]
            rows.append((label, float(dense), float(lca)))
    return rows


def test_byte_counts_of_the_benchmark_configurations(oracle):
    mla = dict(B=1, L=131072, H=16, d_pool=512, d_sel=64, w=1024)
    assert oracle.cache_bytes(oracle.Desc(S=1, g=16, **mla), 2) == (131072 * 576 * 2, (8128 + 1024) * 576 * 2)
    assert oracle.cache_bytes(oracle.Desc(S=1, g=32, **mla), 2) == (150994944, (4064 + 1024) * 1152)
    # one condensed set per query head: 16 * 8128 + 1024 = 131072 entries, no saving at g = 16
    assert oracle.cache_bytes(oracle.Desc(S=16, g=16, **mla), 2) == (150994944, 150994944)
    assert oracle.cache_bytes(oracle.Desc(S=16, g=32, **mla), 2) == (150994944, (16 * 4064 + 1024) * 1152)
    gqa = oracle.Desc(B=1, L=65536, H=32, S=8, d_pool=128, d_sel=128, g=16, w=1024, mode=oracle.MODE_GQA)
    assert oracle.cache_bytes(gqa, 2) == (65536 * 8 * 256 * 2, 8 * (4032 + 1024) * 256 * 2)


def test_ratio_matches_the_sizes_the_paper_prints(oracle):
    """The printed GB figures are rounded to 2 decimals; the formula's ratio must lie inside the
    interval those roundings allow.  A per-query-head cache (S = H) would not."""
    mla = oracle.Desc(B=1, L=131072, H=16, S=1, d_pool=512, d_sel=64, g=16, w=1024)
    gqa = oracle.Desc(B=1, L=131072, H=28, S=4, d_pool=128, d_sel=128, g=16, w=1024, mode=oracle.MODE_GQA)
    per_head = oracle.Desc(B=1, L=131072, H=16, S=16, d_pool=512, d_sel=64, g=16, w=1024)
    for label, dense_gb, lca_gb in _golden():
        lo, hi = (lca_gb - 0.005) / (dense_gb + 0.005), (lca_gb + 0.005) / (dense_gb - 0.005)
        dd, cc = oracle.cache_bytes(gqa if "gqa" in label else mla, 2)
        assert lo <= cc / dd <= hi, (label, cc / dd, lo, hi)
        dd, cc = oracle.cache_bytes(per_head, 2)
        assert not (lo <= cc / dd <= hi)
    np.testing.assert_allclose(cc / dd, 1.0)
