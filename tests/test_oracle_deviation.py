"""Pins for the oracle's per-token deviation statistics (Theorem 1's delta_k, delta_v; appendix on empirical
per-token deviations, Tables 9-10) — CPU only: a numpy re-derivation; groups of equal tokens and g = 1 deviate by
nothing; a two-token group under mean pooling deviates by half the tokens' distance; the maxima are the very
delta_k, delta_v with which the uniform error bound holds."""
import numpy as np
import pytest


def _problem(o, seed, mode, **kw):
    rng = np.random.default_rng(seed)
    base = dict(B=2, L=57, H=4, S=2, d_pool=6, d_sel=4, g=4, w=9, mode=mode, scale=0.7)
    base.update(kw)
    d = o.Desc(**base)
    kvs = (d.B, d.L, d.d_pool) if mode == 0 else (d.B, d.L, d.S, d.d_pool)
    kss = (d.B, d.L, d.d_sel) if mode == 0 else (d.B, d.L, d.S, d.d_sel)
    return d, rng.standard_normal((d.B, d.L, d.H, d.d_qk)), rng.standard_normal(kvs), rng.standard_normal(kss)


@pytest.mark.parametrize("mode", [0, 1])
def test_against_numpy_rederivation(oracle, mode):
    o = oracle
    d, Q, POOL, SEL = _problem(o, 31 + mode, mode)
    c = o.condense(d, o.summary_query(d, Q[:, d.L - d.nq:]), POOL, SEL)
    stats = o.deviation_stats(d, POOL, SEL, c["pool_rep"], c["sel_rep"])
    n = d.m * d.g
    for b in range(d.B):
        for s in range(d.S):
            pool = POOL[b, :n] if mode == 0 else POOL[b, :n, s]
            sel = SEL[b, :n] if mode == 0 else SEL[b, :n, s]
            prep = np.repeat(c["pool_rep"][b, s], d.g, axis=0)
            srep = np.repeat(c["sel_rep"][b, s], d.g, axis=0)
            key, krep = (np.concatenate([pool, sel], -1), np.concatenate([prep, srep], -1)) if mode == 0 else (sel, srep)
            dk, dv = np.linalg.norm(key - krep, axis=-1), np.linalg.norm(pool - prep, axis=-1)
            want = [dk.mean(), (dk / np.linalg.norm(key, axis=-1)).mean(), dk.max(), dv.mean(), (dv / np.linalg.norm(pool, axis=-1)).mean(), dv.max()]
            np.testing.assert_allclose(stats[b, s], want, rtol=1e-12)


def test_no_deviation_for_equal_tokens_and_for_groups_of_one(oracle):
    o = oracle
    d, Q, POOL, SEL = _problem(o, 4, 0)
    POOL[:] = POOL[:, :1]
    SEL[:] = SEL[:, :1]
    c = o.condense(d, o.summary_query(d, Q[:, d.L - d.nq:]), POOL, SEL)
    assert np.abs(o.deviation_stats(d, POOL, SEL, c["pool_rep"], c["sel_rep"])).max() < 1e-14
    d1, Q, POOL, SEL = _problem(o, 5, 1, g=1, w=3)
    c = o.condense(d1, o.summary_query(d1, Q[:, d1.L - d1.nq:]), POOL, SEL)
    assert np.abs(o.deviation_stats(d1, POOL, SEL, c["pool_rep"], c["sel_rep"])).max() < 1e-14
    d0 = o.Desc(B=1, L=5, H=2, S=1, d_pool=4, d_sel=2, g=4, w=8)                    # m = 0: nothing condensed
    assert (o.deviation_stats(d0, np.ones((1, 5, 4)), np.ones((1, 5, 2)), np.zeros((1, 1, 0, 4)), np.zeros((1, 1, 0, 2))) == 0).all()


def test_two_token_groups_under_mean_pooling(oracle):
    o = oracle
    rng = np.random.default_rng(9)
    d = o.Desc(B=1, L=8, H=1, S=1, d_pool=5, d_sel=3, g=2, w=0, mode=1, scale=1.0, pool_reduce=2, sel_reduce=2)   # mean / mean
    POOL, SEL = rng.standard_normal((1, 8, 1, 5)), rng.standard_normal((1, 8, 1, 3))
    c = o.condense(d, np.zeros((1, 1, 3)), POOL, SEL)
    stats = o.deviation_stats(d, POOL, SEL, c["pool_rep"], c["sel_rep"])[0, 0]
    half_v = np.linalg.norm(POOL[0, 0::2, 0] - POOL[0, 1::2, 0], axis=-1) / 2        # each token sits half the distance from the mean
    half_k = np.linalg.norm(SEL[0, 0::2, 0] - SEL[0, 1::2, 0], axis=-1) / 2
    np.testing.assert_allclose([stats[0], stats[2], stats[3], stats[5]], [half_k.mean(), half_k.max(), half_v.mean(), half_v.max()], rtol=1e-13)


def test_the_maxima_are_the_deltas_of_the_uniform_error_bound(oracle):
    """Theorem 1 with the multiplicity-weighted normaliser: ||Attn_t - Attn_t^LCA|| <= V (exp(2 Q delta_k scale) - 1) + delta_v
    with delta_k, delta_v = the maxima this statistic reports (taken over all condensed tokens, so valid for every row)."""
    o = oracle
    rng = np.random.default_rng(10)
    L, g, w = 96, 4, 8
    d = o.Desc(B=1, L=L, H=2, S=1, d_pool=6, d_sel=2, g=g, w=w, scale=0.35, rep_logit_bias=np.log(g))
    POOL = np.cumsum(0.05 * rng.standard_normal((1, L, 6)), axis=1) + rng.standard_normal((1, 1, 6))
    SEL = 0.3 * rng.standard_normal((1, L, 2))
    Q = 0.5 * rng.standard_normal((1, L, 2, 8))
    c = o.condense(d, o.summary_query(d, Q[:, L - g:]), POOL, SEL)
    _, _, dk, _, _, dv = o.deviation_stats(d, POOL, SEL, c["pool_rep"], c["sel_rep"])[0, 0]
    rows = np.arange(L, dtype=np.int32)
    err = np.linalg.norm(o.dense_attn_rows(d, rows, Q, POOL, SEL) - o.lca_attn_rows(d, rows, Q, POOL, SEL, c["pool_rep"], c["sel_rep"]), axis=-1)
    Vn = np.linalg.norm(POOL[0], axis=-1).max()
    for h in range(2):
        Qn = np.linalg.norm(Q[0, :, h], axis=-1)
        assert (err[0, :, h] <= Vn * (np.exp(2 * Qn * dk * d.scale) - 1) + dv + 1e-12).all()
    assert dk > 0 and dv > 0 and (err > 0).sum() > 100
