"""Pins for the alternative pooling strategies of the ablation (section 5.4, Table 5; appendix on alternative
pooling strategies) in the oracle's condensation — CPU only.  Each strategy has a plain definition, re-derived
here in numpy; in addition: the default equals (weighted, max selection); mean pooling is weighted pooling with
uniform weights (the appendix's remark), i.e. what zero queries give; max selection of the pooled component is
the pooled row of the anchor token; a group of equal vectors is reproduced by every strategy."""
import numpy as np
import pytest
from scipy.special import softmax

W, MEAN, MAXSEL, MAXPOOL = 1, 2, 3, 4


def _problem(o, seed, mode, **kw):
    rng = np.random.default_rng(seed)
    base = dict(B=2, L=53, H=4, S=2, d_pool=7, d_sel=5, g=4, w=9, mode=mode, scale=0.8)
    base.update(kw)
    d = o.Desc(**base)
    kvs = (d.B, d.L, d.d_pool) if mode == 0 else (d.B, d.L, d.S, d.d_pool)
    kss = (d.B, d.L, d.d_sel) if mode == 0 else (d.B, d.L, d.S, d.d_sel)
    return d, rng.standard_normal((d.B, d.L, d.H, d.d_qk)), rng.standard_normal(kvs), rng.standard_normal(kss)


def _numpy_reduce(strategy, X, alpha, scores):
    if strategy == W:
        return alpha @ X
    if strategy == MEAN:
        return X.mean(axis=0)
    if strategy == MAXSEL:
        return X[int(np.argmax(scores))]
    return X[int(np.argmax((X * X).sum(-1)))]


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("pool_reduce", [W, MEAN, MAXSEL, MAXPOOL])
@pytest.mark.parametrize("sel_reduce", [W, MEAN, MAXSEL, MAXPOOL])
def test_every_cell_of_the_grid_against_numpy(oracle, mode, pool_reduce, sel_reduce):
    o = oracle
    d, Q, POOL, SEL = _problem(o, 11 + mode, mode, pool_reduce=pool_reduce, sel_reduce=sel_reduce)
    out = o.condense(d, o.summary_query(d, Q[:, d.L - d.nq:]), POOL, SEL)
    hps = d.H // d.S
    for b in range(d.B):
        for s in range(d.S):
            qbar = Q[b, d.L - d.nq:, s * hps:(s + 1) * hps].mean(axis=(0, 1))
            pool = POOL[b] if mode == 0 else POOL[b, :, s]
            sel = SEL[b] if mode == 0 else SEL[b, :, s]
            keys = np.concatenate([pool, sel], -1) if mode == 0 else sel
            for j in range(d.m):
                G = slice(j * d.g, (j + 1) * d.g)
                sc = d.scale * keys[G] @ qbar
                a = softmax(sc)
                np.testing.assert_allclose(out["pool_rep"][b, s, j], _numpy_reduce(pool_reduce, pool[G], a, sc), rtol=1e-12, atol=1e-14)
                np.testing.assert_allclose(out["sel_rep"][b, s, j], _numpy_reduce(sel_reduce, sel[G], a, sc), rtol=1e-12, atol=1e-14)
                assert out["anchor"][b, s, j] == j * d.g + int(np.argmax(sc))     # the anchor reports the arg-max score token whatever the strategies


@pytest.mark.parametrize("mode", [0, 1])
def test_default_is_weighted_pooling_and_max_selection(oracle, mode):
    o = oracle
    d0, Q, POOL, SEL = _problem(o, 5, mode)
    d1 = o.Desc(**{**d0.__dict__, "pool_reduce": W, "sel_reduce": MAXSEL})
    qbar = o.summary_query(d0, Q[:, d0.L - d0.nq:])
    a, b = o.condense(d0, qbar, POOL, SEL), o.condense(d1, qbar, POOL, SEL)
    for k in ("pool_rep", "sel_rep", "anchor", "alpha"):
        np.testing.assert_array_equal(a[k], b[k])


def test_mean_pooling_is_weighted_pooling_with_uniform_weights(oracle):
    o = oracle
    d, Q, POOL, SEL = _problem(o, 8, 0, pool_reduce=MEAN, sel_reduce=MEAN)
    mean = o.condense(d, o.summary_query(d, Q[:, d.L - d.nq:]), POOL, SEL)
    dw = o.Desc(**{**d.__dict__, "pool_reduce": W, "sel_reduce": W})
    uniform = o.condense(dw, np.zeros((d.B, d.S, d.d_qk)), POOL, SEL)              # zero summary query: alpha = 1/g
    np.testing.assert_allclose(mean["pool_rep"], uniform["pool_rep"], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(mean["sel_rep"], uniform["sel_rep"], rtol=1e-13, atol=1e-15)


def test_selection_strategies_copy_rows_and_equal_vectors_survive_everything(oracle):
    o = oracle
    d, Q, POOL, SEL = _problem(o, 9, 1, pool_reduce=MAXSEL, sel_reduce=MAXPOOL)
    out = o.condense(d, o.summary_query(d, Q[:, d.L - d.nq:]), POOL, SEL)
    for b in range(d.B):
        for s in range(d.S):
            for j in range(d.m):
                np.testing.assert_array_equal(out["pool_rep"][b, s, j], POOL[b, out["anchor"][b, s, j], s])
                rows = SEL[b, j * d.g:(j + 1) * d.g, s]
                assert any((out["sel_rep"][b, s, j] == r).all() for r in rows)
                assert np.isclose((out["sel_rep"][b, s, j] ** 2).sum(), (rows ** 2).sum(-1).max())
    # a group whose tokens are all the same vector is reproduced exactly by every strategy
    POOL2, SEL2 = POOL.copy(), SEL.copy()
    POOL2[:, 4:8], SEL2[:, 4:8] = POOL2[:, 4:5], SEL2[:, 4:5]
    for pr in (W, MEAN, MAXSEL, MAXPOOL):
        dd = o.Desc(**{**d.__dict__, "pool_reduce": pr, "sel_reduce": pr})
        out = o.condense(dd, o.summary_query(dd, Q[:, d.L - d.nq:]), POOL2, SEL2)
        np.testing.assert_allclose(out["pool_rep"][:, :, 1], POOL2[:, 4].reshape(d.B, d.S, -1), rtol=1e-14)
        np.testing.assert_allclose(out["sel_rep"][:, :, 1], SEL2[:, 4].reshape(d.B, d.S, -1), rtol=1e-14)
