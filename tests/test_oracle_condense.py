"""Pins for the oracle's condensation step (section 4.2, Eq. 6-8, Proposition 1) — CPU only.

Each check is something the paper or the mathematics fixes independently of the oracle's code:
closed forms, invariants, degenerate cases and a brute-force re-derivation written here in numpy.
"""
import numpy as np
import pytest
from scipy.special import softmax


def _rand_problem(o, seed, B=2, L=70, H=4, S=2, d_pool=6, d_sel=3, g=4, w=9, mode=0, scale=0.7):
    rng = np.random.default_rng(seed)
    d = o.Desc(B=B, L=L, H=H, S=S, d_pool=d_pool, d_sel=d_sel, g=g, w=w, mode=mode, scale=scale)
    kvs = (B, L, d_pool) if mode == 0 else (B, L, S, d_pool)
    kss = (B, L, d_sel) if mode == 0 else (B, L, S, d_sel)
    POOL = rng.standard_normal(kvs)
    SEL = rng.standard_normal(kss)
    Q = rng.standard_normal((B, L, H, d.d_qk))
    return d, Q, POOL, SEL


def _brute_condense(d, Q, POOL, SEL):
    """Eq. 6-8 re-derived with numpy slicing, independent of the C code."""
    B, S, g, m = d.B, d.S, d.g, d.m
    hps = d.H // S
    pool_rep = np.zeros((B, S, m, d.d_pool))
    sel_rep = np.zeros((B, S, m, d.d_sel))
    anchor = np.zeros((B, S, m), dtype=np.int64)
    alpha = np.zeros((B, S, m * g))
    for b in range(B):
        for s in range(S):
            qbar = Q[b, d.L - d.nq:, s * hps:(s + 1) * hps, :].mean(axis=(0, 1))
            if d.mode == 0:
                keys = np.concatenate([POOL[b], SEL[b]], axis=-1)      # [L, d_c + d_r]
                vals, sel = POOL[b], SEL[b]
            else:
                keys, vals, sel = SEL[b, :, s], POOL[b, :, s], SEL[b, :, s]
            for j in range(m):
                G = slice(j * g, (j + 1) * g)
                sc = d.scale * keys[G] @ qbar
                a = softmax(sc)
                pool_rep[b, s, j] = a @ vals[G]
                anchor[b, s, j] = j * g + int(np.argmax(sc))
                sel_rep[b, s, j] = sel[anchor[b, s, j]]
                alpha[b, s, G] = a
    return pool_rep, sel_rep, anchor, alpha


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("g,w,L", [(4, 9, 70), (2, 0, 33), (8, 5, 64), (1, 3, 20), (16, 16, 100)])
def test_condense_matches_brute_force(oracle, mode, g, w, L):
    d, Q, POOL, SEL = _rand_problem(oracle, 11 + g + w, L=L, g=g, w=w, mode=mode)
    qbar = oracle.summary_query(d, Q[:, L - d.nq:])
    out = oracle.condense(d, qbar, POOL, SEL)
    pr, sr, an, al = _brute_condense(d, Q, POOL, SEL)
    assert d.m == (L - w) // g and d.m * g + d.k == L          # every token accounted for (section 4.2)
    np.testing.assert_allclose(out["pool_rep"], pr, rtol=0, atol=1e-12)
    np.testing.assert_array_equal(out["anchor"], an)
    np.testing.assert_array_equal(out["sel_rep"], sr)
    np.testing.assert_allclose(out["alpha"], al, rtol=0, atol=1e-14)


def test_summary_query_is_mean_of_last_queries(oracle):
    d, Q, _, _ = _rand_problem(oracle, 3, H=6, S=3, g=4)
    for n_q in (1, 4, 7):
        d.n_q = n_q
        qbar = oracle.summary_query(d, Q[:, d.L - n_q:])
        ref = Q[:, d.L - n_q:].reshape(d.B, n_q, d.S, d.H // d.S, d.d_qk).mean(axis=(1, 3))
        np.testing.assert_allclose(qbar, ref, atol=1e-15)


def test_alpha_is_a_probability_vector_and_reps_are_convex_combinations(oracle):
    d, Q, POOL, SEL = _rand_problem(oracle, 5, L=200, g=8, w=17, scale=3.0)
    out = oracle.condense(d, oracle.summary_query(d, Q[:, d.L - d.nq:]), POOL, SEL)
    a = out["alpha"].reshape(d.B, d.S, d.m, d.g)
    assert (a >= 0).all()
    np.testing.assert_allclose(a.sum(-1), 1.0, atol=1e-14)
    grp = POOL[:, : d.m * d.g].reshape(d.B, 1, d.m, d.g, d.d_pool)
    assert (out["pool_rep"] <= grp.max(3) + 1e-12).all() and (out["pool_rep"] >= grp.min(3) - 1e-12).all()
    # the anchor is a concrete token of its own group (Eq. 8)
    j = np.arange(d.m)[None, None, :]
    assert ((out["anchor"] >= j * d.g) & (out["anchor"] < (j + 1) * d.g)).all()
    assert (out["margin"] >= 0).all()


def test_zero_summary_query_gives_mean_pooling_and_first_token_anchor(oracle):
    # appendix A.1: mean pooling is weighted pooling with alpha = 1/g
    d, Q, POOL, SEL = _rand_problem(oracle, 6, L=90, g=8, w=10)
    out = oracle.condense(d, np.zeros((d.B, d.S, d.d_qk)), POOL, SEL)
    np.testing.assert_allclose(out["alpha"], 1.0 / d.g, atol=1e-15)
    grp = POOL[:, : d.m * d.g].reshape(d.B, d.m, d.g, d.d_pool).mean(2)
    np.testing.assert_allclose(out["pool_rep"], np.broadcast_to(grp[:, None], out["pool_rep"].shape), atol=1e-14)
    np.testing.assert_array_equal(out["anchor"], np.broadcast_to(np.arange(d.m) * d.g, out["anchor"].shape))
    np.testing.assert_array_equal(out["margin"], 0.0)


def test_constant_group_is_reproduced_exactly(oracle):
    d, Q, POOL, SEL = _rand_problem(oracle, 7, L=64, g=4, w=8)
    POOL[:, 8:12] = POOL[:, 8:9]          # group j = 2 holds one repeated latent
    out = oracle.condense(d, oracle.summary_query(d, Q[:, d.L - d.nq:]), POOL, SEL)
    np.testing.assert_allclose(out["pool_rep"][:, :, 2], np.broadcast_to(POOL[:, None, 8], (d.B, d.S, d.d_pool)),
                               rtol=1e-15, atol=1e-15)


def test_sharp_scores_turn_pooling_into_selection(oracle):
    d, Q, POOL, SEL = _rand_problem(oracle, 8, L=80, g=8, w=8, scale=1e4)
    out = oracle.condense(d, oracle.summary_query(d, Q[:, d.L - d.nq:]), POOL, SEL)
    for b in range(d.B):
        for s in range(d.S):
            np.testing.assert_allclose(out["pool_rep"][b, s], POOL[b, out["anchor"][b, s]], atol=1e-9)
            np.testing.assert_array_equal(out["sel_rep"][b, s], SEL[b, out["anchor"][b, s]])


def test_proposition_1_weighted_mean_minimises_weighted_squared_error(oracle):
    d, Q, POOL, SEL = _rand_problem(oracle, 9, B=1, S=1, H=2, L=48, g=8, w=8)
    out = oracle.condense(d, oracle.summary_query(d, Q[:, d.L - d.nq:]), POOL, SEL)
    rng = np.random.default_rng(0)
    for j in range(d.m):
        c = POOL[0, j * d.g:(j + 1) * d.g]
        a = out["alpha"][0, 0, j * d.g:(j + 1) * d.g]
        loss = lambda x: float((a * ((c - x) ** 2).sum(-1)).sum())
        best = loss(out["pool_rep"][0, 0, j])
        for _ in range(100):
            assert best <= loss(out["pool_rep"][0, 0, j] + 0.1 * rng.standard_normal(d.d_pool))
        # closed form of the minimum: the alpha-weighted variance
        np.testing.assert_allclose(best, (a * (c ** 2).sum(-1)).sum() - (out["pool_rep"][0, 0, j] ** 2).sum(), atol=1e-12)


def test_permuting_a_group_moves_the_anchor_and_keeps_the_representative(oracle):
    d, Q, POOL, SEL = _rand_problem(oracle, 10, B=1, L=60, g=6, w=6)
    qbar = oracle.summary_query(d, Q[:, d.L - d.nq:])
    base = oracle.condense(d, qbar, POOL, SEL)
    perm = np.array([3, 0, 5, 1, 4, 2])
    P2, S2 = POOL.copy(), SEL.copy()
    j = 4
    P2[0, j * 6:(j + 1) * 6] = POOL[0, j * 6 + perm]
    S2[0, j * 6:(j + 1) * 6] = SEL[0, j * 6 + perm]
    out = oracle.condense(d, qbar, P2, S2)
    np.testing.assert_allclose(out["pool_rep"], base["pool_rep"], atol=1e-14)
    np.testing.assert_array_equal(out["sel_rep"], base["sel_rep"])
    for s in range(d.S):
        old = base["anchor"][0, s, j] - j * 6
        assert out["anchor"][0, s, j] - j * 6 == int(np.where(perm == old)[0][0])


def test_ties_go_to_the_lowest_index(oracle):
    d = oracle.Desc(B=1, L=12, H=1, S=1, d_pool=2, d_sel=2, g=4, w=4)
    POOL = np.zeros((1, 12, 2))
    SEL = np.zeros((1, 12, 2))
    POOL[0, [1, 3], 0] = 1.0            # tokens 1 and 3 tie for the maximum in group 0
    POOL[0, [6, 7], 0] = 2.0            # tokens 6 and 7 tie in group 1
    qbar = np.array([[[1.0, 0.0, 0.0, 0.0]]])
    out = oracle.condense(d, qbar, POOL, SEL)
    np.testing.assert_array_equal(out["anchor"][0, 0], [1, 6])
    np.testing.assert_array_equal(out["margin"][0, 0], [0.0, 0.0])


def test_no_groups_when_sequence_is_short(oracle):
    # section 4.3: L < w + g falls back to plain attention; nothing is condensed
    for L, w, g in [(10, 16, 4), (19, 16, 4), (16, 16, 4)]:
        d = oracle.Desc(B=1, L=L, H=1, S=1, d_pool=2, d_sel=2, g=g, w=w)
        assert d.m == 0 and d.k == L
        out = oracle.condense(d, np.zeros((1, 1, 4)), np.zeros((1, L, 2)), np.zeros((1, L, 2)))
        assert out["pool_rep"].shape == (1, 1, 0, 2)


def test_bad_arguments_are_rejected(oracle):
    d = oracle.Desc(B=1, L=12, H=3, S=2, d_pool=2, d_sel=2, g=4, w=4)   # H % S != 0
    with pytest.raises(ValueError):
        oracle.condense(d, np.zeros((1, 2, 4)), np.zeros((1, 12, 2)), np.zeros((1, 12, 2)))
