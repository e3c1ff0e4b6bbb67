"""Pins for the oracle's online cache update (section 4.3, "Decoding and Online Cache Update") — CPU only.

The update condenses the g oldest raw tokens of the tail with the mean query of the last n_q tokens.  What
fixes it independently of the code under test: a numpy re-derivation of Eq. 6-8 on those g tokens written
here; the fact that at the step where the update is due the new representative must equal the LAST group of
a from-scratch condensation of the whole sequence at that length (same tokens, same summary query); the
token accounting m*g + k = L; and a decode loop whose cache, kept by updates alone, must serve the decode
step exactly like a cache built from the same representatives directly.
"""
import numpy as np
import pytest
from scipy.special import softmax


def _seq(o, seed, mode, B=2, L=61, H=4, S=2, d_pool=6, d_sel=4, g=4, w=9, n_q=0, scale=0.6):
    rng = np.random.default_rng(seed)
    d = o.Desc(B=B, L=L, H=H, S=S, d_pool=d_pool, d_sel=d_sel, g=g, w=w, n_q=n_q, mode=mode, scale=scale)
    kvs = (B, L, d_pool) if mode == 0 else (B, L, S, d_pool)
    kss = (B, L, d_sel) if mode == 0 else (B, L, S, d_sel)
    return d, rng.standard_normal((B, L, H, d.d_qk)), rng.standard_normal(kvs), rng.standard_normal(kss)


def _tail(d, X, lo, hi):
    """tokens [lo, hi) of a prefill-layout tensor in the tail layout [B, P, n, width]"""
    return X[:, None, lo:hi] if d.mode == 0 else X[:, lo:hi].transpose(0, 2, 1, 3)


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("S,n_q", [(1, 0), (2, 0), (4, 0), (2, 7), (2, 2)])
def test_update_is_the_last_group_of_a_fresh_condensation(oracle, mode, S, n_q):
    o = oracle
    d, Q, POOL, SEL = _seq(o, 3 + S, mode, L=9 + 4 * 13, S=S, n_q=n_q)      # (L - w) mod g == 0: an update is due
    assert (d.L - d.w) % d.g == 0 and d.m * d.g + d.k == d.L and d.k == d.w
    full = o.condense(d, o.summary_query(d, Q[:, d.L - d.nq:]), POOL, SEL)
    lo = (d.m - 1) * d.g
    upd = o.cache_update(d, Q[:, d.L - d.nq:], _tail(d, POOL, lo, lo + d.g), _tail(d, SEL, lo, lo + d.g))
    np.testing.assert_allclose(upd["pool_rep"], full["pool_rep"][:, :, -1], rtol=0, atol=1e-14)
    np.testing.assert_array_equal(upd["sel_rep"], full["sel_rep"][:, :, -1])
    np.testing.assert_array_equal(upd["anchor"] + lo, full["anchor"][:, :, -1])
    np.testing.assert_allclose(upd["alpha"], full["alpha"][:, :, lo:], rtol=0, atol=1e-15)


@pytest.mark.parametrize("mode", [0, 1])
def test_update_against_numpy_rederivation(oracle, mode):
    o = oracle
    rng = np.random.default_rng(17 + mode)
    B, H, S, g, dp, ds, nq = 2, 6, 3, 5, 7, 3, 4
    d = o.Desc(B=B, L=40, H=H, S=S, d_pool=dp, d_sel=ds, g=g, w=10, n_q=nq, mode=mode, scale=1.3)
    P = d.kv_heads
    qr = rng.standard_normal((B, nq, H, d.d_qk))
    pool_old, sel_old = rng.standard_normal((B, P, g, dp)), rng.standard_normal((B, P, g, ds))
    upd = o.cache_update(d, qr, pool_old, sel_old)
    hps = H // S
    for b in range(B):
        for s in range(S):
            p = 0 if mode == 0 else s
            qbar = qr[b, :, s * hps:(s + 1) * hps].mean(axis=(0, 1))
            keys = np.concatenate([pool_old[b, p], sel_old[b, p]], -1) if mode == 0 else sel_old[b, p]
            sc = d.scale * keys @ qbar
            a = softmax(sc)
            np.testing.assert_allclose(upd["alpha"][b, s], a, rtol=1e-12)
            np.testing.assert_allclose(upd["pool_rep"][b, s], a @ pool_old[b, p], rtol=1e-12, atol=1e-14)
            assert upd["anchor"][b, s] == int(np.argmax(sc))
            np.testing.assert_array_equal(upd["sel_rep"][b, s], sel_old[b, p, int(np.argmax(sc))])
            top = np.sort(sc)
            np.testing.assert_allclose(upd["margin"][b, s], top[-1] - top[-2], rtol=1e-9, atol=1e-12)


def test_uniform_scores_give_the_mean_and_the_first_token(oracle):
    o = oracle
    d = o.Desc(B=1, L=30, H=2, S=1, d_pool=4, d_sel=2, g=6, w=6, mode=0, scale=1.0)
    rng = np.random.default_rng(5)
    pool_old, sel_old = rng.standard_normal((1, 1, 6, 4)), rng.standard_normal((1, 1, 6, 2))
    upd = o.cache_update(d, np.zeros((1, 6, 2, 6)), pool_old, sel_old)          # zero queries: all scores equal
    np.testing.assert_allclose(upd["pool_rep"][0, 0], pool_old[0, 0].mean(0), rtol=1e-14)
    assert upd["anchor"][0, 0] == 0
    np.testing.assert_array_equal(upd["sel_rep"][0, 0], sel_old[0, 0, 0])


@pytest.mark.parametrize("mode", [0, 1])
def test_decode_loop_keeps_every_token_accounted_for(oracle, mode):
    """Run 3g+2 decode steps from a prefill cache.  After each step the cache kept by updates alone has
    m(L) representatives and k(L) raw tokens (m g + k = L), and the decode step over it equals the last row
    of prefill attention with the same representatives (decode = what prefill row L-1 sees)."""
    o = oracle
    g, w, L0 = 4, 6, 6 + 4 * 3 + 2
    d_all, Q, POOL, SEL = _seq(o, 23, mode, B=1, L=L0 + 3 * g + 2, H=4, S=2, g=g, w=w)
    d0 = o.Desc(B=1, L=L0, H=4, S=2, d_pool=d_all.d_pool, d_sel=d_all.d_sel, g=g, w=w, mode=mode, scale=d_all.scale)
    c0 = o.condense(d0, o.summary_query(d0, Q[:, L0 - g:L0]), POOL[:, :L0], SEL[:, :L0])
    reps_p, reps_s = [c0["pool_rep"][:, :, j] for j in range(d0.m)], [c0["sel_rep"][:, :, j] for j in range(d0.m)]
    lo = d0.m * g                                                   # first raw token of the tail
    for L in range(L0 + 1, d_all.L + 1):
        dL = o.Desc(B=1, L=L, H=4, S=2, d_pool=d_all.d_pool, d_sel=d_all.d_sel, g=g, w=w, mode=mode, scale=d_all.scale)
        if L >= w + g and (L - w) % g == 0:                         # the newest token completes a group
            upd = o.cache_update(dL, Q[:, L - g:L], _tail(dL, POOL, lo, lo + g), _tail(dL, SEL, lo, lo + g))
            reps_p.append(upd["pool_rep"]); reps_s.append(upd["sel_rep"])
            lo += g
        assert len(reps_p) == dL.m and L - lo == dL.k and dL.m * g + dL.k == L
        pr, sr = np.stack(reps_p, 2), np.stack(reps_s, 2)
        O = o.decode_attn(dL, Q[:, L - 1], pr, sr, _tail(dL, POOL, lo, L), _tail(dL, SEL, lo, L))
        ref = o.lca_attn_rows(dL, np.array([L - 1], dtype=np.int32), Q[:, L - 1:L], POOL[:, :L], SEL[:, :L], pr, sr)
        np.testing.assert_allclose(O, ref[:, 0], rtol=1e-12, atol=1e-14)
