"""GPU parity: liblca (through its C ABI) against the fp64 oracle on the same seeded inputs.

Stage 1: condensation (anchors bit-exact above the score margin, pooled vectors within tolerance,
selected rows bit-exact copies).  Stage 2: attention fed the GPU's own emitted cache.  Stage 3: end to
end against the all-fp64 oracle.  Small shapes are compared on every row; they span several query
blocks, several key tiles and ragged tails of both.
"""
import math

import numpy as np
import pytest

from paper_2604_12452_amd import inputs
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def _wl(name, **kw):
    base = dict(B=1, L=333, H=4, S=2, d_pool=16, d_sel=8, g=4, w=10, dtype="f32", seed=42)
    base.update(kw)
    return inputs.Workload(name, **base)


def _full_parity(oracle, wl, bias=0.0, dense=True):
    print(f"[case] {wl}", flush=True)
    Q, POOL, SEL = inputs.gen_all(wl)
    Qf, POOLf, SELf = (inputs.to_f64(x, wl.dtype) for x in (Q, POOL, SEL))
    run = hp.GpuRun(wl, Q, POOL, SEL, rep_logit_bias=bias).condense()
    ref, differ = hp.check_condense(oracle, wl, run, Qf[:, wl.L - wl.nq:], POOLf, SELf)
    run.prefill()
    rows = np.arange(wl.L, dtype=np.int32)
    e2, e3 = hp.check_prefill(oracle, wl, run, rows, Qf, POOLf, SELf, ref, differ, bias=bias)
    e_d = None
    if dense:
        run.dense()
        e_d = hp.check_dense(oracle, wl, run, rows, Qf, POOLf, SELf)
    print(f"  stage2 {e2:.2e} stage3 {e3:.2e} dense {e_d}", flush=True)
    return run


# ---- generic kernels (any widths), both element types, both modes --------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("mode", [inputs.MODE_MLA, inputs.MODE_GQA])
@pytest.mark.parametrize("L,g,w,H,S", [(333, 4, 10, 4, 2), (129, 8, 0, 2, 1), (70, 1, 5, 2, 2), (257, 64, 3, 6, 3), (40, 3, 7, 1, 1)])
def test_generic_kernels_small_shapes(oracle, dtype, mode, L, g, w, H, S):
    _full_parity(oracle, _wl("generic", L=L, g=g, w=w, H=H, S=S, dtype=dtype, mode=mode, d_pool=24, d_sel=16, B=2))


@pytest.mark.parametrize("L,w,g", [(40, 64, 4), (10, 8, 4), (1, 1, 1), (5, 0, 8)])
def test_no_groups_falls_back_to_dense(oracle, L, w, g):
    wl = _wl("short", L=L, w=w, g=min(g, 8), n_q=1)
    assert hp.lca_desc(wl).m == 0
    run = _full_parity(oracle, wl)
    assert np.array_equal(hp.from_dev(run.O, wl.dtype), hp.from_dev(run.O_dense, wl.dtype))


# ---- configuration 1: tiny fp32 case, every row -----------------------------------------------------
@pytest.mark.parametrize("S", [1, 4])
def test_cfg1_tiny_fp32_all_rows(oracle, S):
    _full_parity(oracle, inputs.configs()["cfg1"].with_(S=S))


# ---- MFMA kernel at the MLA widths (512 + 64), small L, every row -----------------------------------
@pytest.mark.parametrize("L,g,w,H,S,B", [
    (700, 16, 100, 2, 1, 1),      # several query blocks and key tiles, ragged tails
    (700, 16, 100, 2, 2, 2),      # one condensed set per head
    (513, 32, 0, 1, 1, 1),        # no window: only the remainder stays raw
    (300, 8, 64, 4, 2, 1),
    (257, 1, 31, 1, 1, 1),        # one-token groups: equals dense
    (128, 16, 16, 1, 1, 1),       # exactly one query block
    (100, 16, 200, 2, 1, 1),      # L < w: no groups
    (33, 2, 3, 1, 1, 1),
    (1, 1, 0, 1, 1, 1),           # a single token
    (7, 2, 1, 3, 3, 2),           # fewer rows than a tile, two sequences: segments of a few rows behind one another
    (40, 4, 4, 4, 2, 3),          # three sequences back to back: nothing may leak across a sequence's end
    (200, 16, 48, 128, 1, 1),     # 128 heads over one set: more work items per query block than workgroup slots of an XCD
    (140, 8, 20, 48, 16, 2),      # 48 heads in 16 sets of three
])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_mla_mfma_small_all_rows(oracle, L, g, w, H, S, B, dtype):
    wl = inputs.Workload("mla_small", B=B, L=L, H=H, S=S, d_pool=512, d_sel=64, g=g, w=w, dtype=dtype, seed=7 + L)
    _full_parity(oracle, wl)


@pytest.mark.parametrize("L,g,w,H,S,B,mode", [
    (150, 16, 40, 24, 1, 1, inputs.MODE_MLA),      # 24 heads in one set: 384 (position, head) pairs, two rounds of loads per wavefront
    (96, 8, 10, 40, 2, 2, inputs.MODE_MLA),        # 20 heads per set
    (130, 16, 20, 32, 1, 1, inputs.MODE_MLA),      # more heads per set than wavefronts in the workgroup
    (120, 16, 24, 36, 2, 1, inputs.MODE_GQA),      # 18 query heads per KV head
])
def test_condense_many_heads_per_set(oracle, L, g, w, H, S, B, mode):
    """Condensation alone with more query heads per set than the 16 of the benchmark configurations: the summary query
    walks its (position, head) list in steps of 16 pairs with a carry, which only such head counts exercise in full."""
    d = (512, 64) if mode == inputs.MODE_MLA else (128, 128)
    wl = inputs.Workload("many_heads", B=B, L=L, H=H, S=S, d_pool=d[0], d_sel=d[1], g=g, w=w, dtype="bf16", mode=mode, seed=900 + H)
    Q, POOL, SEL = inputs.gen_all(wl)
    run = hp.GpuRun(wl, Q, POOL, SEL).condense(alpha=True)
    hp.check_condense(oracle, wl, run, inputs.to_f64(Q[:, wl.L - wl.nq:], wl.dtype), inputs.to_f64(POOL, wl.dtype), inputs.to_f64(SEL, wl.dtype))


def _random_shapes(mode, n, seed):
    """Seeded draws of valid shapes for the MFMA kernels: lengths around the tile and block sizes, every group size,
    windows from none to longer than the sequence, several head ratios."""
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        L = int(rng.choice([rng.integers(1, 70), rng.integers(60, 140), rng.integers(120, 300), rng.integers(250, 650)]))
        g = int(rng.choice([1, 2, 3, 4, 8, 16, 32, 64]))
        w = int(rng.choice([0, 1, rng.integers(0, 40), rng.integers(30, 200), L + 5]))
        if mode == inputs.MODE_MLA:
            H, S = [(1, 1), (2, 1), (4, 2), (4, 4), (3, 1)][int(rng.integers(0, 5))]
        else:
            H, S = [(4, 1), (8, 2), (2, 2), (4, 2), (8, 1), (2, 1)][int(rng.integers(0, 6))]
        out.append((L, g, w, H, S, int(rng.integers(1, 3))))
    return out


@pytest.mark.parametrize("L,g,w,H,S,B", _random_shapes(inputs.MODE_MLA, 16, 2024))
def test_mla_mfma_random_shapes(oracle, L, g, w, H, S, B):
    wl = inputs.Workload("mla_rand", B=B, L=L, H=H, S=S, d_pool=512, d_sel=64, g=g, w=w, dtype="bf16", seed=1000 + L + 7 * g + w, n_q=min(g, L))
    _full_parity(oracle, wl)


@pytest.mark.parametrize("L,g,w,H,S,B", _random_shapes(inputs.MODE_GQA, 16, 2025))
def test_gqa_mfma_random_shapes(oracle, L, g, w, H, S, B):
    wl = inputs.Workload("gqa_rand", B=B, L=L, H=H, S=S, d_pool=128, d_sel=128, g=g, w=w, dtype="bf16", mode=inputs.MODE_GQA,
                         theta=500000.0, seed=2000 + L + 7 * g + w, n_q=min(g, L))
    _full_parity(oracle, wl)


@pytest.mark.parametrize("L,g,w,H,S,B", _random_shapes(inputs.MODE_MLA, 8, 2026))
def test_mla_mfma_random_shapes_fp16(oracle, L, g, w, H, S, B):
    wl = inputs.Workload("mla_rand16", B=B, L=L, H=H, S=S, d_pool=512, d_sel=64, g=g, w=w, dtype="f16", seed=3000 + L + 7 * g + w, n_q=min(g, L))
    _full_parity(oracle, wl)


@pytest.mark.parametrize("L,g,w,H,S,B", _random_shapes(inputs.MODE_GQA, 8, 2027))
def test_gqa_mfma_random_shapes_fp16(oracle, L, g, w, H, S, B):
    wl = inputs.Workload("gqa_rand16", B=B, L=L, H=H, S=S, d_pool=128, d_sel=128, g=g, w=w, dtype="f16", mode=inputs.MODE_GQA,
                         theta=500000.0, seed=4000 + L + 7 * g + w, n_q=min(g, L))
    _full_parity(oracle, wl)


def test_mla_mfma_multiplicity_bias(oracle):
    wl = inputs.Workload("mla_bias", B=1, L=400, H=2, S=1, d_pool=512, d_sel=64, g=16, w=32, dtype="bf16", seed=5)
    _full_parity(oracle, wl, bias=math.log(16.0), dense=False)


@pytest.mark.parametrize("mode,d_pool,d_sel,S", [(inputs.MODE_MLA, 512, 64, 1), (inputs.MODE_GQA, 128, 128, 2)])
def test_strongly_redundant_latents(oracle, mode, d_pool, d_sel, S):
    """Neighbouring tokens nearly equal (AR(1) with rho = 0.9999: the regime of a few per cent relative deviation that the
    paper reports for model activations): scores inside a group are close, so near-ties are frequent, and values are large."""
    wl = inputs.Workload("redundant", B=1, L=900, H=4, S=S, d_pool=d_pool, d_sel=d_sel, g=16, w=100, dtype="bf16", mode=mode, seed=15, rho=0.9999,
                         theta=500000.0 if mode == inputs.MODE_GQA else 10000.0)
    _full_parity(oracle, wl)


def test_mla_topic_shift_inputs(oracle):
    wl = inputs.Workload("mla_topics", B=2, L=640, H=2, S=1, d_pool=512, d_sel=64, g=16, w=64, dtype="bf16", seed=9, segments=8)
    _full_parity(oracle, wl)


# ---- MFMA kernel at the GQA widths (128 / 128) --------------------------------------------------------
@pytest.mark.parametrize("B,L,g,w,H,S", [(1, 700, 16, 100, 8, 2), (1, 300, 8, 0, 4, 4), (1, 129, 16, 64, 4, 1), (2, 515, 16, 32, 4, 2),
                                           (2, 260, 4, 7, 16, 2), (1, 31, 4, 2, 8, 2), (1, 1100, 32, 256, 8, 1), (1, 333, 8, 40, 6, 2),
                                           (2, 777, 16, 128, 2, 2), (1, 513, 32, 0, 4, 2), (3, 70, 4, 5, 4, 1), (1, 1, 1, 0, 4, 1),
                                           (1, 300, 16, 50, 14, 2), (2, 200, 8, 30, 7, 1), (1, 150, 4, 10, 6, 1), (1, 130, 16, 20, 5, 1)])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_gqa_mfma_small_all_rows(oracle, B, L, g, w, H, S, dtype):
    """Any number of heads per KV head runs the 128-wide kernel: its 4 wavefronts are 4, 2 or 1 heads (the largest of
    these that divides the heads per KV head) x groups of 64 rows; 7 heads per KV head is the shape of the GQA model the
    paper reports on, 3, 5 and 6 cover the other divisors."""
    wl = inputs.Workload("gqa_small", B=B, L=L, H=H, S=S, d_pool=128, d_sel=128, g=g, w=w, dtype=dtype, mode=inputs.MODE_GQA,
                         theta=500000.0, seed=11 + L)
    _full_parity(oracle, wl)


# ---- configuration 2 at full size: sampled rows -----------------------------------------------------
@pytest.mark.parametrize("S", [1, 16])
def test_cfg2_sampled_rows(oracle, S):
    wl = inputs.configs()["cfg2"].with_(S=S)
    print(f"[case] {wl}", flush=True)
    Q, POOL, SEL = inputs.gen_all(wl)
    POOLf, SELf = inputs.to_f64(POOL, wl.dtype), inputs.to_f64(SEL, wl.dtype)
    run = hp.GpuRun(wl, Q, POOL, SEL).condense()
    Qtail = inputs.to_f64(Q[:, wl.L - wl.nq:], wl.dtype)
    ref, differ = hp.check_condense(oracle, wl, run, Qtail, POOLf, SELf)
    run.prefill().dense()
    rows = inputs.sample_rows(wl, 48)
    Qr = inputs.to_f64(Q[:, rows], wl.dtype)
    e2, e3 = hp.check_prefill(oracle, wl, run, rows, Qr, POOLf, SELf, ref, differ)
    e_d = hp.check_dense(oracle, wl, run, rows[::3], Qr[:, ::3], POOLf, SELf)
    print(f"  stage2 {e2:.2e} stage3 {e3:.2e} dense {e_d:.2e}", flush=True)
    # every row was written
    assert bool(run.O.isfinite().all()) and bool(run.O_dense.isfinite().all())


def test_results_are_deterministic(oracle):
    wl = inputs.Workload("det", B=1, L=600, H=2, S=1, d_pool=512, d_sel=64, g=16, w=64, dtype="bf16", seed=3)
    Q, POOL, SEL = inputs.gen_all(wl)
    a = hp.GpuRun(wl, Q, POOL, SEL).condense().prefill()
    b = hp.GpuRun(wl, Q, POOL, SEL).condense().prefill()
    for x, y in ((a.O, b.O), (a.pool_rep, b.pool_rep), (a.anchor, b.anchor), (a.lse, b.lse)):
        assert bool((x.view(-1) == y.view(-1)).all())


# ---- decode step over the condensed cache -------------------------------------------------------------
@pytest.mark.parametrize("mode,d_pool,d_sel,H,S,dtype", [
    (inputs.MODE_GQA, 128, 128, 8, 2, "bf16"),
    (inputs.MODE_GQA, 128, 128, 4, 4, "bf16"),
    (inputs.MODE_MLA, 512, 64, 16, 1, "bf16"),
    (inputs.MODE_MLA, 512, 64, 16, 4, "bf16"),
    (inputs.MODE_MLA, 512, 64, 8, 8, "bf16"),
    (inputs.MODE_MLA, 128, 32, 4, 1, "f32"),
    (inputs.MODE_GQA, 128, 128, 8, 2, "f16"),
    (inputs.MODE_MLA, 512, 64, 16, 1, "f16"),
    (inputs.MODE_MLA, 512, 64, 8, 8, "f16"),
    (inputs.MODE_GQA, 128, 128, 14, 2, "bf16"),      # 7 heads per KV head
    (inputs.MODE_GQA, 128, 128, 6, 2, "bf16"),
    (inputs.MODE_GQA, 128, 128, 5, 1, "f16"),
    (inputs.MODE_GQA, 128, 128, 6, 1, "bf16"),
])
@pytest.mark.parametrize("L,g,w", [(1000, 16, 100), (77, 4, 9), (50, 16, 64)])
def test_decode_step(oracle, mode, d_pool, d_sel, H, S, dtype, L, g, w):
    import torch
    from paper_2604_12452_amd import lca
    B = 3
    wl = inputs.Workload("decode", B=B, L=L, H=H, S=S, d_pool=d_pool, d_sel=d_sel, g=g, w=w, dtype=dtype, mode=mode, seed=21 + L)
    print(f"[case] {wl}", flush=True)
    Q, POOL, SEL = inputs.gen_all(wl)
    run = hp.GpuRun(wl, Q, POOL, SEL).condense(alpha=False)
    # the cache after L tokens, the newest of which is the one being decoded
    m, k = run.desc.m, run.desc.k
    if mode == inputs.MODE_MLA:
        pool_tail = run.POOL[:, None, m * g:].contiguous()
        sel_tail = run.SEL[:, None, m * g:].contiguous()
    else:
        pool_tail = run.POOL[:, m * g:].permute(0, 2, 1, 3).contiguous()
        sel_tail = run.SEL[:, m * g:].permute(0, 2, 1, 3).contiguous()
    q = run.Q[:, L - 1].contiguous()
    O = torch.full((B, H, d_pool), float("nan"), dtype=lca.torch_dtype(run.desc), device="cuda")
    lca.decode_attn(run.desc, q, run.pool_rep, run.sel_rep, pool_tail, sel_tail, O, run.ws)
    torch.cuda.synchronize()
    od = hp.oracle_desc(oracle, wl)
    ref = oracle.decode_attn(od, hp.from_dev(q, dtype), hp.from_dev(run.pool_rep, dtype), hp.from_dev(run.sel_rep, dtype),
                             hp.from_dev(pool_tail, dtype), hp.from_dev(sel_tail, dtype))
    err = hp.vec_rel_err(hp.from_dev(O, dtype), ref)
    print(f"  decode err {err:.2e}", flush=True)
    assert err <= hp.TOL[dtype]


# ---- rows whose later logits dwarf the first tile's: the kernel's repeat pass ---------------------------
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("dense_only", [False, True])
def test_mla_logits_far_above_first_tile(oracle, dense_only, dtype):
    """A key late in the sequence scores ~100 nats above everything in the first key tile of each row.  The
    MLA kernel fixes its softmax reference at the first tile and must notice that its exponent headroom
    (2^60; fp16: 2^19) is exceeded and repeat the pass; the result must still match the oracle."""
    wl = inputs.Workload("mla_spike", B=1, L=420, H=2, S=1, d_pool=512, d_sel=64, g=16, w=64, dtype=dtype, seed=77)
    Q, POOL, SEL = inputs.gen_all(wl)
    Qf = inputs.to_f64(Q, wl.dtype)
    # make tokens 300 (raw window of the last rows) and 40 (inside a condensed group) line up with the queries' mean direction
    qdir = Qf[0, :, :, :512].mean(axis=(0, 1))
    qdir /= np.linalg.norm(qdir)
    POOLf = inputs.to_f64(POOL, wl.dtype)
    # pick the size so that <q, c> is around 100 for typical q: the queries share a common component along qdir
    Qf[0, :, :, :512] += 2.0 * qdir
    for tok in (40, 300):
        POOLf[0, tok] = 50.0 * qdir
    Q = inputs.to_storage(Qf, wl.dtype)
    POOL = inputs.to_storage(POOLf, wl.dtype)
    Qf, POOLf, SELf = (inputs.to_f64(x, wl.dtype) for x in (Q, POOL, SEL))
    run = hp.GpuRun(wl, Q, POOL, SEL).condense()
    ref, differ = hp.check_condense(oracle, wl, run, Qf[:, wl.L - wl.nq:], POOLf, SELf)
    rows = np.arange(wl.L, dtype=np.int32)
    keys = np.concatenate([POOLf[0], SELf[0]], -1)
    logits = keys[:351] @ Qf[0, 350, 0]
    spread = logits.max() - logits[:32].max()
    assert spread > 60.0, f"the test input must exceed the kernel's headroom (spread {spread:.1f} nats)"
    if dense_only:
        run.dense()
        hp.check_dense(oracle, wl, run, rows, Qf, POOLf, SELf)
    else:
        run.prefill()
        hp.check_prefill(oracle, wl, run, rows, Qf, POOLf, SELf, ref, differ)


@pytest.mark.parametrize("gain", [7.0, 9.0, 11.0, 13.0])
def test_mla_fp16_logits_around_the_type_limit(oracle, gain):
    """fp16 exponentials end at 65504 = 2^16: with the reference 4 binades above a row's first maximum, a later logit
    up to ~2^20 times (13.9 nats) larger still fits, one beyond makes the kernel repeat the item.  The gains put the
    largest logit of the late rows on both sides of that limit; every case must match the oracle."""
    wl = inputs.Workload("mla_limit16", B=1, L=420, H=2, S=1, d_pool=512, d_sel=64, g=16, w=64, dtype="f16", seed=79)
    Q, POOL, SEL = inputs.gen_all(wl)
    Qf, POOLf = inputs.to_f64(Q, wl.dtype), inputs.to_f64(POOL, wl.dtype)
    qdir = Qf[0, :, :, :512].mean(axis=(0, 1))
    qdir /= np.linalg.norm(qdir)
    Qf[0, :, :, :512] += 2.0 * qdir
    for tok in (40, 300):
        POOLf[0, tok] = gain * qdir
    Q, POOL = inputs.to_storage(Qf, wl.dtype), inputs.to_storage(POOLf, wl.dtype)
    Qf, POOLf, SELf = (inputs.to_f64(x, wl.dtype) for x in (Q, POOL, SEL))
    keys = np.concatenate([POOLf[0], SELf[0]], -1)
    spreads = []
    for t in range(301, wl.L):
        for h in range(wl.H):
            lg = keys[:t + 1] @ Qf[0, t, h]
            spreads.append(lg.max() - lg[:32].max())
    print(f"  gain {gain}: largest logit above the first tile's maximum by {min(spreads):.1f} .. {max(spreads):.1f} nats", flush=True)
    run = hp.GpuRun(wl, Q, POOL, SEL).condense()
    ref, differ = hp.check_condense(oracle, wl, run, Qf[:, wl.L - wl.nq:], POOLf, SELf)
    rows = np.arange(wl.L, dtype=np.int32)
    run.prefill()
    hp.check_prefill(oracle, wl, run, rows, Qf, POOLf, SELf, ref, differ)
    run.dense()
    hp.check_dense(oracle, wl, run, rows, Qf, POOLf, SELf)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("dense_only", [False, True])
def test_gqa_logits_far_above_first_tile(oracle, dense_only, dtype):
    """The same situation at the GQA widths: keys of two tokens score ~100 nats above the first key tile, in
    every KV head, so the 128-wide kernel's repeat pass has to run."""
    wl = inputs.Workload("gqa_spike", B=1, L=420, H=8, S=2, d_pool=128, d_sel=128, g=16, w=64, dtype=dtype, mode=inputs.MODE_GQA,
                         theta=500000.0, seed=78)
    Q, POOL, SEL = inputs.gen_all(wl)
    Qf, SELf = inputs.to_f64(Q, wl.dtype), inputs.to_f64(SEL, wl.dtype)
    qdir = Qf[0].mean(axis=(0, 1))
    qdir /= np.linalg.norm(qdir)
    Qf[0] += 2.0 * qdir
    for tok in (100, 300):                  # both beyond the first 64-key tile of plain causal attention
        SELf[0, tok] = 50.0 * qdir
    Q, SEL = inputs.to_storage(Qf, wl.dtype), inputs.to_storage(SELf, wl.dtype)
    Qf, POOLf, SELf = (inputs.to_f64(x, wl.dtype) for x in (Q, POOL, SEL))
    run = hp.GpuRun(wl, Q, POOL, SEL).condense()
    ref, differ = hp.check_condense(oracle, wl, run, Qf[:, wl.L - wl.nq:], POOLf, SELf)
    rows = np.arange(wl.L, dtype=np.int32)
    logits = SELf[0, :351, 0] @ Qf[0, 350, 0]
    spread = logits.max() - logits[:64].max()
    assert spread > 60.0, f"the test input must exceed the kernel's headroom (spread {spread:.1f} nats)"
    if dense_only:
        run.dense()
        hp.check_dense(oracle, wl, run, rows, Qf, POOLf, SELf)
    else:
        run.prefill()
        hp.check_prefill(oracle, wl, run, rows, Qf, POOLf, SELf, ref, differ)


# ---- the ablation's alternative pooling strategies (section 5.4, Table 5) ---------------------------------
REDUCE_NAMES = {1: "weighted", 2: "mean", 3: "maxsel", 4: "maxpool"}


@pytest.mark.parametrize("dtype,mode", [("f32", inputs.MODE_MLA), ("bf16", inputs.MODE_GQA), ("bf16", inputs.MODE_MLA)])
@pytest.mark.parametrize("pool_reduce", [1, 2, 3, 4])
@pytest.mark.parametrize("sel_reduce", [1, 2, 3, 4])
def test_condense_reduce_strategies(oracle, dtype, mode, pool_reduce, sel_reduce):
    """Every cell of the grid: lca_condense with the given strategies against the oracle with the same ones.
    Summed components within tolerance; selected components are bit-exact copies of a row of the group —
    the anchor's row for max selection, a row of (numerically) largest norm for max pooling."""
    wl = _wl("reduce", L=203, g=8, w=11, H=4, S=2, dtype=dtype, mode=mode, d_pool=24, d_sel=16, B=2)
    Q, POOL, SEL = inputs.gen_all(wl)
    Qf, POOLf, SELf = (inputs.to_f64(x, wl.dtype) for x in (Q, POOL, SEL))
    run = hp.GpuRun(wl, Q, POOL, SEL)
    run.desc.pool_reduce, run.desc.sel_reduce = pool_reduce, sel_reduce
    run.condense()
    od = hp.oracle_desc(oracle, wl, pool_reduce=pool_reduce, sel_reduce=sel_reduce)
    ref = oracle.condense(od, oracle.summary_query(od, Qf[:, wl.L - wl.nq:]), POOLf, SELf)
    anchor = run.anchor.cpu().numpy()
    differ = anchor != ref["anchor"]
    assert not (differ & (ref["margin"] > hp.ANCHOR_MARGIN)).any(), "anchor mismatch above the score margin"
    for name, strat, X, got_t, want in (("pool", pool_reduce, POOLf, run.pool_rep, ref["pool_rep"]),
                                        ("sel", sel_reduce, SELf, run.sel_rep, ref["sel_rep"])):
        got = hp.from_dev(got_t, wl.dtype)
        if strat in (1, 2):
            keep = ~differ if strat == 1 else np.ones_like(differ)
            err = hp.vec_rel_err(got[keep], want[keep])
            assert err <= hp.TOL[wl.dtype], f"{name} component ({REDUCE_NAMES[strat]}) rel err {err:.3e}"
            continue
        for b in range(wl.B):
            for s in range(wl.S):
                rows_all = X[b] if wl.mode == inputs.MODE_MLA else X[b, :, s]
                for j in range(od.m):
                    grp = rows_all[j * wl.g:(j + 1) * wl.g]
                    if strat == 3:
                        np.testing.assert_array_equal(got[b, s, j], rows_all[anchor[b, s, j]])
                    else:
                        n2 = (grp * grp).sum(-1)
                        hits = [r for r in range(wl.g) if (got[b, s, j] == grp[r]).all()]
                        assert hits and n2[hits[0]] >= n2.max() * (1 - 1e-5), f"{name} component: not a row of largest norm"


# ---- per-token deviation statistics (Theorem 1's delta_k, delta_v; appendix, Tables 9-10) --------------------
@pytest.mark.parametrize("dtype,mode,d_pool,d_sel,L,g,w,S", [
    ("f32", inputs.MODE_MLA, 24, 16, 333, 4, 10, 2), ("bf16", inputs.MODE_GQA, 128, 128, 700, 16, 100, 2),
    ("bf16", inputs.MODE_MLA, 512, 64, 1200, 16, 64, 1), ("bf16", inputs.MODE_MLA, 24, 16, 40, 16, 64, 1)])
def test_deviation_stats(oracle, dtype, mode, d_pool, d_sel, L, g, w, S):
    """lca_deviation_stats on the cache lca_condense emitted against the oracle on the same (rounded) cache."""
    import torch
    from paper_2604_12452_amd import lca
    wl = _wl("deviation", L=L, g=g, w=w, H=4, S=S, dtype=dtype, mode=mode, d_pool=d_pool, d_sel=d_sel, B=2)
    Q, POOL, SEL = inputs.gen_all(wl)
    run = hp.GpuRun(wl, Q, POOL, SEL).condense(alpha=False)
    stats = torch.full((wl.B, wl.S, 6), float("nan"), dtype=torch.float32, device="cuda")
    lca.deviation_stats(run.desc, run.POOL, run.SEL, run.pool_rep, run.sel_rep, stats, run.ws)
    torch.cuda.synchronize()
    od = hp.oracle_desc(oracle, wl)
    ref = oracle.deviation_stats(od, inputs.to_f64(POOL, dtype), inputs.to_f64(SEL, dtype), hp.from_dev(run.pool_rep, dtype),
                                 hp.from_dev(run.sel_rep, dtype))
    got = stats.cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(got, ref, rtol=2e-5, atol=1e-7)      # fp32 sums of at most a few thousand terms against fp64
    if od.m == 0:
        assert (got == 0).all()


# ---- attention with the value up-projection fused into the kernel's epilogue ---------------------------------
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("L,g,w,H,S,B", [(700, 16, 100, 2, 1, 1), (300, 8, 64, 4, 2, 2), (129, 16, 16, 3, 1, 1), (40, 4, 4, 4, 2, 3), (1, 1, 0, 1, 1, 1)])
def test_mla_prefill_with_fused_up_projection(oracle, dtype, L, g, w, H, S, B):
    """lca_prefill_attn_up against the oracle's attention followed by the oracle's up-projection (every row), and against
    the library's own two-step result: its latent output, rounded as stored, projected in float64."""
    import torch
    from paper_2604_12452_amd import lca
    wl = inputs.Workload("mla_up", B=B, L=L, H=H, S=S, d_pool=512, d_sel=64, g=g, w=w, dtype=dtype, seed=57 + L)
    print(f"[case] {wl}", flush=True)
    Q, POOL, SEL = inputs.gen_all(wl)
    Qf, POOLf, SELf = (inputs.to_f64(x, wl.dtype) for x in (Q, POOL, SEL))
    rng = np.random.default_rng(5 + L)
    W = inputs.to_storage(rng.standard_normal((H, 128, 512)) / np.sqrt(512.0), dtype)      # [H, d_up, d_c]
    Wf = inputs.to_f64(W, dtype)
    run = hp.GpuRun(wl, Q, POOL, SEL).condense()
    ref, differ = hp.check_condense(oracle, wl, run, Qf[:, wl.L - wl.nq:], POOLf, SELf)
    run.prefill()
    tdt = lca.torch_dtype(run.desc)
    O_up = torch.full((B, L, H, 128), float("nan"), dtype=tdt, device="cuda")
    lse = torch.full((B, L, H), float("nan"), dtype=torch.float32, device="cuda")
    lca.prefill_attn_up(run.desc, run.Q, run.POOL, run.SEL, run.pool_rep, run.sel_rep, hp.to_dev(W, dtype), O_up, lse, run.ws)
    torch.cuda.synchronize()
    got = hp.from_dev(O_up, dtype)
    assert np.isfinite(got).all()
    # (a) the oracle end to end: attention over the GPU's own emitted cache (its rounded representatives and anchors), then W
    od = hp.oracle_desc(oracle, wl)
    rows = np.arange(L, dtype=np.int32)
    O_lat, lse_ref = oracle.lca_attn_rows(od, rows, Qf, POOLf, SELf, hp.from_dev(run.pool_rep, dtype), hp.from_dev(run.sel_rep, dtype), want_lse=True)
    want = oracle.up_project(O_lat, Wf)
    err = hp.vec_rel_err(got, want)
    # (b) the two-step path of the library itself
    two_step = oracle.up_project(hp.from_dev(run.O, dtype), Wf)
    err2 = hp.vec_rel_err(got, two_step)
    print(f"  fused up-projection: err {err:.2e} against the oracle, {err2:.2e} against the library's latent output projected in float64", flush=True)
    assert err <= hp.TOL[dtype] and err2 <= hp.TOL[dtype]
    assert np.abs(lse.cpu().numpy().astype(np.float64) - lse_ref).max() <= hp.LSE_TOL[dtype]


# ---- the 1/sqrt(d) factor of Eq. 6 and Eq. 10: desc.scale through every kernel ---------------------------------
_SCALE_KERNELS = {
    # name: (mode, d_pool, d_sel, dtype, H, S)
    "mla_mfma_bf16": (inputs.MODE_MLA, 512, 64, "bf16", 4, 2),
    "mla_mfma_f16": (inputs.MODE_MLA, 512, 64, "f16", 2, 1),
    "gqa_mfma_bf16": (inputs.MODE_GQA, 128, 128, "bf16", 8, 2),
    "gqa_mfma_f16": (inputs.MODE_GQA, 128, 128, "f16", 4, 2),
    "cfg1_widths_f32": (inputs.MODE_MLA, 128, 32, "f32", 4, 1),
    "generic_f32_mla": (inputs.MODE_MLA, 24, 16, "f32", 4, 2),
    "generic_bf16_gqa": (inputs.MODE_GQA, 24, 16, "bf16", 4, 2),
}


@pytest.mark.parametrize("which", ["rsqrt_d", "odd", "large"])
@pytest.mark.parametrize("kernel", sorted(_SCALE_KERNELS))
def test_scale_enters_scores_and_logits(oracle, kernel, which):
    """desc.scale != 1 through condensation (Eq. 6: s_i = scale <qbar, k_i>), LCA prefill and the dense baseline (Eq. 10,
    Eq. 5: logits scale <q, k>), at both matrix-core widths in both 16-bit types and in the general kernels.  'rsqrt_d'
    is the paper's 1/sqrt(d) with unit-variance queries, 'odd' is 0.37 with the benchmark's query distribution, 'large'
    is 3.0 (sharper softmax than any benchmark input).  A scale applied twice, or left out of either place, moves the
    weights and the outputs far beyond the tolerance."""
    mode, d_pool, d_sel, dtype, H, S = _SCALE_KERNELS[kernel]
    d_qk = d_pool + d_sel if mode == inputs.MODE_MLA else d_sel
    scale, qv = {"rsqrt_d": (1.0 / math.sqrt(d_qk), 1), "odd": (0.37, 0), "large": (3.0, 0)}[which]
    wl = inputs.Workload("scale", B=2, L=300, H=H, S=S, d_pool=d_pool, d_sel=d_sel, g=8, w=40, dtype=dtype, mode=mode, seed=61,
                         q_var_dim=qv, scale=scale, theta=500000.0 if mode == inputs.MODE_GQA else 10000.0)
    run = _full_parity(oracle, wl)
    assert abs(run.desc.scale - scale) < 1e-7


@pytest.mark.parametrize("scale", [0.0, -0.5])
@pytest.mark.parametrize("mode,d_pool,d_sel,dtype", [(inputs.MODE_MLA, 512, 64, "bf16"), (inputs.MODE_GQA, 128, 128, "bf16"),
                                                      (inputs.MODE_MLA, 512, 64, "f16"), (inputs.MODE_MLA, 24, 16, "f32")])
def test_zero_and_negative_scale(oracle, scale, mode, d_pool, d_sel, dtype):
    """A zero scale makes every weight uniform (plain averages, lowest index as anchor) and a negative one turns the order of the
    scores around; the matrix-core kernels only take positive scales, so these descriptors run the general attention kernel."""
    wl = inputs.Workload("scale_le0", B=1, L=200, H=4, S=2, d_pool=d_pool, d_sel=d_sel, g=8, w=24, dtype=dtype, mode=mode, seed=62,
                         scale=scale, theta=500000.0 if mode == inputs.MODE_GQA else 10000.0)
    run = _full_parity(oracle, wl)
    if scale == 0.0:
        m = run.desc.m
        assert np.array_equal(run.anchor.cpu().numpy(), np.broadcast_to(np.arange(m) * wl.g, (wl.B, wl.S, m)))


# ---- exact ties: equal rows inside a group (Eq. 8: the lowest index wins) ---------------------------------------------
@pytest.mark.parametrize("g", [2, 3, 4, 8, 16, 32, 64])
@pytest.mark.parametrize("mode,d_pool,d_sel,dtype,S", [
    (inputs.MODE_MLA, 512, 64, "bf16", 1), (inputs.MODE_MLA, 512, 64, "bf16", 4), (inputs.MODE_MLA, 512, 64, "f16", 2),
    (inputs.MODE_GQA, 128, 128, "bf16", 2), (inputs.MODE_GQA, 128, 128, "f16", 1), (inputs.MODE_MLA, 128, 32, "f32", 2),
    (inputs.MODE_MLA, 24, 16, "f32", 2), (inputs.MODE_GQA, 24, 16, "bf16", 2)])
def test_exact_ties_take_the_lowest_index(oracle, g, mode, d_pool, d_sel, dtype, S):
    """In two groups out of three the top-scoring token (of set / KV head 0) is copied over another token of its group, earlier or
    later, so that two tokens hold the group's largest score exactly.  The oracle's margin is then exactly zero there and
    both sides must name the lower of the two positions."""
    wl = inputs.Workload("ties", B=2, L=40 + 12 * g, H=4, S=S, d_pool=d_pool, d_sel=d_sel, g=g, w=40, dtype=dtype, mode=mode, seed=300 + g,
                         theta=500000.0 if mode == inputs.MODE_GQA else 10000.0)
    print(f"[case] {wl}", flush=True)
    Q, POOL, SEL = inputs.gen_all(wl)
    Qf, POOLf, SELf = (inputs.to_f64(x, wl.dtype) for x in (Q, POOL, SEL))
    od = hp.oracle_desc(oracle, wl)
    qbar = oracle.summary_query(od, Qf[:, wl.L - wl.nq:])
    first = oracle.condense(od, qbar, POOLf, SELf)
    planted = np.zeros((wl.B, od.m), dtype=bool)
    expect = np.zeros((wl.B, od.m), dtype=np.int64)
    for b in range(wl.B):
        for j in range(od.m):
            if j % 3 == 2:
                continue
            top = int(first["anchor"][b, 0, j])
            r = top - j * g
            other = j * g + ((r + 1 + (j * 7) % (g - 1)) % g)          # another position of the group, before or after the top one
            assert other != top
            for X in (POOL, SEL):
                X[b, other] = X[b, top]                                 # MLA: the token's rows; GQA: all KV heads' rows of the token
            planted[b, j], expect[b, j] = True, min(top, other)
    POOLf, SELf = inputs.to_f64(POOL, wl.dtype), inputs.to_f64(SEL, wl.dtype)
    ref = oracle.condense(od, qbar, POOLf, SELf)
    assert (ref["margin"][:, 0][planted] == 0.0).all() and np.array_equal(ref["anchor"][:, 0][planted], expect[planted])
    run = hp.GpuRun(wl, Q, POOL, SEL).condense()
    ref2, differ = hp.check_condense(oracle, wl, run, Qf[:, wl.L - wl.nq:], POOLf, SELf)
    got = run.anchor.cpu().numpy()
    assert np.array_equal(got[:, 0][planted], expect[planted]), "a tie between equal rows did not go to the lowest index"
    ties = ref2["margin"] == 0.0
    assert np.array_equal(got[ties], ref2["anchor"][ties])
    print(f"  {int(planted.sum())} planted ties, {int(ties.sum())} exact ties over all sets", flush=True)


# ---- the number of summary queries (Table 8: 8, 16, 32 at g = 16) ----------------------------------------------------
@pytest.mark.parametrize("n_q", [1, 8, 32, 50])
@pytest.mark.parametrize("mode,d_pool,d_sel,dtype,H,S", [
    (inputs.MODE_MLA, 512, 64, "bf16", 16, 1), (inputs.MODE_MLA, 512, 64, "f16", 4, 2), (inputs.MODE_GQA, 128, 128, "bf16", 8, 2),
    (inputs.MODE_MLA, 128, 32, "f32", 4, 1), (inputs.MODE_GQA, 24, 16, "bf16", 4, 4)])
def test_number_of_summary_queries_differs_from_group_size(oracle, n_q, mode, d_pool, d_sel, dtype, H, S):
    """n_q != g with groups present: the summary query averages the last n_q positions whatever the group size is, and
    everything downstream (weights, anchors, representatives, attention over them) follows it."""
    wl = inputs.Workload("n_q", B=2, L=360, H=H, S=S, d_pool=d_pool, d_sel=d_sel, g=16, w=70, n_q=n_q, dtype=dtype, mode=mode, seed=400 + n_q,
                         theta=500000.0 if mode == inputs.MODE_GQA else 10000.0)
    _full_parity(oracle, wl, dense=False)


# ---- representatives counted g times (the normaliser of appendix A.2): rep_logit_bias = ln g -----------------------------
@pytest.mark.parametrize("mode,d_pool,d_sel,dtype,H,S,g", [
    (inputs.MODE_GQA, 128, 128, "bf16", 8, 2, 16), (inputs.MODE_GQA, 128, 128, "f16", 4, 1, 8), (inputs.MODE_GQA, 128, 128, "bf16", 6, 2, 4),
    (inputs.MODE_MLA, 512, 64, "f16", 2, 1, 16), (inputs.MODE_MLA, 24, 16, "f32", 4, 2, 4), (inputs.MODE_GQA, 24, 16, "bf16", 4, 2, 8)])
def test_multiplicity_bias_all_kernels(oracle, mode, d_pool, d_sel, dtype, H, S, g):
    wl = inputs.Workload("bias", B=2, L=400, H=H, S=S, d_pool=d_pool, d_sel=d_sel, g=g, w=32, dtype=dtype, mode=mode, seed=500 + g,
                         theta=500000.0 if mode == inputs.MODE_GQA else 10000.0)
    _full_parity(oracle, wl, bias=math.log(float(g)), dense=False)


@pytest.mark.parametrize("mode,d_pool,d_sel,H,S,dtype", [
    (inputs.MODE_GQA, 128, 128, 8, 2, "bf16"), (inputs.MODE_MLA, 512, 64, 16, 1, "bf16"), (inputs.MODE_MLA, 512, 64, 8, 8, "f16"),
    (inputs.MODE_MLA, 128, 32, 4, 1, "f32")])
def test_decode_step_with_multiplicity_bias_and_scale(oracle, mode, d_pool, d_sel, H, S, dtype):
    """One decode step with rep_logit_bias = ln g and a scale other than 1 against the oracle's decode step (which equals
    the last prefill row by its own pin)."""
    import torch
    from paper_2604_12452_amd import lca
    B, L, g, w = 3, 500, 16, 60
    wl = inputs.Workload("decode_bias", B=B, L=L, H=H, S=S, d_pool=d_pool, d_sel=d_sel, g=g, w=w, dtype=dtype, mode=mode, seed=77, scale=0.6,
                         theta=500000.0 if mode == inputs.MODE_GQA else 10000.0)
    print(f"[case] {wl}", flush=True)
    Q, POOL, SEL = inputs.gen_all(wl)
    bias = math.log(float(g))
    run = hp.GpuRun(wl, Q, POOL, SEL, rep_logit_bias=bias).condense(alpha=False)
    m = run.desc.m
    if mode == inputs.MODE_MLA:
        pool_tail, sel_tail = run.POOL[:, None, m * g:].contiguous(), run.SEL[:, None, m * g:].contiguous()
    else:
        pool_tail, sel_tail = run.POOL[:, m * g:].permute(0, 2, 1, 3).contiguous(), run.SEL[:, m * g:].permute(0, 2, 1, 3).contiguous()
    q = run.Q[:, L - 1].contiguous()
    O = torch.full((B, H, d_pool), float("nan"), dtype=lca.torch_dtype(run.desc), device="cuda")
    lca.decode_attn(run.desc, q, run.pool_rep, run.sel_rep, pool_tail, sel_tail, O, run.ws)
    torch.cuda.synchronize()
    od = hp.oracle_desc(oracle, wl, rep_logit_bias=bias)
    ref = oracle.decode_attn(od, hp.from_dev(q, dtype), hp.from_dev(run.pool_rep, dtype), hp.from_dev(run.sel_rep, dtype),
                             hp.from_dev(pool_tail, dtype), hp.from_dev(sel_tail, dtype))
    nobias = oracle.decode_attn(hp.oracle_desc(oracle, wl), hp.from_dev(q, dtype), hp.from_dev(run.pool_rep, dtype),
                                hp.from_dev(run.sel_rep, dtype), hp.from_dev(pool_tail, dtype), hp.from_dev(sel_tail, dtype))
    got = hp.from_dev(O, dtype)
    err = hp.vec_rel_err(got, ref)
    print(f"  decode err {err:.2e} (the same step without the bias differs by {hp.vec_rel_err(nobias, ref):.2e})", flush=True)
    assert err <= hp.TOL[dtype]
    assert hp.vec_rel_err(nobias, ref) > 10 * hp.TOL[dtype], "the bias must matter on this input, or the case proves nothing"


# ---- condensation with several sets at the MLA widths: the matrix-core kernel ------------------------------------------------
@pytest.mark.parametrize("B,L,H,S,g,w,n_q,scale,dtype", [
    (1, 700, 16, 16, 16, 100, 0, 1.0, "bf16"),        # one set per head, the benchmark's variant
    (2, 1500, 16, 16, 16, 37, 0, 1.0, "f16"),         # more groups than wavefronts in a small grid, two sequences
    (1, 900, 8, 4, 32, 64, 0, 1.0, "bf16"),           # two tiles per group (online softmax across them), two heads per set
    (2, 1000, 12, 3, 48, 20, 5, 0.37, "bf16"),        # three tiles per group, three sets, n_q != g, scale != 1
    (1, 1300, 16, 8, 64, 10, 64, 1.0, "f16"),         # four tiles per group
    (3, 200, 6, 6, 16, 8, 3, -0.5, "bf16"),           # a negative scale turns the order of the scores around
    (1, 300, 5, 5, 16, 12, 0, 0.0, "f16"),            # zero scale: uniform weights, the first row of each group
    (1, 4500, 32, 16, 16, 64, 0, 3.0, "bf16"),        # sharp weights, two heads per set, several tiles per wavefront
])
def test_condense_matrix_core_kernel(oracle, B, L, H, S, g, w, n_q, scale, dtype):
    """lca_condense where it runs on the matrix cores (MLA widths, at least three sets, groups of whole 16-row tiles): weights,
    anchors, copied keys and pooled vectors against the oracle; the summary query and the weights enter the products as hi + lo
    pairs of 16-bit numbers, so the weights must still agree to 1e-4 and the anchors wherever the margin allows."""
    wl = inputs.Workload("condense_mc", B=B, L=L, H=H, S=S, d_pool=512, d_sel=64, g=g, w=w, n_q=n_q, dtype=dtype, seed=600 + L, scale=scale)
    print(f"[case] {wl}", flush=True)
    Q, POOL, SEL = inputs.gen_all(wl)
    run = hp.GpuRun(wl, Q, POOL, SEL).condense(alpha=True)
    hp.check_condense(oracle, wl, run, inputs.to_f64(Q[:, wl.L - wl.nq:], wl.dtype), inputs.to_f64(POOL, wl.dtype), inputs.to_f64(SEL, wl.dtype))
    # without the weights' debug output the kernel takes the same path otherwise: identical representatives
    again = hp.GpuRun(wl, Q, POOL, SEL).condense(alpha=False)
    for x, y in ((run.pool_rep, again.pool_rep), (run.sel_rep, again.sel_rep), (run.anchor, again.anchor)):
        assert bool((x.view(-1) == y.view(-1)).all())


def _random_condense_mc_shapes(n, seed):
    """Seeded draws of shapes the matrix-core condensation kernel takes: 3..16 sets, groups of 1..4 tiles, lengths from fewer
    groups than wavefronts to several groups per wavefront, several sequences, heads per set 1..3, n_q around g."""
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        S = int(rng.integers(3, 17))
        hps = int(rng.choice([1, 1, 2, 3]))
        g = int(rng.choice([16, 16, 32, 48, 64]))
        m = int(rng.choice([1, 2, 3, 5, 17, 40, 130]))
        w = int(rng.choice([0, 1, 16, 33, 100]))
        L = w + m * g + int(rng.integers(0, g))
        n_q = int(rng.choice([0, 1, g // 2, g + 3]))
        out.append((int(rng.integers(1, 4)), L, S * hps, S, g, w, min(n_q, L), str(rng.choice(["bf16", "f16"]))))
    return out


@pytest.mark.parametrize("B,L,H,S,g,w,n_q,dtype", _random_condense_mc_shapes(20, 2028))
def test_condense_matrix_core_kernel_random_shapes(oracle, B, L, H, S, g, w, n_q, dtype):
    wl = inputs.Workload("condense_mc_rand", B=B, L=L, H=H, S=S, d_pool=512, d_sel=64, g=g, w=w, n_q=n_q, dtype=dtype, seed=700 + L + S)
    print(f"[case] {wl}", flush=True)
    Q, POOL, SEL = inputs.gen_all(wl)
    run = hp.GpuRun(wl, Q, POOL, SEL).condense(alpha=True)
    assert run.desc.m == (L - w) // g
    hp.check_condense(oracle, wl, run, inputs.to_f64(Q[:, wl.L - wl.nq:], wl.dtype), inputs.to_f64(POOL, wl.dtype), inputs.to_f64(SEL, wl.dtype))
