"""C-ABI checks that need no GPU: the library loads, exports everything include/lca.h declares, and its
host-side validation rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

from paper_2604_12452_amd import lca

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(lca.LIB_PATH):
        from paper_2604_12452_amd import build
        build.build(verbose=False)
    return lca.load()


def _declared():
    text = open(os.path.join(ROOT, "include", "lca.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return re.findall(r"\b(?:lca_status|const char \*)\s*\*?\s*(\w+)\s*\(", text)


def test_every_declared_symbol_is_exported(lib):
    names = _declared()
    assert set(names) == set(lca.EXPORTS) and len(names) == 17
    for n in names:
        assert hasattr(lib, n)


def _desc(**kw):
    base = dict(B=1, L=8192, H=16, S=1, d_pool=512, d_sel=64, g=16, w=1024)
    base.update(kw)
    return lca.Desc(**base)


def test_workspace_and_cache_bytes_are_host_only(lib):
    assert lca.workspace_size(_desc()) >= 576 * 4
    assert lca.cache_bytes(_desc(L=131072)) == (150994944, 10543104)
    assert lca.cache_bytes(_desc(L=131072, g=32)) == (150994944, 5861376)
    assert lca.cache_bytes(_desc(L=131072, S=16)) == (150994944, 150994944)
    gqa = lca.Desc(B=1, L=65536, H=32, S=8, d_pool=128, d_sel=128, g=16, w=1024, mode=lca.MODE_GQA)
    assert lca.cache_bytes(gqa) == (268435456, 20709376)
    assert lca.workspace_size(_desc(dtype=lca.F16)) == lca.workspace_size(_desc())      # both 16-bit types are accepted
    assert lca.workspace_size(lca.Desc(B=32, L=65537, H=32, S=8, d_pool=128, d_sel=128, g=16, w=1024, mode=lca.MODE_GQA)) > 0


def test_condensed_rows_follow_the_partition_of_section_4_2(lib):
    """m = floor((L - w) / g) groups, k = w + (L - w) mod g raw tokens, every token accounted for (m g + k = L)."""
    for L, w, g in [(131072, 1024, 16), (131072, 1024, 32), (1024, 128, 16), (1000, 100, 16), (77, 9, 4), (100, 200, 16), (40, 40, 4), (5, 0, 8),
                    (65537, 1024, 16)]:
        d = _desc(L=L, w=w, g=g)
        m, k = lca.condensed_rows(d)
        assert (m, k) == (d.m, d.k)
        assert m * g + k == L and m >= 0
        if L > w:
            assert k == w + (L - w) % g and m == (L - w - (L - w) % g) // g
        else:
            assert (m, k) == (0, L)
    assert lca.condensed_rows(_desc(L=65537)) == (4032, 1025)
    cd = _desc().c()
    assert lib.lca_condensed_rows(ctypes.byref(cd), None, None) == lca.ERR_INVALID_ARG


def test_binding_rejects_tensors_that_do_not_fit_the_descriptor(lib):
    """The binding compares every tensor with the size and element type the header documents before the library is
    called: a mismatch raises ValueError and nothing is launched (CPU tensors here; a tensor of the right size and type
    that is not on the device is rejected as well)."""
    import torch
    d = lca.Desc(B=1, L=64, H=2, S=1, d_pool=512, d_sel=64, g=4, w=8)
    m = d.m
    bf = lambda *shape: torch.zeros(shape, dtype=torch.bfloat16)
    Q, POOL, SEL = bf(1, 64, 2, 576), bf(1, 64, 512), bf(1, 64, 64)
    pr, sr, an = bf(1, 1, m, 512), bf(1, 1, m, 64), torch.zeros((1, 1, m), dtype=torch.int32)
    O, ws = bf(1, 64, 2, 512), torch.zeros(1 << 16, dtype=torch.uint8)
    bad = [
        ("Q holds", lambda: lca.condense(d, Q[:, :63].contiguous(), POOL, SEL, pr, sr, an, None, ws)),
        ("POOL has dtype", lambda: lca.condense(d, Q, POOL.float(), SEL, pr, sr, an, None, ws)),
        ("SEL holds", lambda: lca.condense(d, Q, POOL, SEL[:, :, :32].contiguous(), pr, sr, an, None, ws)),
        ("pool_rep holds", lambda: lca.condense(d, Q, POOL, SEL, pr[:, :, :m - 1].contiguous(), sr, an, None, ws)),
        ("anchor_idx has dtype", lambda: lca.condense(d, Q, POOL, SEL, pr, sr, an.long(), None, ws)),
        ("alpha_dbg holds", lambda: lca.condense(d, Q, POOL, SEL, pr, sr, an, torch.zeros(m * 4 - 1), ws)),
        ("O holds", lambda: lca.prefill_attn(d, Q, POOL, SEL, pr, sr, O[:, :, :1].contiguous(), None, ws)),
        ("lse has dtype", lambda: lca.prefill_attn(d, Q, POOL, SEL, pr, sr, O, torch.zeros((1, 64, 2), dtype=torch.float64), ws)),
        ("O is required", lambda: lca.dense_attn(d, Q, POOL, SEL, None, None, ws)),
        ("sel_rep holds", lambda: lca.prefill_attn(d, Q, POOL, SEL, pr, sr[:, :, 1:].contiguous(), O, None, ws)),
        ("pool_tail holds", lambda: lca.decode_attn(lca.Desc(B=1, L=64, H=16, S=1, d_pool=512, d_sel=64, g=4, w=8), bf(1, 16, 576), pr, sr,
                                                    bf(1, 1, d.k - 1, 512), bf(1, 1, d.k, 64), bf(1, 16, 512), ws)),
        ("pool_rep holds", lambda: lca.decode_attn_cached(lca.Desc(B=1, L=64, H=16, S=1, d_pool=512, d_sel=64, g=4, w=8),
                                                          lca.CacheLayout(m_cap=m + 4, k_cap=d.k + 4), bf(1, 16, 576), pr, sr,
                                                          bf(1, 1, d.k + 4, 512), bf(1, 1, d.k + 4, 64), bf(1, 16, 512), ws)),
        ("q_recent holds", lambda: lca.cache_update(d, lca.CacheLayout(m_cap=m, k_cap=12), bf(1, 3, 2, 576), bf(1, 1, 12, 512), bf(1, 1, 12, 64),
                                                    pr, sr, an, ws)),
        ("pool_q8 has dtype", lambda: lca.quantize_cache(d, None, pr, sr, pr, sr, torch.zeros((1, 1, m, 2)))),
        ("stats holds", lambda: lca.deviation_stats(d, POOL, SEL, pr, sr, torch.zeros(5), ws)),
        ("is not a device tensor", lambda: lca.condense(d, Q, POOL, SEL, pr, sr, an, None, ws)),
    ]
    for needle, call in bad:
        with pytest.raises(ValueError) as e:
            call()
        assert needle in str(e.value), (needle, str(e.value))


@pytest.mark.parametrize("kw", [dict(B=0), dict(L=0), dict(H=15, S=2), dict(g=0), dict(g=65), dict(w=-1), dict(n_q=-1),
                                dict(mode=2), dict(dtype=7), dict(d_pool=100), dict(d_sel=4), dict(scale=float("nan")),
                                dict(d_pool=2048)])
def test_invalid_descriptors_are_rejected(lib, kw):
    with pytest.raises(lca.LcaError) as e:
        lca.workspace_size(_desc(**kw))
    assert e.value.status in (lca.ERR_INVALID_ARG, lca.ERR_UNSUPPORTED)
    assert str(e.value)


def test_null_misaligned_and_small_workspace_are_rejected_before_launch(lib):
    d = _desc()
    A = 0x10000   # a made-up, aligned, non-NULL address: validation must fail before it is ever used
    cd = d.c()
    ws = lca.workspace_size(d)
    vp, sz = ctypes.c_void_p, ctypes.c_size_t

    # more summary queries than tokens: rejected by the calls that read them, fine for the others
    big = _desc(n_q=9000).c()
    assert lib.lca_condense(ctypes.byref(big), vp(A), vp(A), vp(A), vp(A), vp(A), vp(A), vp(0), vp(A), sz(1 << 30), vp(0)) == lca.ERR_INVALID_ARG
    assert lca.workspace_size(_desc(n_q=9000)) > 0

    def condense(Q=A, POOL=A, SEL=A, pr=A, sr=A, an=A, ws_ptr=A, ws_bytes=ws):
        return lib.lca_condense(ctypes.byref(cd), vp(Q), vp(POOL), vp(SEL), vp(pr), vp(sr), vp(an), vp(0), vp(ws_ptr), sz(ws_bytes), vp(0))

    assert condense(Q=0) == lca.ERR_INVALID_ARG and b"Q" in lib.lca_last_error()
    assert condense(POOL=A + 2) == lca.ERR_INVALID_ARG and b"aligned" in lib.lca_last_error()
    assert condense(pr=0) == lca.ERR_INVALID_ARG
    assert condense(an=0) == lca.ERR_INVALID_ARG
    assert condense(ws_ptr=0) == lca.ERR_WORKSPACE
    assert condense(ws_bytes=ws - 1) == lca.ERR_WORKSPACE and b"needed" in lib.lca_last_error()
    assert lib.lca_prefill_attn(ctypes.byref(cd), vp(A), vp(A), vp(A), vp(A), vp(A), vp(0), vp(0), vp(A), sz(ws), vp(0)) == lca.ERR_INVALID_ARG
    assert lib.dense_mla_attn(ctypes.byref(cd), vp(A), vp(0), vp(A), vp(A), vp(0), vp(A), sz(ws), vp(0)) == lca.ERR_INVALID_ARG
    assert lib.lca_decode_attn(ctypes.byref(cd), vp(0), vp(A), vp(A), vp(A), vp(A), vp(A), vp(A), sz(ws), vp(0)) in (
        lca.ERR_INVALID_ARG, lca.ERR_UNSUPPORTED)
    und = lca.Desc(B=1, L=100, H=3, S=1, d_pool=64, d_sel=64, g=4, w=4).c()    # no decode kernel for this shape
    assert lib.lca_decode_attn(ctypes.byref(und), vp(A), vp(A), vp(A), vp(A), vp(A), vp(A), vp(A), sz(1 << 20), vp(0)) == lca.ERR_UNSUPPORTED
    assert lib.lca_workspace_size(None, None) == lca.ERR_INVALID_ARG


def test_probes_reject_bad_arguments_before_launch(lib):
    import ctypes
    words = (ctypes.c_uint32 * 4)()
    waves = ctypes.c_int32(-1)
    fake = ctypes.c_void_p(4096)                                       # never dereferenced: every call below is rejected on the host
    assert lib.lca_probe_hbm_read(None, ctypes.c_size_t(1024), fake, None) == lca.ERR_INVALID_ARG
    assert lib.lca_probe_hbm_read(fake, ctypes.c_size_t(1024), None, None) == lca.ERR_INVALID_ARG
    assert lib.lca_probe_hbm_read(fake, ctypes.c_size_t(0), fake, None) == lca.ERR_INVALID_ARG
    assert lib.lca_probe_hbm_read(fake, ctypes.c_size_t(1000), fake, None) == lca.ERR_INVALID_ARG
    assert b"multiple of 16" in lib.lca_last_error()
    assert lib.lca_probe_hbm_read(ctypes.c_void_p(4100), ctypes.c_size_t(1024), fake, None) == lca.ERR_INVALID_ARG   # misaligned
    assert lib.lca_probe_mfma_bf16(ctypes.c_int32(0), ctypes.c_int32(0), fake, ctypes.byref(waves), None) == lca.ERR_INVALID_ARG
    assert lib.lca_probe_mfma_bf16(ctypes.c_int32(65537), ctypes.c_int32(0), fake, ctypes.byref(waves), None) == lca.ERR_INVALID_ARG
    assert lib.lca_probe_mfma_bf16(ctypes.c_int32(10), ctypes.c_int32(0), None, ctypes.byref(waves), None) == lca.ERR_INVALID_ARG
    assert lib.lca_probe_mfma_bf16(ctypes.c_int32(10), ctypes.c_int32(1), fake, None, None) == lca.ERR_INVALID_ARG
    assert lib.lca_probe_mfma_bf16(ctypes.c_int32(10), ctypes.c_int32(2), fake, ctypes.byref(waves), None) == lca.ERR_INVALID_ARG
    assert waves.value == -1 and list(words) == [0, 0, 0, 0]


def test_header_is_plain_c(tmp_path):
    """include/lca.h must be usable from C (no C++-only constructs): gcc -std=c99 -pedantic compiles a translation unit
    that includes it and takes the address of every declared entry point."""
    import subprocess
    names = _declared()
    src = tmp_path / "use_lca.c"
    src.write_text('#include "lca.h"\n' + "void *table[] = {" + ", ".join(f"(void *){n}" for n in names) + "};\n"
                   "int main(void) { lca_desc d; lca_cache_layout l; (void)d; (void)l; return sizeof(table) ? 0 : 1; }\n")
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-Wno-pedantic", "-I", os.path.join(ROOT, "include"), "-c", str(src),
                    "-o", str(tmp_path / "use_lca.o")], check=True)
