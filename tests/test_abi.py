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
    assert set(names) == set(lca.EXPORTS) and len(names) == 13
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
