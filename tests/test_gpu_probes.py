"""The two measurement aids of the library (plain HBM read, back-to-back bf16 matrix-core products) do the work they
are timed for: the read probe's word sums equal the buffer's, the matrix-core probe's outputs equal their closed form."""
import numpy as np
import pytest

from paper_2604_12452_amd import lca

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n_bytes", [16, 4096, 1_000_000 - 1_000_000 % 16, 151_000_000 - 151_000_000 % 16])
def test_read_probe_sums_every_word_once(n_bytes):
    import torch
    print(f"[probe] read {n_bytes} bytes", flush=True)
    rng = np.random.default_rng(n_bytes)
    host = rng.integers(0, 2**32, size=n_bytes // 4, dtype=np.uint32)
    buf = torch.from_numpy(host.view(np.int32)).cuda()
    sums = torch.full((lca.PROBE_WORDS,), -1, dtype=torch.int32, device="cuda")
    lca.probe_hbm_read(buf, sums)
    torch.cuda.synchronize()
    got = int(sums.cpu().numpy().view(np.uint32).astype(np.uint64).sum() % (1 << 32))
    want = int(host.astype(np.uint64).sum() % (1 << 32))
    assert got == want


def test_matrix_core_probe_matches_its_closed_form():
    import torch
    iters = 37
    out = torch.full((lca.PROBE_MFMA_FLOATS,), float("nan"), dtype=torch.float32, device="cuda")
    waves = lca.probe_mfma_bf16(iters, out)
    torch.cuda.synchronize()
    assert waves > 0 and waves % 4 == 0 and waves * 256 <= lca.PROBE_MFMA_FLOATS
    o = out.cpu().numpy().astype(np.float64)
    used = o[: waves * 256].reshape(waves, 64, 4)
    assert np.isfinite(used).all() and np.isnan(o[waves * 256:]).all()          # nothing past the documented extent is written
    i = np.arange(32)
    for c in range(4):
        u = (5 * i + 3 * c) % 7 - 2
        v = (3 * i + 5 * c + 1) % 7 - 2
        assert u.sum() != 0 and v.sum() != 0
        # lane l holds 16 elements of column l % 32 (8 rows in each of two row blocks per half): whatever the rows, the
        # wavefront's total is the sum of all 1024 elements
        assert (used[:, :, c].sum(axis=1) == 16.0 * iters * u.sum() * v.sum()).all()
        # and a lane's own sum is 16 iters v_j times the sum of u over the 16 rows it holds: the two halves of the wavefront
        # together hold every row of column j once
        pair = used[:, :32, c] + used[:, 32:, c]
        assert (pair == 16.0 * iters * u.sum() * v[None, :]).all()


def _hashed_operand(o, c):
    """Operand o (0 = A, 1 = B) of chain c in the hashed pattern, as the header defines it: [x][k], x = row of A / column of B."""
    M = np.uint64(0xFFFFFFFF)
    x = np.arange(32, dtype=np.uint64)[:, None]
    k = np.arange(16, dtype=np.uint64)[None, :]
    h = (((np.uint64(o * 4 + c) * np.uint64(32) + x) * np.uint64(16) + k + np.uint64(1)) & M)
    h = (h * np.uint64(2654435761)) & M
    h ^= h >> np.uint64(15)
    h = (h * np.uint64(2246822519)) & M
    h ^= h >> np.uint64(13)
    sign = ((h >> np.uint64(31)) & np.uint64(1)).astype(np.float64)
    e = 126 + ((h >> np.uint64(8)) & np.uint64(1)).astype(np.int64)
    m = (h & np.uint64(127)).astype(np.float64)
    return (1.0 - 2.0 * sign) * (1.0 + m / 128.0) * np.exp2(e - 127)


def test_matrix_core_probe_with_hashed_operands_matches_a_plain_product():
    import torch
    iters = 37
    out = torch.full((lca.PROBE_MFMA_FLOATS,), float("nan"), dtype=torch.float32, device="cuda")
    waves = lca.probe_mfma_bf16(iters, out, pattern=1)
    torch.cuda.synchronize()
    used = out.cpu().numpy().astype(np.float64)[: waves * 256].reshape(waves, 64, 4)
    assert np.isfinite(used).all()
    for c in range(4):
        A, B = _hashed_operand(0, c), _hashed_operand(1, c).T          # 32 x 16, 16 x 32
        assert len(np.unique(A)) > 100 and (A < 0).any() and (A > 0).any() and (np.abs(A) >= 0.5).all() and (np.abs(A) < 2).all()
        D = iters * (A @ B)
        pair = used[:, :32, c] + used[:, 32:, c]                        # lanes l and l + 32 hold column l between them
        tol = 1e-5 * np.abs(iters * (np.abs(A) @ np.abs(B))).sum(axis=0)
        assert (np.abs(pair - D.sum(axis=0)[None, :]) <= tol[None, :]).all()
        assert (used[:, :, c] == used[:1, :, c]).all()                  # every wavefront computes the same


def test_probe_buffers_are_checked_by_the_binding():
    import torch
    small = torch.zeros(8, dtype=torch.int32, device="cuda")
    with pytest.raises(ValueError):
        lca.probe_hbm_read(torch.zeros(64, dtype=torch.int32, device="cuda"), small)
    with pytest.raises(ValueError):
        lca.probe_mfma_bf16(10, torch.zeros(1024, dtype=torch.float32, device="cuda"))
    with pytest.raises(ValueError):
        lca.probe_hbm_read(torch.zeros(64, dtype=torch.int32), torch.zeros(lca.PROBE_WORDS, dtype=torch.int32, device="cuda"))



def test_library_opened_before_torch_is_imported_still_finds_the_device():
    """The binding opened first in a fresh process, torch only afterwards: both must end up on one HIP runtime (two runtimes
    in one process leave the second without a device, and every launch of the library then fails)."""
    import os
    import subprocess
    import sys
    code = (
        "import sys\n"
        "from paper_2604_12452_amd import lca\n"
        "lca.load()\n"
        "import torch\n"
        "buf = torch.arange(4096, dtype=torch.int32, device='cuda')\n"
        "sums = torch.zeros(lca.PROBE_WORDS, dtype=torch.int32, device='cuda')\n"
        "lca.probe_hbm_read(buf, sums)\n"
        "torch.cuda.synchronize()\n"
        "assert int(sums.sum()) == 4095 * 4096 // 2\n"
        "print('ok')\n")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-c", code], cwd=root, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout + r.stderr


def test_an_error_left_by_the_caller_is_not_taken_for_a_failed_launch():
    """hipGetLastError() after a launch returns the thread's last error whoever caused it: the library reads (clears) the
    state before it launches, so an earlier failed runtime call of the caller's does not fail the library's call."""
    import ctypes
    import torch
    buf = torch.arange(4096, dtype=torch.int32, device="cuda")
    sums = torch.zeros(lca.PROBE_WORDS, dtype=torch.int32, device="cuda")
    lca.load()
    hip = ctypes.CDLL("libamdhip64.so.7")            # by soname: the runtime already in the process
    assert hip.hipSetDevice(12345) != 0              # rejected on the host (no such ordinal); the current device stays, the error is recorded
    assert hip.hipPeekAtLastError() != 0             # ... and is still there (peeking does not clear it)
    lca.probe_hbm_read(buf, sums)
    torch.cuda.synchronize()
    assert int(sums.sum()) == 4095 * 4096 // 2
    assert hip.hipPeekAtLastError() == 0

