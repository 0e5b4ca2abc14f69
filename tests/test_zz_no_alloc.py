"""llvq_validate_static, the entry point for callers that cannot allocate, against llvq_validate."""
import numpy as np
import pytest

from paper_2603_11021_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _words(seed, n):
    # random 48-bit words: about 0.18 % of them lie at or above N(13)
    return synth.rng_for(8, seed).integers(0, 1 << 48, size=n, dtype=np.uint64)


def test_validate_static_matches_validate_on_two_calls_in_a_row():
    from paper_2603_11021_amd import LLVQ
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    dev = torch.device("cuda:0")
    q = LLVQ(13, 0)
    out = torch.full((1,), -1, dtype=torch.int64, device=dev)
    # first a large input (more blocks than one pass of the grid covers), then a smaller one: the partial counts of
    # the first call stay in the library's array and must not leak into the second
    for seed, n in ((0, 3_000_011), (1, 70_001), (2, 0), (3, 257)):
        w = _words(seed, n)
        want_host = int((w >= synth.N_POINTS_M13).sum())
        d48 = torch.from_numpy(synth.pack_u48(w).reshape(-1)).to(dev)
        d64 = torch.from_numpy(w.view(np.int64)).to(dev)
        for d in (d48, d64):
            if n == 0 and d is d48:
                d = torch.empty(0, dtype=torch.uint8, device=dev)
            want = q.llvq_validate(d) if n else 0
            assert want == want_host
            out.fill_(-1)
            got = q.llvq_validate_static(d, out=out)
            assert got.data_ptr() == out.data_ptr()
            assert int(out.cpu()[0]) == want, (seed, n)


def test_validate_static_rejects_bad_arguments():
    import ctypes
    from paper_2603_11021_amd import LLVQ, binding
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    dev = torch.device("cuda:0")
    q = LLVQ(13, 0)
    lib = binding._load()
    d = torch.zeros(6 * 16, dtype=torch.uint8, device=dev)
    out = torch.zeros(2, dtype=torch.int64, device=dev)
    vp = ctypes.c_void_p
    assert lib.llvq_validate_static(q._h, vp(d.data_ptr()), 0, (1 << 32) + 1, vp(out.data_ptr()), None) == -1     # beyond the maximum
    assert b"LLVQ_VALIDATE_STATIC_MAX_BLOCKS" in lib.llvq_last_hip_error(q._h)
    assert lib.llvq_validate_static(q._h, vp(d.data_ptr()), 0, 16, None, None) == -1
    assert lib.llvq_validate_static(q._h, vp(d.data_ptr()), 0, 16, vp(out.data_ptr() + 4), None) == -2           # misaligned result
    assert lib.llvq_validate_static(q._h, vp(d.data_ptr()), 7, 16, vp(out.data_ptr()), None) == -1
