"""CPU-only tests of the library's host side: C-ABI surface, table builder and the index -> block
reconstruction code compiled for the host (tests/host_emul), compared with the oracle."""
import ctypes
import os
import re
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2603_11021_amd", "libllvq.so")
EMUL = os.path.join(ROOT, "tests", "host_emul", "libemul.so")


@pytest.fixture(scope="module")
def emul():
    srcs = [os.path.join(ROOT, "tests", "host_emul", "emul.cpp")] + [
        os.path.join(ROOT, "paper_2603_11021_amd", "csrc", f)
        for f in ("llvq_tables.cpp", "llvq_tables.h", "llvq_decode_core.h", "llvq_encode_core.h", "llvq_wide.h")]
    if not os.path.exists(EMUL) or os.path.getmtime(EMUL) < max(os.path.getmtime(f) for f in srcs):
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-o", EMUL,
                               os.path.join(ROOT, "tests", "host_emul", "emul.cpp"),
                               os.path.join(ROOT, "paper_2603_11021_amd", "csrc", "llvq_tables.cpp")])
    lib = ctypes.CDLL(EMUL)
    lib.emul_num_points.restype = ctypes.c_uint64
    lib.emul_decode_i8.restype = ctypes.c_uint64
    lib.emul_decode_i8.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p]
    lib.emul_encode.restype = ctypes.c_uint64
    lib.emul_encode.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p]
    assert lib.emul_init(13) == 0

    def encode(pts):
        pts = np.ascontiguousarray(pts, dtype=np.int8)
        out = np.empty(pts.shape[0], dtype=np.uint64)
        bad = lib.emul_encode(pts.ctypes.data, pts.shape[0], out.ctypes.data)
        return out, int(bad)

    def decode(idx):
        idx = np.ascontiguousarray(idx, dtype=np.uint64)
        out = np.empty((idx.size, 24), dtype=np.int8)
        bad = lib.emul_decode_i8(idx.ctypes.data, idx.size, out.ctypes.data)
        return out, int(bad)

    decode.lib = lib
    decode.encode = encode
    return decode


def _built_lib():
    if not os.path.exists(LIB):
        pytest.skip("libllvq.so not built (run __graft_entry__.build())")
    return ctypes.CDLL(LIB)


def test_library_exports_every_declared_symbol():
    lib = _built_lib()
    header = open(os.path.join(ROOT, "include", "llvq.h")).read()
    names = sorted(set(re.findall(r"\b(llvq_[a-z0-9_]+)\s*\(", header)))
    assert {"llvq_create", "llvq_destroy", "llvq_decode_i8", "llvq_decode", "llvq_matmul", "llvq_validate"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_no_cpu_fallback_without_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    lib = _built_lib()
    h = ctypes.c_void_p()
    rc = lib.llvq_create(ctypes.byref(h), 13, 0)
    assert rc == -3 and not h.value                       # LLVQ_EHIP: fails loudly, no context
    lib.llvq_strerror.restype = ctypes.c_char_p
    assert b"HIP" in lib.llvq_strerror(rc)
    assert lib.llvq_create(ctypes.byref(h), 20, 0) == -1  # LLVQ_EINVAL
    assert lib.llvq_create(None, 13, 0) == -1


def test_tables_fit_in_lds(emul, oracle13):
    lib = emul.lib
    assert lib.emul_num_classes() == oracle13.num_classes == 383
    assert lib.emul_num_points() == oracle13.num_points
    assert lib.emul_lds_bytes() + 64 * 8 * 4 <= 160 * 1024       # tables + the product kernel's row accumulators


def test_host_decode_matches_oracle_on_shell2(emul, oracle13):
    I = np.arange(196560, dtype=np.uint64)
    got, bad = emul(I)
    want, _ = oracle13.decode(I)
    assert bad == 0 and np.array_equal(got, want)


def test_host_decode_matches_oracle_on_every_class(emul, oracle13):
    rng = np.random.default_rng(21)
    picks = []
    for c in oracle13.classes():
        picks += [c["offset"], c["offset"] + c["size"] - 1]
        picks += [c["offset"] + int(v) for v in rng.integers(0, c["size"], 64)]
    I = np.array(picks, dtype=np.uint64)
    got, bad = emul(I)
    want, _ = oracle13.decode(I)
    assert bad == 0 and np.array_equal(got, want)


def test_host_decode_matches_oracle_on_random_union(emul, oracle13):
    rng = np.random.default_rng(22)
    I = rng.integers(0, oracle13.num_points, 400000, dtype=np.uint64)
    got, bad = emul(I)
    want, _ = oracle13.decode(I)
    assert bad == 0 and np.array_equal(got, want)


def test_host_decode_out_of_range(emul, oracle13):
    got, bad = emul(np.array([oracle13.num_points, 2 ** 48 - 1, 5], dtype=np.uint64))
    assert bad == 2 and not got[:2].any() and got[2].any()


def test_host_encode_inverts_decode_on_every_class(emul, oracle13):
    rng = np.random.default_rng(23)
    picks = []
    for c in oracle13.classes():
        picks += [c["offset"], c["offset"] + c["size"] - 1]
        picks += [c["offset"] + int(v) for v in rng.integers(0, c["size"], 100)]
    I = np.array(picks, dtype=np.uint64)
    pts, _ = oracle13.decode(I)
    got, bad = emul.encode(pts)
    assert bad == 0 and np.array_equal(got, I)


def test_host_encode_matches_oracle_on_random_union_and_shell2(emul, oracle13):
    I = np.concatenate([np.random.default_rng(24).integers(0, oracle13.num_points, 200000, dtype=np.uint64),
                        np.arange(196560, dtype=np.uint64)])
    pts, _ = oracle13.decode(I)
    got, bad = emul.encode(pts)
    want, wbad = oracle13.encode(pts)
    assert bad == wbad == 0 and np.array_equal(got, want) and np.array_equal(got, I)


def test_host_encode_rejects_what_the_oracle_rejects(emul, oracle13):
    from point_cases import spoiled_points
    rng = np.random.default_rng(25)
    pts, _ = oracle13.decode(rng.integers(0, oracle13.num_points, 20000, dtype=np.uint64))
    bad_pts = spoiled_points(pts, rng)
    want, wbad = oracle13.encode(bad_pts)
    got, bad = emul.encode(bad_pts)
    assert 0.8 * bad_pts.shape[0] < wbad < bad_pts.shape[0]               # some spoiled vectors are points again
    assert bad == wbad and np.array_equal(got, want)                        # the oracle marks a non-point with all ones


def test_encoder_tables_fit_in_lds(emul):
    emul.lib.emul_enc_bytes.restype = ctypes.c_uint32
    assert emul.lib.emul_enc_bytes() <= 80 * 1024


def test_synth_pack_u48():
    from paper_2603_11021_amd import synth
    idx = np.array([[0, 1, 2 ** 48 - 1], [0x0102030405, 280974212784719, 7]], dtype=np.uint64)
    b = synth.pack_u48(idx)
    assert b.shape == (2, 3, 6) and b.dtype == np.uint8
    back = sum(b[..., i].astype(np.uint64) << np.uint64(8 * i) for i in range(6))
    assert np.array_equal(back, idx)
    x = synth.activations(synth.rng_for(2), 2, 4096)
    assert x.shape == (2, 4104) and not x[:, 4096:].any() and x[:, :4096].any()


# ---- the decoder of the larger unions (contexts with m_max > 13) -------------------------------------------------
@pytest.fixture(scope="module")
def wide19(emul):
    lib = emul.lib
    lib.emul_wide_num_points.restype = ctypes.c_uint64
    lib.emul_wide_shell_offset.restype = ctypes.c_uint64
    lib.emul_wide_decode_i8.restype = ctypes.c_uint64
    lib.emul_wide_decode_i8.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p]
    assert lib.emul_wide_init(19) == 0

    def decode(idx):
        idx = np.ascontiguousarray(idx, dtype=np.uint64)
        out = np.empty((idx.size, 24), dtype=np.int8)
        bad = lib.emul_wide_decode_i8(idx.ctypes.data, idx.size, out.ctypes.data)
        return out, int(bad)

    decode.lib = lib
    return decode


@pytest.fixture(scope="module")
def oracle19():
    from oracle.llvq_oracle import Oracle
    return Oracle(19)


def test_wide_tables_match_table_1(wide19, oracle19):
    """1,457 classes and the cumulative count of the paper's Table 1, row m = 19"""
    lib = wide19.lib
    assert lib.emul_wide_num_points() == 23546209100646960 == oracle19.num_points
    assert lib.emul_wide_num_classes() == 1457 == len(oracle19.classes())
    assert lib.emul_wide_shell_offset(14) == 280974212784720           # N(13)


def test_wide_decoder_matches_the_oracle_on_every_class(wide19, oracle19):
    rng = np.random.default_rng(191)
    idx = []
    for c in oracle19.classes():
        off, size = int(c["offset"]), int(c["size"])
        idx += [off, off + size - 1] + [off + int(v) for v in rng.integers(0, size, size=40, dtype=np.uint64)]
    idx = np.array(idx, dtype=np.uint64)
    got, bad = wide19(idx)
    want, wbad = oracle19.decode(idx)
    assert bad == 0 and wbad == 0
    assert np.array_equal(got, want)


def test_wide_decoder_matches_the_oracle_on_random_indices_and_small_shells(wide19, oracle19, oracle13):
    rng = np.random.default_rng(192)
    idx = rng.integers(0, oracle19.num_points, size=200000, dtype=np.uint64)
    got, bad = wide19(idx)
    want, _ = oracle19.decode(idx)
    assert bad == 0 and np.array_equal(got, want)
    # the first N(13) indices are the points of the smaller union, in the same order
    idx = rng.integers(0, oracle13.num_points, size=50000, dtype=np.uint64)
    assert np.array_equal(wide19(idx)[0], oracle13.decode(idx)[0])
    # all of shell 2, and out-of-range indices decode to zero
    got, _ = wide19(np.arange(196560, dtype=np.uint64))
    assert np.array_equal(got, oracle13.decode(np.arange(196560, dtype=np.uint64))[0])
    got, bad = wide19(np.array([oracle19.num_points, 2 ** 63], dtype=np.uint64))
    assert bad == 2 and not got.any()
