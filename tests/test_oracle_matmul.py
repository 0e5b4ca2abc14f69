"""Pins for the oracle's shape-gain reconstruction and matrix product (CPU only)."""
import numpy as np


def _inputs(oracle, N, KB, M, seed):
    rng = np.random.default_rng(seed)
    idx = rng.integers(0, oracle.num_points, (N, KB), dtype=np.uint64)
    gain = np.exp(0.5 * rng.standard_normal((N, KB))).astype(np.float16)
    x = rng.standard_normal((M, 24 * KB)).astype(np.float16)
    return idx, gain, x


def test_block_norm_equals_gain(oracle13):
    idx, gain, _ = _inputs(oracle13, 64, 50, 1, 1)
    W = oracle13.dequant(idx, gain)
    nrm = np.sqrt((W ** 2).sum(axis=1))
    assert np.allclose(nrm, gain.astype(np.float64).ravel(), rtol=1e-14, atol=0)


def test_dequant_is_gain_times_unit_lattice_direction(oracle13):
    idx, gain, _ = _inputs(oracle13, 8, 20, 1, 2)
    X, _ = oracle13.decode(idx.ravel())
    Xf = X.astype(np.float64)
    unit = Xf / np.linalg.norm(Xf, axis=1, keepdims=True)
    W = oracle13.dequant(idx, gain)
    assert np.allclose(W, unit * gain.astype(np.float64).ravel()[:, None], rtol=1e-14, atol=0)


def test_matmul_reduces_to_library_gemm(oracle13):
    idx, gain, x = _inputs(oracle13, 96, 31, 5, 3)
    y = oracle13.matmul(x, idx, gain)
    y2 = oracle13.matmul_dense(x, idx, gain)
    assert y.shape == (5, 96)
    assert np.allclose(y, y2, rtol=1e-12, atol=1e-12)


def test_matmul_linearity_and_padding(oracle13):
    idx, gain, x = _inputs(oracle13, 40, 12, 2, 4)
    y = oracle13.matmul(x, idx, gain)
    # linear in the activations (power-of-two factor keeps fp16 exact)
    assert np.allclose(oracle13.matmul((2 * x.astype(np.float32)).astype(np.float16), idx, gain), 2 * y, rtol=1e-13)
    # linear in the gains
    assert np.allclose(oracle13.matmul(x, idx, (gain.astype(np.float32) * 4).astype(np.float16)), 4 * y, rtol=1e-13)
    # a zero-padded tail of the activations contributes nothing, whatever the padded weights decode to
    xz = x.copy()
    xz[:, -24:] = 0
    y_trunc = oracle13.matmul(xz[:, :-24], idx[:, :-1], gain[:, :-1])
    assert np.allclose(oracle13.matmul(xz, idx, gain), y_trunc, rtol=1e-13, atol=1e-13)


def test_half_conversion_matches_numpy(oracle13):
    bits = np.arange(0, 0x7C00, 7, dtype=np.uint16)            # all finite positive halves, strided
    gain = bits.view(np.float16)
    idx = np.zeros(bits.size, dtype=np.uint64)                  # (4,4,0,...) / sqrt(32)
    W = oracle13.dequant(idx, gain)
    assert np.array_equal(W[:, 0], gain.astype(np.float64) * 4.0 / np.sqrt(32.0))
