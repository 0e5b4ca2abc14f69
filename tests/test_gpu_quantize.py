"""GPU parity tests of the quantiser (llvq_quantize): nearest point of the ball cut, against the oracle's search.

The kernel scores candidates in fp32, the oracle in fp64, so where two candidates are closer than fp32 rounding
either is a correct answer: what is compared is what is unique.  The returned vector must be a point of the cut,
its exact (fp64) score must reach the oracle's optimum within 4e-6 relative (24 products and sums in fp32, each
within 2^-24), and on random inputs the points themselves must agree in all but a handful of cases."""
import numpy as np
import pytest

from paper_2603_11021_amd import synth, LLVQ_ANGULAR, LLVQ_EUCLIDEAN, LLVQ_IDX_U64

pytestmark = pytest.mark.gpu
RTOL = 4e-6


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2603_11021_amd import LLVQ
    return LLVQ(13, 0)


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _exact_score(w, pts, metric):
    P = pts.astype(np.float64)
    dots = (w.astype(np.float64) * P).sum(axis=1)
    n2 = (P ** 2).sum(axis=1)
    return dots / np.sqrt(n2) if metric == "angular" else dots - 0.5 * n2


def _check(gpu, oracle, w, metric, min_same):
    code = LLVQ_ANGULAR if metric == "angular" else LLVQ_EUCLIDEAN
    w = w.astype(np.float32)
    pts, idx, score = gpu.llvq_quantize(_dev(w), code, LLVQ_IDX_U64)
    pts, idx, score = pts.cpu().numpy(), idx.cpu().numpy().view(np.uint64), score.cpu().numpy()
    want_pts, want_sc = oracle.nearest(w.astype(np.float64), metric)
    # a point of the cut, and the index is its index
    enc, bad = oracle.encode(pts)
    assert bad == 0 and np.array_equal(enc, idx)
    # its exact score reaches the optimum
    mine = _exact_score(w, pts, metric)
    scale = np.abs(want_sc) + (0.5 * (pts.astype(np.float64) ** 2).sum(axis=1) if metric == "euclidean" else 0.0)
    assert (mine >= want_sc - RTOL * scale).all(), (want_sc - mine).max()
    assert np.allclose(score, mine, rtol=0, atol=RTOL * scale.max())
    same = (pts == want_pts).all(axis=1).mean()
    assert same >= min_same, same
    return same


def test_quantize_gaussian_blocks_angular(gpu, oracle13):
    w = synth.rng_for(10, 1).standard_normal((300, 24))
    _check(gpu, oracle13, w, "angular", 0.99)


def test_quantize_gaussian_blocks_euclidean(gpu, oracle13):
    # scaled so that the typical block falls inside the ball: ||w||^2 ~ 24 * 5.5 = 132 (shell 8)
    w = synth.rng_for(10, 2).standard_normal((200, 24)) * np.sqrt(5.5)
    _check(gpu, oracle13, w, "euclidean", 0.99)


def test_quantize_heavy_tailed_and_sparse_blocks(gpu, oracle13):
    rng = synth.rng_for(10, 3)
    a = rng.standard_t(2.5, size=(60, 24))                          # outliers, as in unrotated weights
    b = rng.standard_normal((60, 24)) * (rng.random((60, 24)) < 0.25)   # many exact zeros
    c = np.round(rng.standard_normal((60, 24)) * 2) / 2             # many ties
    d = np.zeros((2, 24))                                           # no direction at all: any point is as good as any other
    e = rng.standard_normal((6, 24)) * np.array([1e-12, 1e-6, 1e6, 1e12, 1e-3, 1e3])[:, None]   # scale does not matter
    _check(gpu, oracle13, np.concatenate([a, b, c, d, e]), "angular", 0.9)


def test_quantize_lattice_points_return_their_ray(gpu, oracle13):
    rng = np.random.default_rng(61)
    cls = oracle13.classes()
    idx = np.array([c["offset"] + int(rng.integers(0, c["size"])) for c in cls], dtype=np.uint64)
    pts, _ = oracle13.decode(idx)
    w = (pts.astype(np.float64) * rng.uniform(0.05, 2.0, size=(idx.size, 1))).astype(np.float32)
    got, _, score = gpu.llvq_quantize(_dev(w), LLVQ_ANGULAR, LLVQ_IDX_U64)
    G, P = got.cpu().numpy().astype(np.float64), pts.astype(np.float64)
    cos = (G * P).sum(axis=1) / np.linalg.norm(G, axis=1) / np.linalg.norm(P, axis=1)
    assert (cos > 1 - 1e-6).all()
    # Euclidean metric on the integer points themselves: exact in fp32, the point comes back with its index
    got_e, idx_e, _ = gpu.llvq_quantize(_dev(pts.astype(np.float32)), LLVQ_EUCLIDEAN, LLVQ_IDX_U64)
    assert np.array_equal(got_e.cpu().numpy(), pts)
    assert np.array_equal(idx_e.cpu().numpy().view(np.uint64), idx)


def test_quantize_smaller_cut_and_sizes(oracle13):
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2603_11021_amd import LLVQ
    from oracle.llvq_oracle import Oracle
    o4 = Oracle(4)
    g = LLVQ(4, 0)
    for n in (1, 255, 257):
        w = synth.rng_for(10, 100 + n).standard_normal((n, 24))
        _check(g, o4, w, "angular", 0.98)
    e = torch.empty((0, 24), dtype=torch.float32, device="cuda:0")
    pts, idx, score = g.llvq_quantize(e)
    assert pts.shape == (0, 24)
    g.close()


def test_gaussian_source_table_rows_with_gain_bits():
    """The quantiser end to end against figures the paper prints (App. I table, shape-gain rows at 2 bits per
    dimension): angular search over norm(Lambda_24(m)), the norm coded with 0, 1 or 2 bits by a chi_24-matched
    gain code, per-dimension squared error of a unit Gaussian source.  200,000 blocks: the sampling error is far
    below half a unit of the last printed digit."""
    import os
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2603_11021_amd import LLVQ
    rows = [l.split() for l in open(os.path.join(os.path.dirname(__file__), "golden", "gaussian_source_mse.txt"))
            if l.strip() and not l.startswith("#")]
    printed = {(r[0], int(r[1])): float(r[2]) for r in rows}
    rng = np.random.default_rng(2026)
    w = rng.standard_normal((200000, 24)).astype(np.float32)
    dw = _dev(w)
    w64 = w.astype(np.float64)
    nrm = np.linalg.norm(w64, axis=1)
    for m, bits in [(13, 0), (12, 1), (11, 2)]:
        pts, _, _ = LLVQ(m, 0).llvq_quantize(dw, LLVQ_ANGULAR, want_idx=False)
        p = pts.cpu().numpy().astype(np.float64)
        assert ((p ** 2).sum(axis=1) <= 16 * m).all()
        u = p / np.linalg.norm(p, axis=1, keepdims=True)
        levels = synth.chi_gain_levels(bits).astype(np.float64) * np.sqrt(24.0)        # levels for the norm of 24 unit normals
        g = levels[np.abs(nrm[:, None] - levels[None, :]).argmin(axis=1)]
        per_block = ((w64 - g[:, None] * u) ** 2).sum(axis=1) / 24.0
        mse, sem = per_block.mean(), per_block.std() / np.sqrt(per_block.size)
        want = printed[("norm(Lambda24(%d))" % m, bits)]
        assert sem < 1e-4
        assert abs(mse - want) < 0.0005 + 3 * sem, (m, bits, mse)
