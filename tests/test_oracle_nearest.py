"""Pins of the oracle's nearest-point search (paper Sec. 3.1), none of which uses the search itself:
brute force over every point of the small ball cuts, lattice points as inputs, monotonicity in the cut, and the
Gaussian-source distortions the paper prints for shape-gain with 0, 1 and 2 gain bits (App. I table)."""
import os
from math import exp, lgamma, sqrt

import numpy as np
import pytest

from oracle.llvq_oracle import Oracle


@pytest.fixture(scope="module")
def o2():
    return Oracle(2)


@pytest.fixture(scope="module")
def o3():
    return Oracle(3)


def _brute(points, norms2, w, metric):
    dots = w @ points.T
    sc = dots / np.sqrt(norms2)[None, :] if metric == "angular" else dots - 0.5 * norms2[None, :]
    return sc.max(axis=1), sc.argmax(axis=1)


@pytest.mark.parametrize("metric", ["angular", "euclidean"])
def test_nearest_is_the_brute_force_optimum_on_shell_2(o2, metric):
    pts, _ = o2.decode(np.arange(196560, dtype=np.uint64))
    P = pts.astype(np.float64)
    n2 = (P ** 2).sum(axis=1)
    rng = np.random.default_rng(51)
    w = rng.standard_normal((200, 24)) * (1.0 if metric == "angular" else sqrt(32.0 / 24.0))
    w[:20] = np.round(w[:20] * 2) / 2                      # ties and zeros
    got, sc = o2.nearest(w, metric)
    want, _ = _brute(P, n2, w, metric)
    assert np.allclose(sc, want, rtol=1e-12, atol=1e-12)
    # the returned point attains the score and is a point of the cut
    G = got.astype(np.float64)
    mine = (w * G).sum(axis=1) / np.sqrt((G ** 2).sum(axis=1)) if metric == "angular" else (w * G).sum(axis=1) - 0.5 * (G ** 2).sum(axis=1)
    assert np.allclose(mine, want, rtol=1e-12, atol=1e-12)
    _, bad = o2.encode(got)
    assert bad == 0


@pytest.mark.parametrize("metric", ["angular", "euclidean"])
def test_nearest_is_the_brute_force_optimum_on_shells_2_and_3(o3, metric):
    """all 16,969,680 points of Lambda_24(3), in slices"""
    rng = np.random.default_rng(52)
    w = rng.standard_normal((24, 24)) * (1.0 if metric == "angular" else sqrt(44.0 / 24.0))
    best = np.full(w.shape[0], -np.inf)
    step = 1 << 21
    for first in range(0, o3.num_points, step):
        n = min(step, o3.num_points - first)
        pts, bad = o3.decode_range(first, n)
        assert bad == 0
        P = pts.astype(np.float32)
        n2 = (P.astype(np.float64) ** 2).sum(axis=1)
        dots = (w.astype(np.float32) @ P.T).astype(np.float64)
        sc = dots / np.sqrt(n2)[None, :] if metric == "angular" else dots - 0.5 * n2[None, :]
        best = np.maximum(best, sc.max(axis=1))
    got, sc = o3.nearest(w, metric)
    assert np.allclose(sc, best, rtol=2e-6, atol=2e-6)     # the brute force above runs in fp32
    _, bad = o3.encode(got)
    assert bad == 0


def test_nearest_is_the_brute_force_optimum_on_shells_2_to_4():
    """All 415,003,680 points of Lambda_24(4) (Table 1: 196,560 + 16,773,120 + 398,034,000), one pass for both metrics,
    in slices dealt to the host cores.  Shell 4 is the first with a weight-16 class, classes of weight 0 that hold an
    8, and supports carrying two different values (6 and 2), so this pass exercises the parity repair on a position
    that is not interchangeable with the others, which shells 2 and 3 cannot."""
    from concurrent.futures import ThreadPoolExecutor
    o4 = Oracle(4)
    assert o4.num_points == 415003680
    rng = np.random.default_rng(54)
    w = rng.standard_normal((16, 24))
    w[0] = 0.0; w[0, 5] = 3.0                                    # one coordinate: the (8, 0^23) class
    w[1] = 0.0; w[1, [2, 9, 17, 20]] = [1.0, -1.0, 1.0, 1.0]     # (4^4, 0^20)
    w[2] = np.round(w[2])                                        # ties
    w[3] = np.abs(w[3]) * np.where(np.arange(24) < 8, 3.0, 0.3)  # mass on eight coordinates: (6, 2^7, ...) candidates
    w[4, :12] *= 4.0
    inputs = {"angular": w, "euclidean": w * sqrt(56.0 / 24.0)}
    w32 = {k: v.astype(np.float32) for k, v in inputs.items()}
    step = 1 << 21
    firsts = list(range(0, o4.num_points, step))

    def slice_best(first):
        n = min(step, o4.num_points - first)
        pts, bad = o4.decode_range(first, n)
        assert bad == 0
        P = pts.astype(np.float32)
        n2 = (P.astype(np.float64) ** 2).sum(axis=1)
        ang = ((w32["angular"] @ P.T).astype(np.float64) / np.sqrt(n2)[None, :]).max(axis=1)
        euc = ((w32["euclidean"] @ P.T).astype(np.float64) - 0.5 * n2[None, :]).max(axis=1)
        return ang, euc

    best = {k: np.full(16, -np.inf) for k in inputs}
    with ThreadPoolExecutor(max(1, min(8, os.cpu_count() or 1))) as pool:
        for ang, euc in pool.map(slice_best, firsts):
            best["angular"] = np.maximum(best["angular"], ang)
            best["euclidean"] = np.maximum(best["euclidean"], euc)
    for metric, wm in inputs.items():
        got, sc = o4.nearest(wm, metric)
        assert np.allclose(sc, best[metric], rtol=2e-6, atol=2e-6)          # the brute force above runs in fp32
        G = got.astype(np.float64)
        mine = (wm * G).sum(axis=1) / np.sqrt((G ** 2).sum(axis=1)) if metric == "angular" else (wm * G).sum(axis=1) - 0.5 * (G ** 2).sum(axis=1)
        assert np.allclose(mine, sc, rtol=1e-12, atol=1e-12)
        _, bad = o4.encode(got)
        assert bad == 0


def test_a_lattice_point_is_its_own_nearest_direction(oracle13):
    """input = positive multiple of a point of the cut: cosine 1, answer on the same ray (v and 2v can both be in the cut)"""
    rng = np.random.default_rng(53)
    cls = oracle13.classes()
    pick = rng.choice(len(cls), 90, replace=False)
    idx = np.array([cls[j]["offset"] + int(rng.integers(0, cls[j]["size"])) for j in pick], dtype=np.uint64)
    pts, _ = oracle13.decode(idx)
    w = pts.astype(np.float64) * rng.uniform(0.01, 3.0, size=(idx.size, 1))
    got, sc = oracle13.nearest(w)
    assert np.allclose(sc, np.linalg.norm(w, axis=1), rtol=1e-12)
    G, P = got.astype(np.float64), pts.astype(np.float64)
    cos = (G * P).sum(axis=1) / np.linalg.norm(G, axis=1) / np.linalg.norm(P, axis=1)
    assert np.allclose(cos, 1.0, atol=1e-12)
    # Euclidean metric: the point itself
    got_e, _ = oracle13.nearest(pts.astype(np.float64), "euclidean")
    assert np.array_equal(got_e, pts)


def test_larger_cut_is_never_worse_and_beats_random_points(oracle13, o3):
    rng = np.random.default_rng(54)
    w = rng.standard_normal((40, 24))
    _, s13 = oracle13.nearest(w)
    _, s3 = o3.nearest(w)
    assert (s13 >= s3 - 1e-12).all()
    pts, _ = oracle13.decode(rng.integers(0, oracle13.num_points, 200000, dtype=np.uint64))
    P = pts.astype(np.float64)
    sc = (w @ P.T) / np.linalg.norm(P, axis=1)[None, :]
    assert (s13 >= sc.max(axis=1)).all()


def test_gaussian_source_distortion_matches_the_paper(oracle13):
    """shape-gain over norm(Lambda_24(13)) with no gain bits: the gain is the one level of a chi_24 quantiser, E||w||.
    Direction and norm of a Gaussian block are independent, so the per-dimension distortion is
    1 + E||w||^2 (1 - 2 E cos) / 24; the paper prints 0.085 (App. I table, first shape-gain row)."""
    rng = np.random.default_rng(55)
    w = rng.standard_normal((300, 24))
    got, sc = oracle13.nearest(w)
    cos = sc / np.linalg.norm(w, axis=1)
    mean_norm = sqrt(2.0) * exp(lgamma(12.5) - lgamma(12.0))
    mse = 1.0 + mean_norm ** 2 * (1.0 - 2.0 * cos.mean()) / 24.0
    sem = 2.0 * mean_norm ** 2 / 24.0 * cos.std() / sqrt(cos.size)
    rows = [l.split() for l in open(os.path.join(os.path.dirname(__file__), "golden", "gaussian_source_mse.txt"))
            if l.strip() and not l.startswith("#")]
    printed = float(rows[0][2])
    assert rows[0][:2] == ["norm(Lambda24(13))", "0"] and printed == 0.085
    assert sem < 5e-4
    assert abs(mse - printed) < 0.0005 + 3 * sem, mse          # half a unit of the last printed digit + sampling error
    _, bad = oracle13.encode(got)
    assert bad == 0


@pytest.mark.parametrize("m,bits", [(12, 1), (11, 2)])
def test_gaussian_source_distortion_with_gain_bits_matches_the_paper(m, bits):
    """shape-gain over norm(Lambda_24(m)) with a 1- or 2-bit gain code (App. I table: 0.078 for m = 12, 0.080 for
    m = 11), the norm going to the nearest of 2^bits chi_24-matched levels (see the golden file for this reading).
    Direction and norm r of a Gaussian block are independent, so the per-dimension distortion is
    (E r^2 - 2 E[r g(r)] E cos + E g(r)^2) / 24: the expectations over r by numerical integration, E cos from the
    oracle's search on a sample."""
    from scipy import integrate
    from scipy.stats import chi
    L = 1 << bits
    levels = chi.ppf((np.arange(L) + 0.5) / L, 24)
    cuts = np.concatenate([[0.0], (levels[1:] + levels[:-1]) / 2, [np.inf]])
    e_rg = sum(levels[i] * integrate.quad(lambda r: r * chi.pdf(r, 24), cuts[i], cuts[i + 1])[0] for i in range(L))
    e_g2 = sum(levels[i] ** 2 * (chi.cdf(cuts[i + 1], 24) - chi.cdf(cuts[i], 24)) for i in range(L))
    rng = np.random.default_rng(56 + m)
    w = rng.standard_normal((200, 24))
    oracle = Oracle(m)
    got, sc = oracle.nearest(w)
    assert ((got.astype(np.int64) ** 2).sum(axis=1) <= 16 * m).all()
    cos = sc / np.linalg.norm(w, axis=1)
    mse = (24.0 - 2.0 * e_rg * cos.mean() + e_g2) / 24.0
    sem = 2.0 * e_rg / 24.0 * cos.std() / sqrt(cos.size)
    rows = [l.split() for l in open(os.path.join(os.path.dirname(__file__), "golden", "gaussian_source_mse.txt"))
            if l.strip() and not l.startswith("#")]
    printed = {(r[0], int(r[1])): float(r[2]) for r in rows}[("norm(Lambda24(%d))" % m, bits)]
    assert sem < 8e-4
    assert abs(mse - printed) < 0.0005 + 3 * sem, mse
