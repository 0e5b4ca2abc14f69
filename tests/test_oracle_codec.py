"""Pins for the oracle's index <-> point map (CPU only)."""
import os

import numpy as np
import pytest

from lattice_checks import golay_words, is_leech_int, row_hash

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_shell2_exhaustive_bijection_and_membership(oracle13):
    X, bad = oracle13.decode_range(0, 196560)
    assert bad == 0
    Xi = X.astype(np.int64)
    assert ((Xi ** 2).sum(axis=1) == 32).all()                       # shell 2 in the x sqrt(8) scaling
    assert is_leech_int(Xi).all()
    assert np.unique(row_hash(Xi)).size == 196560                   # all distinct => bijection onto Shell(2)
    # class ranges of the paper's example: 1104 + 97152 + 98304
    assert (np.sort(np.abs(Xi[:1104]), axis=1)[:, -2:] == 4).all()
    assert (np.abs(Xi[1104:98256]).max(axis=1) == 2).all()
    assert (np.abs(Xi[98256:]).max(axis=1) == 3).all()


def test_shell2_geometry(oracle13):
    X, _ = oracle13.decode_range(0, 196560)
    Xi = X.astype(np.int64)
    # closed under negation
    h = row_hash(Xi)
    assert np.array_equal(np.sort(h), np.sort(row_hash(-Xi)))
    # kissing configuration: inner products of one vector with all others
    want = {}
    for line in open(os.path.join(GOLDEN, "minimal_vectors.txt")):
        if line.startswith("#") or not line.strip():
            continue
        v, c = line.split()
        want[int(v)] = int(c)
    for probe in (0, 1104, 98256, 150000):
        ip = Xi @ Xi[probe]
        vals, counts = np.unique(ip, return_counts=True)
        assert {int(v): int(c) for v, c in zip(vals, counts)} == want
    # spherical design: sum x x^T = (n * 32 / 24) I
    S = Xi.T @ Xi
    assert np.array_equal(S, 262080 * np.eye(24, dtype=np.int64))


def test_shell3_exhaustive(oracle13):
    n2, n3 = 196560, 16773120
    hashes = []
    S = np.zeros((24, 24), dtype=np.int64)
    step = 1 << 21
    for first in range(n2, n2 + n3, step):
        n = min(step, n2 + n3 - first)
        X, bad = oracle13.decode_range(first, n)
        assert bad == 0
        Xi = X.astype(np.int64)
        assert ((Xi ** 2).sum(axis=1) == 48).all()
        assert is_leech_int(Xi).all()
        hashes.append(row_hash(Xi))
        Xf = X.astype(np.float64)
        S += np.rint(Xf.T @ Xf).astype(np.int64)
    assert np.unique(np.concatenate(hashes)).size == n3             # all distinct => bijection onto Shell(3)
    assert np.array_equal(S, (n3 * 48 // 24) * np.eye(24, dtype=np.int64))


def test_every_class_first_last_random(oracle13):
    rng = np.random.default_rng(11)
    for c in oracle13.classes():
        picks = [c["offset"], c["offset"] + c["size"] - 1] + [c["offset"] + int(rng.integers(0, c["size"])) for _ in range(6)]
        X, bad = oracle13.decode(np.array(picks, dtype=np.uint64))
        assert bad == 0
        Xi = X.astype(np.int64)
        assert ((Xi ** 2).sum(axis=1) == 16 * c["m"]).all()
        assert is_leech_int(Xi).all()
        lead = sorted(v for v, k in c["leader"].items() for _ in range(k))
        assert (np.sort(np.abs(Xi), axis=1) == np.array(lead)).all()
        assert (Xi[:, 0] & 1 == c["odd"]).all()


def test_round_trip_random_indices(oracle13):
    rng = np.random.default_rng(12)
    I = rng.integers(0, oracle13.num_points, 300000, dtype=np.uint64)
    X, bad = oracle13.decode(I)
    assert bad == 0
    assert is_leech_int(X).all()
    J, bad = oracle13.encode(X)
    assert bad == 0
    assert np.array_equal(I, J)


def _random_lattice_points(classes, rng, n):
    """points of the ball cut built without the oracle's decoder: leader, own Golay word, random placement and
    signs, accepted when the membership conditions hold"""
    words = golay_words()
    wt = np.array([bin(int(v)).count("1") for v in words])
    pts = []
    while len(pts) < n:
        c = classes[int(rng.integers(0, len(classes)))]
        vals = [v for v, k in c["leader"].items() for _ in range(k)]
        x = np.zeros(24, dtype=np.int64)
        if c["odd"]:
            cw = int(words[rng.integers(0, 4096)])
            perm = rng.permutation(24)
            for pos, v in zip(perm, vals):
                bit = (cw >> int(pos)) & 1
                x[pos] = v if ((v % 4 == 1) == (bit == 0)) else -v
        else:
            cand = words[wt == c["w"]]
            cw = int(cand[rng.integers(0, cand.size)])
            f1 = [i for i in range(24) if (cw >> i) & 1]
            f0 = [i for i in range(24) if not (cw >> i) & 1]
            v1 = [v for v in vals if v % 4 == 2]
            v0 = [v for v in vals if v % 4 == 0]
            for pos, v in zip(rng.permutation(f1), v1):
                x[pos] = v
            for pos, v in zip(rng.permutation(f0), v0):
                x[pos] = v
            x *= rng.choice([-1, 1], size=24)
        if is_leech_int(x[None, :])[0]:
            pts.append(x)
    return np.array(pts)


def test_decode_inverts_encode_on_independently_built_points(oracle13):
    rng = np.random.default_rng(13)
    P = _random_lattice_points(oracle13.classes(), rng, 3000)
    I, bad = oracle13.encode(P.astype(np.int8))
    assert bad == 0
    assert (I < oracle13.num_points).all()
    X, bad = oracle13.decode(I)
    assert bad == 0
    assert np.array_equal(X.astype(np.int64), P)


def test_encode_rejects_non_members(oracle13):
    x = np.zeros((3, 24), dtype=np.int8)
    x[0, :2] = (4, 2)            # mixed residues, wrong norm
    x[1, :] = 1                  # all ones: sum 24 = 0 mod 8, needs 4
    x[2, :2] = (4, 4)
    I, bad = oracle13.encode(x)
    assert bad == 2 and I[2] == 0
    assert not oracle13.is_member(x[0]) and not oracle13.is_member(x[1]) and oracle13.is_member(x[2])


def test_index_out_of_range_decodes_to_zero(oracle13):
    X, bad = oracle13.decode(np.array([oracle13.num_points, 2 ** 48 - 1], dtype=np.uint64))
    assert bad == 2 and not X.any()


def test_digit_order_of_the_local_index(oracle13):
    """Paper Sec. 3.2 (3) / App. A step 3: r is the least significant digit (it selects the Golay word, i.e. the
    residues of the halved vector), then s (signs only), then I'' (placement)."""
    for c in oracle13.classes():
        if c["size"] < 4 * c["A"] * 2 ** c["B"] or c["A"] == 1:
            continue
        base = c["offset"]
        X, _ = oracle13.decode(np.array([base + r for r in range(4)], dtype=np.uint64))
        Xi = X.astype(np.int64)
        p = Xi[:, :1] & 1
        words = (((Xi - p) >> 1) & 1)
        # consecutive r: different Golay words
        assert len({tuple(w) for w in words.tolist()}) == 4
        if c["B"] > 0:
            Y, _ = oracle13.decode(np.array([base + k * c["A"] for k in range(4)], dtype=np.uint64))
            Yi = Y.astype(np.int64)
            assert (np.abs(Yi) == np.abs(Yi[0])).all()             # same word, same placement ...
            assert len({tuple(v) for v in Yi.tolist()}) == 4         # ... different signs
        Z, _ = oracle13.decode(np.array([base, base + c["A"] * 2 ** c["B"]], dtype=np.uint64))
        Zi = Z.astype(np.int64)
        assert not np.array_equal(np.abs(Zi[0]), np.abs(Zi[1]))      # next I'': another placement


def test_spot_values_format1(oracle13):
    # consequences of the format chosen where the paper leaves the order open (not values printed by the paper)
    N = oracle13.num_points
    X, _ = oracle13.decode(np.array([0, 1103, 1104, 98256, 196559, N - 1], dtype=np.uint64))
    assert X[0].tolist() == [4, 4] + [0] * 22
    assert X[1].tolist() == [0] * 22 + [-4, -4]
    assert [i for i, v in enumerate(X[2]) if v] == [0, 2, 4, 5, 6, 10, 11, 23] and set(X[2].tolist()) == {0, 2}
    assert X[3].tolist() == [-3] + [1] * 23
    assert X[4].tolist() == [-1] * 23 + [3]
    assert X[5].tolist() == [-1] * 21 + [3, 3, -13]
