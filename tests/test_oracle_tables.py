"""Pins for the oracle's static tables: Golay code, shells, classes (CPU only)."""
import os

import numpy as np
import pytest

from lattice_checks import GEN_POLY, clmul, polymod, golay_words, theta_coefficients
from oracle.llvq_oracle import Oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def popcount(a):
    return np.array([bin(int(v)).count("1") for v in a])


def test_generator_polynomial_divides_x23_plus_1():
    # a cyclic code of length 23 needs g(x) | x^23 + 1 over GF(2); degree 11 gives dimension 12
    assert GEN_POLY.bit_length() - 1 == 11
    assert polymod((1 << 23) | 1, GEN_POLY) == 0
    # and g is one of the two degree-11 factors of (x^23+1)/(x+1): the cofactor times (x+1) times g
    other = 0b101011100011  # reciprocal polynomial of g
    assert clmul(clmul(GEN_POLY, other), 0b11) == (1 << 23) | 1


def test_golay_weight_enumerator(oracle13):
    w = oracle13.golay_words()
    assert len(set(w.tolist())) == 4096
    wt = popcount(w)
    counts = {int(k): int((wt == k).sum()) for k in np.unique(wt)}
    assert counts == {0: 1, 8: 759, 12: 2576, 16: 759, 24: 1}          # paper Sec. 2.5: A in {1,759,2576,759,1}


def test_golay_is_linear_selfdual_and_matches_polynomial_construction(oracle13):
    w = oracle13.golay_words()
    s = set(w.tolist())
    rng = np.random.default_rng(5)
    a = w[rng.integers(0, 4096, 20000)]
    b = w[rng.integers(0, 4096, 20000)]
    assert all(int(x) in s for x in (a ^ b))                             # closed under addition
    assert (popcount(a & b) % 2 == 0).all()                              # self-orthogonal, dimension 12 => self-dual
    assert 0xFFFFFF in s
    nz = w[w != 0]
    assert popcount(nz).min() == 8                                       # minimum distance of a linear code
    assert set(golay_words().tolist()) == s                              # same code as message(x) * g(x)


def test_golay_sorted_is_by_weight_then_message(oracle13):
    w = oracle13.golay_words()
    srt = oracle13.golay_sorted()
    wt = popcount(srt)
    assert (np.diff(wt) >= 0).all()
    assert sorted(srt.tolist()) == sorted(w.tolist())
    # inside a weight, the order is the order of the messages
    msg_of = {int(c): u for u, c in enumerate(w)}
    for k in (8, 12, 16):
        msgs = [msg_of[int(c)] for c in srt[wt == k]]
        assert msgs == sorted(msgs)


def test_shell_sizes_equal_theta_series(oracle13):
    theta = theta_coefficients(13)
    assert theta[1] == 0
    for m in range(2, 14):
        assert oracle13.shell_size(m) == theta[m], m
    # the benchmark spec facts
    assert oracle13.shell_size(2) == 196560
    assert oracle13.shell_size(3) == 16773120


def test_table1_of_the_paper():
    o19 = Oracle(19)
    theta = theta_coefficients(19)
    cum = 0
    sizes = {}
    for m in range(2, 20):
        sizes[m] = o19.shell_size(m)
        assert sizes[m] == theta[m]
    for line in open(os.path.join(GOLDEN, "table1_shells.txt")):
        if line.startswith("#") or not line.strip():
            continue
        m, n, N = line.split()
        m = int(m)
        if n != "-":
            assert sizes[m] == int(n)
        assert sum(sizes[k] for k in range(2, m + 1)) == int(N)
    assert o19.num_points == 23546209100646960
    # the index of the 2-bit/dim code fits 48 bits and that of the m=19 code 55 bits
    assert Oracle(13).num_points < 2 ** 48 < Oracle(14).num_points
    assert o19.num_points < 2 ** 55


def test_table2_of_the_paper(oracle13):
    cls = oracle13.classes()
    seen = 0
    for line in open(os.path.join(GOLDEN, "table2_classes.txt")):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        m, parity, count = int(f[0]), f[1], int(f[2])
        mult = [int(v) for v in f[3:]]
        leader = {8 - i: c for i, c in enumerate(mult) if c}
        match = [c for c in cls if c["m"] == m and c["leader"] == leader]
        assert len(match) == 1, (m, leader)
        assert match[0]["size"] == count
        assert match[0]["odd"] == (parity == "odd")
        seen += 1
    assert seen == 15
    # the table lists every class of shells 2..4
    assert sum(1 for c in cls if c["m"] <= 4) == 15


def test_class_table_structure(oracle13):
    cls = oracle13.classes()
    assert len(cls) == 383
    per_shell = [sum(1 for c in cls if c["m"] == m) for m in range(2, 14)]
    assert sum(per_shell) == 383
    # contiguous ranges in index order, shells by increasing radius (paper Sec. 3.2 (1), (2))
    off = 0
    last_m = 2
    for c in cls:
        assert c["offset"] == off
        assert c["m"] >= last_m
        last_m = c["m"]
        off += c["size"]
        assert sum(v * v * k for v, k in c["leader"].items()) == 16 * c["m"]
        assert sum(c["leader"].values()) == 24
        assert c["size"] == c["A"] * c["P1"] * c["P0"] * 2 ** c["B"]
    assert off == oracle13.num_points == 280974212784720
    # "the first 1,104 [indices] belong to the first class, two coordinates equal to 4 and twenty-two equal to 0"
    assert cls[0]["leader"] == {4: 2, 0: 22} and cls[0]["size"] == 1104 and cls[0]["offset"] == 0


def test_class_sizes_by_brute_force_counting_of_sign_and_placement():
    """Cardinality formula checked without the formula: count, for small classes of shell 2 and 3, the points of
    the shell-exhaustive decode that carry each multiset of absolute values."""
    o = Oracle(3)
    X, bad = o.decode_range(0, o.num_points)
    assert bad == 0
    # histogram of absolute values per point, packed into one integer key (7 values 0..6, counts <= 24 < 32)
    A = np.abs(X)
    key = np.zeros(X.shape[0], dtype=np.int64)
    for v in range(7):
        key |= (A == v).sum(axis=1).astype(np.int64) << (5 * v)
    keys, counts = np.unique(key, return_counts=True)
    got = {int(k): int(c) for k, c in zip(keys, counts)}
    for c in o.classes():
        k = sum(cnt << (5 * v) for v, cnt in c["leader"].items())
        assert got[k] == c["size"]
    assert len(got) == 7
