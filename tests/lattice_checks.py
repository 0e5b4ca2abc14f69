"""Independent checks used to pin the oracle (no oracle code is reused here).

Everything is rebuilt from the definitions in the paper's Sec. 2.3: the Golay code from its
generator polynomial by polynomial multiplication over GF(2) (numpy), and the three membership
conditions (i)-(iii) of the integer-coordinate Leech lattice, vectorised.
"""
import numpy as np

GEN_POLY = 0b110001110101  # x^11 + x^10 + x^6 + x^5 + x^4 + x^2 + 1


def clmul(a, b):
    """carry-less product of two GF(2) polynomials given as Python ints"""
    r = 0
    while b:
        if b & 1:
            r ^= a
        a <<= 1
        b >>= 1
    return r


def polymod(a, m):
    dm = m.bit_length()
    while a.bit_length() >= dm:
        a ^= m << (a.bit_length() - dm)
    return a


def golay_words():
    """all 4096 words: message polynomial times the generator, plus an overall parity bit at position 23"""
    words = np.zeros(4096, dtype=np.uint32)
    for u in range(4096):
        c = clmul(u, GEN_POLY)
        if bin(c).count("1") & 1:
            c |= 1 << 23
        words[u] = c
    return words


_member = None


def golay_member_table():
    global _member
    if _member is None:
        t = np.zeros(1 << 24, dtype=bool)
        t[golay_words()] = True
        _member = t
    return _member


def is_leech_int(X):
    """X: int array [n,24] -> bool [n]: conditions (i), (ii), (iii) for L_even U L_odd"""
    X = np.asarray(X).astype(np.int64)
    p = X[:, :1] & 1
    cond1 = ((X & 1) == p).all(axis=1)
    half = (X - p) >> 1                      # exact when (i) holds
    bits = (half & 1).astype(np.uint32)
    code = (bits << np.arange(24, dtype=np.uint32)).sum(axis=1).astype(np.uint32)
    cond2 = golay_member_table()[code]
    want = np.where(p[:, 0] == 1, 4, 0)
    cond3 = (X.sum(axis=1) % 8) == want
    return cond1 & cond2 & cond3


def row_hash(X):
    """64-bit mix of each row; equal rows hash equally, so `#distinct hashes == n` proves all rows distinct"""
    X = np.asarray(X).astype(np.int64) + 32
    h = np.zeros(X.shape[0], dtype=np.uint64)
    with np.errstate(over="ignore"):
        for i in range(X.shape[1]):
            h = h * np.uint64(0x9E3779B97F4A7C15) + X[:, i].astype(np.uint64) + np.uint64(0x632BE59BD9B4E019)
            h ^= h >> np.uint64(29)
    return h


def theta_coefficients(mmax):
    """Leech theta series: number of lattice vectors of squared norm 2m is 65520/691 * (sigma_11(m) - tau(m))."""
    n = mmax + 1
    # tau from q * prod (1-q^k)^24
    poly = [0] * (n + 1)
    poly[0] = 1
    for k in range(1, n + 1):
        for _ in range(24):
            for d in range(n, k - 1, -1):
                poly[d] -= poly[d - k]
    tau = [0] + poly[:n]                     # tau[m] = coefficient of q^(m-1) in the product
    out = {}
    for m in range(1, mmax + 1):
        sigma = sum(d ** 11 for d in range(1, m + 1) if m % d == 0)
        num = 65520 * (sigma - tau[m])
        assert num % 691 == 0
        out[m] = num // 691
    return out
