"""Oracle of the block-wise quantisation with Hessian corrections (paper App. B, Alg. 1; Sec. 3.3; App. F) and of the
closed-form group-scale refinement that may follow it (paper App. J, "Spherically projected GPTQ with group scales").

TEST INFRASTRUCTURE, NOT THE PRODUCT: plain numpy in fp64, written from the definitions -- per block the nearest
direction, the retraction onto the sphere of the block's own radius, and the least-squares propagation of the error
through the factor of the inverse Hessian; afterwards, per row, the Hessian-weighted least-squares gains of the fixed
directions.  The direction quantiser is the oracle's exhaustive nearest-direction search.  Only tests may import this.
"""
import numpy as np


def inverse_hessian_factor(H):
    """Upper-triangular U with U^T U = H^-1 (the factor that App. B, Alg. 1 propagates errors through)."""
    G = np.linalg.inv(np.asarray(H, dtype=np.float64))
    L = np.linalg.cholesky((G + G.T) / 2)          # G = L L^T, L lower
    return L.T


def nearest_level(norms, levels):
    """Scalar gain quantiser (App. B, Alg. 1, the optional Q_gain): every norm goes to the nearest of `levels`
    (ties to the lower level).  Returns the chosen levels as float16."""
    lv = np.sort(np.asarray(levels, dtype=np.float16).astype(np.float64))
    d = np.abs(np.asarray(norms, dtype=np.float64)[:, None] - lv[None, :])
    return lv[np.argmin(d, axis=1)].astype(np.float16)


def retract(v, x, gain_levels=None):
    """The block v replaced by the direction x at a radius of its own (Sec. 3.3, the spherical retraction): the radius
    is the norm of v rounded to float16, or, with gain_levels, the nearest level of the scalar gain quantiser."""
    norms = np.linalg.norm(v, axis=1)
    g = norms.astype(np.float16) if gain_levels is None else nearest_level(norms, gain_levels)
    xf = x.astype(np.float64)
    return g.astype(np.float64)[:, None] * xf / np.linalg.norm(xf, axis=1)[:, None], g


def spherical_gptq(oracle, W, U, direction=None, gain_levels=None):
    """W: [N, 24*KB] weights; U: [K, K] upper factor of H^-1.
    Returns (quantised layer fp64, points int8 [N, KB, 24], gains float16 [N, KB]).
    direction(v) -> int8 points replaces the nearest-direction search (used by the pins to plant any quantiser);
    gain_levels: reconstruction levels of the optional scalar gain quantiser."""
    W = np.array(W, dtype=np.float64)
    U = np.asarray(U, dtype=np.float64)
    N, K = W.shape
    KB = K // 24
    pts = np.zeros((N, KB, 24), dtype=np.int8)
    gain = np.zeros((N, KB), dtype=np.float16)
    for t in range(KB):
        lo, hi = 24 * t, 24 * t + 24
        block = W[:, lo:hi].copy()
        pts[:, t] = direction(block) if direction is not None else oracle.nearest(block)[0]
        W[:, lo:hi], gain[:, t] = retract(block, pts[:, t], gain_levels)
        if hi < K:
            # the error of this block, expressed in the rows of U that belong to it, is taken out of every column to
            # the right: the update that keeps Tr(dW H dW^T) minimal with the processed columns fixed (App. F)
            coeff = np.linalg.solve(U[lo:hi, lo:hi].T, (block - W[:, lo:hi]).T).T
            W[:, hi:] -= coeff @ U[lo:hi, hi:]
    return W, pts, gain


def group_scales(W0, Wq, H, lam=0.0):
    """Per row i the gains s_i that minimise (W0_i - sum_p s_p e_p) H (W0_i - sum_p s_p e_p)^T + lam |s|^2, e_p the row's
    quantised block p padded with zeros to length K (App. J, closed-form group scales): the normal equations
    (M_i + lam I) s_i = r_i with M_i[p, q] = Wq_{i,p} H_{pq} Wq_{i,q}^T and r_i[p] = Wq_{i,p} H_{p,:} W0_i^T.
    Returns s [N, KB]."""
    W0 = np.asarray(W0, dtype=np.float64)
    Wq = np.asarray(Wq, dtype=np.float64)
    H = np.asarray(H, dtype=np.float64)
    N, K = Wq.shape
    KB = K // 24
    s = np.zeros((N, KB))
    for i in range(N):
        E = np.zeros((KB, K))
        for p in range(KB):
            E[p, 24 * p:24 * p + 24] = Wq[i, 24 * p:24 * p + 24]
        M = E @ H @ E.T
        r = E @ H @ W0[i]
        s[i] = np.linalg.solve(M + lam * np.eye(KB), r)
    return s


def apply_group_scales(Wq, gain, s):
    """The refined layer in the stored format: the new gain of a block is gain * s rounded to float16, and the block is
    rescaled by exactly the ratio of the two float16 gains, so that it stays what the decoder reconstructs."""
    g_old = gain.astype(np.float64)
    g_new = (g_old * s).astype(np.float16)
    ratio = np.divide(g_new.astype(np.float64), g_old, out=np.zeros_like(g_old), where=g_old != 0)
    return np.asarray(Wq, dtype=np.float64) * np.repeat(ratio, 24, axis=1), g_new


def proxy_loss(W_hat, W, H):
    """Tr((W_hat - W) H (W_hat - W)^T): the local objective of paper App. F"""
    D = np.asarray(W_hat, dtype=np.float64) - np.asarray(W, dtype=np.float64)
    return float(np.einsum("ik,kl,il->", D, np.asarray(H, dtype=np.float64), D))
