"""Oracle of the block-wise quantisation loop with Hessian corrections (paper App. B, Alg. 1; Sec. 3.3).

TEST INFRASTRUCTURE, NOT THE PRODUCT: plain numpy in fp64, the steps of the algorithm in the paper's order, the
direction quantiser being the oracle's exhaustive nearest-direction search.  Only tests may import this module.
"""
import numpy as np


def inverse_hessian_factor(H):
    """U upper triangular with H^-1 = U^T U (paper App. B, line "U <- chol(H^-1)^T")."""
    G = np.linalg.inv(np.asarray(H, dtype=np.float64))
    L = np.linalg.cholesky((G + G.T) / 2)          # G = L L^T, L lower
    return L.T


def spherical_gptq(oracle, W, U, direction=None):
    """W: [N, 24*KB] weights; U: [K, K] upper factor of H^-1.
    Returns (quantised layer fp64, points int8 [N, KB, 24], gains float16 [N, KB]).
    direction(v) -> int8 points replaces the nearest-direction search (used by the pins to plant any quantiser)."""
    W = np.array(W, dtype=np.float64)
    U = np.asarray(U, dtype=np.float64)
    N, K = W.shape
    KB = K // 24
    pts = np.zeros((N, KB, 24), dtype=np.int8)
    gain = np.zeros((N, KB), dtype=np.float16)
    for t in range(KB):
        Q = slice(24 * t, 24 * t + 24)
        v = W[:, Q].copy()
        x = direction(v) if direction is not None else oracle.nearest(v)[0]
        g = np.linalg.norm(v, axis=1).astype(np.float16)                 # gain reset: the block keeps its norm (fp16)
        xf = x.astype(np.float64)
        vhat = g.astype(np.float64)[:, None] * xf / np.linalg.norm(xf, axis=1)[:, None]
        E = v - vhat
        W[:, Q] = vhat
        pts[:, t], gain[:, t] = x, g
        if 24 * t + 24 < K:
            R = slice(24 * t + 24, K)
            W[:, R] -= (E @ np.linalg.inv(U[Q, Q])) @ U[Q, R]
    return W, pts, gain


def proxy_loss(W_hat, W, H):
    """Tr((W_hat - W) H (W_hat - W)^T): the local objective of paper App. F"""
    D = np.asarray(W_hat, dtype=np.float64) - np.asarray(W, dtype=np.float64)
    return float(np.einsum("ik,kl,il->", D, np.asarray(H, dtype=np.float64), D))
