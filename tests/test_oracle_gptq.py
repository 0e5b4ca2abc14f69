"""Pins of the oracle's block-wise loop with Hessian corrections (paper App. B, App. F): the propagation is checked
against the closed-form minimiser of the local objective computed from H alone, never from the loop's own factor U."""
import numpy as np
import pytest

from oracle.gptq_oracle import inverse_hessian_factor, proxy_loss, spherical_gptq


def _spd(rng, K, cond=30.0):
    X = rng.standard_normal((4 * K, K)) @ np.diag(np.linspace(1.0, np.sqrt(cond), K)) @ np.linalg.qr(rng.standard_normal((K, K)))[0]
    return X.T @ X / X.shape[0] + 0.01 * np.eye(K)


def test_factor_reproduces_the_inverse_hessian():
    rng = np.random.default_rng(71)
    H = _spd(rng, 72)
    U = inverse_hessian_factor(H)
    assert np.allclose(np.triu(U), U) and np.allclose(U.T @ U @ H, np.eye(72), atol=1e-9)


def test_propagation_is_the_minimiser_of_the_local_objective():
    """With ANY quantiser in the loop, after every step the not yet processed columns equal
    W_R - D H_DR H_RR^-1, D the error on the processed columns: the minimiser of Tr(dW H dW^T) over dW_R (App. F)."""
    rng = np.random.default_rng(72)
    N, KB = 5, 4
    K = 24 * KB
    H = _spd(rng, K)
    U = inverse_hessian_factor(H)
    W = rng.standard_normal((N, K))
    planted = rng.integers(-3, 4, size=(KB, N, 24)).astype(np.int8)
    planted[planted == 0] = 1
    step = [0]

    def direction(v):
        step[0] += 1
        return planted[step[0] - 1]

    W_hat, pts, gain = spherical_gptq(None, W, U, direction)
    # replay: the same quantised blocks, corrections from the closed form on H
    Wc = W.copy()
    for t in range(KB):
        Q = slice(24 * t, 24 * t + 24)
        xf = planted[t].astype(np.float64)
        g = np.linalg.norm(Wc[:, Q], axis=1).astype(np.float16).astype(np.float64)
        Wc[:, Q] = g[:, None] * xf / np.linalg.norm(xf, axis=1)[:, None]
        if t + 1 < KB:
            D = Wc[:, :24 * t + 24] - W[:, :24 * t + 24]
            R = slice(24 * t + 24, K)
            Wc[:, R] = W[:, R] - D @ H[:24 * t + 24, R] @ np.linalg.inv(H[R, R])
    assert np.allclose(W_hat, Wc, atol=1e-9)
    assert np.array_equal(pts, planted.transpose(1, 0, 2))


def test_identity_hessian_means_independent_blocks(oracle13):
    rng = np.random.default_rng(73)
    W = rng.standard_normal((3, 48))
    W_hat, pts, gain = spherical_gptq(oracle13, W, np.eye(48))
    for t in range(2):
        v = W[:, 24 * t:24 * t + 24]
        x, _ = oracle13.nearest(v)
        assert np.array_equal(pts[:, t], x)
        # the gain reset keeps the norm of the block (to fp16)
        assert np.allclose(np.linalg.norm(W_hat[:, 24 * t:24 * t + 24], axis=1), np.linalg.norm(v, axis=1), rtol=2 ** -11)


def test_corrections_lower_the_local_objective(oracle13):
    """on a correlated H the loop with corrections beats the same quantiser without them (U = I)"""
    rng = np.random.default_rng(74)
    K = 72
    H = _spd(rng, K, cond=200.0)
    W = rng.standard_normal((12, K))
    with_corr, _, _ = spherical_gptq(oracle13, W, inverse_hessian_factor(H))
    without, _, _ = spherical_gptq(oracle13, W, np.eye(K))
    assert proxy_loss(with_corr, W, H) < 0.9 * proxy_loss(without, W, H)
