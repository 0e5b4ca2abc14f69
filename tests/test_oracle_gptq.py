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


# ---- closed-form group scales (App. J) and the optional scalar gain quantiser (App. B, Alg. 1) ----------------------
from oracle.gptq_oracle import apply_group_scales, group_scales, nearest_level


def test_group_scales_are_the_hessian_weighted_least_squares_gains():
    """s_i against numpy's least-squares routine on the same problem written without normal equations: with H = L L^T,
    minimise |L^T (w0 - E^T s)|_2, E the row's blocks padded to length K."""
    rng = np.random.default_rng(81)
    N, KB = 6, 5
    K = 24 * KB
    H = _spd(rng, K, cond=100.0)
    L = np.linalg.cholesky(H)
    W0 = rng.standard_normal((N, K))
    Wq = W0 + 0.3 * rng.standard_normal((N, K))
    s = group_scales(W0, Wq, H)
    for i in range(N):
        E = np.zeros((KB, K))
        for p in range(KB):
            E[p, 24 * p:24 * p + 24] = Wq[i, 24 * p:24 * p + 24]
        want = np.linalg.lstsq(L.T @ E.T, L.T @ W0[i], rcond=None)[0]
        assert np.allclose(s[i], want, rtol=1e-8, atol=1e-10)


def test_group_scales_undo_a_rescaling_of_the_blocks_for_any_hessian():
    """blocks that are multiples c_p of the original blocks represent the row exactly with gains 1 / c_p, whatever H"""
    rng = np.random.default_rng(82)
    N, KB = 4, 6
    K = 24 * KB
    W0 = rng.standard_normal((N, K))
    c = rng.uniform(0.3, 3.0, size=(N, KB)) * rng.choice([-1.0, 1.0], size=(N, KB))
    Wq = W0 * np.repeat(c, 24, axis=1)
    for cond in (1.0, 500.0):
        s = group_scales(W0, Wq, _spd(rng, K, cond=cond))
        assert np.allclose(s, 1.0 / c, rtol=1e-7)


def test_group_scales_lower_the_objective_and_damping_shrinks_them(oracle13):
    rng = np.random.default_rng(83)
    K = 96
    H = _spd(rng, K, cond=200.0)
    W = rng.standard_normal((10, K))
    Wq, _, gain = spherical_gptq(oracle13, W, inverse_hessian_factor(H))
    s = group_scales(W, Wq, H)
    refined = Wq * np.repeat(s, 24, axis=1)
    assert proxy_loss(refined, W, H) <= proxy_loss(Wq, W, H) * (1 + 1e-12)
    # no other gains do better: perturbing s raises the objective
    for _ in range(5):
        other = Wq * np.repeat(s + 0.01 * rng.standard_normal(s.shape), 24, axis=1)
        assert proxy_loss(other, W, H) >= proxy_loss(refined, W, H)
    s_damped = group_scales(W, Wq, H, lam=0.5)
    assert (np.linalg.norm(s_damped, axis=1) < np.linalg.norm(s, axis=1)).all()
    # stored format: gains stay float16 and the layer stays gain * direction
    W2, g2 = apply_group_scales(Wq, gain, s)
    assert g2.dtype == np.float16
    ratio = np.linalg.norm(W2.reshape(10, -1, 24), axis=2) / np.linalg.norm(Wq.reshape(10, -1, 24), axis=2)
    assert np.allclose(ratio, np.abs(g2.astype(np.float64) / gain.astype(np.float64)), rtol=1e-12)
    assert np.allclose(g2.astype(np.float64), gain.astype(np.float64) * s, rtol=2 ** -10)


def test_scalar_gain_quantiser_takes_the_nearest_level():
    lv = np.array([0.5, 1.0, 2.0, 4.0], dtype=np.float16)
    got = nearest_level(np.array([0.0, 0.74, 0.76, 1.49, 1.51, 2.9, 3.1, 100.0]), lv)
    assert np.array_equal(got, np.array([0.5, 0.5, 1.0, 1.0, 2.0, 2.0, 4.0, 4.0], dtype=np.float16))


def test_loop_with_a_gain_quantiser_writes_only_levels(oracle13):
    rng = np.random.default_rng(84)
    K = 72
    H = _spd(rng, K)
    W = rng.standard_normal((7, K))
    levels = np.array([3.9, 4.6, 5.2, 6.1], dtype=np.float16)
    Wq, pts, gain = spherical_gptq(oracle13, W, inverse_hessian_factor(H), gain_levels=levels)
    assert set(np.unique(gain)) <= set(levels)
    # every block is its level times its unit direction
    x = pts.astype(np.float64)
    rec = gain.astype(np.float64)[:, :, None] * x / np.linalg.norm(x, axis=2, keepdims=True)
    assert np.allclose(rec.reshape(7, K), Wq, atol=1e-12)
    # the first block sees the original weights: its level is the one nearest to the block's norm
    assert np.array_equal(gain[:, 0], nearest_level(np.linalg.norm(W[:, :24], axis=1), levels))
