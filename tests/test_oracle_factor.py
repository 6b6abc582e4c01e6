"""Pins for the oracle's one-time factorizations: SVD (eq. 1), truncation (eq. 2) with its
reconstruction error (eq. 3), and Tucker-2 by truncated HOSVD (eq. 4).  Factors are unique only
up to signs/rotations, so products, singular values and projectors are compared, never factors."""
import math

import numpy as np

import oracle
import synth_inputs as si


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def test_svd_against_lapack_and_orthonormality():
    for (m, n) in ((9, 9), (14, 6), (5, 12), (40, 33)):
        M = _rng(m * 100 + n).standard_normal((m, n))
        U, s, V = oracle.svd(M)
        np.testing.assert_allclose(s, np.linalg.svd(M, compute_uv=False), rtol=1e-11, atol=1e-12)
        assert np.all(np.diff(s) <= 0)
        R = min(m, n)
        assert np.max(np.abs(U.T @ U - np.eye(R))) < 1e-12
        assert np.max(np.abs(V.T @ V - np.eye(R))) < 1e-12
        assert np.max(np.abs((U * s) @ V.T - M)) < 1e-10


def test_svd_tolerates_rank_deficiency():
    rng = _rng(7)
    M = rng.standard_normal((8, 3)) @ rng.standard_normal((3, 10))      # rank 3
    U, s, V = oracle.svd(M)
    assert np.all(s[3:] < 1e-12)
    assert np.max(np.abs((U * s) @ V.T - M)) < 1e-10


def test_full_rank_factors_reconstruct_and_eckart_young():
    rng = _rng(8)
    W = rng.standard_normal((18, 25))
    sig = np.linalg.svd(W, compute_uv=False)
    U, V, s = oracle.svd_factors(W, 18)
    assert np.max(np.abs(U @ V - W)) < 1e-10
    np.testing.assert_allclose(s, sig, rtol=1e-11)
    for r in (1, 4, 11, 17):
        U, V, _ = oracle.svd_factors(W, r)
        err = np.linalg.norm(W - U @ V)                                    # eq. 3 (Frobenius)
        assert abs(err - math.sqrt(np.sum(sig[r:] ** 2))) < 1e-10
        # sigma is split evenly: both factors carry sqrt(sigma) => U^T U = V V^T = diag(sigma)
        np.testing.assert_allclose(U.T @ U, np.diag(sig[:r]), atol=1e-10)
        np.testing.assert_allclose(V @ V.T, np.diag(sig[:r]), atol=1e-10)


def test_config1_closed_forms():
    """W = Q1 diag(exp(-i/100)) Q2^T, 768 x 768: the spectrum and the truncation errors are known
    in closed form (geometric sums)."""
    W, sigma = si.config1_weight()
    r = oracle.quantize_rank(200, 16)
    assert r == 208
    U, V, s = oracle.svd_factors(W, r)
    np.testing.assert_allclose(s, sigma, rtol=0, atol=1e-10)
    q = math.exp(-0.02)

    def tail(a):          # sqrt(sum_{i>=a}^{767} exp(-2 i/100))
        return math.sqrt((q ** a - q ** 768) / (1 - q))

    assert abs(np.linalg.norm(W) - tail(0)) < 1e-10
    assert abs(tail(0) - 7.106451707951675) < 1e-12
    assert abs(np.linalg.norm(W - U @ V) - tail(208)) < 1e-10
    assert abs(tail(208) - 0.8878045445230569) < 1e-12
    assert abs(tail(200) - 0.9617481539550401) < 1e-12
    assert abs(tail(208) / tail(0) - 0.12492937136681857) < 1e-12


def test_tucker2_full_rank_is_exact_and_factors_orthonormal():
    rng = _rng(9)
    S, C, k = 6, 5, 3
    W = rng.standard_normal((S, k, k, C))
    P1, G, P2, tau = oracle.tucker2(W, C, S)
    assert np.max(np.abs(np.einsum("ob,buva,ac->ouvc", P2, G, P1) - W)) < 1e-10
    assert np.max(np.abs(tau)) < 1e-20
    P1, G, P2, _ = oracle.tucker2(W, 3, 4)
    assert G.shape == (4, k, k, 3)
    assert np.max(np.abs(P1 @ P1.T - np.eye(3))) < 1e-12
    assert np.max(np.abs(P2.T @ P2 - np.eye(4))) < 1e-12


def test_tucker2_error_bounds_and_subspaces():
    """Truncated HOSVD: max(tau1,tau2) <= ||W - W'||_F^2 <= tau1 + tau2, tau_n = discarded squared
    mode-n singular values; the factor subspaces are those of the unfoldings (LAPACK projectors)."""
    rng = _rng(10)
    S, C, k, r1, r2 = 8, 7, 3, 4, 5
    W = rng.standard_normal((S, k, k, C)) * np.exp(-np.arange(C) / 2.0)[None, None, None, :]
    P1, G, P2, tau = oracle.tucker2(W, r1, r2)
    Wr = np.einsum("ob,buva,ac->ouvc", P2, G, P1)
    e2 = float(np.sum((W - Wr) ** 2))
    assert max(tau) - 1e-10 <= e2 <= tau[0] + tau[1] + 1e-10
    Mc = W.reshape(-1, C).T                       # C x (S k k)
    Ms = W.reshape(S, -1)                         # S x (k k C)
    uc, sc, _ = np.linalg.svd(Mc, full_matrices=False)
    us, ss, _ = np.linalg.svd(Ms, full_matrices=False)
    np.testing.assert_allclose(tau, [np.sum(sc[r1:] ** 2), np.sum(ss[r2:] ** 2)], rtol=1e-10)
    np.testing.assert_allclose(P1.T @ P1, uc[:, :r1] @ uc[:, :r1].T, atol=1e-9)
    np.testing.assert_allclose(P2 @ P2.T, us[:, :r2] @ us[:, :r2].T, atol=1e-9)
    # the core is the projection of W on both subspaces
    np.testing.assert_allclose(G, np.einsum("ob,ouvc,ac->buva", P2, W, P1), atol=1e-12)


def test_tucker2_k1_is_two_sided_projection():
    rng = _rng(11)
    S, C, r1, r2 = 7, 9, 3, 4
    M = rng.standard_normal((S, C))
    P1, G, P2, _ = oracle.tucker2(M.reshape(S, 1, 1, C), r1, r2)
    u, s, vt = np.linalg.svd(M)
    np.testing.assert_allclose(P2 @ P2.T, u[:, :r2] @ u[:, :r2].T, atol=1e-10)
    np.testing.assert_allclose(P1.T @ P1, vt[:r1].T @ vt[:r1], atol=1e-10)
    np.testing.assert_allclose(P2 @ G[:, 0, 0, :] @ P1, (P2 @ P2.T) @ M @ (P1.T @ P1), atol=1e-10)
