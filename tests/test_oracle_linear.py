"""Pins for the oracle's SVD-decomposed linear layer (Section 2, Fig. 1) and its backward with
freezing (Section 2.2).  Each check uses something other than the oracle's own formula: numpy's
dense matmul, finite differences, closed-form identities, sentinels."""
import numpy as np
import scipy.special

import oracle
import synth_inputs as si


def _case(T, n_in, n_out, r, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    X = rng.standard_normal((T, n_in))
    U, V = si.direct_factors(n_out, n_in, r, rng)
    dY = rng.standard_normal((T, n_out))
    return X, U, V, dY


def test_chain_equals_dense_product():
    """Two consecutive layers == one layer with weight U.V (the layer pair replaces W ~= U V)."""
    for (T, n_in, n_out, r) in ((7, 13, 11, 5), (33, 40, 24, 24), (5, 9, 30, 1)):
        X, U, V, _ = _case(T, n_in, n_out, r, 11)
        b = np.linspace(-1, 1, n_out)
        H, Y = oracle.linear_fwd(X, V, U, b)
        np.testing.assert_allclose(H, X @ V.T, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(Y, X @ (U @ V).T + b, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(oracle.dense_linear_fwd(X, U @ V, b), Y, rtol=1e-12, atol=1e-12)


def test_rank_one_is_outer_product():
    X, U, V, _ = _case(6, 8, 5, 1, 3)
    _, Y = oracle.linear_fwd(X, V, U)
    np.testing.assert_allclose(Y, np.outer(X @ V[0], U[:, 0]), rtol=1e-13, atol=1e-13)


def test_full_rank_svd_pair_equals_original_layer():
    rng = np.random.Generator(np.random.PCG64(5))
    W = rng.standard_normal((12, 9))
    X = rng.standard_normal((4, 9))
    U, V, _ = oracle.svd_factors(W, 9)
    _, Y = oracle.linear_fwd(X, V, U)
    np.testing.assert_allclose(Y, X @ W.T, rtol=1e-10, atol=1e-10)


def _loss(X, V, U):
    _, Y = oracle.linear_fwd(X, V, U)
    return 0.5 * float(np.sum(Y * Y))


def test_backward_matches_finite_differences():
    """L = 0.5 ||Y||^2  =>  dY = Y; central differences on every entry of X, U, V."""
    T, n_in, n_out, r = 3, 5, 4, 2
    X, U, V, _ = _case(T, n_in, n_out, r, 17)
    H, Y = oracle.linear_fwd(X, V, U)
    g = oracle.linear_bwd(Y, X, H, V, U, mask=0)
    h = 1e-6
    for name, arr, grad in (("X", X, g["dX"]), ("U", U, g["dU"]), ("V", V, g["dV"])):
        fd = np.zeros_like(arr)
        for idx in np.ndindex(arr.shape):
            keep = arr[idx]
            arr[idx] = keep + h
            lp = _loss(X, V, U)
            arr[idx] = keep - h
            lm = _loss(X, V, U)
            arr[idx] = keep
            fd[idx] = (lp - lm) / (2 * h)
        err = np.max(np.abs(fd - grad)) / np.max(np.abs(grad))
        assert err < 1e-7, (name, err)


def test_backward_closed_forms_against_dense_gradients():
    """With dW = dY^T X of the undecomposed layer: dU = dW V^T, dV = U^T dW, dX = dY (U V)."""
    T, n_in, n_out, r = 19, 23, 17, 6
    X, U, V, dY = _case(T, n_in, n_out, r, 23)
    H, _ = oracle.linear_fwd(X, V, U)
    g = oracle.linear_bwd(dY, X, H, V, U, mask=0, want_dbias=True)
    dW = dY.T @ X
    np.testing.assert_allclose(g["dU"], dW @ V.T, rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(g["dV"], U.T @ dW, rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(g["dX"], dY @ (U @ V), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(g["dH"], dY @ U, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(g["dbias"], dY.sum(0), rtol=1e-12, atol=1e-12)
    dXd, dWd = oracle.dense_linear_bwd(dY, X, U @ V)
    np.testing.assert_allclose(dXd, g["dX"], rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dWd, dW, rtol=1e-11, atol=1e-11)


def test_frozen_factor_untouched_and_others_unchanged():
    T, n_in, n_out, r = 9, 10, 8, 3
    X, U, V, dY = _case(T, n_in, n_out, r, 29)
    H, _ = oracle.linear_fwd(X, V, U)
    free = oracle.linear_bwd(dY, X, H, V, U, mask=0)
    sent_v = np.full((r, n_in), -7.25)
    sent_u = np.full((n_out, r), 3.5)
    fv = oracle.linear_bwd(dY, X, H, V, U, mask=oracle.FREEZE_L0, dV_init=sent_v, dU_init=sent_u)
    assert np.array_equal(fv["dV"], sent_v)               # frozen: not written
    assert np.array_equal(fv["dU"], free["dU"])           # trainable: same bits as unfrozen run
    assert np.array_equal(fv["dX"], free["dX"]) and np.array_equal(fv["dH"], free["dH"])
    fu = oracle.linear_bwd(dY, X, H, V, U, mask=oracle.FREEZE_L1, dV_init=sent_v, dU_init=sent_u)
    assert np.array_equal(fu["dU"], sent_u)
    assert np.array_equal(fu["dV"], free["dV"])
    assert np.array_equal(fu["dX"], free["dX"])           # gradient still flows through frozen U
    both = oracle.linear_bwd(dY, X, H, V, U, mask=3, dV_init=sent_v, dU_init=sent_u)
    assert np.array_equal(both["dU"], sent_u) and np.array_equal(both["dV"], sent_v)
    # the schedule of Algorithm 2 picks exactly these masks
    assert oracle.freeze_mask(oracle.KIND_SVD, 0) == oracle.FREEZE_L0
    assert oracle.freeze_mask(oracle.KIND_SVD, 1) == oracle.FREEZE_L1


def test_gelu_against_scipy_and_differences():
    z = np.linspace(-6, 6, 241)
    np.testing.assert_allclose(oracle.gelu_fwd(z), z * scipy.special.ndtr(z), rtol=1e-13, atol=1e-15)
    h = 1e-6
    fd = (oracle.gelu_fwd(z + h) - oracle.gelu_fwd(z - h)) / (2 * h)
    dA = np.cos(z)
    np.testing.assert_allclose(oracle.gelu_bwd(dA, z), dA * fd, rtol=1e-8, atol=1e-9)
