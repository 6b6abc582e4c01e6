"""Pins for the oracle's convolutions and the Tucker-2 triple (eq. 4; Section 2: 1x1 -> kxk -> 1x1).
Checked against scipy's correlate2d, linearity (composed dense kernel), the k=1 reduction to the
linear layer, impulse responses, finite differences and adjoint identities."""
import numpy as np
import scipy.signal

import oracle
import synth_inputs as si


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def test_conv_fwd_against_scipy_correlate():
    rng = _rng(1)
    N, Hh, Ww, I, O, k = 2, 6, 7, 3, 4, 3
    X = rng.standard_normal((N, Hh, Ww, I))
    W = rng.standard_normal((O, k, k, I))
    for stride, pad in ((1, 1), (1, 0), (2, 1), (2, 0), (3, 2)):
        Y = oracle.conv_fwd(X, W, stride, pad)
        Xp = np.pad(X, ((0, 0), (pad, pad), (pad, pad), (0, 0)))
        for n in range(N):
            for o in range(O):
                full = sum(scipy.signal.correlate2d(Xp[n, :, :, i], W[o, :, :, i], mode="valid")
                           for i in range(I))
                np.testing.assert_allclose(Y[n, :, :, o], full[::stride, ::stride], rtol=1e-12, atol=1e-12)


def test_impulse_returns_kernel():
    """A unit impulse at the centre, pad = k//2: the output around it is the kernel, flipped in
    space (cross-correlation, no kernel flip in the definition)."""
    k, I, O = 3, 2, 3
    W = _rng(2).standard_normal((O, k, k, I))
    for i in range(I):
        X = np.zeros((1, 5, 5, I))
        X[0, 2, 2, i] = 1.0
        Y = oracle.conv_fwd(X, W, 1, 1)
        for o in range(O):
            np.testing.assert_array_equal(Y[0, 1:4, 1:4, o], W[o, ::-1, ::-1, i])


def test_k1_reduces_to_linear_layer():
    rng = _rng(3)
    N, Hh, Ww, C, S, r = 2, 3, 4, 6, 5, 3
    X = rng.standard_normal((N, Hh, Ww, C))
    P1, G, P2 = si.direct_tucker_factors(S, C, 1, r, r, rng)
    A, B, Y = oracle.tucker_fwd(X, P1, G, P2, 1, 0)
    H, Yl = oracle.linear_fwd(X.reshape(-1, C), G[:, 0, 0, :] @ P1, P2)
    np.testing.assert_allclose(B.reshape(-1, r), H, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(Y.reshape(-1, S), Yl, rtol=1e-12, atol=1e-12)


def test_tucker_chain_equals_dense_conv_with_composed_kernel():
    """Linearity: 1x1 -> kxk -> 1x1 equals one kxk conv with W'[o,u,v,c] = sum_ab P2[o,b] G[b,u,v,a] P1[a,c]
    (eq. 4 read as multilinear products of the core with the two factor matrices)."""
    rng = _rng(4)
    N, Hh, Ww, C, S, r1, r2, k = 2, 6, 5, 7, 6, 4, 3, 3
    X = rng.standard_normal((N, Hh, Ww, C))
    P1, G, P2 = si.direct_tucker_factors(S, C, k, r1, r2, rng)
    Wc = np.einsum("ob,buva,ac->ouvc", P2, G, P1)
    for stride, pad in ((1, 1), (2, 1), (1, 0)):
        _, _, Y = oracle.tucker_fwd(X, P1, G, P2, stride, pad)
        np.testing.assert_allclose(Y, oracle.conv_fwd(X, Wc, stride, pad), rtol=1e-11, atol=1e-12)


def test_conv_adjoints():
    """<conv(A,G), dB> == <A, dgrad(dB,G)> == <G, wgrad(dB,A)>."""
    rng = _rng(5)
    N, Hh, Ww, I, O, k = 2, 7, 6, 3, 4, 3
    for stride, pad in ((1, 1), (2, 1), (2, 0), (1, 2)):
        A = rng.standard_normal((N, Hh, Ww, I))
        G = rng.standard_normal((O, k, k, I))
        B = oracle.conv_fwd(A, G, stride, pad)
        dB = rng.standard_normal(B.shape)
        lhs = float(np.sum(B * dB))
        dA = oracle.conv_dgrad(dB, G, (Hh, Ww), stride, pad)
        dG = oracle.conv_wgrad(dB, A, k, stride, pad)
        assert abs(lhs - float(np.sum(A * dA))) <= 1e-12 * abs(lhs) + 1e-12
        assert abs(lhs - float(np.sum(G * dG))) <= 1e-12 * abs(lhs) + 1e-12


def _tucker_loss(X, P1, G, P2, s, p):
    _, _, Y = oracle.tucker_fwd(X, P1, G, P2, s, p)
    return 0.5 * float(np.sum(Y * Y))


def test_tucker_backward_matches_finite_differences():
    rng = _rng(6)
    N, Hh, Ww, C, S, r1, r2, k = 1, 4, 4, 3, 2, 2, 2, 3
    for stride, pad in ((1, 1), (2, 1)):
        X = rng.standard_normal((N, Hh, Ww, C))
        P1, G, P2 = si.direct_tucker_factors(S, C, k, r1, r2, rng)
        A, B, Y = oracle.tucker_fwd(X, P1, G, P2, stride, pad)
        g = oracle.tucker_bwd(Y, X, A, B, P1, G, P2, 0, stride, pad)
        h = 1e-6
        for name, arr, grad in (("X", X, g["dX"]), ("P1", P1, g["dP1"]), ("G", G, g["dG"]), ("P2", P2, g["dP2"])):
            fd = np.zeros_like(arr)
            for idx in np.ndindex(arr.shape):
                keep = arr[idx]
                arr[idx] = keep + h
                lp = _tucker_loss(X, P1, G, P2, stride, pad)
                arr[idx] = keep - h
                lm = _tucker_loss(X, P1, G, P2, stride, pad)
                arr[idx] = keep
                fd[idx] = (lp - lm) / (2 * h)
            err = np.max(np.abs(fd - grad)) / np.max(np.abs(grad))
            assert err < 1e-7, (name, stride, err)


def test_tucker_freezing():
    rng = _rng(7)
    N, Hh, Ww, C, S, r1, r2, k = 2, 5, 5, 4, 3, 3, 2, 3
    X = rng.standard_normal((N, Hh, Ww, C))
    P1, G, P2 = si.direct_tucker_factors(S, C, k, r1, r2, rng)
    A, B, Y = oracle.tucker_fwd(X, P1, G, P2, 1, 1)
    dY = rng.standard_normal(Y.shape)
    free = oracle.tucker_bwd(dY, X, A, B, P1, G, P2, 0, 1, 1)
    names = ("dP1", "dG", "dP2")
    for mask in range(8):
        g = oracle.tucker_bwd(dY, X, A, B, P1, G, P2, mask, 1, 1)
        for bit, nm in enumerate(names):
            if mask & (1 << bit):
                assert np.all(np.isnan(g[nm]))             # frozen: buffer left as it was (NaN fill)
            else:
                assert np.array_equal(g[nm], free[nm])
        assert np.array_equal(g["dX"], free["dX"])         # data gradient flows regardless
    assert oracle.freeze_mask(oracle.KIND_TUCKER, 0) == 0b101
    assert oracle.freeze_mask(oracle.KIND_TUCKER, 1) == 0b010


def test_dense_conv_gradients_against_composed_tucker():
    """dX of the triple equals dgrad of the composed dense kernel; dG equals the dense wgrad
    projected on the factors: dG[b,u,v,a] = sum_oc P2[o,b] dW'[o,u,v,c] P1[a,c]."""
    rng = _rng(8)
    N, Hh, Ww, C, S, r1, r2, k = 2, 5, 6, 5, 4, 3, 3, 3
    X = rng.standard_normal((N, Hh, Ww, C))
    P1, G, P2 = si.direct_tucker_factors(S, C, k, r1, r2, rng)
    Wc = np.einsum("ob,buva,ac->ouvc", P2, G, P1)
    A, B, Y = oracle.tucker_fwd(X, P1, G, P2, 1, 1)
    dY = rng.standard_normal(Y.shape)
    g = oracle.tucker_bwd(dY, X, A, B, P1, G, P2, 0, 1, 1)
    np.testing.assert_allclose(g["dX"], oracle.conv_dgrad(dY, Wc, (Hh, Ww), 1, 1), rtol=1e-11, atol=1e-12)
    dWc = oracle.conv_wgrad(dY, X, k, 1, 1)
    np.testing.assert_allclose(g["dG"], np.einsum("ob,ouvc,ac->buva", P2, dWc, P1), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(g["dP2"], np.einsum("ouvc,buva,ac->ob", dWc, G, P1), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(g["dP1"], np.einsum("ob,buva,ouvc->ac", P2, G, dWc), rtol=1e-11, atol=1e-12)
