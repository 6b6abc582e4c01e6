"""GPU parity of the on-device factorization (eq. 1, 2: rank-r SVD pair; eq. 4: Tucker-2 by HOSVD)
against the oracle's fp64 Jacobi SVD.  Singular vectors are unique only up to sign (and up to a
rotation inside a repeated singular value), so what is compared is what is unique: the singular
values, the rank-r product U.V, the projectors onto the leading subspaces and the reconstruction;
the rest is checked for validity (orthogonality, the sqrt(sigma) split)."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from parity import host, workspace
from paper_2309_03824_amd import binding as lrd

pytestmark = pytest.mark.gpu


def _f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def _run_svd(W32, r):
    n_out, n_in = W32.shape
    U = torch.empty((n_out, r), dtype=torch.float32, device="cuda")
    V = torch.empty((r, n_in), dtype=torch.float32, device="cuda")
    ws = workspace(lrd.svd_factors_workspace_bytes(n_out, n_in))
    sig, sweeps = lrd.svd_factors(_f32(W32), r, U, V, ws)
    return host(U), host(V), np.array(sig), sweeps


@pytest.mark.parametrize("shape_r", [((96, 160), 24), ((200, 64), 16), ((64, 64), 64), ((33, 70), 9), ((1, 40), 1),
                                     ((256, 768), 64)])
def test_svd_pair_matches_oracle(shape_r):
    (n_out, n_in), r = shape_r
    rng = si.rng_for(6, n_out * 1000 + n_in)
    # a decaying spectrum (as trained weights have) on top of noise: distinct singular values
    W = si.gaussian((n_out, n_in), rng) * 0.05
    k = min(n_out, n_in)
    W += (si.haar_orthogonal(n_out, rng)[:, :k] * np.exp(-np.arange(k) / max(4.0, k / 8.0))) @ si.haar_orthogonal(n_in, rng)[:k, :]
    W32 = W.astype(np.float32)
    Uo, Vo, so = oracle.svd_factors(W32.astype(np.float64), r)
    U, V, s, sweeps = _run_svd(W32, r)
    assert 1 <= sweeps <= 30 or k == 1
    scale = so[0]
    assert np.max(np.abs(s - so)) <= 1e-9 * scale                      # singular values, all of them, descending
    assert np.all(np.diff(s) <= 0)
    assert np.max(np.abs(U @ V - Uo @ Vo)) <= 2e-6 * scale             # rank-r product (fp32 outputs)
    # validity: columns of U and rows of V orthogonal, each carrying sqrt(sigma)
    assert np.max(np.abs(U.T @ U - np.diag(s[:r]))) <= 2e-6 * scale
    assert np.max(np.abs(V @ V.T - np.diag(s[:r]))) <= 2e-6 * scale


def test_svd_pair_of_a_rank_deficient_weight():
    rng = si.rng_for(6, 77)
    W32 = (si.gaussian((48, 10), rng) @ si.gaussian((10, 80), rng)).astype(np.float32)   # rank 10
    Uo, Vo, so = oracle.svd_factors(W32.astype(np.float64), 12)
    U, V, s, _ = _run_svd(W32, 12)
    assert np.max(np.abs(s[:10] - so[:10])) <= 1e-9 * so[0]
    assert np.max(np.abs(s[10:])) <= 1e-6 * so[0]                      # fp32 input: the null space is at rounding level
    assert np.max(np.abs(U @ V - W32)) <= 1e-5 * so[0]                 # rank 12 >= 10 reproduces the weight
    assert np.max(np.abs(U @ V - Uo @ Vo)) <= 1e-5 * so[0]


def test_svd_rejects_bad_arguments():
    W = _f32(np.zeros((8, 8)))
    U = torch.empty((8, 4), dtype=torch.float32, device="cuda")
    V = torch.empty((4, 8), dtype=torch.float32, device="cuda")
    with pytest.raises(lrd.LrdError) as e:
        lrd.svd_factors(W, 9, U, V, workspace(lrd.svd_factors_workspace_bytes(8, 8)))
    assert e.value.status == lrd.ERR_INVALID_ARG
    with pytest.raises(lrd.LrdError) as e:
        lrd.svd_factors(W, 4, U, V, workspace(64))
    assert e.value.status == lrd.ERR_WORKSPACE


def _reconstruct(P1, G, P2):
    # W'[o,u,v,c] = sum_{b,a} P2[o,b] G[b,u,v,a] P1[a,c]
    return np.einsum("ob,buva,ac->ouvc", P2, G, P1)


@pytest.mark.parametrize("geo", [(32, 24, 3, 8, 12), (16, 40, 3, 16, 8), (48, 48, 1, 12, 12), (8, 96, 3, 20, 8),
                                 (64, 64, 3, 32, 32)])
def test_tucker2_matches_oracle(geo):
    S, C, k, r1, r2 = geo
    rng = si.rng_for(6, sum(geo))
    W = si.conv_weight(S, C, k, rng)
    # give both channel modes a decaying spectrum so that the leading subspaces are well separated
    W = np.einsum("ouvc,o,c->ouvc", W, np.exp(-np.arange(S) / (S / 4.0)), np.exp(-np.arange(C) / (C / 4.0)))
    W = np.einsum("po,ouvc,cd->puvd", si.haar_orthogonal(S, rng), W, si.haar_orthogonal(C, rng))
    W32 = np.ascontiguousarray(W, dtype=np.float32)
    P1o, Go, P2o, _ = oracle.tucker2(W32.astype(np.float64), r1, r2)
    P1 = torch.empty((r1, C), dtype=torch.float32, device="cuda")
    G = torch.empty((r2, k, k, r1), dtype=torch.float32, device="cuda")
    P2 = torch.empty((S, r2), dtype=torch.float32, device="cuda")
    sweeps = lrd.tucker2_factors(_f32(W32), r1, r2, P1, G, P2, workspace(lrd.tucker2_factors_workspace_bytes(S, C, k)))
    assert sweeps >= 2
    P1, G, P2 = host(P1), host(G), host(P2)
    scale = np.max(np.abs(W32))
    assert np.max(np.abs(P1 @ P1.T - np.eye(r1))) <= 1e-5                   # orthonormal bases
    assert np.max(np.abs(P2.T @ P2 - np.eye(r2))) <= 1e-5
    assert np.max(np.abs(P1.T @ P1 - P1o.T @ P1o)) <= 1e-5                  # the same leading subspaces
    assert np.max(np.abs(P2 @ P2.T - P2o @ P2o.T)) <= 1e-5
    assert np.max(np.abs(_reconstruct(P1, G, P2) - _reconstruct(P1o, Go, P2o))) <= 1e-5 * scale


@pytest.mark.parametrize("shape_r_b", [((96, 160), 24, 5), ((200, 64), 16, 3), ((40, 40), 40, 7)])
def test_batched_svd_pairs_match_oracle_and_single_calls(shape_r_b):
    """A batch of weights of one shape in one call: every matrix against the oracle, and bit for bit against
    lrd_svd_factors on the same matrix (the batch applies the same rotations in the same order, the extra
    sweeps a slower neighbour forces rotate nothing)."""
    (n_out, n_in), r, B = shape_r_b
    rng = si.rng_for(6, 5000 + n_out + B)
    k = min(n_out, n_in)
    Ws = []
    for b in range(B):
        W = si.gaussian((n_out, n_in), rng) * 0.05
        W += (si.haar_orthogonal(n_out, rng)[:, :k] * np.exp(-np.arange(k) / max(4.0, k / (4.0 + b)))) @ si.haar_orthogonal(n_in, rng)[:k, :]
        Ws.append(W.astype(np.float32))
    W32 = np.stack(Ws)
    U = torch.empty((B, n_out, r), dtype=torch.float32, device="cuda")
    V = torch.empty((B, r, n_in), dtype=torch.float32, device="cuda")
    ws = workspace(lrd.svd_factors_batched_workspace_bytes(B, n_out, n_in))
    sig, sweeps = lrd.svd_factors_batched(_f32(W32), r, U, V, ws)
    assert 1 <= sweeps <= 30
    Uh, Vh = host(U), host(V)
    for b in range(B):
        Uo, Vo, so = oracle.svd_factors(W32[b].astype(np.float64), r)
        s = np.array(sig[b])
        assert np.max(np.abs(s - so)) <= 1e-9 * so[0]
        assert np.max(np.abs(Uh[b] @ Vh[b] - Uo @ Vo)) <= 2e-6 * so[0]
        U1, V1, s1, _ = _run_svd(W32[b], r)
        assert np.array_equal(U1, Uh[b]) and np.array_equal(V1, Vh[b])
