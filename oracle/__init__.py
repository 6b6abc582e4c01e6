"""CPU oracle for low-rank-decomposed layers: TEST INFRASTRUCTURE, not part of the product.

Thin numpy/ctypes front end to ``lrd_ref.c`` (plain fp64 loops written from the paper).  Only the
tests, the smoke check and the benchmark's CPU-baseline leg may import this package; the GPU
library never does and shares no code with it.

Orientation and names (see the header of ``lrd_ref.c``): ``W[out, in] ~= U @ V`` with
``V[r, in]`` = the paper's first decomposed layer L_r(0) and ``U[out, r]`` = L_r(1); Tucker-2 uses
``P1[r1, C]``, ``G[r2, k, k, r1]``, ``P2[S, r2]`` = L_r(0), L_r(1), L_r(2).  Activations are
``[T, features]`` or NHWC.  Freeze-mask bit i set means L_r(i) is frozen (Algorithm 2).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from ctypes import POINTER, c_double, c_int, c_int32, c_int64, c_uint32, c_void_p

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lrd_ref.c")
_LIB = os.path.join(_HERE, "liblrd_ref.so")

FREEZE_L0, FREEZE_L1, FREEZE_L2 = 1, 2, 4
KIND_SVD, KIND_TUCKER = 0, 1
ROUND_NEAREST, ROUND_DOWN, ROUND_UP = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile lrd_ref.c with gcc into liblrd_ref.so (next to the source)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        D = POINTER(c_double)
        lib.lrd_ref_quantize_rank.restype = c_int32
        lib.lrd_ref_quantize_rank.argtypes = [c_int32] * 5
        lib.lrd_ref_freeze_mask.restype = c_uint32
        lib.lrd_ref_freeze_mask.argtypes = [c_int32, c_int64]
        lib.lrd_ref_tucker_rank.restype = c_int
        lib.lrd_ref_tucker_rank.argtypes = [c_int64, c_int64, c_int32, c_double, c_double,
                                            POINTER(c_int32), POINTER(c_int32)]
        lib.lrd_ref_select_rank.restype = c_int32
        lib.lrd_ref_select_rank.argtypes = [ctypes.POINTER(c_double), c_int32, c_int32, c_double, c_double, c_int32,
                                            ctypes.POINTER(c_int32), ctypes.POINTER(c_int32)]
        lib.lrd_ref_sgd_step.restype = None
        lib.lrd_ref_sgd_step.argtypes = [D, D, D, c_int64, c_double, c_double, c_double]
        lib.lrd_ref_svd_rank.restype = c_int32
        lib.lrd_ref_svd_rank.argtypes = [c_int64, c_int64, c_double]
        lib.lrd_ref_linear_fwd.restype = None
        lib.lrd_ref_linear_fwd.argtypes = [D, D, D, D, D, D] + [c_int64] * 4
        lib.lrd_ref_linear_bwd.restype = None
        lib.lrd_ref_linear_bwd.argtypes = [D] * 10 + [c_uint32] + [c_int64] * 4
        lib.lrd_ref_dense_linear_fwd.restype = None
        lib.lrd_ref_dense_linear_fwd.argtypes = [D, D, D, D] + [c_int64] * 3
        lib.lrd_ref_dense_linear_bwd.restype = None
        lib.lrd_ref_dense_linear_bwd.argtypes = [D] * 5 + [c_int64] * 3
        lib.lrd_ref_gelu_fwd.restype = None
        lib.lrd_ref_gelu_fwd.argtypes = [D, D, c_int64]
        lib.lrd_ref_gelu_bwd.restype = None
        lib.lrd_ref_gelu_bwd.argtypes = [D, D, D, c_int64]
        conv_dims = [c_int64] * 5 + [c_int32] * 3
        for name in ("lrd_ref_conv_fwd", "lrd_ref_conv_dgrad", "lrd_ref_conv_wgrad"):
            getattr(lib, name).restype = None
            getattr(lib, name).argtypes = [D, D, D] + conv_dims
        tucker_dims = [c_int64] * 7 + [c_int32] * 3
        lib.lrd_ref_tucker_fwd.restype = None
        lib.lrd_ref_tucker_fwd.argtypes = [D] * 7 + tucker_dims
        lib.lrd_ref_tucker_bwd.restype = None
        lib.lrd_ref_tucker_bwd.argtypes = [D] * 13 + [c_uint32] + tucker_dims
        lib.lrd_ref_svd.restype = c_int
        lib.lrd_ref_svd.argtypes = [D, c_int64, c_int64, D, D, D]
        lib.lrd_ref_svd_factors.restype = c_int
        lib.lrd_ref_svd_factors.argtypes = [D, c_int64, c_int64, c_int64, D, D, D]
        lib.lrd_ref_tucker2.restype = c_int
        lib.lrd_ref_tucker2.argtypes = [D, c_int64, c_int64, c_int32, c_int64, c_int64, D, D, D, D]
        lib.lrd_ref_threads.restype = c_int
        lib.lrd_ref_set_threads.argtypes = [c_int]
        _lib = lib
    return _lib


def _in(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _p(a):
    if a is None:
        return ctypes.cast(c_void_p(0), POINTER(c_double))
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(POINTER(c_double))


def threads() -> int:
    return int(_load().lrd_ref_threads())


def set_threads(n: int) -> None:
    _load().lrd_ref_set_threads(int(n))


# --------------------------------------------------------------------------- integer rules
def quantize_rank(r: int, multiple: int, mode: int = ROUND_NEAREST, r_min: int = 1,
                  r_max: int = 2**31 - 1) -> int:
    return int(_load().lrd_ref_quantize_rank(r, multiple, mode, r_min, r_max))


def freeze_mask(kind: int, epoch: int) -> int:
    return int(_load().lrd_ref_freeze_mask(kind, epoch))


def tucker_rank(C: int, S: int, k: int, alpha: float, beta: float = 1.0):
    r1, r2 = c_int32(0), c_int32(0)
    rc = _load().lrd_ref_tucker_rank(C, S, k, alpha, beta, ctypes.byref(r1), ctypes.byref(r2))
    if rc != 0:
        raise ValueError("bad arguments")
    return int(r1.value), int(r2.value)


SELECT_REQUIRE_FASTER = 4


def select_rank(times, r_min: int, r_max: int, t_dense: float, noise: float = 0.0, mode: int = 0):
    """Algorithm 1's rank choice from measured times; returns (r_opt, keep_decomposed) or raises ValueError.
    mode: 0 first peak (text), 1 arg max (listing); + SELECT_REQUIRE_FASTER for the extension that drops a
    pick which is not faster than the estimated rank."""
    arr = (c_double * len(times))(*[float(v) for v in times])
    if len(times) != r_max - r_min + 1:
        raise ValueError("times must cover r_min..r_max")
    r_opt, keep = c_int32(0), c_int32(0)
    rc = _load().lrd_ref_select_rank(arr, r_min, r_max, t_dense, noise, mode, ctypes.byref(r_opt), ctypes.byref(keep))
    if rc != 0:
        raise ValueError("invalid arguments")
    return int(r_opt.value), bool(keep.value)


def sgd_step(w, m, g, lr: float, momentum: float, weight_decay: float):
    """One SGD-with-momentum step; returns the new (w, m) as fp64 arrays of the input shape."""
    w, m, g = _in(w).copy(), _in(m).copy(), _in(g)
    _load().lrd_ref_sgd_step(_p(w), _p(m), _p(g), w.size, lr, momentum, weight_decay)
    return w, m


def svd_rank(n_in: int, n_out: int, alpha: float) -> int:
    return int(_load().lrd_ref_svd_rank(n_in, n_out, alpha))


# --------------------------------------------------------------------------- linear pair
def linear_fwd(X, V, U, bias=None):
    """Returns (H, Y): H = X V^T, Y = H U^T (+ bias)."""
    X, V, U = _in(X), _in(V), _in(U)
    T, n_in = X.shape
    r = V.shape[0]
    n_out = U.shape[0]
    assert V.shape == (r, n_in) and U.shape == (n_out, r)
    b = None if bias is None else _in(bias)
    H = np.empty((T, r))
    Y = np.empty((T, n_out))
    _load().lrd_ref_linear_fwd(_p(X), _p(V), _p(U), _p(b), _p(H), _p(Y), T, n_in, n_out, r)
    return H, Y


def linear_bwd(dY, X, H, V, U, mask: int = 0, want_dX: bool = True, want_dbias: bool = False,
               dV_init=None, dU_init=None):
    """Returns dict(dH, dX, dV, dU, dbias).  Frozen factors' buffers keep their initial content
    (``dV_init``/``dU_init`` if given, else NaN-filled) so that tests can see they are untouched."""
    dY, X, H, V, U = _in(dY), _in(X), _in(H), _in(V), _in(U)
    T, n_in = X.shape
    r = V.shape[0]
    n_out = U.shape[0]
    dH = np.empty((T, r))
    dX = np.empty((T, n_in)) if want_dX else None
    dV = np.full((r, n_in), np.nan) if dV_init is None else _in(dV_init).copy()
    dU = np.full((n_out, r), np.nan) if dU_init is None else _in(dU_init).copy()
    db = np.empty((n_out,)) if want_dbias else None
    _load().lrd_ref_linear_bwd(_p(dY), _p(X), _p(H), _p(V), _p(U), _p(dH), _p(dX), _p(dV), _p(dU),
                               _p(db), mask, T, n_in, n_out, r)
    return dict(dH=dH, dX=dX, dV=dV, dU=dU, dbias=db)


def dense_linear_fwd(X, W, bias=None):
    X, W = _in(X), _in(W)
    T, n_in = X.shape
    n_out = W.shape[0]
    b = None if bias is None else _in(bias)
    Y = np.empty((T, n_out))
    _load().lrd_ref_dense_linear_fwd(_p(X), _p(W), _p(b), _p(Y), T, n_in, n_out)
    return Y


def dense_linear_bwd(dY, X, W):
    dY, X, W = _in(dY), _in(X), _in(W)
    T, n_in = X.shape
    n_out = W.shape[0]
    dX = np.empty((T, n_in))
    dW = np.empty((n_out, n_in))
    _load().lrd_ref_dense_linear_bwd(_p(dY), _p(X), _p(W), _p(dX), _p(dW), T, n_in, n_out)
    return dX, dW


def gelu_fwd(Z):
    Z = _in(Z)
    A = np.empty_like(Z)
    _load().lrd_ref_gelu_fwd(_p(Z), _p(A), Z.size)
    return A


def gelu_bwd(dA, Z):
    dA, Z = _in(dA), _in(Z)
    dZ = np.empty_like(Z)
    _load().lrd_ref_gelu_bwd(_p(dA), _p(Z), _p(dZ), Z.size)
    return dZ


# --------------------------------------------------------------------------- convolutions
def _out_dim(n, k, s, p):
    return (n + 2 * p - k) // s + 1


def conv_fwd(X, W, stride=1, pad=0):
    """X [N,H,W,I], W [O,k,k,I] -> Y [N,Ho,Wo,O]."""
    X, W = _in(X), _in(W)
    N, Hh, Ww, I = X.shape
    O, k = W.shape[0], W.shape[1]
    assert W.shape == (O, k, k, I)
    Y = np.empty((N, _out_dim(Hh, k, stride, pad), _out_dim(Ww, k, stride, pad), O))
    _load().lrd_ref_conv_fwd(_p(X), _p(W), _p(Y), N, Hh, Ww, I, O, k, stride, pad)
    return Y


def conv_dgrad(dY, W, in_hw, stride=1, pad=0):
    dY, W = _in(dY), _in(W)
    N = dY.shape[0]
    O, k, _, I = W.shape
    Hh, Ww = in_hw
    dX = np.empty((N, Hh, Ww, I))
    _load().lrd_ref_conv_dgrad(_p(dY), _p(W), _p(dX), N, Hh, Ww, I, O, k, stride, pad)
    return dX


def conv_wgrad(dY, X, k, stride=1, pad=0):
    dY, X = _in(dY), _in(X)
    N, Hh, Ww, I = X.shape
    O = dY.shape[3]
    dW = np.empty((O, k, k, I))
    _load().lrd_ref_conv_wgrad(_p(dY), _p(X), _p(dW), N, Hh, Ww, I, O, k, stride, pad)
    return dW


def tucker_fwd(X, P1, G, P2, stride=1, pad=0):
    """Returns (A, B, Y) of the 1x1 -> kxk core -> 1x1 chain."""
    X, P1, G, P2 = _in(X), _in(P1), _in(G), _in(P2)
    N, Hh, Ww, C = X.shape
    r1 = P1.shape[0]
    r2, k = G.shape[0], G.shape[1]
    S = P2.shape[0]
    assert P1.shape == (r1, C) and G.shape == (r2, k, k, r1) and P2.shape == (S, r2)
    Ho, Wo = _out_dim(Hh, k, stride, pad), _out_dim(Ww, k, stride, pad)
    A = np.empty((N, Hh, Ww, r1))
    B = np.empty((N, Ho, Wo, r2))
    Y = np.empty((N, Ho, Wo, S))
    _load().lrd_ref_tucker_fwd(_p(X), _p(P1), _p(G), _p(P2), _p(A), _p(B), _p(Y), N, Hh, Ww, C, S,
                               r1, r2, k, stride, pad)
    return A, B, Y


def tucker_bwd(dY, X, A, B, P1, G, P2, mask=0, stride=1, pad=0, want_dX=True):
    dY, X, A, B, P1, G, P2 = map(_in, (dY, X, A, B, P1, G, P2))
    N, Hh, Ww, C = X.shape
    r1 = P1.shape[0]
    r2, k = G.shape[0], G.shape[1]
    S = P2.shape[0]
    dB = np.empty_like(B)
    dA = np.empty_like(A)
    dX = np.empty_like(X) if want_dX else None
    dP1 = np.full_like(P1, np.nan)
    dG = np.full_like(G, np.nan)
    dP2 = np.full_like(P2, np.nan)
    _load().lrd_ref_tucker_bwd(_p(dY), _p(X), _p(A), _p(B), _p(P1), _p(G), _p(P2), _p(dB), _p(dA),
                               _p(dX), _p(dP1), _p(dG), _p(dP2), mask, N, Hh, Ww, C, S, r1, r2, k,
                               stride, pad)
    return dict(dB=dB, dA=dA, dX=dX, dP1=dP1, dG=dG, dP2=dP2)


# --------------------------------------------------------------------------- factorization
def svd(M):
    """Returns (U[m,R], sigma[R] descending, V[n,R]) with M = U diag(sigma) V^T (eq. 1)."""
    M = _in(M)
    m, n = M.shape
    R = min(m, n)
    U = np.empty((m, R))
    s = np.empty((R,))
    V = np.empty((n, R))
    rc = _load().lrd_ref_svd(_p(M), m, n, _p(U), _p(s), _p(V))
    if rc < 0:
        raise RuntimeError("Jacobi SVD did not converge")
    return U, s, V


def svd_factors(W, r):
    """W [out,in] -> (U [out,r], V [r,in], all singular values); eq. 2 with sqrt(sigma) in each."""
    W = _in(W)
    n_out, n_in = W.shape
    U = np.empty((n_out, r))
    V = np.empty((r, n_in))
    s = np.empty((min(n_out, n_in),))
    rc = _load().lrd_ref_svd_factors(_p(W), n_out, n_in, r, _p(U), _p(V), _p(s))
    if rc < 0:
        raise RuntimeError("svd_factors failed")
    return U, V, s


def tucker2(W, r1, r2):
    """W [S,k,k,C] -> (P1 [r1,C], G [r2,k,k,r1], P2 [S,r2], tau[2]) by truncated HOSVD (eq. 4)."""
    W = _in(W)
    S, k, _, C = W.shape
    P1 = np.empty((r1, C))
    G = np.empty((r2, k, k, r1))
    P2 = np.empty((S, r2))
    tau = np.empty((2,))
    rc = _load().lrd_ref_tucker2(_p(W), S, C, k, r1, r2, _p(P1), _p(G), _p(P2), _p(tau))
    if rc < 0:
        raise RuntimeError("tucker2 failed")
    return P1, G, P2, tau
