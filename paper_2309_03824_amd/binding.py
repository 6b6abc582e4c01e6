"""ctypes binding of liblrd.so: the same entry points as include/lrd.h, taking torch tensors.

Argument marshalling only.  torch supplies device memory and the stream; every arithmetic step
runs in the library's HIP kernels.  There is no CPU fallback: if the library cannot be loaded the
import fails, and a non-OK status raises LrdError.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, c_char_p, c_double, c_int32, c_int64, c_size_t, c_uint32, c_void_p

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblrd.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_ALIGNMENT, ERR_WORKSPACE, ERR_RUNTIME = range(6)
F32, BF16 = 0, 1
KIND_SVD, KIND_TUCKER = 0, 1
FREEZE_L0, FREEZE_L1, FREEZE_L2 = 1, 2, 4
FUSION_AUTO, FUSION_ALWAYS, FUSION_NEVER = 0, 1, 2
ROLE_NONE, ROLE_FWD_DOWN, ROLE_FWD_UP, ROLE_DGRAD_UP, ROLE_DGRAD_DOWN, ROLE_WGRAD_U, ROLE_WGRAD_V = range(7)
ROUND_NEAREST, ROUND_DOWN, ROUND_UP = 0, 1, 2
ACT_NONE, ACT_GELU = 0, 1

EXPORTS = (
    "lrd_status_string", "lrd_quantize_rank", "lrd_freeze_mask", "lrd_tucker_rank", "lrd_svd_rank", "lrd_select_rank",
    "lrd_sgd_step", "lrd_linear_sgd_workspace_bytes", "lrd_linear_bwd_sgd",
    "lrd_linear_group_workspace_bytes", "lrd_linear_group_fwd", "lrd_linear_group_bwd",
    "lrd_linear_bwd_data", "lrd_linear_group_bwd_data", "lrd_linear_wgrad_batched_workspace_bytes", "lrd_linear_wgrad_batched",
    "lrd_svd_factors_workspace_bytes", "lrd_svd_factors", "lrd_svd_factors_batched_workspace_bytes", "lrd_svd_factors_batched", "lrd_tucker2_factors_workspace_bytes", "lrd_tucker2_factors",
    "lrd_linear_workspace_bytes", "lrd_linear_fwd", "lrd_linear_bwd", "lrd_linear_fwd_act", "lrd_linear_bwd_act",
    "lrd_linear_bwd_static", "lrd_linear_bwd_static_fits",
    "lrd_dense_linear_workspace_bytes", "lrd_dense_linear_fwd", "lrd_dense_linear_bwd",
    "lrd_tucker_conv_workspace_bytes", "lrd_tucker_conv_fwd", "lrd_tucker_conv_bwd",
    "lrd_dense_conv_workspace_bytes", "lrd_dense_conv_fwd", "lrd_dense_conv_bwd",
    "lrd_gelu_fwd", "lrd_gelu_bwd",
)
# measurement aids (include/lrd_measure.h): not part of the layer ABI
MEASURE_EXPORTS = ("lrd_set_fusion", "lrd_profile_log_start", "lrd_profile_log_stop", "lrd_measure_mfma_loop", "lrd_measure_lds_read", "lrd_measure_stream")
STREAM_READ, STREAM_WRITE, STREAM_COPY = 0, 1, 2


class LrdError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        super().__init__(f"{where}: {status_string(status)}")


class Sgd(Structure):
    _fields_ = [("lr", ctypes.c_float), ("momentum", ctypes.c_float), ("weight_decay", ctypes.c_float)]


class ProfileRecord(Structure):
    _fields_ = [("role", c_int32), ("gather", c_int32), ("epilogue", c_int32), ("splits", c_int32),
                ("M", c_int64), ("N", c_int64), ("K", c_int64), ("batch", c_int64), ("kernel", ctypes.c_char * 64)]


class ConvGeom(Structure):
    _fields_ = [("N", c_int64), ("H", c_int64), ("W", c_int64), ("C", c_int64), ("S", c_int64),
                ("r1", c_int64), ("r2", c_int64), ("k", c_int32), ("stride", c_int32), ("pad", c_int32)]

    def out_hw(self):
        return ((self.H + 2 * self.pad - self.k) // self.stride + 1,
                (self.W + 2 * self.pad - self.k) // self.stride + 1)


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(LIB_PATH)
    P, I64, SZ, U32 = c_void_p, c_int64, c_size_t, c_uint32
    G = POINTER(ConvGeom)
    lib.lrd_status_string.restype = c_char_p
    lib.lrd_status_string.argtypes = [ctypes.c_int]
    lib.lrd_quantize_rank.restype = c_int32
    lib.lrd_quantize_rank.argtypes = [c_int32] * 5
    lib.lrd_freeze_mask.restype = c_uint32
    lib.lrd_freeze_mask.argtypes = [c_int32, c_int64]
    lib.lrd_tucker_rank.restype = ctypes.c_int
    lib.lrd_tucker_rank.argtypes = [I64, I64, c_int32, c_double, c_double, POINTER(c_int32), POINTER(c_int32)]
    lib.lrd_select_rank.restype = c_int32
    lib.lrd_select_rank.argtypes = [ctypes.POINTER(c_double), c_int32, c_int32, c_double, c_double, c_int32,
                                    ctypes.POINTER(c_int32), ctypes.POINTER(c_int32)]
    lib.lrd_svd_factors_workspace_bytes.restype = c_size_t
    lib.lrd_svd_factors_workspace_bytes.argtypes = [I64, I64]
    lib.lrd_svd_factors.restype = c_int32
    lib.lrd_svd_factors.argtypes = [c_void_p, I64, I64, I64, c_void_p, c_void_p, ctypes.POINTER(c_double),
                                    ctypes.POINTER(c_int32), c_void_p, c_size_t, c_void_p]
    lib.lrd_svd_factors_batched_workspace_bytes.restype = c_size_t
    lib.lrd_svd_factors_batched_workspace_bytes.argtypes = [I64, I64, I64]
    lib.lrd_svd_factors_batched.restype = c_int32
    lib.lrd_svd_factors_batched.argtypes = [c_void_p, I64, I64, I64, I64, c_void_p, c_void_p, ctypes.POINTER(c_double),
                                            ctypes.POINTER(c_int32), c_void_p, c_size_t, c_void_p]
    lib.lrd_tucker2_factors_workspace_bytes.restype = c_size_t
    lib.lrd_tucker2_factors_workspace_bytes.argtypes = [I64, I64, c_int32]
    lib.lrd_tucker2_factors.restype = c_int32
    lib.lrd_tucker2_factors.argtypes = [c_void_p, I64, I64, c_int32, I64, I64, c_void_p, c_void_p, c_void_p,
                                        ctypes.POINTER(c_int32), c_void_p, c_size_t, c_void_p]
    lib.lrd_svd_rank.restype = c_int32
    lib.lrd_svd_rank.argtypes = [I64, I64, c_double]
    lib.lrd_linear_workspace_bytes.restype = SZ
    lib.lrd_linear_workspace_bytes.argtypes = [I64] * 4 + [ctypes.c_int, U32]
    lib.lrd_linear_fwd.restype = ctypes.c_int
    lib.lrd_linear_fwd.argtypes = [P] * 6 + [I64] * 4 + [ctypes.c_int, P, SZ, P]
    lib.lrd_linear_bwd.restype = ctypes.c_int
    lib.lrd_linear_bwd.argtypes = [P] * 9 + [U32] + [I64] * 4 + [ctypes.c_int, P, SZ, P]
    lib.lrd_linear_bwd_static.restype = ctypes.c_int
    lib.lrd_linear_bwd_static.argtypes = [P] * 9 + [U32] + [I64] * 4 + [ctypes.c_int, P]
    lib.lrd_linear_bwd_static_fits.restype = c_int32
    lib.lrd_linear_bwd_static_fits.argtypes = [I64] * 4 + [ctypes.c_int, U32]
    lib.lrd_sgd_step.restype = ctypes.c_int
    lib.lrd_sgd_step.argtypes = [P, P, P, P, ctypes.c_int, I64, ctypes.POINTER(Sgd), P]
    lib.lrd_linear_sgd_workspace_bytes.restype = SZ
    lib.lrd_linear_sgd_workspace_bytes.argtypes = [I64] * 4 + [ctypes.c_int, U32]
    lib.lrd_linear_bwd_sgd.restype = ctypes.c_int
    lib.lrd_linear_bwd_sgd.argtypes = [P] * 11 + [U32, P, c_int32, ctypes.POINTER(Sgd)] + [I64] * 4 + [ctypes.c_int, P, SZ, P]
    lib.lrd_linear_group_workspace_bytes.restype = SZ
    lib.lrd_linear_group_workspace_bytes.argtypes = [I64] * 4 + [c_int32, ctypes.c_int, U32]
    lib.lrd_linear_group_fwd.restype = ctypes.c_int
    lib.lrd_linear_group_fwd.argtypes = [P] * 6 + [I64] * 4 + [c_int32, ctypes.c_int, P, SZ, P]
    lib.lrd_linear_bwd_data.restype = ctypes.c_int
    lib.lrd_linear_bwd_data.argtypes = [P] * 6 + [c_int32] + [I64] * 4 + [ctypes.c_int, P, SZ, P]
    lib.lrd_linear_group_bwd_data.restype = ctypes.c_int
    lib.lrd_linear_group_bwd_data.argtypes = [P] * 5 + [I64] * 4 + [c_int32, ctypes.c_int, P, SZ, P]
    lib.lrd_linear_wgrad_batched_workspace_bytes.restype = SZ
    lib.lrd_linear_wgrad_batched_workspace_bytes.argtypes = [I64] * 5 + [ctypes.c_int, U32]
    lib.lrd_linear_wgrad_batched.restype = ctypes.c_int
    lib.lrd_linear_wgrad_batched.argtypes = [P, I64, P, I64, I64, P, I64, I64, P, I64, P, P, U32] + [I64] * 5 + [ctypes.c_int, P, SZ, P]
    lib.lrd_linear_group_bwd.restype = ctypes.c_int
    lib.lrd_linear_group_bwd.argtypes = [P] * 9 + [U32] + [I64] * 4 + [c_int32, ctypes.c_int, P, SZ, P]
    lib.lrd_linear_fwd_act.restype = ctypes.c_int
    lib.lrd_linear_fwd_act.argtypes = [P] * 7 + [c_int32] + [I64] * 4 + [ctypes.c_int, P, SZ, P]
    lib.lrd_linear_bwd_act.restype = ctypes.c_int
    lib.lrd_linear_bwd_act.argtypes = [P] * 9 + [U32, P, c_int32] + [I64] * 4 + [ctypes.c_int, P, SZ, P]
    lib.lrd_dense_linear_workspace_bytes.restype = SZ
    lib.lrd_dense_linear_workspace_bytes.argtypes = [I64] * 3 + [ctypes.c_int]
    lib.lrd_dense_linear_fwd.restype = ctypes.c_int
    lib.lrd_dense_linear_fwd.argtypes = [P] * 4 + [I64] * 3 + [ctypes.c_int, P, SZ, P]
    lib.lrd_dense_linear_bwd.restype = ctypes.c_int
    lib.lrd_dense_linear_bwd.argtypes = [P] * 5 + [I64] * 3 + [ctypes.c_int, P, SZ, P]
    lib.lrd_tucker_conv_workspace_bytes.restype = SZ
    lib.lrd_tucker_conv_workspace_bytes.argtypes = [G, ctypes.c_int, U32]
    lib.lrd_tucker_conv_fwd.restype = ctypes.c_int
    lib.lrd_tucker_conv_fwd.argtypes = [P] * 7 + [G, ctypes.c_int, P, SZ, P]
    lib.lrd_tucker_conv_bwd.restype = ctypes.c_int
    lib.lrd_tucker_conv_bwd.argtypes = [P] * 11 + [U32, G, ctypes.c_int, P, SZ, P]
    lib.lrd_dense_conv_workspace_bytes.restype = SZ
    lib.lrd_dense_conv_workspace_bytes.argtypes = [G, ctypes.c_int]
    lib.lrd_dense_conv_fwd.restype = ctypes.c_int
    lib.lrd_dense_conv_fwd.argtypes = [P] * 3 + [G, ctypes.c_int, P, SZ, P]
    lib.lrd_dense_conv_bwd.restype = ctypes.c_int
    lib.lrd_dense_conv_bwd.argtypes = [P] * 5 + [G, ctypes.c_int, P, SZ, P]
    lib.lrd_gelu_fwd.restype = ctypes.c_int
    lib.lrd_gelu_fwd.argtypes = [P, P, I64, ctypes.c_int, P]
    lib.lrd_profile_log_start.restype = ctypes.c_int
    lib.lrd_profile_log_start.argtypes = [POINTER(c_void_p), c_int32]
    lib.lrd_profile_log_stop.restype = c_int32
    lib.lrd_profile_log_stop.argtypes = [POINTER(ProfileRecord), c_int32]
    lib.lrd_set_fusion.restype = c_int32
    lib.lrd_set_fusion.argtypes = [c_int32]
    lib.lrd_gelu_bwd.restype = ctypes.c_int
    lib.lrd_gelu_bwd.argtypes = [P, P, P, I64, ctypes.c_int, P]
    lib.lrd_measure_mfma_loop.restype = ctypes.c_int
    lib.lrd_measure_mfma_loop.argtypes = [P, c_int32, c_int32, POINTER(c_double), P]
    lib.lrd_measure_lds_read.restype = ctypes.c_int
    lib.lrd_measure_lds_read.argtypes = [P, c_int32, c_int32, POINTER(c_double), P]
    lib.lrd_measure_stream.restype = ctypes.c_int
    lib.lrd_measure_stream.argtypes = [P, P, SZ, c_int32, P]
    return lib


_lib = _load()


# ------------------------------------------------------------------------------- marshalling
def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor expected")
    return t.data_ptr()


def _dt(t) -> int:
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise ValueError(f"unsupported dtype {t.dtype}")


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _ws(ws):
    return (None, 0) if ws is None else (ws.data_ptr(), ws.numel() * ws.element_size())


def _check(status, where):
    if status != OK:
        raise LrdError(status, where)


def status_string(status: int) -> str:
    return _lib.lrd_status_string(int(status)).decode()


# ------------------------------------------------------------------------------- integer rules
def quantize_rank(r: int, multiple: int, mode: int = ROUND_NEAREST, r_min: int = 1,
                  r_max: int = 2**31 - 1) -> int:
    q = _lib.lrd_quantize_rank(r, multiple, mode, r_min, r_max)
    if q < 0:
        raise LrdError(-q, "lrd_quantize_rank")
    return int(q)


def freeze_mask(kind: int, epoch: int) -> int:
    return int(_lib.lrd_freeze_mask(kind, epoch))


def tucker_rank(C: int, S: int, k: int, alpha: float, beta: float = 1.0):
    r1, r2 = c_int32(0), c_int32(0)
    _check(_lib.lrd_tucker_rank(C, S, k, alpha, beta, ctypes.byref(r1), ctypes.byref(r2)), "lrd_tucker_rank")
    return int(r1.value), int(r2.value)


def svd_rank(n_in: int, n_out: int, alpha: float) -> int:
    r = _lib.lrd_svd_rank(n_in, n_out, alpha)
    if r < 0:
        raise LrdError(-r, "lrd_svd_rank")
    return int(r)


def svd_factors_workspace_bytes(n_out: int, n_in: int) -> int:
    return int(_lib.lrd_svd_factors_workspace_bytes(n_out, n_in))


def svd_factors(W, r: int, U, V, ws, stream=None):
    """Device SVD pair of W [out x in] (fp32 tensors); returns (singular values as a list, sweeps)."""
    n_out, n_in = W.shape
    sig = (c_double * min(n_out, n_in))()
    sweeps = c_int32(0)
    wp, wb = _ws(ws)
    _check(_lib.lrd_svd_factors(_ptr(W), n_out, n_in, r, _ptr(U), _ptr(V), sig, ctypes.byref(sweeps), wp, wb,
                                _stream(stream)), "lrd_svd_factors")
    return list(sig), int(sweeps.value)


def svd_factors_batched_workspace_bytes(batch: int, n_out: int, n_in: int) -> int:
    return int(_lib.lrd_svd_factors_batched_workspace_bytes(batch, n_out, n_in))


def svd_factors_batched(W, r: int, U, V, ws, stream=None):
    """Device SVD pairs of a batch W [B, out, in] (fp32); returns (singular values [B][min] as lists, max sweeps)."""
    B, n_out, n_in = W.shape
    assert U.shape == (B, n_out, r) and V.shape == (B, r, n_in)
    k = min(n_out, n_in)
    sig = (c_double * (B * k))()
    sweeps = c_int32(0)
    wp, wb = _ws(ws)
    _check(_lib.lrd_svd_factors_batched(_ptr(W), B, n_out, n_in, r, _ptr(U), _ptr(V), sig, ctypes.byref(sweeps), wp, wb,
                                        _stream(stream)), "lrd_svd_factors_batched")
    flat = list(sig)
    return [flat[b * k:(b + 1) * k] for b in range(B)], int(sweeps.value)


def tucker2_factors_workspace_bytes(S: int, C: int, k: int) -> int:
    return int(_lib.lrd_tucker2_factors_workspace_bytes(S, C, k))


def tucker2_factors(W, r1: int, r2: int, P1, G, P2, ws, stream=None) -> int:
    """Device Tucker-2 factors of W [S][k][k][C] (fp32 tensors); returns the sweeps used."""
    S, k, _, C = W.shape
    sweeps = c_int32(0)
    wp, wb = _ws(ws)
    _check(_lib.lrd_tucker2_factors(_ptr(W), S, C, k, r1, r2, _ptr(P1), _ptr(G), _ptr(P2), ctypes.byref(sweeps), wp, wb,
                                    _stream(stream)), "lrd_tucker2_factors")
    return int(sweeps.value)


SELECT_FIRST_PEAK, SELECT_ARGMAX, SELECT_REQUIRE_FASTER = 0, 1, 4


def select_rank(times, r_min: int, r_max: int, t_dense: float, noise: float = 0.0, mode: int = SELECT_FIRST_PEAK):
    """Algorithm 1's rank choice from measured step times: returns (r_opt, keep_decomposed)."""
    arr = (c_double * len(times))(*[float(v) for v in times])
    if len(times) != r_max - r_min + 1:
        raise LrdError(1, "lrd_select_rank")
    r_opt, keep = c_int32(0), c_int32(0)
    _check(_lib.lrd_select_rank(arr, r_min, r_max, t_dense, noise, mode, ctypes.byref(r_opt), ctypes.byref(keep)),
           "lrd_select_rank")
    return int(r_opt.value), bool(keep.value)


def set_fusion(mode: int) -> int:
    prev = int(_lib.lrd_set_fusion(mode))
    if prev < 0:
        raise LrdError(ERR_INVALID_ARG, "lrd_set_fusion")
    return prev


class HipEvent:
    """A raw hipEvent_t (created through the HIP runtime), for the product event log."""
    _hip = None

    def __init__(self):
        if HipEvent._hip is None:
            HipEvent._hip = ctypes.CDLL("libamdhip64.so")
            HipEvent._hip.hipEventCreate.argtypes = [POINTER(c_void_p)]
            HipEvent._hip.hipEventElapsedTime.argtypes = [POINTER(ctypes.c_float), c_void_p, c_void_p]
            HipEvent._hip.hipEventDestroy.argtypes = [c_void_p]
        self.handle = c_void_p()
        if HipEvent._hip.hipEventCreate(ctypes.byref(self.handle)) != 0:
            raise RuntimeError("hipEventCreate failed")

    def elapsed_us(self, later: "HipEvent") -> float:
        ms = ctypes.c_float()
        if HipEvent._hip.hipEventElapsedTime(ctypes.byref(ms), self.handle, later.handle) != 0:
            raise RuntimeError("hipEventElapsedTime failed (events not complete?)")
        return ms.value * 1e3

    def __del__(self):
        try:
            HipEvent._hip.hipEventDestroy(self.handle)
        except Exception:
            pass


def measure_mfma_loop(sink, workgroups: int, iters: int, stream=None) -> float:
    """Launches the register-only matrix-instruction loop; returns the flops of the launch."""
    assert sink.dtype == torch.float32 and sink.numel() >= workgroups * 256
    fl = c_double(0.0)
    _check(_lib.lrd_measure_mfma_loop(_ptr(sink), workgroups, iters, ctypes.byref(fl), _stream(stream)), "lrd_measure_mfma_loop")
    return float(fl.value)


def measure_lds_read(sink, workgroups: int, iters: int, stream=None) -> float:
    """Launches the LDS read loop; returns the LDS bytes read by the launch."""
    assert sink.numel() >= workgroups * 256
    nb = c_double(0.0)
    _check(_lib.lrd_measure_lds_read(_ptr(sink), workgroups, iters, ctypes.byref(nb), _stream(stream)), "lrd_measure_lds_read")
    return float(nb.value)


def measure_stream(src, dst, nbytes: int, mode: int, stream=None):
    _check(_lib.lrd_measure_stream(_ptr(src), _ptr(dst), nbytes, mode, _stream(stream)), "lrd_measure_stream")


class ProfileLog:
    """Event log of the library's products (lrd_profile_log_start / _stop): `with ProfileLog(n) as log:`
    runs eager launches; afterwards log.rows() gives one dict per product with its elapsed microseconds."""

    def __init__(self, n_pairs: int):
        self.n = int(n_pairs)
        self.events = [HipEvent() for _ in range(2 * self.n)]          # created ahead of the logged region
        self.array = (c_void_p * (2 * self.n))(*[e.handle for e in self.events])
        self.count = 0
        self.records = None

    def __enter__(self):
        _check(_lib.lrd_profile_log_start(self.array, self.n), "lrd_profile_log_start")
        return self

    def __exit__(self, *exc):
        buf = (ProfileRecord * self.n)()
        self.count = int(_lib.lrd_profile_log_stop(buf, self.n))
        self.records = buf
        return False

    def rows(self):
        """Call after the device has finished the logged work."""
        out = []
        for i in range(min(self.count, self.n)):
            r = self.records[i]
            out.append(dict(role=r.role, gather=r.gather, epilogue=r.epilogue, splits=r.splits, M=r.M, N=r.N, K=r.K, batch=r.batch,
                            kernel=r.kernel.decode(), us=self.events[2 * i].elapsed_us(self.events[2 * i + 1])))
        return out


# ------------------------------------------------------------------------------- linear pair
def linear_workspace_bytes(T, n_in, n_out, r, dtype, freeze_mask=0) -> int:
    return int(_lib.lrd_linear_workspace_bytes(T, n_in, n_out, r, dtype, freeze_mask))


def linear_fwd(X, V, U, bias, Y, H_save, ws=None, stream=None):
    T, n_in = X.shape
    r, n_out = V.shape[0], U.shape[0]
    assert V.shape == (r, n_in) and U.shape == (n_out, r) and Y.shape == (T, n_out)
    assert H_save is None or H_save.shape == (T, r)
    wp, wb = _ws(ws)
    _check(_lib.lrd_linear_fwd(_ptr(X), _ptr(V), _ptr(U), _ptr(bias), _ptr(Y), _ptr(H_save), T, n_in, n_out, r,
                               _dt(X), wp, wb, _stream(stream)), "lrd_linear_fwd")


def linear_bwd(dY, X, H, V, U, dX, dV, dU, dbias, freeze_mask, ws=None, stream=None):
    T, n_out = dY.shape
    r, n_in = V.shape
    assert U.shape == (n_out, r)
    wp, wb = _ws(ws)
    _check(_lib.lrd_linear_bwd(_ptr(dY), _ptr(X), _ptr(H), _ptr(V), _ptr(U), _ptr(dX), _ptr(dV), _ptr(dU),
                               _ptr(dbias), freeze_mask, T, n_in, n_out, r, _dt(dY), wp, wb, _stream(stream)),
           "lrd_linear_bwd")


STATIC_SCRATCH_BYTES = 64 << 20


def linear_bwd_static_fits(T, n_in, n_out, r, dtype, freeze_mask=0) -> bool:
    return bool(_lib.lrd_linear_bwd_static_fits(T, n_in, n_out, r, dtype, freeze_mask))


def linear_bwd_static(dY, X, H, V, U, dX, dV, dU, dbias, freeze_mask, stream=None):
    """lrd_linear_bwd on the library's own fixed scratch array (no workspace argument, no allocation)."""
    T, n_out = dY.shape
    r, n_in = V.shape
    assert U.shape == (n_out, r)
    _check(_lib.lrd_linear_bwd_static(_ptr(dY), _ptr(X), _ptr(H), _ptr(V), _ptr(U), _ptr(dX), _ptr(dV), _ptr(dU),
                                      _ptr(dbias), freeze_mask, T, n_in, n_out, r, _dt(dY), _stream(stream)),
           "lrd_linear_bwd_static")


def sgd_step(w_master, momentum_buf, grad, w_copy, opt: "Sgd", stream=None):
    _check(_lib.lrd_sgd_step(_ptr(w_master), _ptr(momentum_buf), _ptr(grad), _ptr(w_copy),
                             _dt(w_copy) if w_copy is not None else F32, w_master.numel(), ctypes.byref(opt), _stream(stream)),
           "lrd_sgd_step")


def linear_sgd_workspace_bytes(T, n_in, n_out, r, dtype, freeze_mask=0) -> int:
    return int(_lib.lrd_linear_sgd_workspace_bytes(T, n_in, n_out, r, dtype, freeze_mask))


def linear_bwd_sgd(dY, X, H, V, U, dX, V_master, U_master, V_mom, U_mom, dbias, freeze_mask, Z_in, act, opt: "Sgd",
                   ws=None, stream=None):
    T, n_out = dY.shape
    r, n_in = V.shape
    wp, wb = _ws(ws)
    _check(_lib.lrd_linear_bwd_sgd(_ptr(dY), _ptr(X), _ptr(H), _ptr(V), _ptr(U), _ptr(dX), _ptr(V_master), _ptr(U_master),
                                   _ptr(V_mom), _ptr(U_mom), _ptr(dbias), freeze_mask, _ptr(Z_in), act, ctypes.byref(opt),
                                   T, n_in, n_out, r, _dt(dY), wp, wb, _stream(stream)), "lrd_linear_bwd_sgd")


def linear_group_workspace_bytes(T, n_in, n_out, r, groups, dtype, freeze_mask=0) -> int:
    return int(_lib.lrd_linear_group_workspace_bytes(T, n_in, n_out, r, groups, dtype, freeze_mask))


def linear_group_fwd(X, V_cat, U, bias, Y, H_save, ws=None, stream=None):
    """U [G, out, r], V_cat [G*r, in], Y [G, T, out], H_save [T, G*r] or None."""
    T, n_in = X.shape
    G, n_out, r = U.shape
    assert V_cat.shape == (G * r, n_in) and Y.shape == (G, T, n_out)
    wp, wb = _ws(ws)
    _check(_lib.lrd_linear_group_fwd(_ptr(X), _ptr(V_cat), _ptr(U), _ptr(bias), _ptr(Y), _ptr(H_save), T, n_in, n_out, r, G,
                                     _dt(X), wp, wb, _stream(stream)), "lrd_linear_group_fwd")


def linear_group_bwd(dY, X, H, V_cat, U, dX, dV_cat, dU, dbias, freeze_mask, ws=None, stream=None):
    G, T, n_out = dY.shape
    r, n_in = U.shape[2], V_cat.shape[1]
    wp, wb = _ws(ws)
    _check(_lib.lrd_linear_group_bwd(_ptr(dY), _ptr(X), _ptr(H), _ptr(V_cat), _ptr(U), _ptr(dX), _ptr(dV_cat), _ptr(dU),
                                     _ptr(dbias), freeze_mask, T, n_in, n_out, r, G, _dt(dY), wp, wb, _stream(stream)),
           "lrd_linear_group_bwd")


def linear_bwd_data(dY, V, U, dX, dH_save, Z_in=None, act=0, ws=None, stream=None):
    """Data gradient only; dH_save [T x r] receives dY.U for a later lrd_linear_wgrad_batched."""
    T, n_out = dY.shape
    r, n_in = V.shape
    assert U.shape == (n_out, r) and (dX is None or dX.shape == (T, n_in)) and dH_save.shape == (T, r)
    wp, wb = _ws(ws)
    _check(_lib.lrd_linear_bwd_data(_ptr(dY), _ptr(V), _ptr(U), _ptr(dX), _ptr(dH_save), _ptr(Z_in), act, T, n_in, n_out, r,
                                    _dt(dY), wp, wb, _stream(stream)), "lrd_linear_bwd_data")


def linear_group_bwd_data(dY, V_cat, U, dX, dH_save, ws=None, stream=None):
    G, T, n_out = dY.shape
    r, n_in = U.shape[2], V_cat.shape[1]
    assert dH_save.shape == (T, G * r) and (dX is None or dX.shape == (T, n_in))
    wp, wb = _ws(ws)
    _check(_lib.lrd_linear_group_bwd_data(_ptr(dY), _ptr(V_cat), _ptr(U), _ptr(dX), _ptr(dH_save), T, n_in, n_out, r, G,
                                          _dt(dY), wp, wb, _stream(stream)), "lrd_linear_group_bwd_data")


def linear_wgrad_batched_workspace_bytes(layers, T, n_in, n_out, r, dtype, freeze_mask=0) -> int:
    return int(_lib.lrd_linear_wgrad_batched_workspace_bytes(layers, T, n_in, n_out, r, dtype, freeze_mask))


def linear_wgrad_batched(dY, H, dH, X, dV, dU, freeze_mask, ws=None, stream=None):
    """dU[l] = dY[l]^T.H[l], dV[l] = dH[l]^T.X[l] for stacks [layers][T][.]; H and dH may be column
    slices of wider stacks (their row pitch and layer stride are taken from the tensor strides)."""
    ref = dY if dY is not None else dH
    L, T = ref.shape[0], ref.shape[1]
    n_out = dU.shape[1] if dU is not None else 0
    n_in = dV.shape[2] if dV is not None else 0
    r = dU.shape[2] if dU is not None else dV.shape[1]
    dt = _dt(ref)

    def pitch(t, cols):
        if t is None:
            return 0, 0
        assert t.shape == (L, T, cols) and t.stride(2) == 1, (tuple(t.shape), (L, T, cols))
        return t.stride(1), (t.stride(0) if L > 1 else 0)

    ldy, sy = pitch(dY, n_out)
    ldh, sh = pitch(H, r)
    lddh, sdh = pitch(dH, r)
    ldx, sx = pitch(X, n_in)
    assert (dY is None or ldy == n_out) and (X is None or ldx == n_in)
    n_out = n_out or 1
    n_in = n_in or 1
    wp, wb = _ws(ws)
    at = lambda t: None if t is None else t.data_ptr()   # slices of wider stacks: pitch and stride say where
    _check(_lib.lrd_linear_wgrad_batched(at(dY), sy, at(H), ldh or r, sh, at(dH), lddh or r, sdh, at(X), sx, _ptr(dV), _ptr(dU),
                                         freeze_mask, L, T, n_in, n_out, r, dt, wp, wb, _stream(stream)), "lrd_linear_wgrad_batched")


def linear_fwd_act(X, V, U, bias, Y, Y_act, H_save, act, ws=None, stream=None):
    T, n_in = X.shape
    r, n_out = V.shape[0], U.shape[0]
    assert V.shape == (r, n_in) and U.shape == (n_out, r) and Y.shape == (T, n_out)
    wp, wb = _ws(ws)
    _check(_lib.lrd_linear_fwd_act(_ptr(X), _ptr(V), _ptr(U), _ptr(bias), _ptr(Y), _ptr(Y_act), _ptr(H_save), act,
                                   T, n_in, n_out, r, _dt(X), wp, wb, _stream(stream)), "lrd_linear_fwd_act")


def linear_bwd_act(dY, X, H, V, U, dX, dV, dU, dbias, freeze_mask, Z_in, act, ws=None, stream=None):
    T, n_out = dY.shape
    r, n_in = V.shape
    wp, wb = _ws(ws)
    _check(_lib.lrd_linear_bwd_act(_ptr(dY), _ptr(X), _ptr(H), _ptr(V), _ptr(U), _ptr(dX), _ptr(dV), _ptr(dU),
                                   _ptr(dbias), freeze_mask, _ptr(Z_in), act, T, n_in, n_out, r, _dt(dY), wp, wb,
                                   _stream(stream)), "lrd_linear_bwd_act")


def dense_linear_workspace_bytes(T, n_in, n_out, dtype) -> int:
    return int(_lib.lrd_dense_linear_workspace_bytes(T, n_in, n_out, dtype))


def dense_linear_fwd(X, W, bias, Y, ws=None, stream=None):
    T, n_in = X.shape
    n_out = W.shape[0]
    assert W.shape == (n_out, n_in) and Y.shape == (T, n_out)
    wp, wb = _ws(ws)
    _check(_lib.lrd_dense_linear_fwd(_ptr(X), _ptr(W), _ptr(bias), _ptr(Y), T, n_in, n_out, _dt(X), wp, wb,
                                     _stream(stream)), "lrd_dense_linear_fwd")


def dense_linear_bwd(dY, X, W, dX, dW, ws=None, stream=None):
    T, n_out = dY.shape
    n_in = W.shape[1]
    wp, wb = _ws(ws)
    _check(_lib.lrd_dense_linear_bwd(_ptr(dY), _ptr(X), _ptr(W), _ptr(dX), _ptr(dW), T, n_in, n_out, _dt(dY), wp,
                                     wb, _stream(stream)), "lrd_dense_linear_bwd")


# ------------------------------------------------------------------------------- convolutions
def conv_geom(N, H, W, C, S, r1, r2, k, stride, pad) -> ConvGeom:
    return ConvGeom(N, H, W, C, S, r1, r2, k, stride, pad)


def tucker_conv_workspace_bytes(g: ConvGeom, dtype, freeze_mask=0) -> int:
    return int(_lib.lrd_tucker_conv_workspace_bytes(ctypes.byref(g), dtype, freeze_mask))


def tucker_conv_fwd(X, P1, G, P2, Y, A_save, B_save, g: ConvGeom, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(_lib.lrd_tucker_conv_fwd(_ptr(X), _ptr(P1), _ptr(G), _ptr(P2), _ptr(Y), _ptr(A_save), _ptr(B_save),
                                    ctypes.byref(g), _dt(X), wp, wb, _stream(stream)), "lrd_tucker_conv_fwd")


def tucker_conv_bwd(dY, X, A, B, P1, G, P2, dX, dP1, dG, dP2, freeze_mask, g: ConvGeom, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(_lib.lrd_tucker_conv_bwd(_ptr(dY), _ptr(X), _ptr(A), _ptr(B), _ptr(P1), _ptr(G), _ptr(P2), _ptr(dX),
                                    _ptr(dP1), _ptr(dG), _ptr(dP2), freeze_mask, ctypes.byref(g), _dt(dY), wp, wb,
                                    _stream(stream)), "lrd_tucker_conv_bwd")


def dense_conv_workspace_bytes(g: ConvGeom, dtype) -> int:
    return int(_lib.lrd_dense_conv_workspace_bytes(ctypes.byref(g), dtype))


def dense_conv_fwd(X, W, Y, g: ConvGeom, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(_lib.lrd_dense_conv_fwd(_ptr(X), _ptr(W), _ptr(Y), ctypes.byref(g), _dt(X), wp, wb, _stream(stream)),
           "lrd_dense_conv_fwd")


def dense_conv_bwd(dY, X, W, dX, dW, g: ConvGeom, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(_lib.lrd_dense_conv_bwd(_ptr(dY), _ptr(X), _ptr(W), _ptr(dX), _ptr(dW), ctypes.byref(g), _dt(dY), wp, wb,
                                   _stream(stream)), "lrd_dense_conv_bwd")


# ------------------------------------------------------------------------------- glue
def gelu_fwd(Z, A, stream=None):
    _check(_lib.lrd_gelu_fwd(_ptr(Z), _ptr(A), Z.numel(), _dt(Z), _stream(stream)), "lrd_gelu_fwd")


def gelu_bwd(dA, Z, dZ, stream=None):
    _check(_lib.lrd_gelu_bwd(_ptr(dA), _ptr(Z), _ptr(dZ), Z.numel(), _dt(Z), _stream(stream)), "lrd_gelu_bwd")
