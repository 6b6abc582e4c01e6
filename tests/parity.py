"""Helpers of the GPU parity tests: move seeded numpy inputs to the device in the library's dtypes,
hand the oracle the same values (rounded to the storage dtype, widened to fp64), compare."""
import numpy as np
import torch

import synth_inputs as si
from paper_2309_03824_amd import binding as lrd

# max |gpu - oracle| / max |oracle| per output tensor
TOL = {"bf16": 2e-2, "f32": 1e-4}


def dev(a, dt):
    """numpy array -> device tensor in storage dtype dt ('bf16' | 'f32')."""
    if dt == "bf16":
        bits = si.bf16_bits(a).view(np.int16)
        return torch.from_numpy(bits).cuda().view(torch.bfloat16).reshape(a.shape)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def seen(a, dt):
    """The values the device tensor holds, as fp64 (what the oracle must be fed)."""
    return si.round_bf16(a).reshape(np.shape(a)) if dt == "bf16" else si.round_f32(a)


def host(t):
    return t.detach().to(torch.float64).cpu().numpy()


def empty(shape, dt, fill=None):
    td = torch.bfloat16 if dt == "bf16" else torch.float32
    t = torch.empty(shape, dtype=td, device="cuda")
    if fill is not None:
        t.fill_(fill)
    return t


def f32(shape, fill=None):
    t = torch.empty(shape, dtype=torch.float32, device="cuda")
    if fill is not None:
        t.fill_(fill)
    return t


def workspace(nbytes):
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device="cuda")


def rel_err(got, want):
    want = np.asarray(want, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    scale = np.max(np.abs(want))
    if scale == 0:
        return float(np.max(np.abs(got)))
    return float(np.max(np.abs(got - want)) / scale)


def check(got, want, dt, what):
    assert np.all(np.isfinite(got)), what
    e = rel_err(got, want)
    assert e <= TOL[dt], f"{what}: rel err {e:.3e} > {TOL[dt]}"
    return e


def code(dt):
    return lrd.BF16 if dt == "bf16" else lrd.F32
