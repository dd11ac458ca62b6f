"""Helpers for the GPU parity tests: device buffers through torch, column-major
marshalling, the error metric and its tolerances."""
import numpy as np
import torch

import workload

TOL = {"f32": 1e-5, "bf16": 2e-2}     # max-norm relative error allowed against the fp64 oracle


def stream_ptr():
    return torch.cuda.current_stream().cuda_stream


def to_dev(a, dtype="f32"):
    """Logical array -> flat device tensor, first axis fastest."""
    a = np.asarray(a, np.float32)
    t = torch.from_numpy(np.ascontiguousarray(a.T).reshape(-1))
    if dtype == "bf16":
        t = t.to(torch.bfloat16)
    return t.cuda()


def from_dev(t, shape):
    h = t.to(torch.float32).cpu().numpy()
    return h.reshape(tuple(reversed(shape))).T.astype(np.float64)


def quant(a, dtype):
    """The values the device really holds for input `a` stored as `dtype`."""
    a = np.asarray(a, np.float32)
    if dtype == "bf16":
        return workload.round_through_bf16(a.reshape(-1)).reshape(a.shape).astype(np.float64)
    return a.astype(np.float64)


def relerr(got, ref):
    ref = np.asarray(ref, np.float64)
    den = np.abs(ref).max()
    return float(np.abs(np.asarray(got, np.float64) - ref).max() / (den if den > 0 else 1.0))


def check(got, ref, dtype, what=""):
    e = relerr(got, ref)
    assert np.all(np.isfinite(got)), what + ": non-finite output"
    assert e <= TOL[dtype], "%s: max-norm relative error %.3e > %.1e" % (what, e, TOL[dtype])
    return e


def code(dtype):
    return 0 if dtype == "f32" else 1
