"""Helpers shared by the GPU parity tests (test infrastructure only)."""
import numpy as np

from paper_2508_02317_amd.inputs import quantise

TOL = {"f32": 1e-5, "bf16": 2e-2}     # max|got - ref| / max|ref| per output tensor


def torch_dtype(name):
    import torch
    return torch.float32 if name == "f32" else torch.bfloat16


def to_dev(a, dtype_name=None):
    """numpy -> device tensor.  Float arrays already hold values representable in the target dtype."""
    import torch
    a = np.ascontiguousarray(a)
    t = torch.from_numpy(a).cuda()
    if dtype_name is not None:
        t = t.to(torch_dtype(dtype_name))
    return t.contiguous()


def to_np(t):
    import torch
    if t.dtype == torch.bfloat16:
        t = t.float()
    return t.detach().cpu().numpy()


def q(a, dtype_name):
    """Round an fp64 oracle intermediate to the dtype the GPU stage receives (as float32 values)."""
    return quantise(np.asarray(a, dtype=np.float32), dtype_name)


def rel_err(got, ref):
    got = np.asarray(got, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    assert np.all(np.isfinite(got)), "non-finite values in GPU output"
    den = np.max(np.abs(ref))
    num = np.max(np.abs(got - ref))
    return num / den if den > 0 else num


def assert_close(got, ref, dtype_name, what, tol=None):
    e = rel_err(got, ref)
    t = TOL[dtype_name] if tol is None else tol
    assert e <= t, "%s: max-abs/max-ref = %.3e > %.1e" % (what, e, t)
    return e
