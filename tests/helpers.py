"""Shared helpers of the GPU parity tests: move seeded inputs to the device, run the CPU oracle
on the same bits, and measure the error the way the tolerances are stated."""
import numpy as np

# tolerances: tensor-relative infinity-norm error  max|got - ref| / max|ref|
TOL = {"f32": 1e-4, "bf16": 2e-2}


def rel_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.abs(ref).max()
    if den == 0.0:
        return float(np.abs(got).max())
    return float(np.abs(got - ref).max() / den)


def row_rel_err(got, ref):
    """Stricter, reported only: worst row of max|got_i - ref_i| / max|ref_i|."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    num = np.abs(got - ref).max(-1)
    den = np.maximum(np.abs(ref).max(-1), 1e-30)
    return float((num / den).max())


def to_device(x, dtype):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x))
    if dtype == "bf16":
        t = t.to(torch.bfloat16)  # exact: values are already bf16-representable
    return t.cuda()


def to_host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)
