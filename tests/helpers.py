"""Shared helpers of the GPU parity tests: move seeded inputs to the device, run the CPU oracle
on the same bits, and measure the error the way the tolerances are stated."""
import numpy as np

# tolerances: tensor-relative infinity-norm error  max|got - ref| / max|ref|
# f16 runs the bf16 kernels with a unit roundoff of 2^-11 instead of 2^-8: the bf16 bar scaled by 1/8
TOL = {"f32": 1e-4, "bf16": 2e-2, "f16": 2.5e-3}


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
    if dtype == "f16":
        t = t.to(torch.float16)   # exact likewise
    return t.cuda()


def to_host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def ds_terms_rss(oracle, x, causal=True, lens=None, per_unit=False):
    """Root-sum-square of the terms P_ij * A_ij whose (signed) sum is ds: per head (summed over
    the batch, as ds[h] is), or per (batch, head) with per_unit (as ds[b][h] of the padded-batch
    calls is).  lens: rows at or beyond lens[b] do not exist.

    ds is a long sum of terms of both signs; when it happens to cancel, |ds| is far below the
    size of what was added up and a relative error against |ds| alone measures the
    cancellation, not the arithmetic.  The root-sum-square of the terms is the magnitude a
    sum of that many independent terms typically has, and is the floor of the scale the ds
    error is measured against (see rel_err_ds).  Uses only the oracle's similarity matrix
    and a plain matmul for A = dO V^T; it is a scale, never an expected value.
    """
    Q, K, V, dO = (np.asarray(x[k], dtype=np.float64) for k in ("Q", "K", "V", "dO"))
    B, H, N, d = Q.shape
    acc = np.zeros((B, H))
    for b in range(B):
        n = N if lens is None else int(lens[b])
        if n == 0:
            continue
        for h in range(H):
            P = oracle.similarity(Q[b, h, :n], K[b, h, :n])
            A = dO[b, h, :n] @ V[b, h, :n].T
            T = P * A
            if causal:
                T = np.tril(T)
            acc[b, h] = (T ** 2).sum()
    return np.sqrt(acc) if per_unit else np.sqrt(acc.sum(0))


def rel_err_ds(got, ref, rss):
    """max |got - ref| / max(max |ref|, max rss): the stated tensor-relative metric whenever ds
    does not cancel below the size of its own terms (then the two denominators coincide)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = max(np.abs(ref).max(), float(np.max(rss)))
    return float(np.abs(got - ref).max() / den) if den > 0 else float(np.abs(got).max())


def ds_errors(got, ref, rss):
    """{"ds": the asserted metric (rel_err_ds), "ds_plain": max|got-ref|/max|ref|, reported, and
    "ds_cancels": whether the two differ (max|ref| below the scale of the terms)}."""
    ref = np.asarray(ref, dtype=np.float64)
    return {"ds": rel_err_ds(got, ref, rss), "ds_plain": rel_err(got, ref),
            "ds_cancels": bool(np.abs(ref).max() < float(np.max(rss)))}
