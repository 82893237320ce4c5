"""GPU parity on seeded random shapes: every 16-bit and fp32 entry point of the training path
(padded-batch variants, which contain the fixed-length ones as the case of full lengths)
against the CPU oracle, with batch, heads, length, head dimension, segment count, chunk size
and sequence lengths drawn from a seeded generator.  The parametrised tests elsewhere walk
the edges on purpose; this one looks for combinations nobody thought of (COTTN_RANDOM_CASES in
the environment draws more of them)."""
import os

import numpy as np
import pytest

from helpers import TOL, ds_errors, ds_terms_rss, rel_err, to_device, to_host

pytestmark = pytest.mark.gpu


def cases(n):
    rng = np.random.Generator(np.random.Philox(20240918))
    out = []
    for i in range(n):
        dtype = ["bf16", "f16", "f32"][int(rng.integers(0, 3))]
        d = [32, 64, 128][int(rng.integers(0, 3))]
        B, H = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        N = int(rng.integers(1, 420))
        chunk = 0
        if dtype != "f32" and d != 128 and rng.random() < 0.3:
            chunk = [64, 128, 256][int(rng.integers(0, 3))]
        segments = int(rng.integers(0, 9))
        causal = bool(rng.integers(0, 2))
        full = rng.random() < 0.3
        lens = [N if full else int(rng.integers(0, N + 1)) for _ in range(B)]
        saved = bool(rng.integers(0, 2))
        out.append(pytest.param(dtype, d, B, H, N, chunk, segments, causal, lens, saved, 3000 + i,
                                id="%d-%s-d%d-B%dH%dN%d-c%d-g%d-%s" % (
                                    i, dtype, d, B, H, N, chunk, segments, "causal" if causal else "bidir")))
    return out


@pytest.mark.parametrize("dtype,d,B,H,N,chunk,segments,causal,lens,saved,seed", cases(int(os.environ.get("COTTN_RANDOM_CASES", "40"))))
def test_random_shape(oracle, dtype, d, B, H, N, chunk, segments, causal, lens, saved, seed):
    import torch
    import paper_2409_18747_amd.binding as cottn
    from paper_2409_18747_amd import workloads
    x = workloads.draw(B, H, N, d, dtype, seed)
    rng = np.random.Generator(np.random.Philox(seed + 7))
    s_bh = rng.uniform(0.5, 1.5, (B, H)).astype(np.float32)
    Q, K, V, dO = (to_device(x[k], dtype) for k in ("Q", "K", "V", "dO"))
    s = to_device(s_bh, "f32")
    L = torch.tensor(lens, dtype=torch.int32, device="cuda")
    code = {"bf16": cottn.COTTN_BF16, "f16": cottn.COTTN_F16, "f32": cottn.COTTN_F32}[dtype]
    kw = {"chunk": chunk} if causal else {}
    try:
        cottn.cottn_tune_segments(segments)
        op = cottn.OP_FWD_CAUSAL if causal else cottn.OP_FWD_BIDIR
        fwd_ws = None
        if saved:
            need = cottn.cottn_workspace_bytes(op, B, H, N, d, chunk if causal else 0, code)
            fwd_ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
        fwd = cottn.cottn_fwd_causal_varlen if causal else cottn.cottn_fwd_bidir_varlen
        bwd = cottn.cottn_bwd_causal_varlen if causal else cottn.cottn_bwd_bidir_varlen
        O = fwd(Q, K, V, s, L, workspace=fwd_ws, **kw)
        dQ, dK, dV, ds = bwd(Q, K, V, s, L, dO, fwd_workspace=fwd_ws, **kw)
        torch.cuda.synchronize()
    finally:
        cottn.cottn_tune_segments(0)
    O_ref, _ = oracle.fwd_varlen(x["Q"], x["K"], x["V"], s_bh, lens, causal=causal)
    g_ref = oracle.bwd_varlen(x["Q"], x["K"], x["V"], s_bh, x["dO"], lens, causal=causal)
    errs = {"O": rel_err(to_host(O), O_ref)}
    for name, got, want in zip(("dQ", "dK", "dV"), (dQ, dK, dV), g_ref):
        errs[name] = rel_err(to_host(got), want)
    # ds[b][h] is a signed sum that may cancel: measured against the larger of max|ds| and the
    # root-sum-square of its terms (helpers.rel_err_ds), at the same tolerance as every tensor
    dse = ds_errors(to_host(ds), g_ref[3], ds_terms_rss(oracle, x, causal, lens, per_unit=True))
    errs["ds"] = dse["ds"]
    print("random shape:", {k: "%.2e" % v for k, v in errs.items()},
          "ds_plain %.2e%s" % (dse["ds_plain"], " (cancels)" if dse["ds_cancels"] else ""), flush=True)
    for name, e in errs.items():
        assert e <= TOL[dtype], (name, e, errs, dse)
