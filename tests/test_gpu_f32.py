"""GPU parity of the fp32 path (tolerance 1e-4): causal forward and backward, incl. config 1."""
import numpy as np
import pytest

from helpers import TOL, ds_terms_rss, rel_err, rel_err_ds, to_device, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def cottn():
    import paper_2409_18747_amd.binding as b
    yield b
    b.cottn_tune_segments(0)


def run_f32(cottn, oracle, B, H, N, d, seed, segments=0, mutate=None):
    import torch
    from paper_2409_18747_amd import workloads
    x = workloads.draw(B, H, N, d, "f32", seed)
    if mutate:
        mutate(x)
    Q, K, V, dO = (to_device(x[k], "f32") for k in ("Q", "K", "V", "dO"))
    s = to_device(x["s"], "f32")
    cottn.cottn_tune_segments(segments)
    state = torch.full((B, H, d, d), float("nan"), dtype=torch.float32, device="cuda")
    O = cottn.cottn_fwd_causal(Q, K, V, s, state=state)
    dQ, dK, dV, ds = cottn.cottn_bwd_causal(Q, K, V, s, dO)
    torch.cuda.synchronize()
    O_ref = oracle.fwd_quadratic(x["Q"], x["K"], x["V"], x["s"])
    _, S_ref = oracle.fwd_recurrent(x["Q"], x["K"], x["V"], x["s"])
    g_ref = oracle.bwd_quadratic(x["Q"], x["K"], x["V"], x["s"], x["dO"])
    errs = {"O": rel_err(to_host(O), O_ref), "state": rel_err(to_host(state), S_ref)}
    for name, got, want in zip(("dQ", "dK", "dV"), (dQ, dK, dV), g_ref):
        errs[name] = rel_err(to_host(got), want)
    errs["ds"] = rel_err_ds(to_host(ds), g_ref[3], ds_terms_rss(oracle, x))
    print("f32 causal B%d H%d N%d d%d seg%d: %s" %
          (B, H, N, d, segments, {k: "%.2e" % v for k, v in errs.items()}), flush=True)
    for name, e in errs.items():
        assert e <= TOL["f32"], (name, e)
    return O, dQ, dK, dV


def test_config1_small_causal_forward(cottn, oracle):
    """B=1, H=2, N=256, d=32, fp32, seed 0: the smallest benchmark configuration, whole."""
    import torch
    from paper_2409_18747_amd import workloads
    w = workloads.WORKLOADS["cfg1_small_causal_fwd_f32"]
    x = workloads.draw_workload(w)
    Q, K, V = (to_device(x[k], "f32") for k in "QKV")
    s = to_device(x["s"], "f32")
    cottn.cottn_tune_segments(0)
    O = cottn.cottn_fwd_causal(Q, K, V, s, eps=w.eps)
    torch.cuda.synchronize()
    ref = oracle.fwd_quadratic(x["Q"], x["K"], x["V"], x["s"], eps=w.eps)
    e = rel_err(to_host(O), ref)
    print("config 1: rel err %.3e" % e, flush=True)
    assert e <= TOL["f32"]


@pytest.mark.parametrize("N", [1, 31, 32, 33, 100])
@pytest.mark.parametrize("d", [32, 64, 128])
def test_shapes(cottn, oracle, N, d):
    run_f32(cottn, oracle, 2, 2, N, d, seed=500 + N + d, segments=1)


@pytest.mark.parametrize("segments", [2, 5, 64])
def test_segments(cottn, oracle, segments):
    run_f32(cottn, oracle, 1, 3, 300, 64, seed=13, segments=segments)


def test_zero_rows(cottn, oracle):
    import torch

    def mutate(x):
        x["Q"][:, :, 3] = 0.0
        x["K"][:, :, 7] = 0.0

    out = run_f32(cottn, oracle, 1, 2, 70, 32, seed=14, segments=2, mutate=mutate)
    for t in out:
        assert torch.isfinite(t).all()
