"""GPU parity: cottn_fwd_bidir / cottn_bwd_bidir (through the C ABI) against the CPU oracle."""
import numpy as np
import pytest

from helpers import TOL, ds_terms_rss, rel_err, rel_err_ds, to_device, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def cottn():
    import paper_2409_18747_amd.binding as b
    yield b
    b.cottn_tune_segments(0)


def run_bidir(cottn, oracle, B, H, N, d, dtype, seed, segments=0, saved=False):
    import torch
    from paper_2409_18747_amd import workloads
    x = workloads.draw(B, H, N, d, dtype, seed)
    Q, K, V, dO = (to_device(x[k], dtype) for k in ("Q", "K", "V", "dO"))
    s = to_device(x["s"], "f32")
    cottn.cottn_tune_segments(segments)
    state = torch.full((B, H, d, d), float("nan"), dtype=torch.float32, device="cuda")
    fwd_ws = None
    if saved:
        # the backward takes the segment totals of Kh^T V over from the forward's workspace
        code = cottn.COTTN_BF16 if dtype == "bf16" else cottn.COTTN_F32
        need = cottn.cottn_workspace_bytes(cottn.OP_FWD_BIDIR, B, H, N, d, 0, code)
        fwd_ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
    O = cottn.cottn_fwd_bidir(Q, K, V, s, state=state, workspace=fwd_ws)
    dQ, dK, dV, ds = cottn.cottn_bwd_bidir(Q, K, V, s, dO, fwd_workspace=fwd_ws)
    torch.cuda.synchronize()
    O_ref = oracle.fwd_quadratic(x["Q"], x["K"], x["V"], x["s"], causal=False)
    S_ref = oracle.state_total(x["K"], x["V"])
    g_ref = oracle.bwd_quadratic(x["Q"], x["K"], x["V"], x["s"], x["dO"], causal=False)
    errs = {"O": rel_err(to_host(O), O_ref), "state": rel_err(to_host(state), S_ref)}
    for name, got, want in zip(("dQ", "dK", "dV"), (dQ, dK, dV), g_ref):
        errs[name] = rel_err(to_host(got), want)
    errs["ds"] = rel_err_ds(to_host(ds), g_ref[3], ds_terms_rss(oracle, x, causal=False))
    print("bidir %s B%d H%d N%d d%d seg%d saved%d: %s" %
          (dtype, B, H, N, d, segments, saved, {k: "%.2e" % v for k, v in errs.items()}), flush=True)
    for name, e in errs.items():
        assert e <= TOL[dtype], (name, e)


@pytest.mark.parametrize("N", [1, 17, 64, 65, 200, 512])
@pytest.mark.parametrize("d", [32, 64, 128])
def test_bf16(cottn, oracle, N, d):
    run_bidir(cottn, oracle, 2, 3, N, d, "bf16", seed=300 + N + d, segments=0)


@pytest.mark.parametrize("segments", [1, 3, 4, 5, 64])
def test_bf16_segments(cottn, oracle, segments):
    run_bidir(cottn, oracle, 2, 2, 333, 64, "bf16", seed=9, segments=segments)


@pytest.mark.parametrize("segments", [1, 2, 4, 6])
@pytest.mark.parametrize("d,N", [(64, 700), (128, 330), (32, 517)])
def test_bf16_totals_saved_by_forward(cottn, oracle, segments, d, N):
    run_bidir(cottn, oracle, 2, 3, N, d, "bf16", seed=41, segments=segments, saved=True)


def test_f32_ignores_forward_workspace(cottn, oracle):
    run_bidir(cottn, oracle, 1, 2, 150, 64, "f32", seed=42, segments=2, saved=True)


def test_bf16_bert_shape_slice(cottn, oracle):
    # the BERT-shaped workload (H=12, N=512, d=64) with 2 of its 32 batches
    run_bidir(cottn, oracle, 2, 12, 512, 64, "bf16", seed=2, segments=0)


@pytest.mark.parametrize("N,d,segments", [(1, 32, 0), (33, 32, 1), (100, 64, 3), (70, 128, 2)])
def test_f32(cottn, oracle, N, d, segments):
    run_bidir(cottn, oracle, 2, 2, N, d, "f32", seed=400 + N, segments=segments)
