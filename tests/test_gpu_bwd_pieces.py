"""GPU parity: the causal backward of a sequence processed in pieces
(cottn_fwd_causal_from_state first to last, cottn_bwd_causal_from_state last to first, states
handed across the boundaries) against the CPU oracle's gradients of the whole sequence."""
import numpy as np
import pytest

from helpers import TOL, ds_terms_rss, rel_err, rel_err_ds, to_device, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def cottn():
    import paper_2409_18747_amd.binding as b
    yield b
    b.cottn_tune_segments(0)


def run_pieces(cottn, oracle, dtype, d, pieces, segments, saved, seed, B=2, H=3):
    import torch
    from paper_2409_18747_amd import workloads
    N = sum(pieces)
    x = workloads.draw(B, H, N, d, dtype, seed)
    Q, K, V, dO = (to_device(x[k], dtype) for k in ("Q", "K", "V", "dO"))
    s = to_device(x["s"], "f32")
    code = {"bf16": cottn.COTTN_BF16, "f16": cottn.COTTN_F16, "f32": cottn.COTTN_F32}[dtype]
    cottn.cottn_tune_segments(segments)
    bounds = np.concatenate([[0], np.cumsum(pieces)])
    cut = lambda t, i: t[:, :, bounds[i]:bounds[i + 1]].contiguous()
    # forward, first to last: each piece starts from the state the previous one left
    states, workspaces = [None], []
    for i, n in enumerate(pieces):
        ws = None
        if saved:
            need = cottn.cottn_workspace_bytes(cottn.OP_FWD_CAUSAL, B, H, n, d, 0, code)
            ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
        out_state = torch.empty(B, H, d, d, dtype=torch.float32, device="cuda")
        if states[-1] is None:
            cottn.cottn_fwd_causal(cut(Q, i), cut(K, i), cut(V, i), s, state=out_state, workspace=ws)
        else:
            cottn.cottn_fwd_causal_from_state(cut(Q, i), cut(K, i), cut(V, i), s, states[-1],
                                              state=out_state, workspace=ws)
        states.append(out_state)
        workspaces.append(ws)
    # backward, last to first: each piece is handed the reverse state of what follows it
    rev = None
    grads = [None] * len(pieces)
    ds_total = torch.zeros(H, dtype=torch.float32, device="cuda")
    for i in reversed(range(len(pieces))):
        rev_out = torch.full((B, H, d, d), float("nan"), dtype=torch.float32, device="cuda")
        dQ, dK, dV, ds = cottn.cottn_bwd_causal_from_state(
            cut(Q, i), cut(K, i), cut(V, i), s, cut(dO, i), state_in=states[i], rev_state_in=rev,
            rev_state_out=rev_out, fwd_workspace=workspaces[i])
        grads[i] = (dQ, dK, dV)
        ds_total += ds
        rev = rev_out
    torch.cuda.synchronize()
    ref = oracle.bwd_quadratic(x["Q"], x["K"], x["V"], x["s"], x["dO"], causal=True)
    errs = {}
    for k, name in enumerate(("dQ", "dK", "dV")):
        got = np.concatenate([to_host(g[k]) for g in grads], axis=2)
        errs[name] = rel_err(got, ref[k])
    errs["ds"] = rel_err_ds(to_host(ds_total), ref[3], ds_terms_rss(oracle, x))
    # the reverse state that leaves the first piece is the sum of qh_i^T dO_i over all rows
    errs["rev_state"] = rel_err(to_host(rev), oracle.state_total(x["Q"], x["dO"]))
    print("pieces %s d%d %s seg%d saved%d: %s" % (dtype, d, pieces, segments, saved,
                                                   {k: "%.1e" % v for k, v in errs.items()}), flush=True)
    for name, e in errs.items():
        assert e <= TOL[dtype], (name, e)


@pytest.mark.parametrize("saved", [False, True])
@pytest.mark.parametrize("segments", [0, 1, 3, 6])
@pytest.mark.parametrize("d,pieces", [(64, [130, 100, 70]), (128, [64, 200]), (32, [1, 255, 17, 90])])
def test_bf16(cottn, oracle, d, pieces, segments, saved):
    run_pieces(cottn, oracle, "bf16", d, pieces, segments, saved, seed=900 + d + segments)


@pytest.mark.parametrize("dtype,d", [("f16", 64), ("f32", 64), ("f32", 32), ("f16", 128)])
@pytest.mark.parametrize("segments", [0, 3])
def test_other_types(cottn, oracle, dtype, d, segments):
    run_pieces(cottn, oracle, dtype, d, [90, 150, 33], segments, saved=(dtype == "f16"), seed=950 + d)


def test_empty_piece_passes_the_states_on(cottn):
    """N = 0 through the C ABI itself (the tensor-based binding has no pointer for an empty
    tensor): ds is zero and the reverse state passes through unchanged."""
    import ctypes
    import torch
    B, H, d = 2, 3, 64
    dummy = torch.zeros(16, dtype=torch.bfloat16, device="cuda")
    s = torch.ones(H, device="cuda")
    g = torch.Generator(device="cuda"); g.manual_seed(6)
    rev_in = torch.randn(B, H, d, d, device="cuda", generator=g)
    rev_out = torch.full_like(rev_in, float("nan"))
    ds = torch.full((H,), float("nan"), device="cuda")
    ws = torch.empty(4096, dtype=torch.uint8, device="cuda")
    ptr = lambda t: ctypes.c_void_p(t.data_ptr())
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    for given, want in ((rev_in, rev_in), (None, torch.zeros_like(rev_in))):
        st = cottn.lib.cottn_bwd_causal_from_state(
            ptr(dummy), ptr(dummy), ptr(dummy), ptr(s), ptr(dummy), None,
            None if given is None else ptr(given), ptr(dummy), ptr(dummy), ptr(dummy), ptr(ds),
            ptr(rev_out), None, 0, ptr(ws), 4096, B, H, 0, d, 0, cottn.COTTN_BF16, 1e-6, stream)
        torch.cuda.synchronize()
        assert st == 0
        assert torch.equal(rev_out, want)
        assert torch.all(ds == 0)


def test_one_piece_equals_the_plain_call(cottn, oracle):
    """Without states the piecewise entry point is cottn_bwd_causal, bit for bit."""
    import torch
    from paper_2409_18747_amd import workloads
    B, H, N, d = 2, 2, 333, 64
    x = workloads.draw(B, H, N, d, "bf16", 980)
    Q, K, V, dO = (to_device(x[k], "bf16") for k in ("Q", "K", "V", "dO"))
    s = to_device(x["s"], "f32")
    cottn.cottn_tune_segments(3)
    a = cottn.cottn_bwd_causal(Q, K, V, s, dO)
    b = cottn.cottn_bwd_causal_from_state(Q, K, V, s, dO)
    torch.cuda.synchronize()
    for u, v in zip(a, b):
        assert torch.equal(u, v)
