"""GPU parity for IEEE half-precision storage: the 16-bit MFMA kernels compiled for fp16, every
entry point, against the CPU oracle (tolerance: the bf16 bar scaled by the ratio of the unit
roundoffs, see helpers.TOL)."""
import numpy as np
import pytest

from helpers import TOL, ds_terms_rss, rel_err, rel_err_ds, to_device, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def cottn():
    import paper_2409_18747_amd.binding as b
    yield b
    b.cottn_tune_segments(0)


@pytest.mark.parametrize("segments", [0, 1, 3, 6])
@pytest.mark.parametrize("d,N", [(64, 517), (128, 330), (32, 700)])
def test_causal(cottn, oracle, segments, d, N):
    import torch
    from paper_2409_18747_amd import workloads
    B, H = 2, 3
    x = workloads.draw(B, H, N, d, "f16", 800 + d + segments)
    Q, K, V, dO = (to_device(x[k], "f16") for k in ("Q", "K", "V", "dO"))
    s = to_device(x["s"], "f32")
    cottn.cottn_tune_segments(segments)
    state = torch.full((B, H, d, d), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(cottn.cottn_workspace_bytes(cottn.OP_FWD_CAUSAL, B, H, N, d, 0, cottn.COTTN_F16), 256),
                     dtype=torch.uint8, device="cuda")
    O = cottn.cottn_fwd_causal(Q, K, V, s, state=state, workspace=ws)
    g1 = cottn.cottn_bwd_causal(Q, K, V, s, dO)
    g2 = cottn.cottn_bwd_causal(Q, K, V, s, dO, fwd_workspace=ws)
    torch.cuda.synchronize()
    assert O.dtype == torch.float16
    O_ref = oracle.fwd_quadratic(x["Q"], x["K"], x["V"], x["s"])
    S_ref = oracle.state_total(x["K"], x["V"])
    ref = oracle.bwd_quadratic(x["Q"], x["K"], x["V"], x["s"], x["dO"])
    errs = {"O": rel_err(to_host(O), O_ref), "state": rel_err(to_host(state), S_ref)}
    for g, tag in ((g1, ""), (g2, "'")):
        for name, got, want in zip(("dQ", "dK", "dV"), g, ref):
            errs[name + tag] = rel_err(to_host(got), want)
        errs["ds" + tag] = rel_err_ds(to_host(g[3]), ref[3], ds_terms_rss(oracle, x))
    print("f16 causal d%d N%d seg%d: %s" % (d, N, segments, {k: "%.1e" % v for k, v in errs.items()}), flush=True)
    for name, e in errs.items():
        assert e <= TOL["f16"], (name, e)


@pytest.mark.parametrize("segments", [0, 3, 6])
@pytest.mark.parametrize("d,N", [(64, 333), (128, 200), (32, 512)])
def test_bidirectional(cottn, oracle, segments, d, N):
    import torch
    from paper_2409_18747_amd import workloads
    B, H = 2, 2
    x = workloads.draw(B, H, N, d, "f16", 820 + d + segments)
    Q, K, V, dO = (to_device(x[k], "f16") for k in ("Q", "K", "V", "dO"))
    s = to_device(x["s"], "f32")
    cottn.cottn_tune_segments(segments)
    ws = torch.empty(max(cottn.cottn_workspace_bytes(cottn.OP_FWD_BIDIR, B, H, N, d, 0, cottn.COTTN_F16), 256),
                     dtype=torch.uint8, device="cuda")
    O = cottn.cottn_fwd_bidir(Q, K, V, s, workspace=ws)
    g = cottn.cottn_bwd_bidir(Q, K, V, s, dO, fwd_workspace=ws)
    torch.cuda.synchronize()
    O_ref = oracle.fwd_quadratic(x["Q"], x["K"], x["V"], x["s"], causal=False)
    ref = oracle.bwd_quadratic(x["Q"], x["K"], x["V"], x["s"], x["dO"], causal=False)
    errs = {"O": rel_err(to_host(O), O_ref)}
    for name, got, want in zip(("dQ", "dK", "dV"), g, ref):
        errs[name] = rel_err(to_host(got), want)
    errs["ds"] = rel_err_ds(to_host(g[3]), ref[3], ds_terms_rss(oracle, x, causal=False))
    print("f16 bidir d%d N%d seg%d: %s" % (d, N, segments, {k: "%.1e" % v for k, v in errs.items()}), flush=True)
    for name, e in errs.items():
        assert e <= TOL["f16"], (name, e)


@pytest.mark.parametrize("d", [32, 64, 128])
def test_decode_steps_and_pieces(cottn, oracle, d):
    """Prefill, a piece continued from its state, then single steps, all in fp16."""
    import torch
    from paper_2409_18747_amd import workloads
    B, H, n1, n2, n3 = 2, 3, 150, 70, 6
    N = n1 + n2 + n3
    x = workloads.draw(B, H, N, d, "f16", 840 + d, with_dO=False)
    s = to_device(x["s"], "f32")
    Q, K, V = (to_device(x[n], "f16") for n in "QKV")
    cut = lambda t, a, b: t[:, :, a:b].contiguous()
    st1 = torch.empty(B, H, d, d, dtype=torch.float32, device="cuda")
    st2 = torch.empty_like(st1)
    O1 = cottn.cottn_fwd_causal(cut(Q, 0, n1), cut(K, 0, n1), cut(V, 0, n1), s, state=st1)
    O2 = cottn.cottn_fwd_causal_from_state(cut(Q, n1, n1 + n2), cut(K, n1, n1 + n2), cut(V, n1, n1 + n2), s,
                                           st1, state=st2)
    o3 = [cottn.cottn_step(Q[:, :, t].contiguous(), K[:, :, t].contiguous(), V[:, :, t].contiguous(), s, st2)
          for t in range(n1 + n2, N)]
    torch.cuda.synchronize()
    ref, S_ref = oracle.fwd_recurrent(x["Q"], x["K"], x["V"], x["s"])
    got = np.concatenate([to_host(O1), to_host(O2), np.stack([to_host(o) for o in o3], axis=2)], axis=2)
    assert rel_err(got, ref) <= TOL["f16"]
    assert rel_err(to_host(st2), S_ref) <= TOL["f16"]


def test_padded_batch(cottn, oracle):
    import torch
    from paper_2409_18747_amd import workloads
    B, H, N, d = 3, 2, 260, 64
    lens = [260, 0, 97]
    x = workloads.draw(B, H, N, d, "f16", 860)
    rng = np.random.Generator(np.random.Philox(861))
    s_bh = rng.uniform(0.5, 1.5, (B, H)).astype(np.float32)
    Q, K, V, dO = (to_device(x[k], "f16") for k in ("Q", "K", "V", "dO"))
    s = to_device(s_bh, "f32")
    L = torch.tensor(lens, dtype=torch.int32, device="cuda")
    O = cottn.cottn_fwd_causal_varlen(Q, K, V, s, L)
    g = cottn.cottn_bwd_causal_varlen(Q, K, V, s, L, dO)
    torch.cuda.synchronize()
    O_ref, _ = oracle.fwd_varlen(x["Q"], x["K"], x["V"], s_bh, lens)
    ref = oracle.bwd_varlen(x["Q"], x["K"], x["V"], s_bh, x["dO"], lens)
    assert rel_err(to_host(O), O_ref) <= TOL["f16"]
    for got, want in zip(g[:3], ref[:3]):
        assert rel_err(to_host(got), want) <= TOL["f16"]
    assert rel_err(to_host(g[3]), ref[3]) <= 4 * TOL["f16"]


@pytest.mark.parametrize("eps", [1e-6, 1e-3])
def test_zero_norm_rows(cottn, oracle, eps):
    """Key and query rows that are exactly zero (padding by zeroed rows, Sec. 4) while their
    value rows are not: every other row must come out finite and right, which requires that no
    row is ever multiplied by a zero row's factor 1/eps inside the kernels (fp16 would
    overflow).  The gradient of a zero row itself is 1/eps times a quantity of order one (the
    derivative of x/max(|x|, eps) at the clamp): representable in fp16 only for the larger
    eps; with the default eps those rows overflow fp16 storage and are left out."""
    import torch
    from paper_2409_18747_amd import workloads
    B, H, N, d = 2, 2, 200, 64
    x = workloads.draw(B, H, N, d, "f16", 870)
    zero_k, zero_q = [5, 70, 71, 199], [64]
    x["K"][:, :, zero_k] = 0.0
    x["Q"][:, :, zero_q] = 0.0
    Q, K, V, dO = (to_device(x[k], "f16") for k in ("Q", "K", "V", "dO"))
    s = to_device(x["s"], "f32")
    cottn.cottn_tune_segments(2)
    for causal in (True, False):
        if causal:
            O = cottn.cottn_fwd_causal(Q, K, V, s, eps=eps)
            g = cottn.cottn_bwd_causal(Q, K, V, s, dO, eps=eps)
        else:
            O = cottn.cottn_fwd_bidir(Q, K, V, s, eps=eps)
            g = cottn.cottn_bwd_bidir(Q, K, V, s, dO, eps=eps)
        torch.cuda.synchronize()
        O_ref = oracle.fwd_quadratic(x["Q"], x["K"], x["V"], x["s"], eps=eps, causal=causal)
        ref = [t.copy() for t in
               oracle.bwd_quadratic(x["Q"], x["K"], x["V"], x["s"], x["dO"], eps=eps, causal=causal)]
        got = [to_host(t).copy() for t in g]
        if eps < 1e-4:   # (1/eps) * O(1) is beyond fp16's largest finite value
            for t in (got[0], ref[0]):
                t[:, :, zero_q] = 0.0
            for t in (got[1], ref[1]):
                t[:, :, zero_k] = 0.0
        assert rel_err(to_host(O), O_ref) <= TOL["f16"]
        for name, a, b in zip(("dQ", "dK", "dV"), got, ref):
            assert np.isfinite(a).all(), (causal, name)
            assert rel_err(a, b) <= TOL["f16"], (causal, name)
