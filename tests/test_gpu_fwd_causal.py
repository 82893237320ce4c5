"""GPU parity: cottn_fwd_causal (through the C ABI) against the CPU oracle, element by element."""
import numpy as np
import pytest

from helpers import TOL, rel_err, row_rel_err, to_device, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def cottn():
    import paper_2409_18747_amd.binding as b
    yield b
    b.cottn_tune_segments(0)


def run_fwd(cottn, oracle, B, H, N, d, dtype, seed, chunk=0, segments=0, want_state=True, scale=1.0):
    import torch
    from paper_2409_18747_amd import workloads
    x = workloads.draw(B, H, N, d, dtype, seed, value_scale=scale, with_dO=False)
    Q, K, V = (to_device(x[k], dtype) for k in "QKV")
    s = to_device(x["s"], "f32")
    state = torch.full((B, H, d, d), float("nan"), dtype=torch.float32, device="cuda") if want_state else None
    cottn.cottn_tune_segments(segments)
    O = cottn.cottn_fwd_causal(Q, K, V, s, state=state, chunk=chunk)
    torch.cuda.synchronize()
    if N <= 2048:
        ref = oracle.fwd_quadratic(x["Q"], x["K"], x["V"], x["s"], causal=True)
        _, Sref = oracle.fwd_recurrent(x["Q"], x["K"], x["V"], x["s"])
    else:
        ref, Sref = oracle.fwd_recurrent(x["Q"], x["K"], x["V"], x["s"])
    got = to_host(O)
    e = rel_err(got, ref)
    print("fwd_causal %s B%d H%d N%d d%d chunk%d seg%d: rel %.3e row-rel %.3e" %
          (dtype, B, H, N, d, chunk, segments, e, row_rel_err(got, ref)), flush=True)
    assert e <= TOL[dtype]
    if want_state:
        es = rel_err(to_host(state), Sref)
        assert es <= TOL[dtype], es
    return got


@pytest.mark.parametrize("N", [1, 15, 16, 63, 64, 65, 200, 256, 261])
@pytest.mark.parametrize("d", [32, 64, 128])
def test_bf16_one_segment(cottn, oracle, N, d):
    run_fwd(cottn, oracle, 2, 3, N, d, "bf16", seed=100 + N + d, segments=1)


@pytest.mark.parametrize("segments", [2, 3, 5, 64])
@pytest.mark.parametrize("d,N", [(64, 517), (128, 330), (32, 700)])
def test_bf16_segmented_matches(cottn, oracle, segments, d, N):
    run_fwd(cottn, oracle, 2, 2, N, d, "bf16", seed=7, segments=segments)


@pytest.mark.parametrize("chunk,d", [(128, 32), (128, 64), (256, 32), (256, 64)])
def test_bf16_chunk_sizes(cottn, oracle, chunk, d):
    for segments in (1, 3):
        run_fwd(cottn, oracle, 1, 3, 900, d, "bf16", seed=11, chunk=chunk, segments=segments)


def test_bf16_default_plan_gpt_shape(cottn, oracle):
    # the benchmark shape with fewer batches; default segment heuristic
    run_fwd(cottn, oracle, 2, 12, 1024, 64, "bf16", seed=1, segments=0)


def test_bf16_zero_rows_and_determinism(cottn, oracle):
    import torch
    from paper_2409_18747_amd import workloads
    B, H, N, d = 1, 2, 150, 64
    x = workloads.draw(B, H, N, d, "bf16", 5, with_dO=False)
    x["Q"][:, :, 10] = 0.0   # padded rows (Sec. 4: padding is applied by zeroing rows)
    x["K"][:, :, 20:23] = 0.0
    x["V"][:, :, 20:23] = 0.0
    Q, K, V = (to_device(x[k], "bf16") for k in "QKV")
    s = to_device(x["s"], "f32")
    cottn.cottn_tune_segments(2)
    O1 = cottn.cottn_fwd_causal(Q, K, V, s)
    O2 = cottn.cottn_fwd_causal(Q, K, V, s)
    torch.cuda.synchronize()
    assert torch.isfinite(O1.float()).all()
    assert torch.equal(O1, O2)
    ref = oracle.fwd_quadratic(x["Q"], x["K"], x["V"], x["s"])
    assert rel_err(to_host(O1), ref) <= TOL["bf16"]
    assert np.all(to_host(O1)[:, :, 10] == 0.0)


@pytest.mark.parametrize("dtype,d,cuts,segments", [
    ("bf16", 64, (0, 300, 301, 700, 1000), 0),
    ("bf16", 64, (0, 517, 1100), 3),
    ("bf16", 128, (0, 64, 330), 2),
    ("bf16", 32, (0, 1, 200, 450), 0),
    ("f32", 32, (0, 100, 260), 0),
    ("f32", 64, (0, 33, 150), 3),
])
def test_sequence_fed_in_pieces(cottn, oracle, dtype, d, cuts, segments):
    """A sequence fed piece by piece through cottn_fwd_causal_from_state gives the rows and the
    final state of one pass over the whole sequence (Sec. 5: the state carries all the later
    tokens need)."""
    import torch
    from paper_2409_18747_amd import workloads
    B, H, N = 2, 3, cuts[-1]
    x = workloads.draw(B, H, N, d, dtype, 91, with_dO=False)
    s = to_device(x["s"], "f32")
    cottn.cottn_tune_segments(segments)
    ref, S_ref = oracle.fwd_recurrent(x["Q"], x["K"], x["V"], x["s"])
    state = torch.zeros(B, H, d, d, dtype=torch.float32, device="cuda")
    outs = []
    for a, b in zip(cuts[:-1], cuts[1:]):
        Q, K, V = (to_device(x[k][:, :, a:b], dtype) for k in "QKV")
        nxt = torch.full_like(state, float("nan"))
        if a == 0:
            O = cottn.cottn_fwd_causal(Q, K, V, s, state=nxt)
        else:
            O = cottn.cottn_fwd_causal_from_state(Q, K, V, s, state, state=nxt)
        state = nxt
        outs.append(to_host(O))
    torch.cuda.synchronize()
    got = np.concatenate(outs, axis=2)
    e, es = rel_err(got, ref), rel_err(to_host(state), S_ref)
    print("pieces %s d%d cuts %s: rel %.3e state %.3e" % (dtype, d, cuts, e, es), flush=True)
    assert e <= TOL[dtype] and es <= TOL[dtype]


def test_prefill_from_decode_state(cottn, oracle):
    """The state of a few cottn_step calls continues into a multi-token piece."""
    import torch
    from paper_2409_18747_amd import workloads
    B, H, d, n_steps, N = 2, 2, 64, 5, 200
    x = workloads.draw(B, H, n_steps + N, d, "bf16", 92, with_dO=False)
    s = to_device(x["s"], "f32")
    state = torch.zeros(B, H, d, d, dtype=torch.float32, device="cuda")
    for t in range(n_steps):
        q, k, v = (to_device(x[n][:, :, t], "bf16") for n in "QKV")
        cottn.cottn_step(q, k, v, s, state)
    Q, K, V = (to_device(x[n][:, :, n_steps:], "bf16") for n in "QKV")
    O = cottn.cottn_fwd_causal_from_state(Q, K, V, s, state)
    torch.cuda.synchronize()
    ref, _ = oracle.fwd_recurrent(x["Q"], x["K"], x["V"], x["s"])
    assert rel_err(to_host(O), ref[:, :, n_steps:]) <= TOL["bf16"]


def test_empty_piece_copies_the_state(cottn):
    """N = 0 through the C ABI itself (the tensor-based binding has no pointer for an empty
    tensor): the state passes through unchanged."""
    import ctypes
    import torch
    B, H, d = 2, 3, 64
    dummy = torch.zeros(16, dtype=torch.bfloat16, device="cuda")
    s = torch.ones(H, device="cuda")
    g = torch.Generator(device="cuda"); g.manual_seed(5)
    state_in = torch.randn(B, H, d, d, device="cuda", generator=g)
    state = torch.full_like(state_in, float("nan"))
    ptr = lambda t: ctypes.c_void_p(t.data_ptr())
    st = cottn.lib.cottn_fwd_causal_from_state(ptr(dummy), ptr(dummy), ptr(dummy), ptr(s), ptr(state_in),
                                               ptr(dummy), ptr(state), None, 0, B, H, 0, d, 0,
                                               cottn.COTTN_BF16, 1e-6,
                                               ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    assert st == 0
    assert torch.equal(state, state_in)


@pytest.mark.parametrize("k", [1, 4, 7])
def test_multi_token_step_equals_single_steps(cottn, oracle, k):
    """A k-token step (speculative decoding) is cottn_fwd_causal_from_state with N = k: same
    outputs and same final state as k calls of cottn_step, to bf16 output rounding."""
    import torch
    from paper_2409_18747_amd import workloads
    B, H, d, warm = 3, 4, 128, 40
    x = workloads.draw(B, H, warm + k, d, "bf16", 93, with_dO=False)
    s = to_device(x["s"], "f32")
    Q, K, V = (to_device(x[n], "bf16") for n in "QKV")
    state0 = torch.empty(B, H, d, d, dtype=torch.float32, device="cuda")
    cottn.cottn_fwd_causal(Q[:, :, :warm].contiguous(), K[:, :, :warm].contiguous(),
                           V[:, :, :warm].contiguous(), s, state=state0)
    # k single steps
    st_a = state0.clone()
    o_a = [cottn.cottn_step(Q[:, :, warm + t].contiguous(), K[:, :, warm + t].contiguous(),
                            V[:, :, warm + t].contiguous(), s, st_a) for t in range(k)]
    # one k-token call
    st_b = torch.empty_like(state0)
    O_b = cottn.cottn_fwd_causal_from_state(Q[:, :, warm:].contiguous(), K[:, :, warm:].contiguous(),
                                            V[:, :, warm:].contiguous(), s, state0, state=st_b)
    torch.cuda.synchronize()
    ref, S_ref = oracle.fwd_recurrent(x["Q"], x["K"], x["V"], x["s"])
    got_a = np.stack([to_host(o) for o in o_a], axis=2)
    assert rel_err(got_a, ref[:, :, warm:]) <= TOL["bf16"]
    assert rel_err(to_host(O_b), ref[:, :, warm:]) <= TOL["bf16"]
    assert rel_err(to_host(st_a), S_ref) <= TOL["bf16"] and rel_err(to_host(st_b), S_ref) <= TOL["bf16"]
    assert rel_err(to_host(O_b), got_a) <= 2.0 ** -6
