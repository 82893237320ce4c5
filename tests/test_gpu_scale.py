"""GPU parity: the stabiliser map of Sec. 3.3 (cottn_scale_from_m / cottn_scale_backward, through
the C ABI) against the CPU oracle, alone and chained around the attention forward + backward."""
import numpy as np
import pytest

from helpers import TOL, rel_err, to_device, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def cottn():
    import paper_2409_18747_amd.binding as b
    yield b
    b.cottn_tune_segments(0)


@pytest.mark.parametrize("H", [1, 12, 16, 300])
@pytest.mark.parametrize("n", [1, 2, 512, 65536])
def test_map_and_gradient(cottn, oracle, H, n):
    import torch
    rng = np.random.Generator(np.random.Philox(500 + H + n))
    m = rng.uniform(-4.0, 4.0, H).astype(np.float32)
    m[0] = 0.5  # the paper's initial value
    ds = rng.standard_normal(H).astype(np.float32)
    s = cottn.cottn_scale_from_m(to_device(m, "f32"), n)
    dm = cottn.cottn_scale_backward(to_device(m, "f32"), n, to_device(ds, "f32"))
    torch.cuda.synchronize()
    s_ref = oracle.scale_from_m(m, n)
    dm_ref = oracle.scale_backward(m, n, ds)
    # element-wise here: every value is a smooth positive function, no cancellation
    np.testing.assert_allclose(to_host(s), s_ref, rtol=1e-5)
    np.testing.assert_allclose(to_host(dm), dm_ref, rtol=1e-4, atol=1e-7 * np.abs(dm_ref).max())


@pytest.mark.parametrize("dtype,N,d", [("bf16", 300, 64), ("f32", 100, 32)])
def test_chain_m_to_dm(cottn, oracle, dtype, N, d):
    """m -> s -> causal attention -> ds -> dm, every step in the library, against the oracle chain."""
    import torch
    from paper_2409_18747_amd import workloads
    B, H = 2, 4
    x = workloads.draw(B, H, N, d, dtype, 77)
    m = np.array([0.5, -1.0, 0.0, 2.0], dtype=np.float32)
    Q, K, V, dO = (to_device(x[k], dtype) for k in ("Q", "K", "V", "dO"))
    md = to_device(m, "f32")
    s = cottn.cottn_scale_from_m(md, N)
    O = cottn.cottn_fwd_causal(Q, K, V, s)
    dQ, dK, dV, ds = cottn.cottn_bwd_causal(Q, K, V, s, dO)
    dm = cottn.cottn_scale_backward(md, N, ds)
    torch.cuda.synchronize()
    s_ref = oracle.scale_from_m(m, N)
    O_ref = oracle.fwd_quadratic(x["Q"], x["K"], x["V"], s_ref)
    g_ref = oracle.bwd_quadratic(x["Q"], x["K"], x["V"], s_ref, x["dO"])
    dm_ref = oracle.scale_backward(m, N, g_ref[3])
    assert rel_err(to_host(O), O_ref) <= TOL[dtype]
    assert rel_err(to_host(dQ), g_ref[0]) <= TOL[dtype]
    assert rel_err(to_host(dm), dm_ref) <= TOL[dtype]
