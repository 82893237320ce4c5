"""The causal forward that allocates nothing (its workspace is an array inside the library) gives,
through the C ABI, exactly what cottn_fwd_causal gives with a caller's workspace: same kernels,
same values.  Two calls in a row share the library's array, the second on a smaller input."""
import pytest

from helpers import to_device

pytestmark = pytest.mark.gpu


def one_call(cottn, B, H, N, d, dtype, seed, chunk=0, with_state=True):
    import torch
    from paper_2409_18747_amd import workloads
    x = workloads.draw(B, H, N, d, dtype, seed)
    Q, K, V = (to_device(x[k], dtype) for k in ("Q", "K", "V"))
    s = to_device(x["s"], "f32")
    code = {"bf16": cottn.COTTN_BF16, "f16": cottn.COTTN_F16, "f32": cottn.COTTN_F32}[dtype]
    need = cottn.cottn_workspace_bytes(cottn.OP_FWD_CAUSAL, B, H, N, d, chunk, code)
    assert 0 < need <= cottn.STATIC_WORKSPACE_BYTES, need  # the case must use the array
    print("fwd_causal_static %s B%d H%d N%d d%d chunk%d: %d workspace bytes, %d segments" %
          (dtype, B, H, N, d, chunk, need,
           cottn.cottn_segments(cottn.OP_FWD_CAUSAL, B, H, N, d, chunk, code)), flush=True)
    O_ref = torch.full_like(Q, float("nan"))
    S_ref = torch.full((B, H, d, d), float("nan"), dtype=torch.float32, device="cuda")
    cottn.cottn_fwd_causal(Q, K, V, s, O=O_ref, state=S_ref if with_state else None, chunk=chunk)
    O = torch.full_like(Q, float("nan"))
    S = torch.full_like(S_ref, float("nan"))
    out = cottn.cottn_fwd_causal_static(Q, K, V, s, O, state=S if with_state else None, chunk=chunk)
    torch.cuda.synchronize()
    assert out is O
    assert torch.isfinite(O.float()).all()
    assert torch.equal(O, O_ref)
    if with_state:
        assert torch.equal(S, S_ref)


def test_two_calls_in_a_row_second_smaller():
    import paper_2409_18747_amd.binding as cottn
    cottn.cottn_tune_segments(0)
    # few segments (the scan adds the totals up itself), then a smaller input that leaves most
    # of what the first call wrote in the array untouched
    one_call(cottn, 4, 6, 1024, 64, "bf16", seed=71)
    one_call(cottn, 1, 2, 333, 64, "bf16", seed=72)
    # many segments (carried prefixes), then fewer rows of another head dimension and type
    one_call(cottn, 1, 2, 8192, 64, "bf16", seed=73)
    one_call(cottn, 1, 3, 700, 32, "f16", seed=74, with_state=False)
    one_call(cottn, 2, 2, 300, 64, "f32", seed=75)
