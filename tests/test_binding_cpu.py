"""Host-only checks of the Python binding: it refuses tensors whose shape, dtype, length or
device do not match what the kernels will assume from Q, before calling the library (the
kernels index every buffer blindly, so a mismatch would be an out-of-bounds access on the GPU).
Every call here raises on the host; nothing is launched."""
import pytest
import torch


@pytest.fixture(scope="module")
def cottn():
    import paper_2409_18747_amd.binding as b
    return b


def rows(B=1, H=2, N=8, d=64, dtype=torch.bfloat16):
    return torch.zeros(B, H, N, d, dtype=dtype)


def test_row_tensors_must_match_q(cottn):
    Q, s = rows(), torch.ones(2)
    with pytest.raises(ValueError, match="K must match Q"):
        cottn.cottn_fwd_causal(Q, rows(N=4), Q, s)                      # shorter K
    with pytest.raises(ValueError, match="V must match Q"):
        cottn.cottn_fwd_causal(Q, Q, rows(dtype=torch.float16), s)      # other dtype
    with pytest.raises(ValueError, match="O must match Q"):
        cottn.cottn_fwd_bidir(Q, Q, Q, s, O=rows(d=32))
    with pytest.raises(ValueError, match="dO must match Q"):
        cottn.cottn_bwd_causal(Q, Q, Q, s, rows(H=1))
    with pytest.raises(ValueError, match="dK must match Q"):
        cottn.cottn_bwd_bidir(Q, Q, Q, s, Q, dK=rows(B=2))
    with pytest.raises(ValueError, match=r"Q must be \[B, H, N, d\]"):
        cottn.cottn_fwd_causal(Q[0], Q[0], Q[0], s)
    with pytest.raises(TypeError, match="float32, bfloat16 or float16"):
        cottn.cottn_fwd_causal(rows(dtype=torch.float64), Q, Q, s)


def test_scale_state_and_lengths_are_checked(cottn):
    Q = rows()
    with pytest.raises(ValueError, match="s must be float32 with 2 elements"):
        cottn.cottn_fwd_causal(Q, Q, Q, torch.ones(3))
    with pytest.raises(ValueError, match="s must be float32"):
        cottn.cottn_fwd_causal(Q, Q, Q, torch.ones(2, dtype=torch.float64))
    with pytest.raises(ValueError, match="state must be float32 with 8192 elements"):
        cottn.cottn_fwd_causal(Q, Q, Q, torch.ones(2), state=torch.zeros(1, 2, 64, 32))
    with pytest.raises(ValueError, match="ds must be float32 with 2 elements"):
        cottn.cottn_bwd_causal(Q, Q, Q, torch.ones(2), Q, ds=torch.zeros(1))
    # padded batches: s and ds are per (batch, head), lengths int32 [B]
    with pytest.raises(TypeError, match="seq_len must be an int32 tensor of B = 1"):
        cottn.cottn_fwd_causal_varlen(Q, Q, Q, torch.ones(1, 2), torch.tensor([8]))      # int64
    with pytest.raises(TypeError, match="seq_len must be an int32 tensor of B = 1"):
        cottn.cottn_fwd_bidir_varlen(Q, Q, Q, torch.ones(1, 2), torch.tensor([8, 8], dtype=torch.int32))
    with pytest.raises(ValueError, match="s must be float32 with 2 elements"):
        cottn.cottn_bwd_causal_varlen(Q, Q, Q, torch.ones(2, 2), torch.tensor([8], dtype=torch.int32), Q)
    q = torch.zeros(1, 2, 64, dtype=torch.bfloat16)
    with pytest.raises(ValueError, match="k must match q"):
        cottn.cottn_step(q, q[:, :1], q, torch.ones(2), torch.zeros(1, 2, 64, 64))
    with pytest.raises(ValueError, match="state must be float32 with 8192 elements"):
        cottn.cottn_step(q, q, q, torch.ones(2), torch.zeros(1, 2, 64, 64, dtype=torch.float64))


def test_host_tensors_are_refused(cottn):
    """Everything matches but the memory is the host's: refused, not handed to a kernel."""
    Q = rows()
    with pytest.raises(ValueError, match="must live on the GPU"):
        cottn.cottn_fwd_causal(Q, Q, Q, torch.ones(2))
    q = torch.zeros(1, 2, 64, dtype=torch.bfloat16)
    with pytest.raises(ValueError, match="must live on the GPU"):
        cottn.cottn_step(q, q, q, torch.ones(2), torch.zeros(1, 2, 64, 64))
