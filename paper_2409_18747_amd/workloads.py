"""Seeded synthetic inputs shaped like the paper's workloads.

This module holds NO attention arithmetic: only the random draws, the rounding of the
draws to the storage dtype, and the table of workload shapes.  It is the one module that
both the tests' CPU checker and the GPU path are fed from, so both consume identical bits.

The paper trains BERT (bidirectional, Sec. 6) and GPT-J (causal, Sec. 6) on text corpora
that are not available here; these workloads keep only the *shapes* of those models'
attention calls (heads, head dimension, sequence length) and draw i.i.d. Gaussian values.

Draw order within one seed: Q, K, V, dO, s.
"""
from dataclasses import dataclass, field

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    N: int
    d: int
    dtype: str          # "f32", "bf16" or "f16": storage type of Q, K, V, O and the gradients
    causal: bool
    backward: bool
    seed: int
    value_scale: float = 1.0
    eps: float = 1e-6
    extra: dict = field(default_factory=dict)


# The five benchmark configurations (B, H, N, d as in [B, H, N, d] tensors).
WORKLOADS = {
    "cfg1_small_causal_fwd_f32": Workload("cfg1_small_causal_fwd_f32", 1, 2, 256, 32, "f32",
                                          True, False, 0),
    "cfg2_gpt_causal_fwdbwd_bf16": Workload("cfg2_gpt_causal_fwdbwd_bf16", 8, 12, 1024, 64,
                                            "bf16", True, True, 1),
    "cfg3_bert_bidir_fwdbwd_bf16": Workload("cfg3_bert_bidir_fwdbwd_bf16", 32, 12, 512, 64,
                                            "bf16", False, True, 2),
    "cfg4_long_causal_fwdbwd_bf16": Workload("cfg4_long_causal_fwdbwd_bf16", 1, 16, 65536, 64,
                                             "bf16", True, True, 3, value_scale=0.5),
    # decode: 256 sequences; N here is the prefill length, extra["steps"] single-token steps
    "cfg5_decode_bf16": Workload("cfg5_decode_bf16", 256, 16, 2048, 128, "bf16", True, False, 4,
                                 extra={"steps": 4096}),
}


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """The uint16 bit patterns of bf16-representable float32 values."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> 16).astype(np.uint16).reshape(x.shape)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return round_to_bf16(x)
    if dtype == "f16":
        # numpy's float16 conversion rounds to nearest even; back to float32 is exact
        return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).astype(np.float32)
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    raise ValueError("dtype must be 'f32', 'bf16' or 'f16'")


def draw(B, H, N, d, dtype="f32", seed=0, value_scale=1.0, with_dO=True, d_value=None):
    """Q, K, V (and dO) ~ value_scale * N(0, 1) of shape [B, H, N, d], s ~ U(0.5, 1.5) of shape [H].
    With d_value, V and dO are [B, H, N, d_value] (the paper's separate head dimension of the
    values, Sec. 2.1).

    Values are float32 arrays already rounded to ``dtype``, so converting them to that
    dtype anywhere is exact.  Returns a dict with keys Q, K, V, dO (optional), s.
    """
    rng = np.random.Generator(np.random.Philox(seed))
    out = {}
    for name in ("Q", "K", "V", "dO"):
        width = d if (d_value is None or name in ("Q", "K")) else d_value
        x = rng.standard_normal((B, H, N, width), dtype=np.float32)
        if value_scale != 1.0:
            x = x * np.float32(value_scale)
        if name == "dO" and not with_dO:
            continue
        out[name] = _store(x, dtype)
    out["s"] = rng.uniform(0.5, 1.5, size=(H,)).astype(np.float32)
    return out


def draw_workload(w: Workload, B=None, N=None):
    """Inputs of a named workload; B and N may be overridden to take a smaller slice of work."""
    return draw(B or w.B, w.H, N or w.N, w.d, w.dtype, w.seed, w.value_scale,
                with_dO=True)


def draw_tokens(B, H, T, d, dtype="bf16", seed=0):
    """q, k, v streams for decode: three [T, B, H, d] arrays (one [B, H, d] slab per step)."""
    rng = np.random.Generator(np.random.Philox(seed))
    return tuple(_store(rng.standard_normal((T, B, H, d), dtype=np.float32), dtype)
                 for _ in range(3))
