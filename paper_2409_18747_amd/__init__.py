"""Cosine attention (Cottention) for MI355X: thin Python binding over the C-ABI library.

The HIP library is loaded on first use of a ``cottn_*`` name, so importing
``paper_2409_18747_amd.workloads`` (pure numpy input generators) does not need it.
"""

_BINDING_NAMES = (
    "cottn_fwd_causal", "cottn_bwd_causal", "cottn_fwd_bidir", "cottn_bwd_bidir", "cottn_step",
    "cottn_workspace_bytes", "cottn_status_string", "cottn_segments", "CottnError", "lib",
    "COTTN_F32", "COTTN_BF16", "OP_FWD_CAUSAL", "OP_BWD_CAUSAL", "OP_FWD_BIDIR", "OP_BWD_BIDIR",
    "OP_STEP", "library_path",
)


def __getattr__(name):
    if name in _BINDING_NAMES:
        from . import binding
        return getattr(binding, name)
    raise AttributeError(name)
