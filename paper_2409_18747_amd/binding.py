"""ctypes binding of libcottn.so: the same names as the C ABI (include/cottn.h), taking torch
tensors.  Argument marshalling only — every step of the computation runs in the HIP kernels.
PyTorch supplies device memory and the stream handle, nothing else.

The library must have been built (``python -m paper_2409_18747_amd.build``); there is no
fallback: a missing library raises at first use.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
library_path = os.path.join(_HERE, "libcottn.so")

COTTN_F32, COTTN_BF16, COTTN_F16 = 0, 1, 2
OP_FWD_CAUSAL, OP_BWD_CAUSAL, OP_FWD_BIDIR, OP_BWD_BIDIR, OP_STEP = range(5)


class CottnError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: status %d (%s)" % (where, status, cottn_status_string(status)))


def _load():
    if not os.path.exists(library_path):
        raise ImportError(
            "libcottn.so is not built: run `python -m paper_2409_18747_amd.build` "
            "(there is no CPU or PyTorch fallback)")
    lib = ctypes.CDLL(library_path)
    vp, fp, i, f, sz = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    lib.cottn_workspace_bytes.restype = sz
    lib.cottn_workspace_bytes.argtypes = [i] * 7
    lib.cottn_segments.restype = i
    lib.cottn_segments.argtypes = [i] * 7
    lib.cottn_tune_segments.restype = None
    lib.cottn_tune_segments.argtypes = [i]
    lib.cottn_status_string.restype = ctypes.c_char_p
    lib.cottn_status_string.argtypes = [i]
    lib.cottn_fwd_causal.restype = i
    lib.cottn_fwd_causal.argtypes = [vp, vp, vp, fp, vp, fp, vp, sz, i, i, i, i, i, i, f, vp]
    lib.cottn_fwd_causal_static.restype = i
    lib.cottn_fwd_causal_static.argtypes = [vp, vp, vp, fp, vp, fp, i, i, i, i, i, i, f, vp]
    lib.cottn_fwd_causal_from_state.restype = i
    lib.cottn_fwd_causal_from_state.argtypes = [vp, vp, vp, fp, fp, vp, fp, vp, sz, i, i, i, i, i, i, f,
                                                vp]
    lib.cottn_bwd_causal.restype = i
    lib.cottn_bwd_causal.argtypes = [vp, vp, vp, fp, vp, vp, vp, vp, fp, vp, sz, vp, sz, i, i, i, i, i, i,
                                     f, vp]
    lib.cottn_bwd_causal_from_state.restype = i
    lib.cottn_bwd_causal_from_state.argtypes = [vp, vp, vp, fp, vp, fp, fp, vp, vp, vp, fp, fp, vp, sz,
                                                vp, sz, i, i, i, i, i, i, f, vp]
    lib.cottn_fwd_bidir.restype = i
    lib.cottn_fwd_bidir.argtypes = [vp, vp, vp, fp, vp, fp, vp, sz, i, i, i, i, i, f, vp]
    lib.cottn_bwd_bidir.restype = i
    lib.cottn_bwd_bidir.argtypes = [vp, vp, vp, fp, vp, vp, vp, vp, fp, vp, sz, vp, sz, i, i, i, i, i, f,
                                    vp]
    ip = ctypes.c_void_p
    lib.cottn_fwd_causal_varlen.restype = i
    lib.cottn_fwd_causal_varlen.argtypes = [vp, vp, vp, fp, ip, vp, fp, vp, sz, i, i, i, i, i, i, f, vp]
    lib.cottn_bwd_causal_varlen.restype = i
    lib.cottn_bwd_causal_varlen.argtypes = [vp, vp, vp, fp, ip, vp, vp, vp, vp, fp, vp, sz, vp, sz, i, i,
                                            i, i, i, i, f, vp]
    lib.cottn_fwd_bidir_varlen.restype = i
    lib.cottn_fwd_bidir_varlen.argtypes = [vp, vp, vp, fp, ip, vp, fp, vp, sz, i, i, i, i, i, f, vp]
    lib.cottn_bwd_bidir_varlen.restype = i
    lib.cottn_bwd_bidir_varlen.argtypes = [vp, vp, vp, fp, ip, vp, vp, vp, vp, fp, vp, sz, vp, sz, i, i,
                                           i, i, i, f, vp]
    lib.cottn_scale_from_m_varlen.restype = i
    lib.cottn_scale_from_m_varlen.argtypes = [fp, ip, fp, i, i, vp]
    lib.cottn_scale_backward_varlen.restype = i
    lib.cottn_scale_backward_varlen.argtypes = [fp, ip, fp, fp, i, i, vp]
    lib.cottn_step.restype = i
    lib.cottn_step.argtypes = [vp, vp, vp, fp, fp, vp, i, i, i, i, f, vp]
    lib.cottn_workspace_bytes_dkdv.restype = sz
    lib.cottn_workspace_bytes_dkdv.argtypes = [i] * 8
    lib.cottn_segments_dkdv.restype = i
    lib.cottn_segments_dkdv.argtypes = [i] * 8
    lib.cottn_fwd_causal_dkdv.restype = i
    lib.cottn_fwd_causal_dkdv.argtypes = [vp, vp, vp, fp, vp, fp, vp, sz, i, i, i, i, i, i, i, f, vp]
    lib.cottn_bwd_causal_dkdv.restype = i
    lib.cottn_bwd_causal_dkdv.argtypes = [vp, vp, vp, fp, vp, vp, vp, vp, fp, vp, sz, vp, sz, i, i, i, i,
                                          i, i, i, f, vp]
    lib.cottn_fwd_bidir_dkdv.restype = i
    lib.cottn_fwd_bidir_dkdv.argtypes = [vp, vp, vp, fp, vp, fp, vp, sz, i, i, i, i, i, i, f, vp]
    lib.cottn_bwd_bidir_dkdv.restype = i
    lib.cottn_bwd_bidir_dkdv.argtypes = [vp, vp, vp, fp, vp, vp, vp, vp, fp, vp, sz, vp, sz, i, i, i, i,
                                         i, i, f, vp]
    lib.cottn_step_dkdv.restype = i
    lib.cottn_step_dkdv.argtypes = [vp, vp, vp, fp, fp, vp, i, i, i, i, i, f, vp]
    lib.cottn_scale_from_m.restype = i
    lib.cottn_scale_from_m.argtypes = [fp, fp, i, f, vp]
    lib.cottn_scale_backward.restype = i
    lib.cottn_scale_backward.argtypes = [fp, fp, fp, i, f, vp]
    lib.cottn_profile_start.restype = i
    lib.cottn_profile_stop.restype = i
    lib.cottn_profile_count.restype = i
    lib.cottn_profile_name.restype = ctypes.c_char_p
    lib.cottn_profile_name.argtypes = [i]
    lib.cottn_profile_launches.restype = ctypes.c_long
    lib.cottn_profile_launches.argtypes = [i]
    lib.cottn_profile_ms.restype = ctypes.c_double
    lib.cottn_profile_ms.argtypes = [i]
    return lib


lib = _load()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return COTTN_F32
    if t.dtype == torch.bfloat16:
        return COTTN_BF16
    if t.dtype == torch.float16:
        return COTTN_F16
    raise TypeError("tensors must be float32, bfloat16 or float16, got %s" % t.dtype)


def _ptr(t):
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensors must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check(status, where):
    if status != 0:
        raise CottnError(status, where)


def _rows_like(Q, **tensors):
    """Q is a device tensor [B, H, N, d] (_dims checked the rank); every other row tensor given (None = absent) has
    its shape, dtype and device.  The kernels take all of that from Q alone, so a mismatch would
    be read or written out of bounds on the device: refuse it here."""
    for name, t in tensors.items():
        if t is None:
            continue
        if tuple(t.shape) != tuple(Q.shape) or t.dtype != Q.dtype or t.device != Q.device:
            raise ValueError("%s must match Q (%s %s on %s), got %s %s on %s" % (
                name, tuple(Q.shape), Q.dtype, Q.device, tuple(t.shape), t.dtype, t.device))


def _tokens_like(q, **tensors):
    for name, t in tensors.items():
        if tuple(t.shape) != tuple(q.shape) or t.dtype != q.dtype or t.device != q.device:
            raise ValueError("%s must match q (%s %s on %s), got %s %s on %s" % (
                name, tuple(q.shape), q.dtype, q.device, tuple(t.shape), t.dtype, t.device))


def _on_gpu(t):
    if not t.is_cuda:
        raise ValueError("tensors must live on the GPU, got %s" % t.device)


def _f32(name, t, numel, device, optional=False):
    """t is a float32 tensor of `numel` elements on `device` (the kernels index it blindly)."""
    if t is None:
        if optional:
            return
        raise ValueError("%s is required" % name)
    if t.dtype != torch.float32 or t.numel() != numel or t.device != device:
        raise ValueError("%s must be float32 with %d elements on %s, got %s with %d on %s" % (
            name, numel, device, t.dtype, t.numel(), t.device))


def _check_lengths(seq_len, B, device):
    if seq_len.dtype != torch.int32 or seq_len.numel() != B or seq_len.device != device:
        raise TypeError("seq_len must be an int32 tensor of B = %d elements on %s" % (B, device))


def cottn_status_string(status: int) -> str:
    return lib.cottn_status_string(int(status)).decode()


def cottn_workspace_bytes(op, B, H, N, d, chunk=0, dtype=COTTN_BF16) -> int:
    n = lib.cottn_workspace_bytes(op, B, H, N, d, chunk, dtype)
    if n == ctypes.c_size_t(-1).value:
        raise CottnError(2, "cottn_workspace_bytes")
    return n


def cottn_segments(op, B, H, N, d, chunk=0, dtype=COTTN_BF16) -> int:
    return lib.cottn_segments(op, B, H, N, d, chunk, dtype)


def cottn_tune_segments(segments: int) -> None:
    lib.cottn_tune_segments(int(segments))


def _workspace(op, B, H, N, d, chunk, dtype, device, workspace, stream=None):
    need = cottn_workspace_bytes(op, B, H, N, d, chunk, dtype)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=device)
        # a temporary is dropped when the call returns, while the kernels may still be queued:
        # tell the allocator which stream uses it, so the memory is not handed out before they ran
        if stream is not None:
            workspace.record_stream(stream)
    elif workspace is not None and (not workspace.is_cuda or workspace.device != device):
        raise ValueError("workspace must live on %s" % device)
    have = workspace.numel() * workspace.element_size() if workspace is not None else 0
    return workspace, have


def _bytes(t, device):
    if t is None:
        return 0
    if t.device != device:
        raise ValueError("fwd_workspace must live on %s" % device)
    return t.numel() * t.element_size()


def _dims(Q):
    if Q.dim() != 4:
        raise ValueError("Q must be [B, H, N, d], got shape %s" % (tuple(Q.shape),))
    B, H, N, d = Q.shape
    return B, H, N, d, _dtype_code(Q)


def _grads(Q, dQ, dK, dV, ds, ds_shape):
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(Q) if dK is None else dK
    dV = torch.empty_like(Q) if dV is None else dV
    ds = torch.empty(ds_shape, dtype=torch.float32, device=Q.device) if ds is None else ds
    return dQ, dK, dV, ds


def cottn_fwd_causal(Q, K, V, s, O=None, state=None, workspace=None, chunk=0, eps=1e-6,
                     stream=None):
    """O = s_h (Qhat Khat^T (.) M) V; returns O (allocated if not given).  `state`, if given,
    receives sum_j khat_j^T v_j as float32 [B, H, d, d]."""
    B, H, N, d, dt = _dims(Q)
    if O is None:
        O = torch.empty_like(Q)
    _rows_like(Q, K=K, V=V, O=O)
    _f32("s", s, H, Q.device)
    _f32("state", state, B * H * d * d, Q.device, optional=True)
    _on_gpu(Q)
    workspace, have = _workspace(OP_FWD_CAUSAL, B, H, N, d, chunk, dt, Q.device, workspace, stream)
    st = lib.cottn_fwd_causal(_ptr(Q), _ptr(K), _ptr(V), _ptr(s), _ptr(O), _ptr(state),
                              _ptr(workspace), have, B, H, N, d, chunk, dt, eps, _stream(stream))
    _check(st, "cottn_fwd_causal")
    return O


STATIC_WORKSPACE_BYTES = 16 << 20  # COTTN_STATIC_WORKSPACE_BYTES of include/cottn.h


def cottn_fwd_causal_static(Q, K, V, s, O, state=None, chunk=0, eps=1e-6, stream=None):
    """cottn_fwd_causal without a workspace argument, for callers that cannot allocate: the
    segment states live in an array inside the library.  O must be given (nothing is allocated
    here either); returns O."""
    B, H, N, d, dt = _dims(Q)
    _rows_like(Q, K=K, V=V, O=O)
    _f32("s", s, H, Q.device)
    _f32("state", state, B * H * d * d, Q.device, optional=True)
    _on_gpu(Q)
    st = lib.cottn_fwd_causal_static(_ptr(Q), _ptr(K), _ptr(V), _ptr(s), _ptr(O), _ptr(state), B, H,
                                     N, d, chunk, dt, eps, _stream(stream))
    _check(st, "cottn_fwd_causal_static")
    return O


def cottn_fwd_causal_from_state(Q, K, V, s, state_in, O=None, state=None, workspace=None, chunk=0,
                                eps=1e-6, stream=None):
    """cottn_fwd_causal for a piece of a longer sequence: starts from `state_in` (float32
    [B, H, d, d]) and leaves the state after the piece in `state` (a different tensor)."""
    B, H, N, d, dt = _dims(Q)
    if O is None:
        O = torch.empty_like(Q)
    _rows_like(Q, K=K, V=V, O=O)
    _f32("s", s, H, Q.device)
    _f32("state_in", state_in, B * H * d * d, Q.device)
    _f32("state", state, B * H * d * d, Q.device, optional=True)
    _on_gpu(Q)
    workspace, have = _workspace(OP_FWD_CAUSAL, B, H, N, d, chunk, dt, Q.device, workspace, stream)
    st = lib.cottn_fwd_causal_from_state(_ptr(Q), _ptr(K), _ptr(V), _ptr(s), _ptr(state_in), _ptr(O),
                                         _ptr(state), _ptr(workspace), have, B, H, N, d, chunk, dt,
                                         eps, _stream(stream))
    _check(st, "cottn_fwd_causal_from_state")
    return O


def cottn_bwd_causal(Q, K, V, s, dO, dQ=None, dK=None, dV=None, ds=None, workspace=None, chunk=0,
                     eps=1e-6, stream=None, fwd_workspace=None):
    """Gradients of cottn_fwd_causal wrt raw Q, K, V and s; returns (dQ, dK, dV, ds).

    fwd_workspace: the workspace tensor the matching cottn_fwd_causal call used (untouched
    since), or None; see include/cottn.h."""
    B, H, N, d, dt = _dims(Q)
    dQ, dK, dV, ds = _grads(Q, dQ, dK, dV, ds, (H,))
    _rows_like(Q, K=K, V=V, dO=dO, dQ=dQ, dK=dK, dV=dV)
    _f32("s", s, H, Q.device)
    _f32("ds", ds, H, Q.device)
    _on_gpu(Q)
    workspace, have = _workspace(OP_BWD_CAUSAL, B, H, N, d, chunk, dt, Q.device, workspace, stream)
    st = lib.cottn_bwd_causal(_ptr(Q), _ptr(K), _ptr(V), _ptr(s), _ptr(dO), _ptr(dQ), _ptr(dK),
                              _ptr(dV), _ptr(ds), _ptr(fwd_workspace), _bytes(fwd_workspace, Q.device),
                              _ptr(workspace), have, B, H, N, d, chunk, dt, eps, _stream(stream))
    _check(st, "cottn_bwd_causal")
    return dQ, dK, dV, ds


def cottn_bwd_causal_from_state(Q, K, V, s, dO, state_in=None, rev_state_in=None, dQ=None, dK=None,
                                dV=None, ds=None, rev_state_out=None, workspace=None, chunk=0,
                                eps=1e-6, stream=None, fwd_workspace=None):
    """cottn_bwd_causal for one piece of a sequence processed in pieces: state_in is the
    forward-time state before the piece, rev_state_in the reverse-time state after it;
    returns (dQ, dK, dV, ds) and fills rev_state_out (float32 [B, H, d, d]) when given."""
    B, H, N, d, dt = _dims(Q)
    dQ, dK, dV, ds = _grads(Q, dQ, dK, dV, ds, (H,))
    _rows_like(Q, K=K, V=V, dO=dO, dQ=dQ, dK=dK, dV=dV)
    _f32("s", s, H, Q.device)
    _f32("ds", ds, H, Q.device)
    for name, t in (("state_in", state_in), ("rev_state_in", rev_state_in),
                    ("rev_state_out", rev_state_out)):
        _f32(name, t, B * H * d * d, Q.device, optional=True)
    _on_gpu(Q)
    workspace, have = _workspace(OP_BWD_CAUSAL, B, H, N, d, chunk, dt, Q.device, workspace, stream)
    st = lib.cottn_bwd_causal_from_state(_ptr(Q), _ptr(K), _ptr(V), _ptr(s), _ptr(dO), _ptr(state_in),
                                         _ptr(rev_state_in), _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(ds),
                                         _ptr(rev_state_out), _ptr(fwd_workspace),
                                         _bytes(fwd_workspace, Q.device), _ptr(workspace), have, B, H,
                                         N, d, chunk, dt, eps, _stream(stream))
    _check(st, "cottn_bwd_causal_from_state")
    return dQ, dK, dV, ds


def cottn_fwd_bidir(Q, K, V, s, O=None, state=None, workspace=None, eps=1e-6, stream=None):
    """O = s_h Qhat (Khat^T V); returns O."""
    B, H, N, d, dt = _dims(Q)
    if O is None:
        O = torch.empty_like(Q)
    _rows_like(Q, K=K, V=V, O=O)
    _f32("s", s, H, Q.device)
    _f32("state", state, B * H * d * d, Q.device, optional=True)
    _on_gpu(Q)
    workspace, have = _workspace(OP_FWD_BIDIR, B, H, N, d, 0, dt, Q.device, workspace, stream)
    st = lib.cottn_fwd_bidir(_ptr(Q), _ptr(K), _ptr(V), _ptr(s), _ptr(O), _ptr(state),
                             _ptr(workspace), have, B, H, N, d, dt, eps, _stream(stream))
    _check(st, "cottn_fwd_bidir")
    return O


def cottn_bwd_bidir(Q, K, V, s, dO, dQ=None, dK=None, dV=None, ds=None, workspace=None, eps=1e-6,
                    stream=None, fwd_workspace=None):
    """Gradients of cottn_fwd_bidir; returns (dQ, dK, dV, ds).  fwd_workspace: the workspace
    tensor of the matching cottn_fwd_bidir call (untouched since), or None."""
    B, H, N, d, dt = _dims(Q)
    dQ, dK, dV, ds = _grads(Q, dQ, dK, dV, ds, (H,))
    _rows_like(Q, K=K, V=V, dO=dO, dQ=dQ, dK=dK, dV=dV)
    _f32("s", s, H, Q.device)
    _f32("ds", ds, H, Q.device)
    _on_gpu(Q)
    workspace, have = _workspace(OP_BWD_BIDIR, B, H, N, d, 0, dt, Q.device, workspace, stream)
    st = lib.cottn_bwd_bidir(_ptr(Q), _ptr(K), _ptr(V), _ptr(s), _ptr(dO), _ptr(dQ), _ptr(dK),
                             _ptr(dV), _ptr(ds), _ptr(fwd_workspace), _bytes(fwd_workspace, Q.device),
                             _ptr(workspace), have, B, H, N, d, dt, eps, _stream(stream))
    _check(st, "cottn_bwd_bidir")
    return dQ, dK, dV, ds


def cottn_fwd_causal_varlen(Q, K, V, s, seq_len, O=None, state=None, workspace=None, chunk=0,
                            eps=1e-6, stream=None):
    """cottn_fwd_causal for a padded batch: seq_len int32 [B], s float32 [B, H]."""
    B, H, N, d, dt = _dims(Q)
    if O is None:
        O = torch.empty_like(Q)
    _rows_like(Q, K=K, V=V, O=O)
    _check_lengths(seq_len, B, Q.device)
    _f32("s", s, B * H, Q.device)
    _f32("state", state, B * H * d * d, Q.device, optional=True)
    _on_gpu(Q)
    workspace, have = _workspace(OP_FWD_CAUSAL, B, H, N, d, chunk, dt, Q.device, workspace, stream)
    st = lib.cottn_fwd_causal_varlen(_ptr(Q), _ptr(K), _ptr(V), _ptr(s), _ptr(seq_len), _ptr(O),
                                     _ptr(state), _ptr(workspace), have, B, H, N, d, chunk, dt, eps,
                                     _stream(stream))
    _check(st, "cottn_fwd_causal_varlen")
    return O


def cottn_bwd_causal_varlen(Q, K, V, s, seq_len, dO, dQ=None, dK=None, dV=None, ds=None,
                            workspace=None, chunk=0, eps=1e-6, stream=None, fwd_workspace=None):
    """cottn_bwd_causal for a padded batch; returns (dQ, dK, dV, ds) with ds float32 [B, H]."""
    B, H, N, d, dt = _dims(Q)
    dQ, dK, dV, ds = _grads(Q, dQ, dK, dV, ds, (B, H))
    _rows_like(Q, K=K, V=V, dO=dO, dQ=dQ, dK=dK, dV=dV)
    _check_lengths(seq_len, B, Q.device)
    _f32("s", s, B * H, Q.device)
    _f32("ds", ds, B * H, Q.device)
    _on_gpu(Q)
    workspace, have = _workspace(OP_BWD_CAUSAL, B, H, N, d, chunk, dt, Q.device, workspace, stream)
    st = lib.cottn_bwd_causal_varlen(_ptr(Q), _ptr(K), _ptr(V), _ptr(s), _ptr(seq_len), _ptr(dO),
                                     _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(ds), _ptr(fwd_workspace),
                                     _bytes(fwd_workspace, Q.device), _ptr(workspace), have, B, H, N,
                                     d, chunk, dt, eps, _stream(stream))
    _check(st, "cottn_bwd_causal_varlen")
    return dQ, dK, dV, ds


def cottn_fwd_bidir_varlen(Q, K, V, s, seq_len, O=None, state=None, workspace=None, eps=1e-6,
                           stream=None):
    """cottn_fwd_bidir for a padded batch: seq_len int32 [B], s float32 [B, H]."""
    B, H, N, d, dt = _dims(Q)
    if O is None:
        O = torch.empty_like(Q)
    _rows_like(Q, K=K, V=V, O=O)
    _check_lengths(seq_len, B, Q.device)
    _f32("s", s, B * H, Q.device)
    _f32("state", state, B * H * d * d, Q.device, optional=True)
    _on_gpu(Q)
    workspace, have = _workspace(OP_FWD_BIDIR, B, H, N, d, 0, dt, Q.device, workspace, stream)
    st = lib.cottn_fwd_bidir_varlen(_ptr(Q), _ptr(K), _ptr(V), _ptr(s), _ptr(seq_len), _ptr(O),
                                    _ptr(state), _ptr(workspace), have, B, H, N, d, dt, eps,
                                    _stream(stream))
    _check(st, "cottn_fwd_bidir_varlen")
    return O


def cottn_bwd_bidir_varlen(Q, K, V, s, seq_len, dO, dQ=None, dK=None, dV=None, ds=None,
                           workspace=None, eps=1e-6, stream=None, fwd_workspace=None):
    """cottn_bwd_bidir for a padded batch; returns (dQ, dK, dV, ds) with ds float32 [B, H]."""
    B, H, N, d, dt = _dims(Q)
    dQ, dK, dV, ds = _grads(Q, dQ, dK, dV, ds, (B, H))
    _rows_like(Q, K=K, V=V, dO=dO, dQ=dQ, dK=dK, dV=dV)
    _check_lengths(seq_len, B, Q.device)
    _f32("s", s, B * H, Q.device)
    _f32("ds", ds, B * H, Q.device)
    _on_gpu(Q)
    workspace, have = _workspace(OP_BWD_BIDIR, B, H, N, d, 0, dt, Q.device, workspace, stream)
    st = lib.cottn_bwd_bidir_varlen(_ptr(Q), _ptr(K), _ptr(V), _ptr(s), _ptr(seq_len), _ptr(dO),
                                    _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(ds), _ptr(fwd_workspace),
                                    _bytes(fwd_workspace, Q.device), _ptr(workspace), have, B, H, N,
                                    d, dt, eps, _stream(stream))
    _check(st, "cottn_bwd_bidir_varlen")
    return dQ, dK, dV, ds


def cottn_scale_from_m_varlen(m, seq_len, s=None, stream=None):
    """s[b, h] = seq_len[b]^(-sigmoid(m[h]))."""
    B, H = seq_len.numel(), m.numel()
    _f32("m", m, H, m.device)
    _check_lengths(seq_len, B, m.device)
    s = torch.empty(B, H, dtype=torch.float32, device=m.device) if s is None else s
    _f32("s", s, B * H, m.device)
    _on_gpu(m)
    _check(lib.cottn_scale_from_m_varlen(_ptr(m), _ptr(seq_len), _ptr(s), B, H, _stream(stream)),
           "cottn_scale_from_m_varlen")
    return s


def cottn_scale_backward_varlen(m, seq_len, ds, dm=None, stream=None):
    """dm[h] = sum_b ds[b, h] * d s[b, h] / d m[h]."""
    B, H = seq_len.numel(), m.numel()
    _f32("m", m, H, m.device)
    _check_lengths(seq_len, B, m.device)
    _f32("ds", ds, B * H, m.device)
    dm = torch.empty(H, dtype=torch.float32, device=m.device) if dm is None else dm
    _f32("dm", dm, H, m.device)
    _on_gpu(m)
    _check(lib.cottn_scale_backward_varlen(_ptr(m), _ptr(seq_len), _ptr(ds), _ptr(dm), B, H,
                                           _stream(stream)), "cottn_scale_backward_varlen")
    return dm


def cottn_step(q, k, v, s, state, o=None, eps=1e-6, stream=None):
    """state += khat^T v (in place); returns o = s_h qhat state.  q, k, v are [B, H, d]."""
    if q.dim() != 3:
        raise ValueError("q must be [B, H, d], got shape %s" % (tuple(q.shape),))
    B, H, d = q.shape
    dt = _dtype_code(q)
    if o is None:
        o = torch.empty_like(q)
    _tokens_like(q, k=k, v=v, o=o)
    _f32("s", s, H, q.device)
    _f32("state", state, B * H * d * d, q.device)
    _on_gpu(q)
    st = lib.cottn_step(_ptr(q), _ptr(k), _ptr(v), _ptr(s), _ptr(state), _ptr(o), B, H, d, dt,
                        eps, _stream(stream))
    _check(st, "cottn_step")
    return o


def cottn_scale_from_m(m, n, s=None, stream=None):
    """s[h] = n^(-sigmoid(m[h])): the stabiliser of Sec. 3.3 as the factor the attention calls take."""
    H = m.numel()
    _f32("m", m, H, m.device)
    s = torch.empty(H, dtype=torch.float32, device=m.device) if s is None else s
    _f32("s", s, H, m.device)
    _on_gpu(m)
    _check(lib.cottn_scale_from_m(_ptr(m), _ptr(s), H, float(n), _stream(stream)), "cottn_scale_from_m")
    return s


def cottn_scale_backward(m, n, ds, dm=None, stream=None):
    """dm[h] = ds[h] * ds_h/dm_h for s_h = n^(-sigmoid(m_h))."""
    H = m.numel()
    _f32("m", m, H, m.device)
    _f32("ds", ds, H, m.device)
    dm = torch.empty(H, dtype=torch.float32, device=m.device) if dm is None else dm
    _f32("dm", dm, H, m.device)
    _on_gpu(m)
    _check(lib.cottn_scale_backward(_ptr(m), _ptr(ds), _ptr(dm), H, float(n), _stream(stream)),
           "cottn_scale_backward")
    return dm


# ---- d_key != d_value: Q, K (dQ, dK) are [B, H, N, dk]; V, dO (O, dV) are [B, H, N, dv] ----------

def cottn_workspace_bytes_dkdv(op, B, H, N, dk, dv, chunk=0, dtype=COTTN_BF16) -> int:
    n = lib.cottn_workspace_bytes_dkdv(op, B, H, N, dk, dv, chunk, dtype)
    if n == ctypes.c_size_t(-1).value:
        raise CottnError(2, "cottn_workspace_bytes_dkdv")
    return n


def cottn_segments_dkdv(op, B, H, N, dk, dv, chunk=0, dtype=COTTN_BF16) -> int:
    return lib.cottn_segments_dkdv(op, B, H, N, dk, dv, chunk, dtype)


def _dims_dkdv(Q, V):
    """B, H, N, dk (of Q), dv (of V), dtype code; V must agree with Q in everything but width."""
    B, H, N, dk, dt = _dims(Q)
    if V.dim() != 4 or tuple(V.shape[:3]) != (B, H, N) or V.dtype != Q.dtype or V.device != Q.device:
        raise ValueError("V must be [%d, %d, %d, d_value] %s on %s, got %s %s on %s" % (
            B, H, N, Q.dtype, Q.device, tuple(V.shape), V.dtype, V.device))
    return B, H, N, dk, V.shape[-1], dt


def _workspace_dkdv(op, B, H, N, dk, dv, chunk, dtype, device, workspace, stream):
    need = cottn_workspace_bytes_dkdv(op, B, H, N, dk, dv, chunk, dtype)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=device)
        if stream is not None:
            workspace.record_stream(stream)
    elif workspace is not None and (not workspace.is_cuda or workspace.device != device):
        raise ValueError("workspace must live on %s" % device)
    have = workspace.numel() * workspace.element_size() if workspace is not None else 0
    return workspace, have


def cottn_fwd_causal_dkdv(Q, K, V, s, O=None, state=None, workspace=None, chunk=0, eps=1e-6,
                          stream=None):
    """cottn_fwd_causal with d_key = Q.shape[-1] and d_value = V.shape[-1]; returns O (like V).
    `state`, if given, receives float32 [B, H, d_key, d_value]."""
    B, H, N, dk, dv, dt = _dims_dkdv(Q, V)
    if O is None:
        O = torch.empty_like(V)
    _rows_like(Q, K=K)
    _rows_like(V, O=O)
    _f32("s", s, H, Q.device)
    _f32("state", state, B * H * dk * dv, Q.device, optional=True)
    _on_gpu(Q)
    workspace, have = _workspace_dkdv(OP_FWD_CAUSAL, B, H, N, dk, dv, chunk, dt, Q.device, workspace, stream)
    st = lib.cottn_fwd_causal_dkdv(_ptr(Q), _ptr(K), _ptr(V), _ptr(s), _ptr(O), _ptr(state),
                                   _ptr(workspace), have, B, H, N, dk, dv, chunk, dt, eps,
                                   _stream(stream))
    _check(st, "cottn_fwd_causal_dkdv")
    return O


def _grads_dkdv(Q, V, dQ, dK, dV, ds, H):
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(Q) if dK is None else dK
    dV = torch.empty_like(V) if dV is None else dV
    ds = torch.empty(H, dtype=torch.float32, device=Q.device) if ds is None else ds
    return dQ, dK, dV, ds


def cottn_bwd_causal_dkdv(Q, K, V, s, dO, dQ=None, dK=None, dV=None, ds=None, workspace=None,
                          chunk=0, eps=1e-6, stream=None, fwd_workspace=None):
    """cottn_bwd_causal with d_key = Q.shape[-1] and d_value = V.shape[-1] (dO like V);
    returns (dQ, dK, dV, ds)."""
    B, H, N, dk, dv, dt = _dims_dkdv(Q, V)
    dQ, dK, dV, ds = _grads_dkdv(Q, V, dQ, dK, dV, ds, H)
    _rows_like(Q, K=K, dQ=dQ, dK=dK)
    _rows_like(V, dO=dO, dV=dV)
    _f32("s", s, H, Q.device)
    _f32("ds", ds, H, Q.device)
    _on_gpu(Q)
    workspace, have = _workspace_dkdv(OP_BWD_CAUSAL, B, H, N, dk, dv, chunk, dt, Q.device, workspace, stream)
    st = lib.cottn_bwd_causal_dkdv(_ptr(Q), _ptr(K), _ptr(V), _ptr(s), _ptr(dO), _ptr(dQ), _ptr(dK),
                                   _ptr(dV), _ptr(ds), _ptr(fwd_workspace),
                                   _bytes(fwd_workspace, Q.device), _ptr(workspace), have, B, H, N, dk,
                                   dv, chunk, dt, eps, _stream(stream))
    _check(st, "cottn_bwd_causal_dkdv")
    return dQ, dK, dV, ds


def cottn_fwd_bidir_dkdv(Q, K, V, s, O=None, state=None, workspace=None, eps=1e-6, stream=None):
    """cottn_fwd_bidir with d_key = Q.shape[-1] and d_value = V.shape[-1]; returns O (like V)."""
    B, H, N, dk, dv, dt = _dims_dkdv(Q, V)
    if O is None:
        O = torch.empty_like(V)
    _rows_like(Q, K=K)
    _rows_like(V, O=O)
    _f32("s", s, H, Q.device)
    _f32("state", state, B * H * dk * dv, Q.device, optional=True)
    _on_gpu(Q)
    workspace, have = _workspace_dkdv(OP_FWD_BIDIR, B, H, N, dk, dv, 0, dt, Q.device, workspace, stream)
    st = lib.cottn_fwd_bidir_dkdv(_ptr(Q), _ptr(K), _ptr(V), _ptr(s), _ptr(O), _ptr(state),
                                  _ptr(workspace), have, B, H, N, dk, dv, dt, eps, _stream(stream))
    _check(st, "cottn_fwd_bidir_dkdv")
    return O


def cottn_bwd_bidir_dkdv(Q, K, V, s, dO, dQ=None, dK=None, dV=None, ds=None, workspace=None,
                         eps=1e-6, stream=None, fwd_workspace=None):
    """cottn_bwd_bidir with d_key = Q.shape[-1] and d_value = V.shape[-1]; returns (dQ, dK, dV, ds)."""
    B, H, N, dk, dv, dt = _dims_dkdv(Q, V)
    dQ, dK, dV, ds = _grads_dkdv(Q, V, dQ, dK, dV, ds, H)
    _rows_like(Q, K=K, dQ=dQ, dK=dK)
    _rows_like(V, dO=dO, dV=dV)
    _f32("s", s, H, Q.device)
    _f32("ds", ds, H, Q.device)
    _on_gpu(Q)
    workspace, have = _workspace_dkdv(OP_BWD_BIDIR, B, H, N, dk, dv, 0, dt, Q.device, workspace, stream)
    st = lib.cottn_bwd_bidir_dkdv(_ptr(Q), _ptr(K), _ptr(V), _ptr(s), _ptr(dO), _ptr(dQ), _ptr(dK),
                                  _ptr(dV), _ptr(ds), _ptr(fwd_workspace),
                                  _bytes(fwd_workspace, Q.device), _ptr(workspace), have, B, H, N, dk,
                                  dv, dt, eps, _stream(stream))
    _check(st, "cottn_bwd_bidir_dkdv")
    return dQ, dK, dV, ds


def cottn_step_dkdv(q, k, v, s, state, o=None, eps=1e-6, stream=None):
    """cottn_step with q, k [B, H, d_key] and v [B, H, d_value]; state float32 [B, H, d_key, d_value]
    updated in place; returns o (like v)."""
    if q.dim() != 3 or v.dim() != 3:
        raise ValueError("q and v must be [B, H, d], got shapes %s and %s" % (tuple(q.shape), tuple(v.shape)))
    B, H, dk = q.shape
    dv = v.shape[-1]
    dt = _dtype_code(q)
    if tuple(v.shape[:2]) != (B, H) or v.dtype != q.dtype or v.device != q.device:
        raise ValueError("v must be [%d, %d, d_value] %s on %s" % (B, H, q.dtype, q.device))
    if o is None:
        o = torch.empty_like(v)
    _tokens_like(q, k=k)
    _tokens_like(v, o=o)
    _f32("s", s, H, q.device)
    _f32("state", state, B * H * dk * dv, q.device)
    _on_gpu(q)
    st = lib.cottn_step_dkdv(_ptr(q), _ptr(k), _ptr(v), _ptr(s), _ptr(state), _ptr(o), B, H, dk, dv,
                             dt, eps, _stream(stream))
    _check(st, "cottn_step_dkdv")
    return o


def profile_start():
    _check(lib.cottn_profile_start(), "cottn_profile_start")


def profile_stop():
    """Returns {kernel name: (launches, total ms)} gathered since profile_start()."""
    _check(lib.cottn_profile_stop(), "cottn_profile_stop")
    return {lib.cottn_profile_name(i).decode(): (lib.cottn_profile_launches(i), lib.cottn_profile_ms(i))
            for i in range(lib.cottn_profile_count())}
