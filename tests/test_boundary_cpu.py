"""Host-only checks of the C-ABI boundary: the library loads without a GPU, exports every
symbol the header declares, sizes workspaces consistently and rejects bad arguments before
anything would be enqueued.  No compute call is made."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "cottn.h")
LIB = os.path.join(ROOT, "paper_2409_18747_amd", "libcottn.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        pytest.fail("libcottn.so is not built: run python -m paper_2409_18747_amd.build")
    l = ctypes.CDLL(LIB)
    l.cottn_workspace_bytes.restype = ctypes.c_size_t
    l.cottn_workspace_bytes.argtypes = [ctypes.c_int] * 7
    l.cottn_segments.restype = ctypes.c_int
    l.cottn_segments.argtypes = [ctypes.c_int] * 7
    l.cottn_status_string.restype = ctypes.c_char_p
    vp, i, f, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    l.cottn_fwd_causal.argtypes = [vp, vp, vp, vp, vp, vp, vp, sz, i, i, i, i, i, i, f, vp]
    l.cottn_bwd_causal.argtypes = [vp] * 10 + [sz, vp, sz, i, i, i, i, i, i, f, vp]
    l.cottn_fwd_bidir.argtypes = [vp, vp, vp, vp, vp, vp, vp, sz, i, i, i, i, i, f, vp]
    l.cottn_bwd_bidir.argtypes = [vp] * 10 + [sz, vp, sz, i, i, i, i, i, f, vp]
    l.cottn_step.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, f, vp]
    l.cottn_fwd_causal_from_state.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, sz, i, i, i, i, i, i, f, vp]
    l.cottn_bwd_causal_from_state.argtypes = [vp] * 13 + [sz, vp, sz, i, i, i, i, i, i, f, vp]
    l.cottn_fwd_causal_varlen.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, sz, i, i, i, i, i, i, f, vp]
    l.cottn_bwd_bidir_varlen.argtypes = [vp] * 11 + [sz, vp, sz, i, i, i, i, i, f, vp]
    l.cottn_scale_from_m_varlen.argtypes = [vp, vp, vp, i, i, vp]
    l.cottn_fwd_causal_static.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, f, vp]
    l.cottn_workspace_bytes_dkdv.restype = ctypes.c_size_t
    l.cottn_workspace_bytes_dkdv.argtypes = [ctypes.c_int] * 8
    l.cottn_segments_dkdv.argtypes = [ctypes.c_int] * 8
    l.cottn_fwd_causal_dkdv.argtypes = [vp, vp, vp, vp, vp, vp, vp, sz, i, i, i, i, i, i, i, f, vp]
    l.cottn_bwd_bidir_dkdv.argtypes = [vp] * 10 + [sz, vp, sz, i, i, i, i, i, i, f, vp]
    l.cottn_step_dkdv.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, i, f, vp]
    l.cottn_scale_from_m.argtypes = [vp, vp, i, f, vp]
    l.cottn_scale_backward.argtypes = [vp, vp, vp, i, f, vp]
    yield l
    l.cottn_tune_segments(0)


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cottn_[a-z_]+)\s*\(", text)))


def test_header_declares_the_entry_points():
    names = declared_functions()
    for required in ("cottn_fwd_causal", "cottn_bwd_causal", "cottn_fwd_bidir", "cottn_bwd_bidir",
                     "cottn_step", "cottn_workspace_bytes", "cottn_status_string",
                     "cottn_scale_from_m", "cottn_scale_backward", "cottn_fwd_causal_from_state",
                     "cottn_bwd_causal_from_state",
                     "cottn_fwd_causal_varlen", "cottn_bwd_causal_varlen", "cottn_fwd_bidir_varlen",
                     "cottn_bwd_bidir_varlen", "cottn_scale_from_m_varlen",
                     "cottn_scale_backward_varlen"):
        assert required in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), name


NOSIZE = ctypes.c_size_t(-1).value
F32, BF16 = 0, 1


def test_workspace_sizes(lib):
    lib.cottn_tune_segments(0)
    # decode needs none
    assert lib.cottn_workspace_bytes(4, 256, 16, 1, 128, 0, BF16) == 0
    # one segment: forward needs nothing, backward only the ds partial sums
    lib.cottn_tune_segments(1)
    assert lib.cottn_segments(0, 8, 12, 1024, 64, 0, BF16) == 1
    assert lib.cottn_workspace_bytes(0, 8, 12, 1024, 64, 0, BF16) == 0
    assert lib.cottn_workspace_bytes(1, 8, 12, 1024, 64, 0, BF16) == 512  # 96 floats, padded
    # G segments: one fp32 d x d state per (b, h, segment); the backward keeps two arrays
    lib.cottn_tune_segments(4)
    assert lib.cottn_segments(0, 8, 12, 1024, 64, 0, BF16) == 4
    one = 8 * 12 * 4 * 64 * 64 * 4
    assert lib.cottn_workspace_bytes(0, 8, 12, 1024, 64, 0, BF16) == one
    assert lib.cottn_workspace_bytes(1, 8, 12, 1024, 64, 0, BF16) == 2 * one + 1536
    assert lib.cottn_workspace_bytes(2, 8, 12, 1024, 64, 0, BF16) == one
    # never more segments than chunks
    lib.cottn_tune_segments(1000)
    assert lib.cottn_segments(0, 1, 1, 100, 64, 0, BF16) == 2
    assert lib.cottn_segments(0, 1, 1, 100, 64, 0, F32) == 4
    lib.cottn_tune_segments(0)
    # linear in N at a fixed split (the paper's memory claim, Sec. 7): doubling N with the
    # heuristic split never more than doubles the workspace
    a = lib.cottn_workspace_bytes(1, 1, 16, 32768, 64, 0, BF16)
    b = lib.cottn_workspace_bytes(1, 1, 16, 65536, 64, 0, BF16)
    assert b <= 2 * a


def test_heuristic_split_per_operation(lib):
    """The split the library chooses by itself: the causal forward and backward agree (the
    backward takes the forward's states over only then), so do the bidirectional pair, and the
    bidirectional calls, which have no chain of chunks to shorten, are cut finer but never into
    more segments than their kernels add up themselves (four)."""
    lib.cottn_tune_segments(0)
    for B, H, N, d in [(8, 12, 1024, 64), (32, 12, 512, 64), (1, 16, 65536, 64), (2, 3, 333, 32),
                       (8, 12, 1024, 128), (1, 1, 64, 64)]:
        assert lib.cottn_segments(0, B, H, N, d, 0, BF16) == lib.cottn_segments(1, B, H, N, d, 0, BF16)
        assert lib.cottn_segments(2, B, H, N, d, 0, BF16) == lib.cottn_segments(3, B, H, N, d, 0, BF16)
    assert lib.cottn_segments(0, 8, 12, 1024, 64, 0, BF16) == 4     # 384 workgroups
    assert lib.cottn_segments(0, 32, 12, 512, 64, 0, BF16) == 1     # 384 units fill the chip
    assert lib.cottn_segments(2, 32, 12, 512, 64, 0, BF16) == 2     # 768 workgroups
    assert lib.cottn_segments(2, 8, 12, 1024, 64, 0, BF16) == 4     # capped at four
    assert lib.cottn_segments(0, 1, 16, 65536, 64, 0, BF16) == 32   # long chains: 512 workgroups


@pytest.mark.parametrize("args", [
    (0, 0, 1, 8, 64, 0, BF16),      # B < 1
    (0, 1, 0, 8, 64, 0, BF16),      # H < 1
    (0, 1, 1, -1, 64, 0, BF16),     # N < 0
    (0, 1, 1, 8, 48, 0, BF16),      # unsupported d
    (0, 1, 1, 8, 64, 32, BF16),     # bf16 chunk must be 64/128/256
    (0, 1, 1, 8, 128, 128, BF16),   # d = 128 supports chunk 64 only
    (0, 1, 1, 8, 64, 64, F32),      # fp32 chunk must be 32
    (0, 1, 1, 8, 64, 0, 3),         # dtype
    (0, 1, 1, 8, 64, 32, 2),        # fp16 follows the bf16 chunk rules
    (7, 1, 1, 8, 64, 0, BF16),      # op
])
def test_unsupported_arguments_have_no_size(lib, args):
    assert lib.cottn_workspace_bytes(*args) == NOSIZE


def test_status_strings(lib):
    seen = set()
    for code in range(8):
        s = lib.cottn_status_string(code)
        assert s and s not in seen
        seen.add(s)
    assert lib.cottn_status_string(99) == b"unknown status"


def test_argument_errors_are_reported_before_any_launch(lib):
    """All of these return on the host; none touches HIP (this runs without a GPU)."""
    E_NULL, E_SHAPE, E_DTYPE, E_ALIGN, E_WS, E_ARG = 1, 2, 3, 4, 5, 7
    buf = ctypes.create_string_buffer(1 << 16)
    base = (ctypes.addressof(buf) + 255) & ~255
    p = lambda off=0: ctypes.c_void_p(base + off)
    eps = 1e-6
    lib.cottn_tune_segments(0)
    fwd = lib.cottn_fwd_causal
    assert fwd(None, p(), p(), p(), p(), None, None, 0, 1, 1, 8, 64, 0, BF16, eps, None) == E_NULL
    assert fwd(p(), p(), p(), None, p(), None, None, 0, 1, 1, 8, 64, 0, BF16, eps, None) == E_NULL
    assert fwd(p(), p(), p(), p(), p(), None, None, 0, 1, 1, 8, 64, 0, 5, eps, None) == E_DTYPE
    assert fwd(p(), p(), p(), p(), p(), None, None, 0, 1, 1, 8, 40, 0, BF16, eps, None) == E_SHAPE
    assert fwd(p(), p(), p(), p(), p(), None, None, 0, 1, 1, 8, 64, 96, BF16, eps, None) == E_SHAPE
    assert fwd(p(), p(), p(), p(), p(), None, None, 0, 0, 1, 8, 64, 0, BF16, eps, None) == E_SHAPE
    assert fwd(p(), p(), p(), p(), p(), None, None, 0, 1, 1, 8, 64, 0, BF16, 0.0, None) == E_ARG
    assert fwd(p(2), p(), p(), p(), p(), None, None, 0, 1, 1, 8, 64, 0, BF16, eps, None) == E_ALIGN
    assert fwd(p(), p(), p(), p(), p(), p(4), None, 0, 1, 1, 8, 64, 0, BF16, eps, None) == E_ALIGN
    # two segments of a 2-chunk sequence need a workspace
    lib.cottn_tune_segments(2)
    need = lib.cottn_workspace_bytes(0, 1, 1, 128, 64, 0, BF16)
    assert need == 2 * 64 * 64 * 4
    assert fwd(p(), p(), p(), p(), p(), None, None, 0, 1, 1, 128, 64, 0, BF16, eps, None) == E_WS
    assert fwd(p(), p(), p(), p(), p(), None, p(), need - 1, 1, 1, 128, 64, 0, BF16, eps, None) == E_WS
    assert fwd(p(), p(), p(), p(), p(), None, p(16), need, 1, 1, 128, 64, 0, BF16, eps, None) == E_ALIGN
    lib.cottn_tune_segments(0)
    bwd = lib.cottn_bwd_causal
    assert bwd(p(), p(), p(), p(), None, p(), p(), p(), p(), None, 0, p(), 1 << 12, 1, 1, 8, 64, 0, BF16, eps, None) == E_NULL
    assert bwd(p(), p(), p(), p(), p(), p(), p(), p(), None, None, 0, p(), 1 << 12, 1, 1, 8, 64, 0, BF16, eps, None) == E_NULL
    assert bwd(p(), p(), p(), p(), p(), p(), p(), p(), p(), None, 0, None, 0, 1, 1, 8, 64, 0, BF16, eps, None) == E_WS
    assert bwd(p(), p(), p(), p(), p(), p(), p(), p(), p(), None, 0, p(), 1 << 12, 1, 1, 8, 64, 0, 9, eps, None) == E_DTYPE
    # a forward workspace that is handed over must be as large and as aligned as the forward
    # needed it (two segments here); with one segment there is nothing to take over
    lib.cottn_tune_segments(2)
    fneed = lib.cottn_workspace_bytes(0, 1, 1, 128, 64, 0, BF16)
    bneed = lib.cottn_workspace_bytes(1, 1, 1, 128, 64, 0, BF16)
    assert bwd(p(), p(), p(), p(), p(), p(), p(), p(), p(), p(), fneed - 1, p(), bneed, 1, 1, 128, 64, 0, BF16, eps, None) == E_WS
    assert bwd(p(), p(), p(), p(), p(), p(), p(), p(), p(), p(16), fneed, p(), bneed, 1, 1, 128, 64, 0, BF16, eps, None) == E_ALIGN
    lib.cottn_tune_segments(0)
    assert lib.cottn_fwd_bidir(p(), p(), None, p(), p(), None, p(), 1 << 15, 1, 1, 8, 64, BF16, eps, None) == E_NULL
    assert lib.cottn_fwd_bidir(p(), p(), p(), p(), p(), None, None, 0, 1, 1, 8, 64, BF16, eps, None) == E_WS
    assert lib.cottn_bwd_bidir(p(), p(), p(), p(), p(), p(), p(), p(), p(), None, 0, p(), 16, 1, 1, 8, 64, BF16, eps, None) == E_WS
    assert lib.cottn_bwd_bidir(p(), p(), p(), p(), p(), p(), p(), p(), p(), None, 0, p(), 1 << 15, 1, 1, 8, 96, BF16, eps, None) == E_SHAPE
    cont = lib.cottn_fwd_causal_from_state
    st_buf = p()
    assert cont(p(), p(), p(), p(), None, p(), None, None, 0, 1, 1, 8, 64, 0, BF16, eps, None) == E_NULL
    assert cont(p(), p(), p(), p(), p(4), p(), None, None, 0, 1, 1, 8, 64, 0, BF16, eps, None) == E_ALIGN
    assert cont(p(), p(), p(), p(), st_buf, p(), st_buf, None, 0, 1, 1, 8, 64, 0, BF16, eps, None) == E_ARG
    assert cont(p(), p(), p(), p(), p(), p(), None, None, 0, 1, 1, 8, 48, 0, BF16, eps, None) == E_SHAPE
    piece = lib.cottn_bwd_causal_from_state
    tail = (None, 0, p(), 1 << 12, 1, 1, 8, 64, 0, BF16, eps, None)
    assert piece(p(), p(), p(), p(), None, None, None, p(), p(), p(), p(), None, *tail) == E_NULL
    assert piece(p(), p(), p(), p(), p(), p(4), None, p(), p(), p(), p(), None, *tail) == E_ALIGN
    assert piece(p(), p(), p(), p(), p(), None, p(8), p(), p(), p(), p(), None, *tail) == E_ALIGN
    assert piece(p(), p(), p(), p(), p(), None, st_buf, p(), p(), p(), p(), st_buf, *tail) == E_ARG
    vl = lib.cottn_fwd_causal_varlen
    assert vl(p(), p(), p(), p(), None, p(), None, None, 0, 1, 1, 8, 64, 0, BF16, eps, None) == E_NULL
    assert vl(p(), p(), p(), p(), p(2), p(), None, None, 0, 1, 1, 8, 64, 0, BF16, eps, None) == E_ALIGN
    assert vl(p(), p(), p(), p(), p(), p(), None, None, 0, 1, 1, 8, 64, 0, 7, eps, None) == E_DTYPE
    assert lib.cottn_bwd_bidir_varlen(p(), p(), p(), p(), None, p(), p(), p(), p(), p(), None, 0, p(), 1 << 15, 1, 1, 8, 64, BF16, eps, None) == E_NULL
    assert lib.cottn_scale_from_m_varlen(p(), None, p(), 2, 4, None) == E_NULL
    assert lib.cottn_scale_from_m_varlen(p(), p(), p(), 0, 4, None) == E_SHAPE
    assert lib.cottn_scale_from_m(p(), None, 4, 128.0, None) == E_NULL
    assert lib.cottn_scale_from_m(p(), p(), 0, 128.0, None) == E_SHAPE
    assert lib.cottn_scale_from_m(p(), p(), 4, 0.5, None) == E_ARG
    assert lib.cottn_scale_from_m(p(), p(), 4, float("nan"), None) == E_ARG
    assert lib.cottn_scale_from_m(p(2), p(), 4, 128.0, None) == E_ALIGN
    assert lib.cottn_scale_backward(p(), p(), None, 4, 128.0, None) == E_NULL
    assert lib.cottn_scale_backward(p(), p(), p(), 4, float("inf"), None) == E_ARG
    step = lib.cottn_step
    assert step(p(), p(), p(), p(), None, p(), 1, 1, 64, BF16, eps, None) == E_NULL
    assert step(p(), p(), p(), p(), p(), p(), 1, 1, 100, BF16, eps, None) == E_SHAPE
    assert step(p(), p(), p(), p(), p(), p(), 1, 1, 64, 3, eps, None) == E_DTYPE
    assert step(p(), p(), p(), p(), p(), p(), 1, 1, 64, BF16, -1.0, None) == E_ARG
    assert step(p(), p(8), p(), p(), p(), p(), 1, 1, 64, BF16, eps, None) == E_ALIGN


def test_static_workspace_forward_rejects_on_the_host(lib):
    """cottn_fwd_causal_static checks its arguments, and that the segment states fit the array
    inside the library, before it touches HIP."""
    E_NULL, E_SHAPE, E_WS = 1, 2, 5
    buf = ctypes.create_string_buffer(1 << 12)
    base = (ctypes.addressof(buf) + 255) & ~255
    p = lambda: ctypes.c_void_p(base)
    f = lib.cottn_fwd_causal_static
    lib.cottn_tune_segments(0)
    assert f(p(), None, p(), p(), p(), None, 1, 1, 8, 64, 0, BF16, 1e-6, None) == E_NULL
    assert f(p(), p(), p(), p(), p(), None, 1, 1, 8, 72, 0, BF16, 1e-6, None) == E_SHAPE
    limit = 16 << 20
    # B8 H16 N65536 d64 in 32 segments: 8*16*32 fp32 64x64 states = 64 MiB
    lib.cottn_tune_segments(32)
    assert lib.cottn_workspace_bytes(0, 8, 16, 65536, 64, 0, BF16) == 64 << 20
    assert f(p(), p(), p(), p(), p(), None, 8, 16, 65536, 64, 0, BF16, 1e-6, None) == E_WS
    lib.cottn_tune_segments(0)
    # the benchmarked shape fits
    assert 0 < lib.cottn_workspace_bytes(0, 8, 12, 1024, 64, 0, BF16) <= limit


def test_rectangular_head_dimensions_on_the_host(lib):
    """d_key != d_value (Sec. 2.1): workspace sizes follow dk * dv, the one-dimension calls are
    the dk = dv case, and unsupported combinations are refused before any launch."""
    E_NULL, E_SHAPE, E_WS = 1, 2, 5
    lib.cottn_tune_segments(4)
    wb = lib.cottn_workspace_bytes_dkdv
    assert wb(0, 8, 12, 1024, 64, 64, 0, BF16) == lib.cottn_workspace_bytes(0, 8, 12, 1024, 64, 0, BF16)
    assert wb(0, 8, 12, 1024, 32, 128, 0, BF16) == 8 * 12 * 4 * 32 * 128 * 4
    assert wb(1, 8, 12, 1024, 128, 64, 0, BF16) == 2 * 8 * 12 * 4 * 128 * 64 * 4 + 1536
    assert wb(3, 2, 2, 512, 64, 32, 0, BF16) == 2 * 2 * 2 * 4 * 64 * 32 * 4 + 256   # ds partials: max(G, dk*dv/256) = 8 per unit
    assert lib.cottn_segments_dkdv(0, 8, 12, 1024, 64, 128, 0, BF16) == 4
    lib.cottn_tune_segments(0)
    assert wb(4, 256, 16, 1, 32, 128, 0, BF16) == 0             # decode needs none
    assert wb(0, 1, 1, 8, 64, 128, 128, BF16) == NOSIZE          # rectangular: chunk 64 only
    assert wb(0, 1, 1, 8, 64, 96, 0, BF16) == NOSIZE             # unsupported d_value
    assert wb(0, 1, 1, 8, 64, 32, 0, F32) == 0                   # fp32: any pair; one segment needs none
    assert wb(0, 1, 1, 8, 64, 32, 64, F32) == NOSIZE             # fp32 chunk is 32
    buf = ctypes.create_string_buffer(1 << 16)
    base = (ctypes.addressof(buf) + 255) & ~255
    p = lambda: ctypes.c_void_p(base)
    eps = 1e-6
    f = lib.cottn_fwd_causal_dkdv
    assert f(p(), p(), None, p(), p(), None, None, 0, 1, 1, 8, 32, 64, 0, BF16, eps, None) == E_NULL
    assert f(p(), p(), p(), p(), p(), None, None, 0, 1, 1, 8, 32, 48, 0, BF16, eps, None) == E_SHAPE
    assert f(p(), p(), p(), p(), p(), None, None, 0, 1, 1, 8, 32, 64, 128, BF16, eps, None) == E_SHAPE
    assert f(p(), p(), p(), p(), p(), None, None, 0, 1, 1, 8, 32, 64, 64, F32, eps, None) == E_SHAPE
    assert lib.cottn_bwd_bidir_dkdv(p(), p(), p(), p(), p(), p(), p(), p(), p(), None, 0, p(), 16,
                                    1, 1, 8, 64, 128, BF16, eps, None) == E_WS
    assert lib.cottn_step_dkdv(p(), p(), p(), p(), p(), p(), 1, 1, 64, 100, BF16, eps, None) == E_SHAPE
    assert lib.cottn_step_dkdv(p(), p(), p(), p(), None, p(), 1, 1, 64, 128, BF16, eps, None) == E_NULL
