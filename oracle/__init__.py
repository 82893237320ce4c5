"""numpy/ctypes front end of the fp64 CPU oracle (``cottn_oracle.cpp``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke`` and by the
``cpu_baseline`` leg of ``bench.py``; the product package never imports it, and it never
imports the product package.  Every function converts its inputs to contiguous float64
(bf16/fp32 values convert exactly) and returns fresh float64 arrays.

Shapes: Q, K (and dQ, dK) are [B, H, N, d_key]; V, dO (and O, dV) are [B, H, N, d_value]
(Sec. 2.1 keeps the two head dimensions apart; every configuration of the paper has them
equal); s is [H]; states are [B, H, d_key, d_value] and do not contain the scale s.
"""
import ctypes
import os

import numpy as np

from .build import LIB, build

_lib = None
_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_int)


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = ctypes.CDLL(LIB)
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def _f64(x):
    return np.ascontiguousarray(np.asarray(x, dtype=np.float64))


def _p(a):
    return a.ctypes.data_as(_dp) if a is not None else None


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(ctypes.c_int(n))


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _dims(Q, V):
    """B, H, N, d_key (of Q, K), d_value (of V, O, dO) as C ints."""
    B, H, N, d = Q.shape
    e = V.shape[-1]
    assert V.shape[:-1] == Q.shape[:-1], (Q.shape, V.shape)
    return ctypes.c_int(B), ctypes.c_int(H), ctypes.c_int(N), ctypes.c_int(d), ctypes.c_int(e)


def normalize_rows(X, eps=1e-6):
    """Row L2 normalisation x / max(||x||, eps) over the last axis (Sec. 3.2)."""
    X = _f64(X)
    d = X.shape[-1]
    out = np.empty_like(X)
    den = np.empty(X.shape[:-1], dtype=np.float64)
    _load().oracle_normalize_rows(_p(X), ctypes.c_long(X.size // d), ctypes.c_int(d),
                                  ctypes.c_double(eps), _p(out), _p(den))
    return out, den


def similarity(Q, K, eps=1e-6):
    """Unmasked cosine-similarity matrix [N, N] of one unit; Q, K are [N, d] (Sec. 3.1)."""
    Q, K = _f64(Q), _f64(K)
    N, d = Q.shape
    P = np.empty((N, N), dtype=np.float64)
    _load().oracle_similarity(_p(Q), _p(K), ctypes.c_int(N), ctypes.c_int(d),
                              ctypes.c_double(eps), _p(P))
    return P


def fwd_quadratic(Q, K, V, s, eps=1e-6, causal=True):
    """The definition: s_h (Qhat Khat^T (.) M) V, or without mask (Sec. 4)."""
    Q, K, V, s = _f64(Q), _f64(K), _f64(V), _f64(s)
    O = np.empty_like(V)
    _load().oracle_fwd_quadratic(_p(Q), _p(K), _p(V), _p(s), *_dims(Q, V), ctypes.c_double(eps),
                                 ctypes.c_int(1 if causal else 0), _p(O))
    return O


def fwd_recurrent(Q, K, V, s, eps=1e-6, S0=None):
    """The RNN form (Sec. 5); returns (O, final state)."""
    Q, K, V, s = _f64(Q), _f64(K), _f64(V), _f64(s)
    B, H, N, d = Q.shape
    S0 = _f64(S0) if S0 is not None else None
    O = np.empty_like(V)
    S = np.empty((B, H, d, V.shape[-1]), dtype=np.float64)
    _load().oracle_fwd_recurrent(_p(Q), _p(K), _p(V), _p(s), *_dims(Q, V), ctypes.c_double(eps),
                                 _p(S0), _p(O), _p(S))
    return O, S


def state_total(K, V, eps=1e-6):
    """Khat^T V over the whole sequence, [B, H, d_key, d_value] (Sec. 4, eq. subQuadCos right bracket)."""
    K, V = _f64(K), _f64(V)
    B, H, N, d = K.shape
    S = np.empty((B, H, d, V.shape[-1]), dtype=np.float64)
    _load().oracle_state_total(_p(K), _p(V), *_dims(K, V), ctypes.c_double(eps), _p(S))
    return S


def step(q, k, v, s, S, eps=1e-6):
    """One decode step; q, k are [B, H, d_key], v [B, H, d_value]; returns (o, new state)
    without touching S."""
    q, k, v, s = _f64(q), _f64(k), _f64(v), _f64(s)
    S = _f64(S).copy()
    B, H, d = q.shape
    o = np.empty_like(v)
    _load().oracle_step(_p(q), _p(k), _p(v), _p(s), _p(S), ctypes.c_int(B), ctypes.c_int(H),
                        ctypes.c_int(d), ctypes.c_int(v.shape[-1]), ctypes.c_double(eps), _p(o))
    return o, S


def bwd_quadratic(Q, K, V, s, dO, eps=1e-6, causal=True):
    """Brute-force gradients wrt raw Q, K, V and s; returns (dQ, dK, dV, ds)."""
    Q, K, V, s, dO = _f64(Q), _f64(K), _f64(V), _f64(s), _f64(dO)
    dQ, dK, dV = np.empty_like(Q), np.empty_like(Q), np.empty_like(V)
    ds = np.empty_like(s)
    _load().oracle_bwd_quadratic(_p(Q), _p(K), _p(V), _p(s), _p(dO), *_dims(Q, V),
                                 ctypes.c_double(eps), ctypes.c_int(1 if causal else 0),
                                 _p(dQ), _p(dK), _p(dV), _p(ds))
    return dQ, dK, dV, ds


def bwd_recurrent(Q, K, V, s, dO, eps=1e-6):
    """Linear-time causal gradients (forward and reverse cumulative sums, Sec. 4)."""
    Q, K, V, s, dO = _f64(Q), _f64(K), _f64(V), _f64(s), _f64(dO)
    dQ, dK, dV = np.empty_like(Q), np.empty_like(Q), np.empty_like(V)
    ds = np.empty_like(s)
    _load().oracle_bwd_recurrent(_p(Q), _p(K), _p(V), _p(s), _p(dO), *_dims(Q, V),
                                 ctypes.c_double(eps), _p(dQ), _p(dK), _p(dV), _p(ds))
    return dQ, dK, dV, ds


def _rows(rows):
    r = np.ascontiguousarray(np.asarray(rows, dtype=np.int32).reshape(-1, 3))
    return r, r.ctypes.data_as(_ip), ctypes.c_int(r.shape[0])


def fwd_rows(Q, K, V, s, rows, eps=1e-6, causal=True):
    """Rows (b, h, i) of the definition, each from its own sum; returns [len(rows), d_value]."""
    Q, K, V, s = _f64(Q), _f64(K), _f64(V), _f64(s)
    r, rp, n = _rows(rows)
    out = np.empty((r.shape[0], V.shape[-1]), dtype=np.float64)
    _load().oracle_fwd_rows(_p(Q), _p(K), _p(V), _p(s), *_dims(Q, V), ctypes.c_double(eps),
                            ctypes.c_int(1 if causal else 0), rp, n, _p(out))
    return out


def bwd_rows(Q, K, V, s, dO, rows, eps=1e-6, causal=True):
    """Rows (b, h, t) of the brute-force dQ, dK ([len(rows), d_key]) and dV ([len(rows), d_value])."""
    Q, K, V, s, dO = _f64(Q), _f64(K), _f64(V), _f64(s), _f64(dO)
    r, rp, n = _rows(rows)
    d = Q.shape[-1]
    dQ = np.empty((r.shape[0], d), dtype=np.float64)
    dK, dV = np.empty_like(dQ), np.empty((r.shape[0], V.shape[-1]), dtype=np.float64)
    _load().oracle_bwd_rows(_p(Q), _p(K), _p(V), _p(s), _p(dO), *_dims(Q, V), ctypes.c_double(eps),
                            ctypes.c_int(1 if causal else 0), rp, n, _p(dQ), _p(dK), _p(dV))
    return dQ, dK, dV


def scale_from_m(m, n):
    """The paper's stabiliser (Sec. 3.3): the similarity is divided by n^sigma(m_h), with n the
    sequence length and m_h a learned scalar per head, i.e. s_h = n^(-sigma(m_h))."""
    m = _f64(m)
    sig = 1.0 / (1.0 + np.exp(-m))
    return np.power(float(n), -sig)


def scale_backward(m, n, ds):
    """dL/dm_h from dL/ds_h through s_h = n^(-sigma(m_h)):
    ds_h/dm_h = -ln(n) sigma(m_h) (1 - sigma(m_h)) n^(-sigma(m_h))."""
    m = _f64(m)
    ds = _f64(ds)
    sig = 1.0 / (1.0 + np.exp(-m))
    return ds * (-np.log(float(n))) * sig * (1.0 - sig) * np.power(float(n), -sig)


# ---- padded batches ---------------------------------------------------------------------------
# Sequences of different lengths share one [B, H, N, d] tensor; rows at or beyond seq_len[b]
# do not exist (Sec. 4: padding is masked by zeroing rows).  The oracle simply runs each
# sequence on its own rows; rows that do not exist are zero in every output.  s is [B, H]
# (the stabiliser of Sec. 3.3 depends on each sequence's own length) and so is ds.


def fwd_varlen(Q, K, V, s, seq_len, eps=1e-6, causal=True):
    """Returns (O, state): O zero on rows that do not exist; state [B, H, d, d] over the rows that do."""
    Q, K, V, s = _f64(Q), _f64(K), _f64(V), _f64(s)
    B, H, N, d = Q.shape
    O = np.zeros_like(V)
    S = np.zeros((B, H, d, V.shape[-1]))
    for b in range(B):
        n = int(min(N, max(0, seq_len[b])))
        if n == 0:
            continue
        sl = (slice(b, b + 1), slice(None), slice(0, n))
        O[sl] = fwd_quadratic(Q[sl], K[sl], V[sl], s[b], eps=eps, causal=causal)
        S[b] = state_total(K[sl], V[sl], eps=eps)[0]
    return O, S


def bwd_varlen(Q, K, V, s, dO, seq_len, eps=1e-6, causal=True):
    """Returns (dQ, dK, dV, ds) with ds [B, H]; gradients are zero on rows that do not exist."""
    Q, K, V, s, dO = _f64(Q), _f64(K), _f64(V), _f64(s), _f64(dO)
    B, H, N, d = Q.shape
    dQ, dK, dV = np.zeros_like(Q), np.zeros_like(Q), np.zeros_like(V)
    ds = np.zeros((B, H))
    for b in range(B):
        n = int(min(N, max(0, seq_len[b])))
        if n == 0:
            continue
        sl = (slice(b, b + 1), slice(None), slice(0, n))
        dQ[sl], dK[sl], dV[sl], ds[b] = bwd_quadratic(Q[sl], K[sl], V[sl], s[b], dO[sl], eps=eps,
                                                      causal=causal)
    return dQ, dK, dV, ds


def scale_from_m_varlen(m, seq_len):
    """s[b, h] = max(seq_len[b], 1)^(-sigma(m[h]))."""
    return np.stack([scale_from_m(m, max(int(n), 1)) for n in seq_len])


def scale_backward_varlen(m, seq_len, ds):
    """dm[h] = sum over b of ds[b, h] * d s[b, h] / d m[h]."""
    ds = _f64(ds)
    return sum(scale_backward(m, max(int(n), 1), ds[b]) for b, n in enumerate(seq_len))
