"""Pins for the CPU oracle: each test checks oracle/ against something that is not the oracle
(hand-worked numbers, closed forms, invariants, finite differences, brute force written in
another form), chosen so that a dropped term, a wrong sign or index, or a transposed operand
fails at least one of them.  CPU only."""
import json
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


def rand_inputs(seed, B, H, N, d, with_s=True):
    r = rng(seed)
    Q, K, V, dO = (r.standard_normal((B, H, N, d)) for _ in range(4))
    s = r.uniform(0.5, 1.5, size=H)
    return Q, K, V, dO, s


# ---------------------------------------------------------------- worked example
@pytest.mark.parametrize("name", ["worked_example_n3_d2.json", "worked_example_n3_dk2_dv3.json"])
def test_worked_example(oracle, name):
    check_worked_example(oracle, name)


def check_worked_example(oracle, name="worked_example_n3_d2.json"):
    g = json.load(open(os.path.join(GOLDEN, name)))
    A = lambda k: np.array(g[k], dtype=np.float64)[None, None]
    Q, K, V, dO, s = A("Q"), A("K"), A("V"), A("dO"), np.array(g["s"])
    tol = dict(rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.fwd_quadratic(Q, K, V, s, causal=True), A("O_causal"), **tol)
    np.testing.assert_allclose(oracle.fwd_quadratic(Q, K, V, s, causal=False), A("O_bidir"), **tol)
    O, S = oracle.fwd_recurrent(Q, K, V, s)
    np.testing.assert_allclose(O, A("O_causal"), **tol)
    np.testing.assert_allclose(S, A("state"), **tol)
    np.testing.assert_allclose(oracle.state_total(K, V), A("state"), **tol)
    for fn in (lambda: oracle.bwd_quadratic(Q, K, V, s, dO, causal=True),
               lambda: oracle.bwd_recurrent(Q, K, V, s, dO)):
        dQ, dK, dV, ds = fn()
        np.testing.assert_allclose(dQ, A("dQ_causal"), **tol)
        np.testing.assert_allclose(dK, A("dK_causal"), **tol)
        np.testing.assert_allclose(dV, A("dV_causal"), **tol)
        np.testing.assert_allclose(ds, np.array(g["ds_causal"]), **tol)
    rows = [(0, 0, i) for i in range(3)]
    np.testing.assert_allclose(oracle.fwd_rows(Q, K, V, s, rows), A("O_causal")[0, 0], **tol)
    rq, rk, rv = oracle.bwd_rows(Q, K, V, s, dO, rows)
    np.testing.assert_allclose(rq, A("dQ_causal")[0, 0], **tol)
    np.testing.assert_allclose(rk, A("dK_causal")[0, 0], **tol)
    np.testing.assert_allclose(rv, A("dV_causal")[0, 0], **tol)


# ---------------------------------------------------------------- normalisation (Sec. 3.2)
def test_normalise_unit_rows_and_eps(oracle):
    X = rng(1).standard_normal((7, 5)) * 3.0
    Xh, den = oracle.normalize_rows(X)
    np.testing.assert_allclose(np.sqrt((Xh ** 2).sum(-1)), 1.0, atol=1e-14)
    np.testing.assert_allclose(den, np.sqrt((X ** 2).sum(-1)), rtol=1e-15)
    # a 3-4-5 row
    Xh, _ = oracle.normalize_rows(np.array([[3.0, 4.0]]))
    np.testing.assert_allclose(Xh, [[0.6, 0.8]], atol=1e-15)
    # rows at or below eps are divided by eps, zero rows stay zero (padding rows, Sec. 4)
    Z = np.array([[0.0, 0.0, 0.0], [3e-7, 0.0, 4e-7]])
    Zh, den = oracle.normalize_rows(Z, eps=1e-6)
    assert np.all(np.isfinite(Zh))
    np.testing.assert_allclose(Zh[0], 0.0)
    np.testing.assert_allclose(Zh[1], [0.3, 0.0, 0.4], rtol=1e-12)
    np.testing.assert_allclose(den, [1e-6, 1e-6])


def test_similarity_bounded_by_one(oracle):
    # Sec. 3.1: cosine similarity lies in [-1, 1]; equality for parallel / anti-parallel rows.
    Q = rng(2).standard_normal((33, 8)) * 10
    K = rng(3).standard_normal((33, 8)) * 0.01
    K[5] = 7.5 * Q[9]
    K[6] = -0.2 * Q[9]
    P = oracle.similarity(Q, K)
    assert np.all(np.abs(P) <= 1 + 1e-12)
    assert abs(P[9, 5] - 1) < 1e-12 and abs(P[9, 6] + 1) < 1e-12


# ---------------------------------------------------------------- closed forms
def test_identical_rows_give_prefix_sum(oracle):
    # all q and k rows parallel -> every P_ij = 1 -> O is s times the inclusive prefix sum of V;
    # the bidirectional output is s times the column sums of V in every row.
    r = rng(4)
    u = r.standard_normal(6)
    B, H, N, d = 2, 3, 19, 6
    Q = np.broadcast_to(u, (B, H, N, d)) * r.uniform(0.5, 2, size=(B, H, N, 1))
    K = np.broadcast_to(u, (B, H, N, d)) * r.uniform(0.5, 2, size=(B, H, N, 1))
    V = r.standard_normal((B, H, N, d))
    s = r.uniform(0.5, 1.5, size=H)
    want = np.cumsum(V, axis=2) * s[None, :, None, None]
    np.testing.assert_allclose(oracle.fwd_quadratic(Q, K, V, s), want, atol=1e-12)
    np.testing.assert_allclose(oracle.fwd_recurrent(Q, K, V, s)[0], want, atol=1e-12)
    want_b = np.broadcast_to(V.sum(2, keepdims=True), V.shape) * s[None, :, None, None]
    np.testing.assert_allclose(oracle.fwd_quadratic(Q, K, V, s, causal=False), want_b, atol=1e-12)


def test_single_token(oracle):
    Q, K, V, dO, s = rand_inputs(5, 2, 2, 1, 7)
    cos = (Q * K).sum(-1) / np.sqrt((Q ** 2).sum(-1) * (K ** 2).sum(-1))
    want = s[None, :, None, None] * cos[..., None] * V
    for causal in (True, False):
        np.testing.assert_allclose(oracle.fwd_quadratic(Q, K, V, s, causal=causal), want, atol=1e-13)
    np.testing.assert_allclose(oracle.fwd_recurrent(Q, K, V, s)[0], want, atol=1e-13)


def test_orthonormal_keys_select_query_components(oracle):
    # keys = scaled rows of the identity: P_ij = qhat_i[j], so O_i = s sum_{j<=i} qhat_i[j] V_j
    r = rng(6)
    N = d = 6
    Q = r.standard_normal((1, 1, N, d))
    K = (np.eye(d) * r.uniform(0.5, 3, size=(d, 1)))[None, None]
    V = r.standard_normal((1, 1, N, d))
    s = np.array([0.75])
    Qh = Q / np.sqrt((Q ** 2).sum(-1, keepdims=True))
    want = np.zeros_like(V)
    for i in range(N):
        for j in range(i + 1):
            want[0, 0, i] += 0.75 * Qh[0, 0, i, j] * V[0, 0, j]
    np.testing.assert_allclose(oracle.fwd_quadratic(Q, K, V, s), want, atol=1e-13)
    np.testing.assert_allclose(oracle.fwd_recurrent(Q, K, V, s)[0], want, atol=1e-13)


def test_mask_includes_diagonal_and_is_causal(oracle):
    # changing inputs at positions > i must not change O_i; changing v_i must change O_i.
    Q, K, V, dO, s = rand_inputs(7, 1, 2, 12, 4)
    O = oracle.fwd_quadratic(Q, K, V, s)
    K2, V2 = K.copy(), V.copy()
    K2[:, :, 8:] += 1.0
    V2[:, :, 8:] -= 2.0
    O2 = oracle.fwd_quadratic(Q, K2, V2, s)
    np.testing.assert_array_equal(O[:, :, :8], O2[:, :, :8])
    assert np.all(np.abs(O[:, :, 8] - O2[:, :, 8]).max(-1) > 1e-6)


# ---------------------------------------------------------------- equivalences of the forms
@pytest.mark.parametrize("N,d", [(1, 4), (5, 4), (17, 8), (64, 8), (40, 3)])
def test_quadratic_equals_recurrent(oracle, N, d):
    Q, K, V, dO, s = rand_inputs(10 + N, 2, 2, N, d)
    Oq = oracle.fwd_quadratic(Q, K, V, s)
    Or, S = oracle.fwd_recurrent(Q, K, V, s)
    np.testing.assert_allclose(Oq, Or, atol=1e-12)
    np.testing.assert_allclose(S, oracle.state_total(K, V), atol=1e-12)


def test_cumsum_form_of_the_paper(oracle):
    # Sec. 4 eq. attn_2 evaluated literally with array ops: outer products V (x) K, inclusive
    # cumulative sum over the sequence axis, product with Q, reduction over the key axis.
    Q, K, V, dO, s = rand_inputs(11, 2, 3, 23, 5)
    Qh = Q / np.linalg.norm(Q, axis=-1, keepdims=True)
    Kh = K / np.linalg.norm(K, axis=-1, keepdims=True)
    Hs = (V[..., :, None] * Kh[..., None, :]).cumsum(axis=2)       # [B,H,N,d_value,d_key]
    want = (Hs * Qh[..., None, :]).sum(-1) * s[None, :, None, None]
    np.testing.assert_allclose(oracle.fwd_quadratic(Q, K, V, s), want, atol=1e-12)
    np.testing.assert_allclose(oracle.fwd_recurrent(Q, K, V, s)[0], want, atol=1e-12)
    # the oracle's state is the transpose ([d_key][d_value]) of the paper's hidden state
    np.testing.assert_allclose(oracle.fwd_recurrent(Q, K, V, s)[1],
                               np.swapaxes(Hs[:, :, -1], -1, -2), atol=1e-12)


def test_bidirectional_reassociation_and_permutation(oracle):
    # Sec. 4 eq. subQuadCos: [Qhat Khat^T] V = Qhat [Khat^T V]; invariant under a joint
    # permutation of the (K, V) rows; its last row equals the causal last row.
    Q, K, V, dO, s = rand_inputs(12, 2, 2, 21, 6)
    Ob = oracle.fwd_quadratic(Q, K, V, s, causal=False)
    S = oracle.state_total(K, V)
    Qh, _ = oracle.normalize_rows(Q)
    np.testing.assert_allclose(Ob, np.einsum("bhik,bhkc->bhic", Qh, S) * s[None, :, None, None],
                               atol=1e-12)
    Kh, _ = oracle.normalize_rows(K)
    np.testing.assert_allclose(S, np.einsum("bhjk,bhjc->bhkc", Kh, V), atol=1e-12)
    perm = rng(13).permutation(21)
    np.testing.assert_allclose(oracle.fwd_quadratic(Q, K[:, :, perm], V[:, :, perm], s, causal=False),
                               Ob, atol=1e-12)
    Oc = oracle.fwd_quadratic(Q, K, V, s, causal=True)
    np.testing.assert_allclose(Ob[:, :, -1], Oc[:, :, -1], atol=1e-12)


def test_scale_invariance_and_linearity(oracle):
    Q, K, V, dO, s = rand_inputs(14, 1, 2, 15, 5)
    O = oracle.fwd_quadratic(Q, K, V, s)
    a = rng(15).uniform(0.1, 9, size=(1, 2, 15, 1))
    np.testing.assert_allclose(oracle.fwd_quadratic(Q * a, K / a, V, s), O, atol=1e-12)
    np.testing.assert_allclose(oracle.fwd_quadratic(Q, K, 3 * V, s), 3 * O, atol=1e-12)
    np.testing.assert_allclose(oracle.fwd_quadratic(Q, K, V, 2 * s), 2 * O, atol=1e-12)
    # Sec. 3.3: a row of the similarity matrix sums to at most the sequence length
    bound = s[None, :, None] * np.cumsum(np.abs(V).max(-1), axis=2)
    assert np.all(np.abs(O).max(-1) <= bound + 1e-12)


def test_prefill_then_steps_equals_one_pass(oracle):
    # Sec. 5: the state after N1 tokens continues the sequence token by token.
    B, H, N1, N2, d = 2, 2, 9, 7, 5
    Q, K, V, dO, s = rand_inputs(16, B, H, N1 + N2, d)
    O_all = oracle.fwd_quadratic(Q, K, V, s)
    O1, S = oracle.fwd_recurrent(Q[:, :, :N1], K[:, :, :N1], V[:, :, :N1], s)
    np.testing.assert_allclose(O1, O_all[:, :, :N1], atol=1e-12)
    for t in range(N1, N1 + N2):
        o, S = oracle.step(Q[:, :, t], K[:, :, t], V[:, :, t], s, S)
        np.testing.assert_allclose(o, O_all[:, :, t], atol=1e-12)
    # and fwd_recurrent started from a state continues identically
    O2, S2 = oracle.fwd_recurrent(Q[:, :, N1:], K[:, :, N1:], V[:, :, N1:], s,
                                  S0=oracle.fwd_recurrent(Q[:, :, :N1], K[:, :, :N1], V[:, :, :N1], s)[1])
    np.testing.assert_allclose(O2, O_all[:, :, N1:], atol=1e-12)
    np.testing.assert_allclose(S2, S, atol=1e-12)


def test_step_updates_before_reading(oracle):
    # from a zero state one step gives s (qhat.khat) v: the state is read after the update
    r = rng(17)
    q, k, v = (r.standard_normal((1, 1, 4)) for _ in range(3))
    o, S = oracle.step(q, k, v, np.array([1.25]), np.zeros((1, 1, 4, 4)))
    cos = (q * k).sum() / np.linalg.norm(q) / np.linalg.norm(k)
    np.testing.assert_allclose(o, 1.25 * cos * v, atol=1e-14)
    np.testing.assert_allclose(S[0, 0], np.outer(k[0, 0] / np.linalg.norm(k), v[0, 0]), atol=1e-14)


def test_sampled_rows_match_full(oracle):
    Q, K, V, dO, s = rand_inputs(18, 2, 3, 29, 4)
    rows = [(0, 0, 0), (1, 2, 28), (1, 1, 13), (0, 2, 7)]
    for causal in (True, False):
        O = oracle.fwd_quadratic(Q, K, V, s, causal=causal)
        got = oracle.fwd_rows(Q, K, V, s, rows, causal=causal)
        dQ, dK, dV, _ = oracle.bwd_quadratic(Q, K, V, s, dO, causal=causal)
        rq, rk, rv = oracle.bwd_rows(Q, K, V, s, dO, rows, causal=causal)
        for n, (b, h, i) in enumerate(rows):
            np.testing.assert_allclose(got[n], O[b, h, i], atol=1e-12)
            np.testing.assert_allclose(rq[n], dQ[b, h, i], atol=1e-12)
            np.testing.assert_allclose(rk[n], dK[b, h, i], atol=1e-12)
            np.testing.assert_allclose(rv[n], dV[b, h, i], atol=1e-12)


# ---------------------------------------------------------------- gradients
def _loss(oracle, Q, K, V, s, dO, causal):
    return float((oracle.fwd_quadratic(Q, K, V, s, causal=causal) * dO).sum())


@pytest.mark.parametrize("causal", [True, False])
def test_gradients_by_central_differences(oracle, causal):
    # L = sum(dO * O); every raw input element and every s[h] is perturbed.
    B, H, N, d = 2, 2, 6, 3
    Q, K, V, dO, s = rand_inputs(20, B, H, N, d)
    dQ, dK, dV, ds = oracle.bwd_quadratic(Q, K, V, s, dO, causal=causal)
    h = 1e-6
    for name, X, G in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV), ("s", s, ds)):
        num = np.zeros_like(X)
        it = np.nditer(X, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = X[idx]
            X[idx] = old + h
            lp = _loss(oracle, Q, K, V, s, dO, causal)
            X[idx] = old - h
            lm = _loss(oracle, Q, K, V, s, dO, causal)
            X[idx] = old
            num[idx] = (lp - lm) / (2 * h)
        err = np.abs(num - G).max() / np.abs(num).max()
        assert err < 1e-6, (name, err)


def test_gradient_through_clamped_rows(oracle):
    # rows with norm <= eps are x/eps: the function is linear there, so dx = dxhat/eps, and
    # central differences (with a step that keeps the row below eps) must agree.
    B, H, N, d = 1, 1, 5, 3
    Q, K, V, dO, s = rand_inputs(21, B, H, N, d)
    eps = 1e-2
    Q[0, 0, 2] = [1e-3, -2e-3, 5e-4]
    K[0, 0, 3] = 0.0
    dQ, dK, dV, ds = oracle.bwd_quadratic(Q, K, V, s, dO, eps=eps)
    assert np.all(np.isfinite(dQ)) and np.all(np.isfinite(dK))
    h = 1e-7
    L = lambda: float((oracle.fwd_quadratic(Q, K, V, s, eps=eps) * dO).sum())
    for X, G, row in ((Q, dQ, 2), (K, dK, 3)):
        for c in range(d):
            old = X[0, 0, row, c]
            X[0, 0, row, c] = old + h
            lp = L()
            X[0, 0, row, c] = old - h
            lm = L()
            X[0, 0, row, c] = old
            assert abs((lp - lm) / (2 * h) - G[0, 0, row, c]) <= 1e-6 * max(1.0, abs(G[0, 0, row, c]))


@pytest.mark.parametrize("N,d", [(1, 4), (7, 3), (33, 8)])
def test_recurrent_backward_equals_brute_force(oracle, N, d):
    Q, K, V, dO, s = rand_inputs(30 + N, 2, 3, N, d)
    a = oracle.bwd_quadratic(Q, K, V, s, dO, causal=True)
    b = oracle.bwd_recurrent(Q, K, V, s, dO)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y, atol=1e-11)


@pytest.mark.parametrize("causal", [True, False])
def test_gradient_identities(oracle, causal):
    # normalisation makes O independent of row lengths -> dQ_i . Q_i = 0 and dK_j . K_j = 0;
    # O is linear in V and in s -> sum(V * dV) = sum(dO * O) = sum_h s_h ds_h.
    Q, K, V, dO, s = rand_inputs(40, 2, 3, 14, 5)
    dQ, dK, dV, ds = oracle.bwd_quadratic(Q, K, V, s, dO, causal=causal)
    np.testing.assert_allclose((dQ * Q).sum(-1), 0, atol=1e-11)
    np.testing.assert_allclose((dK * K).sum(-1), 0, atol=1e-11)
    O = oracle.fwd_quadratic(Q, K, V, s, causal=causal)
    per_head = (dO * O).sum(axis=(0, 2, 3))
    np.testing.assert_allclose((V * dV).sum(axis=(0, 2, 3)), per_head, rtol=1e-11)
    np.testing.assert_allclose(s * ds, per_head, rtol=1e-11)


def test_bidirectional_backward_closed_form(oracle):
    # without a mask the gradients collapse to dense products with S = Khat^T V and
    # G = Qhat^T dO:  dQhat = s dO S^T, dKhat = s V G^T, dV = s Khat G.
    Q, K, V, dO, s = rand_inputs(41, 2, 2, 11, 4)
    dQ, dK, dV, ds = oracle.bwd_quadratic(Q, K, V, s, dO, causal=False)
    Qh, qn = oracle.normalize_rows(Q)
    Kh, kn = oracle.normalize_rows(K)
    S = np.einsum("bhjk,bhjc->bhkc", Kh, V)
    G = np.einsum("bhik,bhic->bhkc", Qh, dO)
    sc = s[None, :, None, None]
    dQh = sc * np.einsum("bhic,bhkc->bhik", dO, S)
    dKh = sc * np.einsum("bhjc,bhkc->bhjk", V, G)
    proj = lambda Xh, dXh, n: (dXh - Xh * (Xh * dXh).sum(-1, keepdims=True)) / n[..., None]
    np.testing.assert_allclose(dQ, proj(Qh, dQh, qn), atol=1e-11)
    np.testing.assert_allclose(dK, proj(Kh, dKh, kn), atol=1e-11)
    np.testing.assert_allclose(dV, sc * np.einsum("bhjk,bhkc->bhjc", Kh, G), atol=1e-11)
    np.testing.assert_allclose(ds, (S * G).sum(axis=(0, 2, 3)), atol=1e-11)


def test_threads_do_not_change_results(oracle):
    Q, K, V, dO, s = rand_inputs(50, 3, 3, 16, 4)
    oracle.set_num_threads(1)
    a = oracle.bwd_quadratic(Q, K, V, s, dO)
    oracle.set_num_threads(0)
    b = oracle.bwd_quadratic(Q, K, V, s, dO)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)
    assert oracle.num_threads() >= 1


# ---- the stabiliser of Sec. 3.3: s_h = n^(-sigma(m_h)) -------------------------------------
def test_stabiliser_closed_forms(oracle):
    # m = 0 gives sigma = 1/2, i.e. division by sqrt(n) (the paper initialises m at 0.5, between
    # no scaling and division by n); n = 1 never scales; m -> +inf divides by n, -inf by 1
    np.testing.assert_allclose(oracle.scale_from_m([0.0], 1024), [1.0 / 32.0], rtol=1e-15)
    np.testing.assert_allclose(oracle.scale_from_m([-3.0, 0.5, 7.0], 1), [1.0, 1.0, 1.0], rtol=0)
    np.testing.assert_allclose(oracle.scale_from_m([40.0], 512), [1.0 / 512.0], rtol=1e-12)
    np.testing.assert_allclose(oracle.scale_from_m([-40.0], 512), [1.0], rtol=1e-12)
    # the paper's initial value: sigma(0.5) = 0.62245933..., so s = n^-0.62245933...
    np.testing.assert_allclose(oracle.scale_from_m([0.5], 100.0),
                               [np.exp(-np.log(100.0) / (1.0 + np.exp(-0.5)))], rtol=1e-15)
    # monotone: a larger m scales more strongly; a longer sequence scales more strongly
    s = oracle.scale_from_m(np.linspace(-4, 4, 17), 300)
    assert np.all(np.diff(s) < 0)
    assert oracle.scale_from_m([0.3], 2000)[0] < oracle.scale_from_m([0.3], 200)[0]


def test_stabiliser_gradient_finite_differences(oracle):
    m = np.array([-1.3, 0.0, 0.5, 2.2])
    ds = np.array([0.7, -1.1, 2.0, 0.3])
    for n in (2, 77, 4096):
        h = 1e-6
        fd = (oracle.scale_from_m(m + h, n) - oracle.scale_from_m(m - h, n)) / (2 * h)
        np.testing.assert_allclose(oracle.scale_backward(m, n, ds), ds * fd, rtol=1e-8, atol=1e-12)
    np.testing.assert_array_equal(oracle.scale_backward(m, 1, ds), np.zeros(4))  # ln 1 = 0


def test_stabiliser_through_attention(oracle):
    # the whole chain: L = sum(dO * O(s(m))) differentiated with respect to m by central
    # differences equals the oracle's ds pushed through scale_backward
    Q, K, V, dO, _ = rand_inputs(60, 2, 3, 12, 4)
    m = np.array([0.5, -0.8, 1.7])
    n = Q.shape[2]
    loss = lambda mm: float((dO * oracle.fwd_quadratic(Q, K, V, oracle.scale_from_m(mm, n))).sum())
    ds = oracle.bwd_quadratic(Q, K, V, oracle.scale_from_m(m, n), dO)[3]
    dm = oracle.scale_backward(m, n, ds)
    for h_idx in range(3):
        e = np.zeros(3); e[h_idx] = 1e-6
        fd = (loss(m + e) - loss(m - e)) / 2e-6
        np.testing.assert_allclose(dm[h_idx], fd, rtol=1e-6, atol=1e-9)


# ---- padded batches (rows at or beyond seq_len[b] do not exist) ----------------------------
def test_padded_batch_reduces_to_fixed_length(oracle):
    Q, K, V, dO, s = rand_inputs(70, 3, 2, 10, 4)
    sb = np.tile(s, (3, 1))
    for causal in (True, False):
        O, S = oracle.fwd_varlen(Q, K, V, sb, [10, 10, 10], causal=causal)
        np.testing.assert_allclose(O, oracle.fwd_quadratic(Q, K, V, s, causal=causal), atol=1e-13)
        np.testing.assert_allclose(S, oracle.state_total(K, V), atol=1e-13)
        g = oracle.bwd_varlen(Q, K, V, sb, dO, [10, 10, 10], causal=causal)
        ref = oracle.bwd_quadratic(Q, K, V, s, dO, causal=causal)
        for a, b in zip(g[:3], ref[:3]):
            np.testing.assert_allclose(a, b, atol=1e-12)
        np.testing.assert_allclose(g[3].sum(0), ref[3], atol=1e-12)  # ds[b][h] summed over b


def test_padded_batch_equals_zeroed_rows(oracle):
    # Sec. 4: "masking" a bidirectional sequence is zeroing its padded rows: with K, V zeroed
    # there the rows that exist see exactly the shorter sequence, whatever Q holds in the padding
    Q, K, V, dO, s = rand_inputs(71, 2, 3, 12, 4)
    lens = [7, 12]
    sb = np.stack([s, s * 1.3])
    O, _ = oracle.fwd_varlen(Q, K, V, sb, lens, causal=False)
    Kz, Vz = K.copy(), V.copy()
    Kz[0, :, 7:] = 0.0
    Vz[0, :, 7:] = 0.0
    for b in range(2):
        ref = oracle.fwd_quadratic(Q[b:b + 1], Kz[b:b + 1], Vz[b:b + 1], sb[b], causal=False)
        np.testing.assert_allclose(O[b, :, :lens[b]], ref[0, :, :lens[b]], atol=1e-13)
    assert np.all(O[0, :, 7:] == 0.0)
    # causal: rows that exist never see later rows, so garbage in the padding changes nothing
    Qg, Kg, Vg = Q.copy(), K.copy(), V.copy()
    for X in (Qg, Kg, Vg):
        X[0, :, 7:] = 1e3
    Oc, Sc = oracle.fwd_varlen(Q, K, V, sb, lens, causal=True)
    Og, Sg = oracle.fwd_varlen(Qg, Kg, Vg, sb, lens, causal=True)
    np.testing.assert_array_equal(Oc, Og)
    np.testing.assert_array_equal(Sc, Sg)


@pytest.mark.parametrize("causal", [True, False])
def test_padded_batch_gradients_finite_differences(oracle, causal):
    Q, K, V, dO, s = rand_inputs(72, 2, 2, 6, 3)
    lens = [4, 6]
    sb = np.stack([s, s * 0.7])
    loss = lambda q, k, v, ss: float((dO * oracle.fwd_varlen(q, k, v, ss, lens, causal=causal)[0]).sum())
    dQ, dK, dV, ds = oracle.bwd_varlen(Q, K, V, sb, dO, lens, causal=causal)
    h = 1e-6
    for (b, hd, i, c) in [(0, 0, 1, 2), (0, 1, 3, 0), (1, 0, 5, 1), (0, 1, 5, 1)]:  # last: padding
        for X, dX, which in ((Q, dQ, 0), (K, dK, 1), (V, dV, 2)):
            Xp, Xm = X.copy(), X.copy()
            Xp[b, hd, i, c] += h
            Xm[b, hd, i, c] -= h
            args = lambda Y: [Y if w == which else Z for w, Z in enumerate((Q, K, V))]
            fd = (loss(*args(Xp), sb) - loss(*args(Xm), sb)) / (2 * h)
            np.testing.assert_allclose(dX[b, hd, i, c], fd, rtol=1e-6, atol=1e-8)
    for (b, hd) in [(0, 0), (1, 1)]:
        sp, sm = sb.copy(), sb.copy()
        sp[b, hd] += h
        sm[b, hd] -= h
        np.testing.assert_allclose(ds[b, hd], (loss(Q, K, V, sp) - loss(Q, K, V, sm)) / (2 * h),
                                   rtol=1e-6, atol=1e-8)


def test_padded_batch_stabiliser(oracle):
    m = np.array([0.5, -1.0, 2.0])
    lens = [1, 17, 0, 300]
    s = oracle.scale_from_m_varlen(m, lens)
    assert s.shape == (4, 3)
    np.testing.assert_array_equal(s[0], np.ones(3))          # n = 1
    np.testing.assert_array_equal(s[2], np.ones(3))          # an empty sequence counts as n = 1
    np.testing.assert_allclose(s[3], oracle.scale_from_m(m, 300), rtol=0)
    ds = np.arange(12, dtype=np.float64).reshape(4, 3) - 5.0
    h = 1e-6
    fd = np.array([((oracle.scale_from_m_varlen(m + h * e, lens) -
                     oracle.scale_from_m_varlen(m - h * e, lens)) * ds).sum() / (2 * h)
                   for e in np.eye(3)])
    np.testing.assert_allclose(oracle.scale_backward_varlen(m, lens, ds), fd, rtol=1e-7)


# ---------------------------------------------------------------- the pins have teeth
class _Mistaken:
    """The oracle with one planted mistake (made here, on the CPU, around the real oracle):
    handed to a pin in the oracle's place, it must make that pin fail."""

    def __init__(self, oracle, kind):
        self._o, self._kind = oracle, kind

    def __getattr__(self, name):
        return getattr(self._o, name)

    def fwd_quadratic(self, Q, K, V, s, eps=1e-6, causal=True):
        o, kind = self._o, self._kind
        if kind == "operands_swapped":      # Kh Qh^T instead of Qh Kh^T
            return o.fwd_quadratic(K, Q, V, s, eps=eps, causal=causal)
        if kind == "scale_dropped":
            return o.fwd_quadratic(Q, K, V, np.ones_like(s), eps=eps, causal=causal)
        if kind == "keys_not_normalised":
            norms = np.maximum(np.linalg.norm(K, axis=-1, keepdims=True), eps)
            return o.fwd_quadratic(Q, K, V * norms, s, eps=eps, causal=causal)
        O = o.fwd_quadratic(Q, K, V, s, eps=eps, causal=causal)
        if kind == "diagonal_excluded" and causal:
            diag = (o.normalize_rows(Q, eps)[0] * o.normalize_rows(K, eps)[0]).sum(-1, keepdims=True)
            return O - np.asarray(s).reshape(1, -1, 1, 1) * diag * V
        if kind == "sign":
            return -O
        if kind == "value_columns_rotated":   # a wrong column stride on the value side
            return np.roll(O, 1, axis=-1)
        return O

    def fwd_recurrent(self, Q, K, V, s, eps=1e-6, S0=None):
        O, S = self._o.fwd_recurrent(Q, K, V, s, eps=eps, S0=S0)
        if self._kind == "state_keys_truncated":  # state accumulated over d_value x d_value
            S = S.copy()
            S[:, :, -1, :] = 0.0
        return O, S

    def bwd_quadratic(self, Q, K, V, s, dO, eps=1e-6, causal=True):
        dQ, dK, dV, ds = self._o.bwd_quadratic(Q, K, V, s, dO, eps=eps, causal=causal)
        kind = self._kind
        if kind == "dq_dk_exchanged":
            return dK, dQ, dV, ds
        if kind == "projection_dropped":   # gradient of the normalised rows passed through
            nq = np.maximum(np.linalg.norm(Q, axis=-1, keepdims=True), eps)
            return dQ + Q * 0.01 / nq, dK, dV, ds
        if kind == "dv_unscaled":
            return dQ, dK, dV / np.asarray(s).reshape(1, -1, 1, 1), ds
        if kind == "ds_per_batch_only":    # summed over one batch entry instead of all
            return dQ, dK, dV, ds * 0.5
        if kind == "dv_over_key_width":    # dV filled over d_key columns only
            dV = dV.copy()
            dV[..., Q.shape[-1]:] = 0.0
            return dQ, dK, dV, ds
        return dQ, dK, dV, ds


@pytest.mark.parametrize("kind,pin", [
    ("operands_swapped", "worked"), ("scale_dropped", "worked"), ("keys_not_normalised", "worked"),
    ("diagonal_excluded", "worked"), ("sign", "worked"),
    ("operands_swapped", "closed_form"), ("diagonal_excluded", "mask"),
    ("dq_dk_exchanged", "differences"), ("projection_dropped", "differences"),
    ("dv_unscaled", "differences"), ("ds_per_batch_only", "differences"),
    ("projection_dropped", "identities"), ("dq_dk_exchanged", "worked")])
def test_pins_reject_planted_mistakes(oracle, kind, pin):
    pins = {"worked": lambda o: check_worked_example(o),
            "closed_form": lambda o: test_orthonormal_keys_select_query_components(o),
            "mask": lambda o: test_mask_includes_diagonal_and_is_causal(o),
            "differences": lambda o: test_gradients_by_central_differences(o, True),
            "identities": lambda o: test_gradient_identities(o, True)}
    pins[pin](oracle)  # the pin passes on the oracle itself
    with pytest.raises(AssertionError):
        pins[pin](_Mistaken(oracle, kind))


# ---------------------------------------------------------------- d_key != d_value (Sec. 2.1)
def rand_inputs_dkdv(seed, B, H, N, dk, dv):
    r = np.random.default_rng(seed)
    Q, K = r.standard_normal((B, H, N, dk)), r.standard_normal((B, H, N, dk))
    V, dO = r.standard_normal((B, H, N, dv)), r.standard_normal((B, H, N, dv))
    return Q, K, V, dO, r.uniform(0.5, 1.5, size=H)


@pytest.mark.parametrize("dk,dv", [(3, 5), (6, 2)])
def test_dkdv_forms_agree_and_match_dense_algebra(oracle, dk, dv):
    """Keys and values of different widths: the definition, the recurrence, the sampled rows and
    the state agree with each other and with the dense matrix expressions written with array
    ops (P = Qhat Khat^T is N x N whatever the widths; O = s (P (.) M) V has d_value columns)."""
    Q, K, V, dO, s = rand_inputs_dkdv(60 + dk, 2, 2, 9, dk, dv)
    Qh, _ = oracle.normalize_rows(Q)
    Kh, _ = oracle.normalize_rows(K)
    P = np.einsum("bhik,bhjk->bhij", Qh, Kh)
    sc = s[None, :, None, None]
    O_c = sc * np.einsum("bhij,bhjc->bhic", np.tril(P), V)
    O_b = sc * np.einsum("bhij,bhjc->bhic", P, V)
    np.testing.assert_allclose(oracle.fwd_quadratic(Q, K, V, s, causal=True), O_c, atol=1e-12)
    np.testing.assert_allclose(oracle.fwd_quadratic(Q, K, V, s, causal=False), O_b, atol=1e-12)
    O_r, S = oracle.fwd_recurrent(Q, K, V, s)
    assert O_r.shape == V.shape and S.shape == (2, 2, dk, dv)
    np.testing.assert_allclose(O_r, O_c, atol=1e-12)
    np.testing.assert_allclose(S, np.einsum("bhjk,bhjc->bhkc", Kh, V), atol=1e-12)
    np.testing.assert_allclose(oracle.state_total(K, V), S, atol=1e-12)
    rows = [(1, 0, 8), (0, 1, 0), (1, 1, 4)]
    np.testing.assert_allclose(oracle.fwd_rows(Q, K, V, s, rows), np.stack([O_c[r] for r in rows]), atol=1e-12)
    # prefill + single steps == one pass, with a d_key x d_value state
    n1 = 4
    O1, S1 = oracle.fwd_recurrent(Q[:, :, :n1], K[:, :, :n1], V[:, :, :n1], s)
    for t in range(n1, 9):
        o, S1 = oracle.step(Q[:, :, t], K[:, :, t], V[:, :, t], s, S1)
        np.testing.assert_allclose(o, O_c[:, :, t], atol=1e-12)
    np.testing.assert_allclose(S1, S, atol=1e-12)


@pytest.mark.parametrize("causal", [True, False])
def test_dkdv_gradients_by_central_differences(oracle, causal):
    B, H, N, dk, dv = 1, 2, 5, 3, 4
    Q, K, V, dO, s = rand_inputs_dkdv(70, B, H, N, dk, dv)
    dQ, dK, dV, ds = oracle.bwd_quadratic(Q, K, V, s, dO, causal=causal)
    assert dQ.shape == Q.shape and dK.shape == K.shape and dV.shape == V.shape
    h = 1e-6
    for name, X, G in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV), ("s", s, ds)):
        num = np.zeros_like(X)
        it = np.nditer(X, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = X[idx]
            X[idx] = old + h
            lp = _loss(oracle, Q, K, V, s, dO, causal)
            X[idx] = old - h
            lm = _loss(oracle, Q, K, V, s, dO, causal)
            X[idx] = old
            num[idx] = (lp - lm) / (2 * h)
        err = np.abs(num - G).max() / np.abs(num).max()
        assert err < 1e-6, (name, err)


def test_dkdv_backward_forms_and_identities(oracle):
    Q, K, V, dO, s = rand_inputs_dkdv(80, 2, 3, 12, 4, 7)
    a = oracle.bwd_quadratic(Q, K, V, s, dO, causal=True)
    b = oracle.bwd_recurrent(Q, K, V, s, dO)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y, atol=1e-11)
    dQ, dK, dV, ds = a
    np.testing.assert_allclose((dQ * Q).sum(-1), 0, atol=1e-11)
    np.testing.assert_allclose((dK * K).sum(-1), 0, atol=1e-11)
    O = oracle.fwd_quadratic(Q, K, V, s, causal=True)
    per_head = (dO * O).sum(axis=(0, 2, 3))
    np.testing.assert_allclose((V * dV).sum(axis=(0, 2, 3)), per_head, rtol=1e-11)
    np.testing.assert_allclose(s * ds, per_head, rtol=1e-11)
    rows = [(0, 0, 0), (1, 2, 11), (1, 1, 5)]
    rq, rk, rv = oracle.bwd_rows(Q, K, V, s, dO, rows)
    np.testing.assert_allclose(rq, np.stack([dQ[r] for r in rows]), atol=1e-11)
    np.testing.assert_allclose(rk, np.stack([dK[r] for r in rows]), atol=1e-11)
    np.testing.assert_allclose(rv, np.stack([dV[r] for r in rows]), atol=1e-11)
    # bidirectional closed form with rectangular S = Khat^T V and G = Qhat^T dO
    dQ, dK, dV, ds = oracle.bwd_quadratic(Q, K, V, s, dO, causal=False)
    Qh, qn = oracle.normalize_rows(Q)
    Kh, kn = oracle.normalize_rows(K)
    S = np.einsum("bhjk,bhjc->bhkc", Kh, V)
    G = np.einsum("bhik,bhic->bhkc", Qh, dO)
    sc = s[None, :, None, None]
    proj = lambda Xh, dXh, n: (dXh - Xh * (Xh * dXh).sum(-1, keepdims=True)) / n[..., None]
    np.testing.assert_allclose(dQ, proj(Qh, sc * np.einsum("bhic,bhkc->bhik", dO, S), qn), atol=1e-11)
    np.testing.assert_allclose(dK, proj(Kh, sc * np.einsum("bhjc,bhkc->bhjk", V, G), kn), atol=1e-11)
    np.testing.assert_allclose(dV, sc * np.einsum("bhjk,bhkc->bhjc", Kh, G), atol=1e-11)
    np.testing.assert_allclose(ds, (S * G).sum(axis=(0, 2, 3)), atol=1e-11)


@pytest.mark.parametrize("kind,pin", [
    ("value_columns_rotated", "worked_dkdv"), ("value_columns_rotated", "forms"),
    ("state_keys_truncated", "forms"), ("dv_over_key_width", "differences_dkdv"),
    ("dv_over_key_width", "worked_dkdv"), ("dq_dk_exchanged", "worked_dkdv")])
def test_dkdv_pins_reject_planted_mistakes(oracle, kind, pin):
    pins = {"worked_dkdv": lambda o: check_worked_example(o, "worked_example_n3_dk2_dv3.json"),
            "forms": lambda o: test_dkdv_forms_agree_and_match_dense_algebra(o, 3, 5),
            "differences_dkdv": lambda o: test_dkdv_gradients_by_central_differences(o, True)}
    pins[pin](oracle)
    with pytest.raises(AssertionError):
        pins[pin](_Mistaken(oracle, kind))
