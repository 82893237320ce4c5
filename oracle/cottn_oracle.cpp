// CPU oracle for cosine attention (Cottention).  TEST INFRASTRUCTURE ONLY.
//
// This file is the slow, plain, fp64 statement of what the GPU library must
// compute.  It is used by the tests, by the smoke check and by the benchmark's
// "cpu_baseline" leg, and by nothing else: the product path never calls it and
// shares no code, header, table or helper with it.
//
// Everything is written straight from the paper's definitions:
//   * row L2 normalisation N(X) = X / ||X||_2            (Sec. 3.2, eq. "cosine")
//   * O = (N(Q) N(K)^T (.) M) V, M lower-triangular ones  (Sec. 4, eq. "attn_1")
//   * the cumulative-sum / RNN form H_t = H_{t-1} + k (x) v, O_t = q H_t
//                                                         (Sec. 4 eq. "attn_2", Sec. 5 eq. "hidden_state_obs")
//   * the bidirectional form [N(Q) N(K)^T] V              (Sec. 4, eq. "subQuadCos", left side)
//   * the three gradient formulas of Sec. 4 (dL/dQ, dL/dK, dL/dV) followed by
//     the chain rule through the normalisation and the per-head scale.
//
// Readings taken where the paper is silent (all listed in the design notes):
//   - normalisation divides by max(||x||, eps) (the semantics of the library
//     call in the appendix listing); rows with ||x|| <= eps are x/eps, and
//     their backward is dx = dxhat/eps.
//   - the mask includes the diagonal (inclusive cumulative sum; the RNN reads
//     the state after updating it).
//   - the stabiliser is taken as a given positive per-head number s[h] that
//     multiplies the output (Sec. 3.3 allows applying it before, during or
//     after the product).
//   - the recurrent state is stored [d_key][d_value] = sum_j khat_j^T v_j and
//     does NOT contain s[h].
//   - gradients are with respect to the raw (un-normalised) Q, K, V and to s.
//
// All tensors are contiguous row-major double arrays: Q,K,dQ,dK are [B][H][N][d]
// and V,O,dO,dV are [B][H][N][e] (d = d_key, e = d_value of Sec. 2.1; every
// configuration of the paper has e = d); s and ds are [H]; states are
// [B][H][d][e].
// No blocking, no fusion, no reordering beyond what the formulas state.
//
// Pins (tests/test_oracle_pins.py): hand-worked example, closed forms
// (identical rows -> prefix sum of V, orthonormal keys, N = 1), the bound
// |P_ij| <= 1, scale invariance, quadratic == recurrent, central finite
// differences for every gradient, gradient orthogonality and trace
// identities, permutation invariance of the bidirectional form, prefill +
// single steps == one causal pass.  No function here is "parity unpinned".

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstddef>
#include <cstdint>
#include <thread>
#include <vector>

namespace {

int g_threads = 0;  // 0 = hardware_concurrency

int thread_count() {
  int n = g_threads;
  if (n <= 0) n = static_cast<int>(std::thread::hardware_concurrency());
  return n < 1 ? 1 : n;
}

// Run fn(unit) for unit in [0, units) on up to thread_count() threads.
template <class F>
void for_each_unit(long units, F fn) {
  int nt = static_cast<int>(std::min<long>(thread_count(), units));
  if (nt <= 1) {
    for (long u = 0; u < units; ++u) fn(u);
    return;
  }
  std::atomic<long> next{0};
  std::vector<std::thread> pool;
  pool.reserve(nt);
  for (int t = 0; t < nt; ++t)
    pool.emplace_back([&] {
      for (;;) {
        long u = next.fetch_add(1);
        if (u >= units) break;
        fn(u);
      }
    });
  for (auto& th : pool) th.join();
}

// xhat = x / max(||x||_2, eps); returns the denominator actually used and
// whether the row was clamped.  (Sec. 3.2, N(X).)
double normalise_row(const double* x, int d, double eps, double* xhat, bool* clamped) {
  double ss = 0.0;
  for (int k = 0; k < d; ++k) ss += x[k] * x[k];
  double nrm = std::sqrt(ss);
  bool c = !(nrm > eps);
  double den = c ? eps : nrm;
  for (int k = 0; k < d; ++k) xhat[k] = x[k] / den;
  if (clamped) *clamped = c;
  return den;
}

double dot(const double* a, const double* b, int d) {
  double acc = 0.0;
  for (int k = 0; k < d; ++k) acc += a[k] * b[k];
  return acc;
}

// Normalised copy of one (b,h) unit: rows [N][d].
struct NormRows {
  std::vector<double> hat;   // [N][d]
  std::vector<double> den;   // [N]  max(||x||, eps)
  std::vector<char> clamped; // [N]
  NormRows(const double* X, int N, int d, double eps) : hat(size_t(N) * d), den(N), clamped(N) {
    for (int i = 0; i < N; ++i) {
      bool c;
      den[i] = normalise_row(X + size_t(i) * d, d, eps, hat.data() + size_t(i) * d, &c);
      clamped[i] = c;
    }
  }
  const double* row(int i, int d) const { return hat.data() + size_t(i) * d; }
};

// Chain rule through xhat = x / max(||x||, eps) for one row.
//   ||x|| > eps : dx = (dxhat - xhat (xhat . dxhat)) / ||x||
//   otherwise   : dx = dxhat / eps
void normalise_backward_row(const double* xhat, const double* dxhat, double den, bool clamped,
                            int d, double* dx) {
  if (clamped) {
    for (int k = 0; k < d; ++k) dx[k] = dxhat[k] / den;
    return;
  }
  double proj = dot(xhat, dxhat, d);
  for (int k = 0; k < d; ++k) dx[k] = (dxhat[k] - xhat[k] * proj) / den;
}

}  // namespace

extern "C" {

void oracle_set_num_threads(int n) { g_threads = n; }
int oracle_num_threads() { return thread_count(); }

// Xhat[r] = X[r] / max(||X[r]||, eps), den[r] = that denominator (may be null).
void oracle_normalize_rows(const double* X, long rows, int d, double eps, double* Xhat,
                           double* den) {
  for (long r = 0; r < rows; ++r) {
    double dn = normalise_row(X + size_t(r) * d, d, eps, Xhat + size_t(r) * d, nullptr);
    if (den) den[r] = dn;
  }
}

// Similarity matrix of one unit: P[i][j] = qhat_i . khat_j for all i, j
// (no mask).  Used by the |P| <= 1 pin.  (Sec. 3.1, eq. "cosine_sim".)
void oracle_similarity(const double* Q, const double* K, int N, int d, double eps, double* P) {
  NormRows q(Q, N, d, eps), k(K, N, d, eps);
  for (int i = 0; i < N; ++i)
    for (int j = 0; j < N; ++j) P[size_t(i) * N + j] = dot(q.row(i, d), k.row(j, d), d);
}

// In everything below the keys and queries have d features and the values,
// outputs and output gradients have e features (Sec. 2.1 writes d_H_key and
// d_H_value; the paper's experiments use e = d): Q, K, dQ, dK are [B][H][N][d],
// V, O, dO, dV are [B][H][N][e], and a state is [d][e] = [d_key][d_value].

// The definition.  causal != 0: O_i = s_h sum_{j<=i} (qhat_i . khat_j) v_j
// (Sec. 4 eq. "attn_1" with the multiplicative lower-triangular mask);
// causal == 0: the sum runs over all j (Sec. 4 eq. "subQuadCos", left side).
void oracle_fwd_quadratic(const double* Q, const double* K, const double* V, const double* s,
                          int B, int H, int N, int d, int e, double eps, int causal, double* O) {
  for_each_unit(long(B) * H, [&](long u) {
    int h = int(u % H);
    size_t kbase = size_t(u) * N * d, vbase = size_t(u) * N * e;
    NormRows q(Q + kbase, N, d, eps), k(K + kbase, N, d, eps);
    const double* v = V + vbase;
    double* o = O + vbase;
    for (int i = 0; i < N; ++i) {
      double* oi = o + size_t(i) * e;
      for (int c = 0; c < e; ++c) oi[c] = 0.0;
      int jend = causal ? i : N - 1;
      for (int j = 0; j <= jend; ++j) {
        double p = dot(q.row(i, d), k.row(j, d), d);
        const double* vj = v + size_t(j) * e;
        for (int c = 0; c < e; ++c) oi[c] += p * vj[c];
      }
      for (int c = 0; c < e; ++c) oi[c] *= s[h];
    }
  });
}

// The recurrent form (Sec. 5 eq. "hidden_state_obs"): S starts from S0 (zero
// when S0 is null; Fig. 1 caption: H_0 = 0), then for each t
//   S <- S + khat_t^T v_t ;  O_t = s_h qhat_t S      (state read after update)
// S is [d_key][d_value].  S_final (may be null) receives the last state.
void oracle_fwd_recurrent(const double* Q, const double* K, const double* V, const double* s,
                          int B, int H, int N, int d, int e, double eps, const double* S0,
                          double* O, double* S_final) {
  for_each_unit(long(B) * H, [&](long u) {
    int h = int(u % H);
    size_t kbase = size_t(u) * N * d, vbase = size_t(u) * N * e;
    size_t sbase = size_t(u) * d * e;
    std::vector<double> S(size_t(d) * e, 0.0), qh(d), kh(d);
    if (S0) std::copy(S0 + sbase, S0 + sbase + size_t(d) * e, S.begin());
    for (int t = 0; t < N; ++t) {
      normalise_row(Q + kbase + size_t(t) * d, d, eps, qh.data(), nullptr);
      normalise_row(K + kbase + size_t(t) * d, d, eps, kh.data(), nullptr);
      const double* vt = V + vbase + size_t(t) * e;
      for (int a = 0; a < d; ++a)
        for (int c = 0; c < e; ++c) S[size_t(a) * e + c] += kh[a] * vt[c];
      double* ot = O + vbase + size_t(t) * e;
      for (int c = 0; c < e; ++c) {
        double acc = 0.0;
        for (int a = 0; a < d; ++a) acc += qh[a] * S[size_t(a) * e + c];
        ot[c] = s[h] * acc;
      }
    }
    if (S_final) std::copy(S.begin(), S.end(), S_final + sbase);
  });
}

// S[b][h] = Khat^T V over all N rows ([d_key][d_value]); the right-hand
// bracket of eq. "subQuadCos".
void oracle_state_total(const double* K, const double* V, int B, int H, int N, int d, int e,
                        double eps, double* S) {
  for_each_unit(long(B) * H, [&](long u) {
    size_t kbase = size_t(u) * N * d, vbase = size_t(u) * N * e;
    double* Su = S + size_t(u) * d * e;
    std::fill(Su, Su + size_t(d) * e, 0.0);
    std::vector<double> kh(d);
    for (int t = 0; t < N; ++t) {
      normalise_row(K + kbase + size_t(t) * d, d, eps, kh.data(), nullptr);
      const double* vt = V + vbase + size_t(t) * e;
      for (int a = 0; a < d; ++a)
        for (int c = 0; c < e; ++c) Su[size_t(a) * e + c] += kh[a] * vt[c];
    }
  });
}

// One decode step for B*H independent states (Sec. 5): q, k are [B][H][d], v and
// o [B][H][e]; S [B][H][d][e] is updated in place with khat^T v and then read
// with qhat.
void oracle_step(const double* q, const double* k, const double* v, const double* s, double* S,
                 int B, int H, int d, int e, double eps, double* o) {
  for_each_unit(long(B) * H, [&](long u) {
    int h = int(u % H);
    std::vector<double> qh(d), kh(d);
    normalise_row(q + size_t(u) * d, d, eps, qh.data(), nullptr);
    normalise_row(k + size_t(u) * d, d, eps, kh.data(), nullptr);
    const double* vu = v + size_t(u) * e;
    double* Su = S + size_t(u) * d * e;
    for (int a = 0; a < d; ++a)
      for (int c = 0; c < e; ++c) Su[size_t(a) * e + c] += kh[a] * vu[c];
    for (int c = 0; c < e; ++c) {
      double acc = 0.0;
      for (int a = 0; a < d; ++a) acc += qh[a] * Su[size_t(a) * e + c];
      o[size_t(u) * e + c] = s[h] * acc;
    }
  });
}

// Brute-force backward.  With P_ij = qhat_i . khat_j and A_ij = dO_i . v_j on
// the unmasked pairs (j <= i when causal, all pairs otherwise), the gradient
// formulas of Sec. 4 read, row by row,
//   dqhat_i = s_h sum_j A_ij khat_j      (dL/dQ = (dO V^T (.) M) K)
//   dkhat_j = s_h sum_i A_ij qhat_i      (dL/dK = (dO V^T (.) M)^T Q)
//   dv_j    = s_h sum_i P_ij dO_i        (dL/dV = (Q K^T (.) M)^T dO)
// and, since O = s_h * (unscaled output), ds_h = sum_{b,i,j} P_ij A_ij.
// dQ, dK then go through the normalisation's chain rule.
void oracle_bwd_quadratic(const double* Q, const double* K, const double* V, const double* s,
                          const double* dO, int B, int H, int N, int d, int e, double eps,
                          int causal, double* dQ, double* dK, double* dV, double* ds) {
  std::vector<double> ds_unit(size_t(B) * H, 0.0);
  for_each_unit(long(B) * H, [&](long u) {
    int h = int(u % H);
    size_t kbase = size_t(u) * N * d, vbase = size_t(u) * N * e;
    NormRows q(Q + kbase, N, d, eps), k(K + kbase, N, d, eps);
    const double* v = V + vbase;
    const double* g = dO + vbase;
    std::vector<double> dqh(size_t(N) * d, 0.0), dkh(size_t(N) * d, 0.0);
    double* dv = dV + vbase;
    std::fill(dv, dv + size_t(N) * e, 0.0);
    double ds_acc = 0.0;
    for (int i = 0; i < N; ++i) {
      int jend = causal ? i : N - 1;
      for (int j = 0; j <= jend; ++j) {
        double p = dot(q.row(i, d), k.row(j, d), d);
        double a = dot(g + size_t(i) * e, v + size_t(j) * e, e);
        ds_acc += p * a;
        for (int c = 0; c < d; ++c) {
          dqh[size_t(i) * d + c] += s[h] * a * k.row(j, d)[c];
          dkh[size_t(j) * d + c] += s[h] * a * q.row(i, d)[c];
        }
        for (int c = 0; c < e; ++c) dv[size_t(j) * e + c] += s[h] * p * g[size_t(i) * e + c];
      }
    }
    for (int i = 0; i < N; ++i) {
      normalise_backward_row(q.row(i, d), dqh.data() + size_t(i) * d, q.den[i], q.clamped[i], d,
                             dQ + kbase + size_t(i) * d);
      normalise_backward_row(k.row(i, d), dkh.data() + size_t(i) * d, k.den[i], k.clamped[i], d,
                             dK + kbase + size_t(i) * d);
    }
    ds_unit[u] = ds_acc;
  });
  for (int h = 0; h < H; ++h) ds[h] = 0.0;
  for (long u = 0; u < long(B) * H; ++u) ds[u % H] += ds_unit[u];
}

// Linear-time causal backward in the paper's own arrangement (Sec. 4, last
// paragraph, and the appendix's description): dqhat comes from a forward-time
// cumulative sum of khat (x) v; dkhat and dv come from a cumulative sum of
// qhat (x) dO that runs backward in time.  Used where the brute force is too
// slow; pinned against it on small inputs.
void oracle_bwd_recurrent(const double* Q, const double* K, const double* V, const double* s,
                          const double* dO, int B, int H, int N, int d, int e, double eps,
                          double* dQ, double* dK, double* dV, double* ds) {
  std::vector<double> ds_unit(size_t(B) * H, 0.0);
  for_each_unit(long(B) * H, [&](long u) {
    int h = int(u % H);
    size_t kbase = size_t(u) * N * d, vbase = size_t(u) * N * e;
    NormRows q(Q + kbase, N, d, eps), k(K + kbase, N, d, eps);
    const double* v = V + vbase;
    const double* g = dO + vbase;
    std::vector<double> S(size_t(d) * e, 0.0), R(size_t(d) * e, 0.0), tmp(d);
    double ds_acc = 0.0;
    // forward in time: S_t = sum_{j<=t} khat_j^T v_j ; dqhat_t[a] = s sum_c dO_t[c] S_t[a][c]
    for (int t = 0; t < N; ++t) {
      for (int a = 0; a < d; ++a)
        for (int c = 0; c < e; ++c) S[size_t(a) * e + c] += k.row(t, d)[a] * v[size_t(t) * e + c];
      for (int a = 0; a < d; ++a) {
        double acc = 0.0;
        for (int c = 0; c < e; ++c) acc += g[size_t(t) * e + c] * S[size_t(a) * e + c];
        tmp[a] = s[h] * acc;
        ds_acc += q.row(t, d)[a] * acc;
      }
      normalise_backward_row(q.row(t, d), tmp.data(), q.den[t], q.clamped[t], d,
                             dQ + kbase + size_t(t) * d);
    }
    // backward in time: R_t = sum_{i>=t} qhat_i^T dO_i
    for (int t = N - 1; t >= 0; --t) {
      for (int a = 0; a < d; ++a)
        for (int c = 0; c < e; ++c) R[size_t(a) * e + c] += q.row(t, d)[a] * g[size_t(t) * e + c];
      for (int a = 0; a < d; ++a) {
        double acc = 0.0;
        for (int c = 0; c < e; ++c) acc += v[size_t(t) * e + c] * R[size_t(a) * e + c];
        tmp[a] = s[h] * acc;
      }
      normalise_backward_row(k.row(t, d), tmp.data(), k.den[t], k.clamped[t], d,
                             dK + kbase + size_t(t) * d);
      for (int c = 0; c < e; ++c) {
        double acc = 0.0;
        for (int a = 0; a < d; ++a) acc += k.row(t, d)[a] * R[size_t(a) * e + c];
        dV[vbase + size_t(t) * e + c] = s[h] * acc;
      }
    }
    ds_unit[u] = ds_acc;
  });
  for (int h = 0; h < H; ++h) ds[h] = 0.0;
  for (long u = 0; u < long(B) * H; ++u) ds[u % H] += ds_unit[u];
}

// Sampled rows of the definition, for sizes where the whole quadratic form is
// too slow.  rows[r] = {b, h, i}.  Each output row is computed on its own from
// the definition (cost O(N d) per row).
//   O_out[r]  = row i of the forward output
void oracle_fwd_rows(const double* Q, const double* K, const double* V, const double* s, int B,
                     int H, int N, int d, int e, double eps, int causal, const int* rows,
                     int nrows, double* O_out) {
  (void)B;
  for_each_unit(nrows, [&](long r) {
    int b = rows[3 * r], h = rows[3 * r + 1], i = rows[3 * r + 2];
    size_t kbase = (size_t(b) * H + h) * size_t(N) * d, vbase = (size_t(b) * H + h) * size_t(N) * e;
    std::vector<double> qh(d), kh(d), acc(e, 0.0);
    normalise_row(Q + kbase + size_t(i) * d, d, eps, qh.data(), nullptr);
    int jend = causal ? i : N - 1;
    for (int j = 0; j <= jend; ++j) {
      normalise_row(K + kbase + size_t(j) * d, d, eps, kh.data(), nullptr);
      double p = dot(qh.data(), kh.data(), d);
      for (int c = 0; c < e; ++c) acc[c] += p * V[vbase + size_t(j) * e + c];
    }
    for (int c = 0; c < e; ++c) O_out[size_t(r) * e + c] = s[h] * acc[c];
  });
}

// Sampled rows of the brute-force backward: for rows[r] = {b, h, t} returns
// dQ_t, dK_t ([nrows][d]) and dV_t ([nrows][e]), every one from its own defining sum.
void oracle_bwd_rows(const double* Q, const double* K, const double* V, const double* s,
                     const double* dO, int B, int H, int N, int d, int e, double eps, int causal,
                     const int* rows, int nrows, double* dQ_out, double* dK_out, double* dV_out) {
  (void)B;
  for_each_unit(nrows, [&](long r) {
    int b = rows[3 * r], h = rows[3 * r + 1], t = rows[3 * r + 2];
    size_t kbase = (size_t(b) * H + h) * size_t(N) * d, vbase = (size_t(b) * H + h) * size_t(N) * e;
    std::vector<double> qt(d), kt(d), other(d), dqh(d, 0.0), dkh(d, 0.0), dv(e, 0.0);
    bool qc, kc;
    double qden = normalise_row(Q + kbase + size_t(t) * d, d, eps, qt.data(), &qc);
    double kden = normalise_row(K + kbase + size_t(t) * d, d, eps, kt.data(), &kc);
    // dqhat_t = s sum_{j in mask(t)} (dO_t . v_j) khat_j
    int jend = causal ? t : N - 1;
    for (int j = 0; j <= jend; ++j) {
      normalise_row(K + kbase + size_t(j) * d, d, eps, other.data(), nullptr);
      double a = dot(dO + vbase + size_t(t) * e, V + vbase + size_t(j) * e, e);
      for (int c = 0; c < d; ++c) dqh[c] += s[h] * a * other[c];
    }
    // dkhat_t = s sum_{i: t in mask(i)} (dO_i . v_t) qhat_i ; dv_t = s sum_i (qhat_i . khat_t) dO_i
    int ibeg = causal ? t : 0;
    for (int i = ibeg; i < N; ++i) {
      normalise_row(Q + kbase + size_t(i) * d, d, eps, other.data(), nullptr);
      double a = dot(dO + vbase + size_t(i) * e, V + vbase + size_t(t) * e, e);
      double p = dot(other.data(), kt.data(), d);
      for (int c = 0; c < d; ++c) dkh[c] += s[h] * a * other[c];
      for (int c = 0; c < e; ++c) dv[c] += s[h] * p * dO[vbase + size_t(i) * e + c];
    }
    normalise_backward_row(qt.data(), dqh.data(), qden, qc, d, dQ_out + size_t(r) * d);
    normalise_backward_row(kt.data(), dkh.data(), kden, kc, d, dK_out + size_t(r) * d);
    for (int c = 0; c < e; ++c) dV_out[size_t(r) * e + c] = dv[c];
  });
}

}  // extern "C"
