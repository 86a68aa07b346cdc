// CPU oracle for one step of bidirectional Top_K SGD with error feedback
// (Algorithm 2 of "Downlink Compression Improves Top_K Sparsification").
//
// THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, obviously
// correct implementation used only to check the HIP library and to give a CPU
// baseline time.  It shares no code with the HIP path and nothing in the
// product may call it.
//
// Everything is the plain definition written out:
//   * Top_K (the operator the paper describes in words in its abstract and
//     introduction: keep the K components of largest magnitude, zero the rest)
//     is a full stable sort of all d coordinates on the magnitude, largest
//     first.  The paper gives no rule for equal magnitudes; the stable sort makes
//     the lower index win.  "Magnitude" is the 31-bit pattern of the fp32 value
//     with the sign bit cleared, compared as an unsigned integer, which orders
//     NaN > Inf > finite > denormal > zero and makes +0 and -0 equal.
//   * The residual bookkeeping eps = a - Top_K(a) and delta = g - Top_K(g)
//     (Algorithm 2, worker and server residual lines) is written as "copy, then
//     store +0 at the kept positions".
//   * Every multiply-add of the algorithm is one correctly rounded fused
//     multiply-add (std::fmaf).
//
// Build: g++ -O2 -ffp-contract=off -shared -fPIC (no fast-math, no FTZ/DAZ).
//
// oracle_unidir_step (Algorithm 1) is pinned by agreeing, on w and eps, with
// oracle_bidir_step run with K_dn = d (which tests pin to Algorithm 1 independently).
//
// Parity pins (see tests/test_oracle_*.py): brute-force subset enumeration on
// tiny inputs, the three Top_K invariants, the contraction bound of the
// paper's Eq. "topk_bound", reduction to dense SGD (Eq. 2) when K = d,
// reduction to Algorithm 1 when K_dn = d, the conservation identity of Lemma 1
// on dyadic inputs (exact), and the closed-form optimum of the appendix toy
// example.  The bit-level conventions (tie rule, NaN order, +0 at kept
// positions, fused rounding, accumulation starting from delta) are readings of
// this build, not of the paper: the paper does not pin them.

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <thread>
#include <vector>

namespace {

struct KeyIdx {
  uint32_t key;  // magnitude bit pattern
  uint32_t idx;  // coordinate
};

inline uint32_t bits_of(float x) {
  uint32_t u;
  std::memcpy(&u, &x, sizeof u);
  return u;
}

inline uint32_t magnitude_key(float x) { return bits_of(x) & 0x7FFFFFFFu; }

// Top_K of x[0..d): writes the K kept (index, value) pairs in ascending index
// order and, if residual != nullptr, residual = x with +0 at the kept positions.
// residual may alias x.
void topk_plain(const float* x, uint64_t d, uint64_t K, uint32_t* idx, float* val,
                float* residual) {
  std::vector<KeyIdx> order(d);
  for (uint64_t i = 0; i < d; ++i) {
    order[i].key = magnitude_key(x[i]);
    order[i].idx = static_cast<uint32_t>(i);
  }
  // Largest magnitude first; equal magnitudes keep their index order.
  std::stable_sort(order.begin(), order.end(),
                   [](const KeyIdx& a, const KeyIdx& b) { return a.key > b.key; });
  std::vector<uint32_t> kept(K);
  for (uint64_t j = 0; j < K; ++j) kept[j] = order[j].idx;
  std::sort(kept.begin(), kept.end());
  for (uint64_t j = 0; j < K; ++j) {
    idx[j] = kept[j];
    val[j] = x[kept[j]];
  }
  if (residual != nullptr) {
    if (residual != x) std::memcpy(residual, x, d * sizeof(float));
    for (uint64_t j = 0; j < K; ++j) residual[kept[j]] = 0.0f;
  }
}

// Worker side of Algorithm 2 for one worker q: a = eps + alpha*g, send
// Top_K(a), keep eps = a - Top_K(a).
void worker_row(const float* g, float* eps, uint64_t d, float alpha_in, uint64_t K_up,
                uint32_t* up_idx, float* up_val) {
  for (uint64_t i = 0; i < d; ++i) eps[i] = std::fmaf(alpha_in, g[i], eps[i]);
  topk_plain(eps, d, K_up, up_idx, up_val, eps);
}

}  // namespace

extern "C" {

// Top_K operator on one vector.  residual may be null.  Returns 0, or -1 on bad
// arguments (K > d or d >= 2^32).
int oracle_topk(const float* x, uint64_t d, uint64_t K, uint32_t* idx, float* val,
                float* residual) {
  if (K > d || d >= (1ull << 32)) return -1;
  topk_plain(x, d, K, idx, val, residual);
  return 0;
}

// Worker lines of Algorithm 2 for all N workers.  g, eps are N x d row-major;
// eps is updated in place; up_idx/up_val are N x K_up.  Rows are independent and
// are spread over nthreads threads (each row is still computed sequentially).
int oracle_worker_stage(const float* g, float* eps, int32_t N, uint64_t d, float alpha_in,
                        uint64_t K_up, uint32_t* up_idx, float* up_val, int32_t nthreads) {
  if (N <= 0 || K_up > d || d >= (1ull << 32)) return -1;
  if (nthreads < 1) nthreads = 1;
  if (nthreads > N) nthreads = N;
  auto run = [&](int t) {
    for (int q = t; q < N; q += nthreads)
      worker_row(g + (uint64_t)q * d, eps + (uint64_t)q * d, d, alpha_in, K_up,
                 up_idx + (uint64_t)q * K_up, up_val + (uint64_t)q * K_up);
  };
  if (nthreads == 1) {
    run(0);
  } else {
    std::vector<std::thread> pool;
    for (int t = 0; t < nthreads; ++t) pool.emplace_back(run, t);
    for (auto& th : pool) th.join();
  }
  return 0;
}

// Server aggregation line of Algorithm 2: g_t = sum_q p_q Top_K(a^q) + delta.
// The accumulator starts at delta and the workers are added in ascending q, one
// fused multiply-add each.  delta is overwritten with g_t.  union_nnz (nullable)
// receives the number of distinct coordinates named by the uplinks.
int oracle_aggregate(const uint32_t* up_idx, const float* up_val, const float* p, int32_t N,
                     uint64_t K_up, float* delta, uint64_t d, uint64_t* union_nnz) {
  if (N <= 0 || K_up > d) return -1;
  std::vector<uint8_t> touched;
  if (union_nnz) touched.assign(d, 0);
  for (int q = 0; q < N; ++q) {
    for (uint64_t j = 0; j < K_up; ++j) {
      uint32_t i = up_idx[(uint64_t)q * K_up + j];
      if (i >= d) return -2;
      delta[i] = std::fmaf(p[q], up_val[(uint64_t)q * K_up + j], delta[i]);
      if (union_nnz) touched[i] = 1;
    }
  }
  if (union_nnz) {
    uint64_t c = 0;
    for (uint64_t i = 0; i < d; ++i) c += touched[i];
    *union_nnz = c;
  }
  return 0;
}

// Server compression lines of Algorithm 2: send Top_K(g_t), keep
// delta = g_t - Top_K(g_t).  delta holds g_t on entry.
int oracle_downlink(float* delta, uint64_t d, uint64_t K_dn, uint32_t* dn_idx, float* dn_val) {
  if (K_dn > d || d >= (1ull << 32)) return -1;
  topk_plain(delta, d, K_dn, dn_idx, dn_val, delta);
  return 0;
}

// Model update line of Algorithm 2 on the K received pairs:
// w[i] = w[i] - alpha_out * val, one fused multiply-add.
int oracle_update(const uint32_t* idx, const float* val, uint64_t K, float alpha_out, float* w,
                  uint64_t d) {
  for (uint64_t j = 0; j < K; ++j) {
    if (idx[j] >= d) return -2;
    w[idx[j]] = std::fmaf(-alpha_out, val[j], w[idx[j]]);
  }
  return 0;
}

// One whole iteration of the loop body of Algorithm 2.
int oracle_bidir_step(const float* g, float* eps, float* delta, float* w, const float* p,
                      int32_t N, uint64_t d, uint64_t K_up, uint64_t K_dn, float alpha_in,
                      float alpha_out, uint32_t* up_idx, float* up_val, uint32_t* dn_idx,
                      float* dn_val, uint64_t* union_nnz, int32_t nthreads) {
  int rc = oracle_worker_stage(g, eps, N, d, alpha_in, K_up, up_idx, up_val, nthreads);
  if (rc) return rc;
  rc = oracle_aggregate(up_idx, up_val, p, N, K_up, delta, d, union_nnz);
  if (rc) return rc;
  rc = oracle_downlink(delta, d, K_dn, dn_idx, dn_val);
  if (rc) return rc;
  return oracle_update(dn_idx, dn_val, K_dn, alpha_out, w, d);
}

// One whole iteration of the loop body of Algorithm 1 (unidirectional Top_K SGD): the
// worker lines are those of Algorithm 2; the server forms g_t = sum_q p_q Top_K(a^q)
// (accumulator starts at +0, workers in ascending q, one fused multiply-add each) and
// sends it uncompressed; the workers apply w = w - alpha_out * g_t.  g_t is non-zero at
// most at the coordinates some uplink names, so the message is returned sparse: those
// coordinates in ascending order with their g_t values (dn_idx/dn_val need room for
// N*K_up pairs; *dn_count receives how many were written).
int oracle_unidir_step(const float* g, float* eps, float* w, const float* p, int32_t N,
                       uint64_t d, uint64_t K_up, float alpha_in, float alpha_out,
                       uint32_t* up_idx, float* up_val, uint32_t* dn_idx, float* dn_val,
                       uint64_t* dn_count, int32_t nthreads) {
  int rc = oracle_worker_stage(g, eps, N, d, alpha_in, K_up, up_idx, up_val, nthreads);
  if (rc) return rc;
  std::vector<float> gt(d, 0.0f);
  std::vector<uint8_t> named(d, 0);
  for (int q = 0; q < N; ++q) {
    for (uint64_t j = 0; j < K_up; ++j) {
      const uint32_t i = up_idx[(uint64_t)q * K_up + j];
      gt[i] = std::fmaf(p[q], up_val[(uint64_t)q * K_up + j], gt[i]);
      named[i] = 1;
    }
  }
  uint64_t n = 0;
  for (uint64_t i = 0; i < d; ++i) {
    if (!named[i]) continue;
    dn_idx[n] = static_cast<uint32_t>(i);
    dn_val[n] = gt[i];
    ++n;
    w[i] = std::fmaf(-alpha_out, gt[i], w[i]);
  }
  *dn_count = n;
  return 0;
}

// One iteration of Algorithm 2 together with the per-step estimates of the constants the
// paper measures in its section on convergence-bound constants:
//   rho      = |Top_K(delta_{t-1} + sum_q p_q a^q) - Top_K(delta_{t-1} + sum_q Top_K(p_q a^q))|_2
//              / |alpha_{t-1} sum_q p_q g^q|_2                       (left/right side of Assumption 5)
//   rho_hat  = |Top_K(sum_q p_q a^q) - sum_q Top_K(p_q a^q)|_2 / |alpha_{t-1} sum_q p_q g^q|_2
//                                                                    (Assumption 6, unidirectional)
//   1-gamma  = |Top_K(x) - x|_2^2 / |x|_2^2 for every compression of the step (x = a^q, x = g_t)
//   nnz      = distinct coordinates named by the uplinks / d          (communication section)
// The dense sums are fp32 fused multiply-add chains in ascending q (from +0, or from
// delta_{t-1}), Top_K(p_q a^q) is read as p_q Top_K(a^q) as in Algorithm 2, the second
// Top_K in rho is the step's own downlink message, the first uses K_dn and the one in
// rho_hat K_up.  Norms accumulate in fp64.
// diag: 8 + N doubles: rho, rho_hat, max(1-gamma), |alpha sum p g|, numerator of rho,
// numerator of rho_hat, nnz fraction, 1-gamma of the server, then 1-gamma of each worker.
int oracle_bidir_step_diag(const float* g, float* eps, float* delta, float* w, const float* p,
                           int32_t N, uint64_t d, uint64_t K_up, uint64_t K_dn, float alpha_in,
                           float alpha_out, uint32_t* up_idx, float* up_val, uint32_t* dn_idx,
                           float* dn_val, double* diag, int32_t nthreads) {
  if (N <= 0 || K_up > d || K_dn > d || K_up == 0 || K_dn == 0) return -1;
  std::vector<float> s(d, 0.0f), u(d, 0.0f), v(delta, delta + d);
  for (int q = 0; q < N; ++q) {
    const float* gq = g + (uint64_t)q * d;
    const float* eq = eps + (uint64_t)q * d;
    for (uint64_t i = 0; i < d; ++i) {
      const float a = std::fmaf(alpha_in, gq[i], eq[i]);
      s[i] = std::fmaf(p[q], gq[i], s[i]);
      u[i] = std::fmaf(p[q], a, u[i]);
      v[i] = std::fmaf(p[q], a, v[i]);
    }
  }
  uint64_t nnz = 0;
  int rc = oracle_bidir_step(g, eps, delta, w, p, N, d, K_up, K_dn, alpha_in, alpha_out, up_idx,
                             up_val, dn_idx, dn_val, &nnz, nthreads);
  if (rc) return rc;
  auto sq = [](double x) { return x * x; };
  // denominator
  double den = 0.0;
  for (uint64_t i = 0; i < d; ++i) den += sq((double)alpha_in * (double)s[i]);
  den = std::sqrt(den);
  // rho: Top_K(v) against the step's downlink message
  std::vector<uint32_t> ti(std::max(K_up, K_dn));
  std::vector<float> tv(std::max(K_up, K_dn));
  std::vector<double> dense(d, 0.0);
  topk_plain(v.data(), d, K_dn, ti.data(), tv.data(), nullptr);
  for (uint64_t j = 0; j < K_dn; ++j) dense[ti[j]] += tv[j];
  for (uint64_t j = 0; j < K_dn; ++j) dense[dn_idx[j]] -= dn_val[j];
  double num_rho = 0.0;
  for (uint64_t i = 0; i < d; ++i) num_rho += sq(dense[i]);
  num_rho = std::sqrt(num_rho);
  // rho_hat: Top_K(u) against sum_q p_q Top_K(a^q)
  std::vector<float> m(d, 0.0f);
  for (int q = 0; q < N; ++q)
    for (uint64_t j = 0; j < K_up; ++j) {
      const uint64_t at = (uint64_t)q * K_up + j;
      m[up_idx[at]] = std::fmaf(p[q], up_val[at], m[up_idx[at]]);
    }
  std::fill(dense.begin(), dense.end(), 0.0);
  topk_plain(u.data(), d, K_up, ti.data(), tv.data(), nullptr);
  for (uint64_t j = 0; j < K_up; ++j) dense[ti[j]] += tv[j];
  double num_hat = 0.0;
  for (uint64_t i = 0; i < d; ++i) num_hat += sq(dense[i] - (double)m[i]);
  num_hat = std::sqrt(num_hat);
  // 1 - gamma of every compression: residual energy over input energy
  double worst = 0.0;
  for (int q = 0; q < N; ++q) {
    double res = 0.0, sent = 0.0;
    for (uint64_t i = 0; i < d; ++i) res += sq(eps[(uint64_t)q * d + i]);
    for (uint64_t j = 0; j < K_up; ++j) sent += sq(up_val[(uint64_t)q * K_up + j]);
    const double r = res + sent > 0.0 ? res / (res + sent) : 0.0;
    diag[8 + q] = r;
    worst = std::max(worst, r);
  }
  {
    double res = 0.0, sent = 0.0;
    for (uint64_t i = 0; i < d; ++i) res += sq(delta[i]);
    for (uint64_t j = 0; j < K_dn; ++j) sent += sq(dn_val[j]);
    diag[7] = res + sent > 0.0 ? res / (res + sent) : 0.0;
    worst = std::max(worst, diag[7]);
  }
  diag[0] = den > 0.0 ? num_rho / den : 0.0;
  diag[1] = den > 0.0 ? num_hat / den : 0.0;
  diag[2] = worst;
  diag[3] = den;
  diag[4] = num_rho;
  diag[5] = num_hat;
  diag[6] = (double)nnz / (double)d;
  return 0;
}

}  // extern "C"
