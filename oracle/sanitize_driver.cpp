// Stand-alone driver that runs the CPU oracle under AddressSanitizer and
// UndefinedBehaviorSanitizer (host only; TEST INFRASTRUCTURE like the oracle itself).
//
// Built by oracle.build_sanitized() as one executable together with bts_oracle.cpp and run
// by tests/test_oracle_sanitizers.py.  It replays, through every exported function of the
// oracle, inputs chosen to reach the edges of its buffers:
//   1. Top_K against the selection rule written out by rank (a coordinate is kept iff fewer
//      than K coordinates precede it in the order "larger magnitude pattern first, lower
//      index first") for every d <= 7 over an alphabet with NaN, Inf, denormal, +0, -0 and
//      tied magnitudes, every K in 0..d;
//   2. a run of Algorithm 2 over several steps on dyadic inputs, where every fp32 operation
//      is exact, checked against the conservation identity of Lemma 1
//      (w_t - sum_q p_q eps_t^q - delta_t = w_0 - sum_s alpha sum_q p_q g_s^q) with == ;
//   3. one call each of the unidirectional step and of the step with diagnostics.
// Exit status 0 = all checks passed and no sanitizer report (reports abort the process).

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <limits>
#include <vector>

extern "C" {
int oracle_topk(const float* x, uint64_t d, uint64_t K, uint32_t* idx, float* val,
                float* residual);
int oracle_bidir_step(const float* g, float* eps, float* delta, float* w, const float* p,
                      int32_t N, uint64_t d, uint64_t K_up, uint64_t K_dn, float alpha_in,
                      float alpha_out, uint32_t* up_idx, float* up_val, uint32_t* dn_idx,
                      float* dn_val, uint64_t* union_nnz, int32_t nthreads);
int oracle_unidir_step(const float* g, float* eps, float* w, const float* p, int32_t N,
                       uint64_t d, uint64_t K_up, float alpha_in, float alpha_out,
                       uint32_t* up_idx, float* up_val, uint32_t* dn_idx, float* dn_val,
                       uint64_t* dn_count, int32_t nthreads);
int oracle_bidir_step_diag(const float* g, float* eps, float* delta, float* w, const float* p,
                           int32_t N, uint64_t d, uint64_t K_up, uint64_t K_dn, float alpha_in,
                           float alpha_out, uint32_t* up_idx, float* up_val, uint32_t* dn_idx,
                           float* dn_val, double* diag, int32_t nthreads);
}

namespace {

int failures = 0;

void fail(const char* what, long a, long b) {
  std::fprintf(stderr, "FAIL %s (%ld, %ld)\n", what, a, b);
  ++failures;
}

uint32_t bits(float x) {
  uint32_t u;
  std::memcpy(&u, &x, 4);
  return u;
}

float from_bits(uint32_t u) {
  float x;
  std::memcpy(&x, &u, 4);
  return x;
}

// 1. Top_K by rank on every vector of length d over the alphabet
long check_topk_exhaustive() {
  const float alphabet[] = {0.0f, -0.0f, 1.0f, -1.0f, 2.5f, from_bits(0x00000001u) /* denormal */,
                            std::numeric_limits<float>::infinity(), from_bits(0x7FC00001u) /* NaN */};
  const int A = sizeof(alphabet) / sizeof(alphabet[0]);
  long cases = 0;
  for (int d = 1; d <= 7; ++d) {
    long combos = 1;
    for (int i = 0; i < d; ++i) combos *= A;
    const long stride = combos > 4096 ? combos / 4096 : 1;   // a spread of at most ~4096 vectors
    for (long code = 0; code < combos; code += stride) {
      std::vector<float> x(d);
      long c = code;
      for (int i = 0; i < d; ++i) {
        x[i] = alphabet[c % A];
        c /= A;
      }
      for (int K = 0; K <= d; ++K) {
        std::vector<uint32_t> idx(K);
        std::vector<float> val(K), res(d);
        if (oracle_topk(x.data(), d, K, idx.data(), val.data(), res.data()) != 0)
          fail("oracle_topk rc", d, K);
        int out = 0;
        for (int i = 0; i < d; ++i) {
          int before = 0;
          for (int j = 0; j < d; ++j) {
            const uint32_t ki = bits(x[i]) & 0x7FFFFFFFu, kj = bits(x[j]) & 0x7FFFFFFFu;
            if (kj > ki || (kj == ki && j < i)) ++before;
          }
          const bool kept = before < K;
          if (kept) {
            if (out >= K || idx[out] != (uint32_t)i || bits(val[out]) != bits(x[i]))
              fail("kept coordinate", code, K);
            if (bits(res[i]) != 0u) fail("residual at a kept coordinate", code, K);
            ++out;
          } else if (bits(res[i]) != bits(x[i])) {
            fail("residual elsewhere", code, K);
          }
        }
        if (out != K) fail("count", code, K);
        ++cases;
      }
    }
  }
  return cases;
}

// 2. Lemma 1 on dyadic inputs: small integers / 8 as gradients, p_q = 1/4, alpha = 1/4
void check_lemma1() {
  const int N = 4, T = 6;
  const uint64_t d = 37, K_up = 5, K_dn = 3;
  const float alpha = 0.25f;
  std::vector<float> p(N, 0.25f), eps(N * d, 0.0f), delta(d, 0.0f), w(d), w0(d);
  std::vector<double> drift(d, 0.0);
  uint32_t s = 12345u;
  auto next = [&]() {
    s = s * 1664525u + 1013904223u;
    return (int)((s >> 20) % 33) - 16;
  };
  for (uint64_t i = 0; i < d; ++i) w0[i] = w[i] = (float)next() / 4.0f;
  std::vector<float> g(N * d);
  std::vector<uint32_t> ui(N * K_up), di(K_dn);
  std::vector<float> uv(N * K_up), dv(K_dn);
  for (int t = 0; t < T; ++t) {
    for (auto& v : g) v = (float)next() / 8.0f;
    uint64_t nnz = 0;
    if (oracle_bidir_step(g.data(), eps.data(), delta.data(), w.data(), p.data(), N, d, K_up, K_dn,
                          alpha, 1.0f, ui.data(), uv.data(), di.data(), dv.data(), &nnz, 2) != 0)
      fail("oracle_bidir_step rc", t, 0);
    if (nnz > (uint64_t)N * K_up) fail("union nnz bound", t, (long)nnz);
    for (uint64_t i = 0; i < d; ++i) {
      double sum = 0.0;
      for (int q = 0; q < N; ++q) sum += 0.25 * (double)g[q * d + i];
      drift[i] += (double)alpha * sum;
      double corrected = (double)w[i] - (double)delta[i];
      for (int q = 0; q < N; ++q) corrected -= 0.25 * (double)eps[q * d + i];
      if (corrected != (double)w0[i] - drift[i]) fail("Lemma 1", t, (long)i);
    }
  }
}

// 3. the other entry points, for their memory accesses
void touch_other_entry_points() {
  const int N = 3;
  const uint64_t d = 29, K_up = 4, K_dn = 2;
  std::vector<float> g(N * d), eps(N * d, 0.0f), delta(d, 0.0f), w(d, 1.0f), p(N, 1.0f / 3.0f);
  for (uint64_t i = 0; i < N * d; ++i) g[i] = std::sin((float)i) * (float)(1 + i % 5);
  std::vector<uint32_t> ui(N * K_up), di(N * K_up);
  std::vector<float> uv(N * K_up), dv(N * K_up);
  uint64_t cnt = 0;
  if (oracle_unidir_step(g.data(), eps.data(), w.data(), p.data(), N, d, K_up, 0.1f, 1.0f,
                         ui.data(), uv.data(), di.data(), dv.data(), &cnt, 3) != 0 ||
      cnt == 0 || cnt > N * K_up)
    fail("oracle_unidir_step", (long)cnt, 0);
  std::vector<double> diag(8 + N, -1.0);
  if (oracle_bidir_step_diag(g.data(), eps.data(), delta.data(), w.data(), p.data(), N, d, K_up,
                             K_dn, 0.1f, 1.0f, ui.data(), uv.data(), di.data(), dv.data(),
                             diag.data(), 1) != 0)
    fail("oracle_bidir_step_diag rc", 0, 0);
  for (double v : diag)
    if (!(v >= 0.0)) fail("diagnostic not set", 0, 0);
}

}  // namespace

int main() {
  const long cases = check_topk_exhaustive();
  check_lemma1();
  touch_other_entry_points();
  std::printf("sanitized oracle run: %ld Top_K cases, Lemma 1 run, %d failures\n", cases, failures);
  return failures == 0 ? 0 : 1;
}
