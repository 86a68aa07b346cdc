// Per-step estimates of the constants the paper measures (section on convergence-bound
// constants): rho (Assumption 5), rho_hat (Assumption 6), 1 - gamma (Assumption 2 / Eq.
// "topk_bound") and the fraction of coordinates named by the uplinks (communication
// section).  Not part of the hot path: one extra dense read of g and eps before the step
// and O(d + N K) work after it.
//
//   before the step   s = sum_q p_q g^q,  u = sum_q p_q a^q,  v = delta_{t-1} + sum_q p_q a^q
//                     with a^q = fma(alpha, g^q, eps^q); fp32 fma chains in ascending q.
//   after the step    A = Top_{K_dn}(v), C = Top_{K_up}(u) (dense select on the scratch rows),
//                     m = sum_q p_q Top_K(a^q) as a sparse list,
//                     rho = |A - b| / |alpha s|, rho_hat = |C - m| / |alpha s| with b the
//                     step's downlink message; 1 - gamma = |residual|^2 / (|residual|^2 +
//                     |sent|^2) for every worker row and for the server.
// All norms accumulate in fp64 (per-block partial sums, summed by one finishing block).

#include "bts_device.h"

namespace bts {

namespace {

constexpr int kParts = 1024;     // partial sums per dense quantity
constexpr int kRowParts = 256;   // partial sums per row quantity

__device__ __forceinline__ double block_sum_f64(double v, double* lds) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  const int w = threadIdx.x / kWave, nw = blockDim.x / kWave;
  if (lane_id() == 0) lds[w] = v;
  __syncthreads();
  double t = 0.0;
  if (threadIdx.x == 0)
    for (int i = 0; i < nw; ++i) t += lds[i];
  __syncthreads();
  return t;      // valid in thread 0
}

// One thread per VEC consecutive coordinates (4 when d is a multiple of 4, so that every
// row start is 16-byte aligned; else 1), workers in ascending q.
template <int VEC>
__global__ __launch_bounds__(kBlock) void k_diag_dense(
    const float* __restrict__ g, const float* __restrict__ eps, const float* __restrict__ delta,
    const float* __restrict__ p, uint32_t N, uint64_t d, float alpha, float* __restrict__ u_out,
    float* __restrict__ v_out, double* __restrict__ part_s2) {
  __shared__ double lds[kBlock / kWave];
  double s2 = 0.0;
  const uint64_t groups = d / VEC;
  for (uint64_t gi = (uint64_t)blockIdx.x * kBlock + threadIdx.x; gi < groups;
       gi += (uint64_t)gridDim.x * kBlock) {
    const uint64_t i = gi * VEC;
    float s[VEC], u[VEC], v[VEC];
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
      s[j] = 0.0f;
      u[j] = 0.0f;
      v[j] = delta[i + j];
    }
#pragma unroll 4
    for (uint32_t q = 0; q < N; ++q) {
      float gq[VEC], eq[VEC];
      if (VEC == 4) {
        const uint64_t at = (uint64_t)q * d + i;
        const f4 gv = __builtin_nontemporal_load(reinterpret_cast<const f4*>(g + at));
        const f4 ev = __builtin_nontemporal_load(reinterpret_cast<const f4*>(eps + at));
        gq[0] = gv.x; gq[1 % VEC] = gv.y; gq[2 % VEC] = gv.z; gq[3 % VEC] = gv.w;
        eq[0] = ev.x; eq[1 % VEC] = ev.y; eq[2 % VEC] = ev.z; eq[3 % VEC] = ev.w;
      } else {
        gq[0] = g[(uint64_t)q * d + i];
        eq[0] = eps[(uint64_t)q * d + i];
      }
      const float pq = p[q];
#pragma unroll
      for (int j = 0; j < VEC; ++j) {
        const float a = __fmaf_rn(alpha, gq[j], eq[j]);
        s[j] = __fmaf_rn(pq, gq[j], s[j]);
        u[j] = __fmaf_rn(pq, a, u[j]);
        v[j] = __fmaf_rn(pq, a, v[j]);
      }
    }
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
      u_out[i + j] = u[j];
      v_out[i + j] = v[j];
      s2 += (double)s[j] * (double)s[j];
    }
  }
  const double t = block_sum_f64(s2, lds);
  if (threadIdx.x == 0) part_s2[blockIdx.x] = t;
}

// Squared distance of two sparse vectors given as ascending (index, value) lists.
// nb may come from a device counter (nb_dev != nullptr).
__global__ __launch_bounds__(kBlock) void k_sparse_dist2(
    const uint32_t* __restrict__ ia, const float* __restrict__ va, uint32_t na,
    const uint32_t* __restrict__ ib, const float* __restrict__ vb, uint32_t nb_host,
    const uint32_t* __restrict__ nb_dev, double* __restrict__ part) {
  __shared__ double lds[kBlock / kWave];
  const uint32_t nb = nb_dev != nullptr ? *nb_dev : nb_host;
  double acc = 0.0;
  for (uint64_t t = (uint64_t)blockIdx.x * kBlock + threadIdx.x; t < (uint64_t)na + nb;
       t += (uint64_t)gridDim.x * kBlock) {
    const bool from_a = t < na;
    const uint32_t j = from_a ? (uint32_t)t : (uint32_t)(t - na);
    const uint32_t key = from_a ? ia[j] : ib[j];
    const uint32_t* other = from_a ? ib : ia;
    const uint32_t n_other = from_a ? nb : na;
    uint32_t lo = 0, hi = n_other;
    while (lo < hi) {
      const uint32_t mid = lo + ((hi - lo) >> 1);
      if (other[mid] < key) lo = mid + 1; else hi = mid;
    }
    const bool found = lo < n_other && other[lo] == key;
    if (from_a) {
      const double diff = (double)va[j] - (found ? (double)vb[lo] : 0.0);
      acc += diff * diff;
    } else if (!found) {
      acc += (double)vb[j] * (double)vb[j];
    }
  }
  const double t = block_sum_f64(acc, lds);
  if (threadIdx.x == 0) part[blockIdx.x] = t;
}

// Sum of squares of each row of a rows x len matrix: kRowParts partial sums per row.
// 16-byte loads where the row allows it, four independent accumulators.
__global__ __launch_bounds__(kBlock) void k_rows_sumsq(const float* __restrict__ x, uint64_t len,
                                                       double* __restrict__ part) {
  __shared__ double lds[kBlock / kWave];
  const float* row = x + (uint64_t)blockIdx.y * len;
  double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
  const uint64_t tid = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  const uint64_t nthr = (uint64_t)gridDim.x * kBlock;
  // scalar head up to the first 16-byte boundary, vector body, scalar tail
  const uint64_t mis = (reinterpret_cast<uintptr_t>(row) >> 2) & 3u;
  const uint64_t head = min(len, (4 - mis) & 3u);
  const uint64_t nvec = (len - head) / 4;
  const f4* body = reinterpret_cast<const f4*>(row + head);
  for (uint64_t i = tid; i < nvec; i += nthr) {
    const f4 t = __builtin_nontemporal_load(body + i);
    a0 += (double)t.x * (double)t.x;
    a1 += (double)t.y * (double)t.y;
    a2 += (double)t.z * (double)t.z;
    a3 += (double)t.w * (double)t.w;
  }
  if (blockIdx.x == 0) {
    for (uint64_t i = threadIdx.x; i < head; i += kBlock) a0 += (double)row[i] * (double)row[i];
    for (uint64_t i = head + nvec * 4 + threadIdx.x; i < len; i += kBlock)
      a1 += (double)row[i] * (double)row[i];
  }
  const double t = block_sum_f64((a0 + a1) + (a2 + a3), lds);
  if (threadIdx.x == 0) part[(uint64_t)blockIdx.y * kRowParts + blockIdx.x] = t;
}

// diag: rho, rho_hat, max(1-gamma), |alpha s|, |A - b|, |C - m|, nnz fraction,
// 1-gamma of the server, then 1-gamma of each worker.
__global__ __launch_bounds__(kBlock) void k_diag_finish(const double* __restrict__ part,
                                                        uint32_t N, uint64_t d, float alpha,
                                                        const uint32_t* __restrict__ m_cnt,
                                                        double* __restrict__ diag) {
  __shared__ double lds[kBlock / kWave];
  __shared__ double s_val[3];
  const double* p_s2 = part;
  const double* p_rho = part + kParts;
  const double* p_hat = part + 2 * kParts;
  const double* p_res = part + 3 * kParts;                       // N rows
  const double* p_sent = p_res + (uint64_t)N * kRowParts;        // N rows
  const double* p_sres = p_sent + (uint64_t)N * kRowParts;       // server
  const double* p_ssent = p_sres + kRowParts;
  for (int which = 0; which < 3; ++which) {
    const double* src = which == 0 ? p_s2 : (which == 1 ? p_rho : p_hat);
    double acc = 0.0;
    for (int i = threadIdx.x; i < kParts; i += kBlock) acc += src[i];
    const double t = block_sum_f64(acc, lds);
    if (threadIdx.x == 0) s_val[which] = t;
  }
  __syncthreads();
  double worst = 0.0;
  for (uint32_t q = threadIdx.x; q <= N; q += kBlock) {          // q == N: the server
    const double* r = q < N ? p_res + (uint64_t)q * kRowParts : p_sres;
    const double* s = q < N ? p_sent + (uint64_t)q * kRowParts : p_ssent;
    double res = 0.0, sent = 0.0;
    for (int i = 0; i < kRowParts; ++i) {
      res += r[i];
      sent += s[i];
    }
    const double ratio = res + sent > 0.0 ? res / (res + sent) : 0.0;
    diag[q < N ? 8 + q : 7] = ratio;
    worst = fmax(worst, ratio);
  }
  // max over threads
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) worst = fmax(worst, __shfl_xor(worst, o, kWave));
  if (lane_id() == 0) lds[threadIdx.x / kWave] = worst;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int i = 0; i < kBlock / kWave; ++i) worst = fmax(worst, lds[i]);
    const double den = fabs((double)alpha) * sqrt(s_val[0]);
    const double num_rho = sqrt(s_val[1]), num_hat = sqrt(s_val[2]);
    diag[0] = den > 0.0 ? num_rho / den : 0.0;
    diag[1] = den > 0.0 ? num_hat / den : 0.0;
    diag[2] = worst;
    diag[3] = den;
    diag[4] = num_rho;
    diag[5] = num_hat;
    diag[6] = (double)(*m_cnt) / (double)d;
  }
}

#define BTS_LAUNCH_CHECK()                       \
  do {                                           \
    hipError_t e_ = hipGetLastError();           \
    if (e_ != hipSuccess) return e_;             \
  } while (0)

}  // namespace

size_t diag_part_doubles(uint32_t N) {
  return 3ull * kParts + 2ull * N * kRowParts + 2ull * kRowParts;
}

hipError_t diag_before_step(hipStream_t s, const DiagScratch& ds, const float* g,
                            const float* eps, const float* delta, const float* p, uint32_t N,
                            uint64_t d, float alpha) {
  const bool vec = d % 4 == 0 && (reinterpret_cast<uintptr_t>(g) & 15u) == 0 &&
                   (reinterpret_cast<uintptr_t>(eps) & 15u) == 0;
  if (vec)
    k_diag_dense<4><<<dim3(kParts), dim3(kBlock), 0, s>>>(g, eps, delta, p, N, d, alpha, ds.u,
                                                          ds.v, ds.part);
  else
    k_diag_dense<1><<<dim3(kParts), dim3(kBlock), 0, s>>>(g, eps, delta, p, N, d, alpha, ds.u,
                                                          ds.v, ds.part);
  return hipGetLastError();
}

hipError_t diag_after_step(hipStream_t s, const DiagScratch& ds, const DenseScratch& dense,
                           const float* eps, const float* delta, const float* p, uint32_t N,
                           uint64_t d, uint32_t K_up, uint32_t K_dn, float alpha,
                           const uint32_t* up_idx, const float* up_val, const uint32_t* dn_idx,
                           const float* dn_val, const AggScratch& agg, double* diag) {
  double* part = ds.part;
  double* p_rho = part + kParts;
  double* p_hat = part + 2 * kParts;
  double* p_res = part + 3 * kParts;
  double* p_sent = p_res + (uint64_t)N * kRowParts;
  double* p_sres = p_sent + (uint64_t)N * kRowParts;
  double* p_ssent = p_sres + kRowParts;
  // A = Top_{K_dn}(v), C = Top_{K_up}(u)
  hipError_t e = dense_select(s, dense, nullptr, ds.v, 1, d, K_dn, 0.0f, ds.a_idx, ds.a_val,
                              nullptr, false, nullptr, nullptr);
  if (e != hipSuccess) return e;
  e = dense_select(s, dense, nullptr, ds.u, 1, d, K_up, 0.0f, ds.c_idx, ds.c_val, nullptr, false,
                   nullptr, nullptr);
  if (e != hipSuccess) return e;
  // m = sum_q p_q Top_K(a^q), sparse
  e = aggregate_update_unidirectional(s, up_idx, up_val, p, N, K_up, nullptr, d, 0.0f, ds.m_idx,
                                      ds.m_val, ds.m_cnt, agg);
  if (e != hipSuccess) return e;
  k_sparse_dist2<<<dim3(kParts), dim3(kBlock), 0, s>>>(ds.a_idx, ds.a_val, K_dn, dn_idx, dn_val,
                                                       K_dn, nullptr, p_rho);
  BTS_LAUNCH_CHECK();
  k_sparse_dist2<<<dim3(kParts), dim3(kBlock), 0, s>>>(ds.c_idx, ds.c_val, K_up, ds.m_idx,
                                                       ds.m_val, 0, ds.m_cnt, p_hat);
  BTS_LAUNCH_CHECK();
  k_rows_sumsq<<<dim3(kRowParts, N), dim3(kBlock), 0, s>>>(eps, d, p_res);
  BTS_LAUNCH_CHECK();
  k_rows_sumsq<<<dim3(kRowParts, N), dim3(kBlock), 0, s>>>(up_val, K_up, p_sent);
  BTS_LAUNCH_CHECK();
  k_rows_sumsq<<<dim3(kRowParts, 1), dim3(kBlock), 0, s>>>(delta, d, p_sres);
  BTS_LAUNCH_CHECK();
  k_rows_sumsq<<<dim3(kRowParts, 1), dim3(kBlock), 0, s>>>(dn_val, K_dn, p_ssent);
  BTS_LAUNCH_CHECK();
  k_diag_finish<<<dim3(1), dim3(kBlock), 0, s>>>(part, N, d, alpha, ds.m_cnt, diag);
  BTS_LAUNCH_CHECK();
  return hipSuccess;
}

}  // namespace bts
