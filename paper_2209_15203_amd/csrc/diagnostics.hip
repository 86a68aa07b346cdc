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

// Workers in ascending q.  VEC = 4 when d is a multiple of 4 (every row start is then
// 16-byte aligned): a thread owns TILE groups of 4 consecutive coordinates, one workgroup a
// span of TILE * 1024 consecutive coordinates, so that for each worker it reads TILE * 4 KB
// in one piece from g and from eps (2 * TILE 16-byte loads per lane in flight; TILE = 4
// without unrolling over the workers was the best of a sweep over TILE 1-4, unrolling 1-8 and
// 1024-4096 workgroups: 9.6 ms for 64 workers x 1.1e8 coordinates, 5.9 TB/s).  VEC = 1: one
// coordinate per thread.
constexpr int kDiagTile = 4;

template <int VEC, int TILE>
__global__ __launch_bounds__(kBlock) void k_diag_dense(
    const float* __restrict__ g, const float* __restrict__ eps, const float* __restrict__ delta,
    const float* __restrict__ p, uint32_t N, uint64_t d, float alpha, float* __restrict__ u_out,
    float* __restrict__ v_out, double* __restrict__ part_s2) {
  __shared__ double lds[kBlock / kWave];
  double s2 = 0.0;
  constexpr uint64_t kSpan = (uint64_t)TILE * kBlock * VEC;       // coordinates per workgroup pass
  for (uint64_t base = (uint64_t)blockIdx.x * kSpan; base < d; base += (uint64_t)gridDim.x * kSpan) {
    float s[TILE][VEC], u[TILE][VEC], v[TILE][VEC];
    uint64_t at[TILE];
    bool in[TILE];
#pragma unroll
    for (int t = 0; t < TILE; ++t) {
      at[t] = base + ((uint64_t)t * kBlock + threadIdx.x) * VEC;
      in[t] = at[t] + VEC <= d;                                  // d % VEC == 0
#pragma unroll
      for (int j = 0; j < VEC; ++j) {
        s[t][j] = 0.0f;
        u[t][j] = 0.0f;
        v[t][j] = in[t] ? delta[at[t] + j] : 0.0f;
      }
    }
#pragma unroll 1
    for (uint32_t q = 0; q < N; ++q) {
      float gq[TILE][VEC], eq[TILE][VEC];
#pragma unroll
      for (int t = 0; t < TILE; ++t) {
        if (!in[t]) continue;
        const uint64_t e = (uint64_t)q * d + at[t];
        if (VEC == 4) {
          const f4 gv = __builtin_nontemporal_load(reinterpret_cast<const f4*>(g + e));
          const f4 ev = __builtin_nontemporal_load(reinterpret_cast<const f4*>(eps + e));
          gq[t][0] = gv.x; gq[t][1 % VEC] = gv.y; gq[t][2 % VEC] = gv.z; gq[t][3 % VEC] = gv.w;
          eq[t][0] = ev.x; eq[t][1 % VEC] = ev.y; eq[t][2 % VEC] = ev.z; eq[t][3 % VEC] = ev.w;
        } else {
          gq[t][0] = g[e];
          eq[t][0] = eps[e];
        }
      }
      const float pq = p[q];
#pragma unroll
      for (int t = 0; t < TILE; ++t) {
        if (!in[t]) continue;
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
          const float a = __fmaf_rn(alpha, gq[t][j], eq[t][j]);
          s[t][j] = __fmaf_rn(pq, gq[t][j], s[t][j]);
          u[t][j] = __fmaf_rn(pq, a, u[t][j]);
          v[t][j] = __fmaf_rn(pq, a, v[t][j]);
        }
      }
    }
#pragma unroll
    for (int t = 0; t < TILE; ++t) {
      if (!in[t]) continue;
#pragma unroll
      for (int j = 0; j < VEC; ++j) {
        u_out[at[t] + j] = u[t][j];
        v_out[at[t] + j] = v[t][j];
        s2 += (double)s[t][j] * (double)s[t][j];
      }
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
// 16-byte loads where the row allows it, four independent accumulators; launched with 1024
// threads per block on the dense rows (the grid is only kRowParts blocks wide) and 256 on
// the messages.  only (nullable): rows whose word is zero are left alone.
__global__ __launch_bounds__(1024) void k_rows_sumsq(const float* __restrict__ x, uint64_t len,
                                                     double* __restrict__ part,
                                                     const uint32_t* __restrict__ only) {
  __shared__ double lds[1024 / kWave];
  if (only != nullptr && only[blockIdx.y] == 0) return;
  const float* row = x + (uint64_t)blockIdx.y * len;
  double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
  const uint64_t tid = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const uint64_t nthr = (uint64_t)gridDim.x * blockDim.x;
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
    for (uint64_t i = threadIdx.x; i < head; i += blockDim.x) a0 += (double)row[i] * (double)row[i];
    for (uint64_t i = head + nvec * 4 + threadIdx.x; i < len; i += blockDim.x)
      a1 += (double)row[i] * (double)row[i];
  }
  const double t = block_sum_f64((a0 + a1) + (a2 + a3), lds);
  if (threadIdx.x == 0) part[(uint64_t)blockIdx.y * kRowParts + blockIdx.x] = t;
}

// Residual energy of each worker row from the partial sums the single-pass select left
// behind: per wave chunk the squares of the coordinates it did not capture, per directory
// tile the squares of the captured entries it did not keep.  Block b of a row adds up the
// slots b, b + kRowParts, ... of both arrays (thread-strided, then the block's tree: a
// fixed order) into the row's partial sum b.  Rows the select handed to the dense path are
// skipped (k_rows_sumsq sums those from eps).
__global__ __launch_bounds__(kBlock) void k_row_energy(const double* __restrict__ chunks,
                                                       const double* __restrict__ tiles,
                                                       uint32_t nwc_pad, uint32_t ntiles,
                                                       const uint32_t* __restrict__ need,
                                                       double* __restrict__ part) {
  __shared__ double lds[kBlock / kWave];
  const uint32_t row = blockIdx.y;
  if (need[row] != 0) return;
  double acc = 0.0;
  const uint32_t first = blockIdx.x * kBlock + threadIdx.x, step = kRowParts * kBlock;
  const double* c = chunks + (uint64_t)row * nwc_pad;
  for (uint32_t i = first; i < nwc_pad; i += step) acc += c[i];
  const double* t = tiles + (uint64_t)row * ntiles;
  for (uint32_t i = first; i < ntiles; i += step) acc += t[i];
  const double total = block_sum_f64(acc, lds);
  if (threadIdx.x == 0) part[(uint64_t)row * kRowParts + blockIdx.x] = total;
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
    k_diag_dense<4, kDiagTile><<<dim3(kParts), dim3(kBlock), 0, s>>>(g, eps, delta, p, N, d, alpha,
                                                                     ds.u, ds.v, ds.part);
  else
    k_diag_dense<1, 1><<<dim3(kParts), dim3(kBlock), 0, s>>>(g, eps, delta, p, N, d, alpha, ds.u,
                                                             ds.v, ds.part);
  return hipGetLastError();
}

hipError_t diag_after_step(hipStream_t s, const DiagScratch& ds, const DenseScratch& dense,
                           const float* eps, const float* delta, const float* p, uint32_t N,
                           uint64_t d, uint32_t K_up, uint32_t K_dn, float alpha,
                           const uint32_t* up_idx, const float* up_val, const uint32_t* dn_idx,
                           const float* dn_val, const AggScratch& agg, const RowEnergy& energy,
                           const OneRowSelect& sel_v, const OneRowSelect& sel_u, double* diag) {
  double* part = ds.part;
  double* p_rho = part + kParts;
  double* p_hat = part + 2 * kParts;
  double* p_res = part + 3 * kParts;
  double* p_sent = p_res + (uint64_t)N * kRowParts;
  double* p_sres = p_sent + (uint64_t)N * kRowParts;
  double* p_ssent = p_sres + kRowParts;
  // A = Top_{K_dn}(v), C = Top_{K_up}(u): the single-pass select where the shape prefers it
  auto select_row = [&](const OneRowSelect& os, float* x, uint32_t K, uint32_t* idx, float* val) {
    if (os.plan != nullptr && os.plan->enabled && os.plan->preferred)
      return fast_select(s, *os.scratch, *os.plan, nullptr, x, 1, d, K, 0.0f, idx, val, nullptr,
                         nullptr, dense, false);
    return dense_select(s, dense, nullptr, x, 1, d, K, 0.0f, idx, val, nullptr, false, nullptr,
                        nullptr);
  };
  hipError_t e = select_row(sel_v, ds.v, K_dn, ds.a_idx, ds.a_val);
  if (e != hipSuccess) return e;
  e = select_row(sel_u, ds.u, K_up, ds.c_idx, ds.c_val);
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
  if (energy.chunks != nullptr) {
    // the select's dense pass already summed what it left behind; only rows it handed to
    // the dense path (rare) are read again
    k_row_energy<<<dim3(kRowParts, N), dim3(kBlock), 0, s>>>(energy.chunks, energy.tiles, energy.nwc_pad,
                                                  energy.ntiles, energy.need, p_res);
    BTS_LAUNCH_CHECK();
    k_rows_sumsq<<<dim3(kRowParts, N), dim3(1024), 0, s>>>(eps, d, p_res, energy.need);
  } else {
    k_rows_sumsq<<<dim3(kRowParts, N), dim3(1024), 0, s>>>(eps, d, p_res, nullptr);
  }
  BTS_LAUNCH_CHECK();
  k_rows_sumsq<<<dim3(kRowParts, N), dim3(kBlock), 0, s>>>(up_val, K_up, p_sent, nullptr);
  BTS_LAUNCH_CHECK();
  k_rows_sumsq<<<dim3(kRowParts, 1), dim3(1024), 0, s>>>(delta, d, p_sres, nullptr);
  BTS_LAUNCH_CHECK();
  k_rows_sumsq<<<dim3(kRowParts, 1), dim3(kBlock), 0, s>>>(dn_val, K_dn, p_ssent, nullptr);
  BTS_LAUNCH_CHECK();
  k_diag_finish<<<dim3(1), dim3(kBlock), 0, s>>>(part, N, d, alpha, ds.m_cnt, diag);
  BTS_LAUNCH_CHECK();
  return hipSuccess;
}

}  // namespace bts
