// Server side of Algorithm 2 apart from the compression: the weighted aggregation
//     g_t = sum_q p_q Top_K(a^q) + delta_{t-1}
// and the model update  w_t = w_{t-1} - Top_K(g_t)  on the received pairs.
//
// Aggregation is deterministic without float atomics: the coordinate axis is cut into
// ranges of kAggWidth coordinates, one workgroup owns a range, and inside it the workers
// are applied one after the other in ascending q (a worker never names a coordinate twice,
// so the pairs of one worker are applied in parallel; a workgroup barrier separates
// consecutive workers).  Each worker's pairs that fall into the range are found by binary
// search in its sorted index list.  The range's pairs are staged in LDS and the touched
// part of delta is gathered into an LDS accumulator first, so that the N dependent
// rounds run at LDS latency instead of HBM latency.

#include "bts_device.h"

namespace bts {

namespace {

constexpr int kAggBlock = 256;
constexpr int kAggTile = 256;          // workers whose range bounds are held in LDS at a time
constexpr uint32_t kAggWidth = 4096;   // coordinates per range
constexpr uint32_t kAggStage = 1024;   // pairs staged in LDS at a time

__device__ __forceinline__ uint32_t lower_bound_u32(const uint32_t* __restrict__ a, uint32_t n,
                                                    uint32_t key) {
  uint32_t lo = 0, hi = n;
  while (lo < hi) {
    const uint32_t mid = lo + ((hi - lo) >> 1);
    if (a[mid] < key) lo = mid + 1; else hi = mid;
  }
  return lo;
}

// Where each worker's sorted index list enters and leaves each range: pair j of worker q
// opens range r if its predecessor lies in another range and closes it if its successor
// does.  The table is all zero between calls (the aggregation clears what it reads).
__global__ void k_range_bounds(const uint32_t* __restrict__ up_idx, uint32_t N, uint32_t K_up,
                               uint64_t d, uint32_t* __restrict__ start,
                               uint32_t* __restrict__ end) {
  const uint32_t q = blockIdx.y;
  const uint32_t j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= K_up) return;
  const uint32_t* row = up_idx + (uint64_t)q * K_up;
  if (row[j] >= d) return;                       // invalid input never reaches the table
  const uint32_t r = row[j] / kAggWidth;
  if (j == 0 || row[j - 1] / kAggWidth != r) start[(uint64_t)r * N + q] = j;
  if (j + 1 == K_up || row[j + 1] / kAggWidth != r) end[(uint64_t)r * N + q] = j + 1;
}

// MODE 0: bidirectional server (Algorithm 2): delta[i] = delta[i] + sum_q p_q v_q[i].
// MODE 1: count the distinct coordinates named in each range and nothing else.
// MODE 2: unidirectional server and update (Algorithm 1): g_t[i] = sum_q p_q v_q[i] from +0,
//         the named coordinates and their g_t written in ascending order to the message at
//         range_off[range] + rank, and w[i] = fma(-alpha_out, g_t[i], w[i]).
template <int MODE>
__global__ __launch_bounds__(kAggBlock) void k_aggregate(
    const uint32_t* __restrict__ up_idx, const float* __restrict__ up_val,
    const float* __restrict__ p, uint32_t N, uint32_t K_up, float* __restrict__ dense,
    uint64_t d, uint32_t* __restrict__ range_nnz, uint32_t* __restrict__ tab_start,
    uint32_t* __restrict__ tab_end, const uint32_t* __restrict__ range_off, float neg_alpha,
    uint32_t* __restrict__ msg_idx, float* __restrict__ msg_val) {
  __shared__ float acc[kAggWidth];                  // g_t of the touched coordinates
  __shared__ uint32_t touched[kAggWidth / 32];
  __shared__ uint32_t s_lo[kAggTile], s_pref[kAggTile + 1];
  __shared__ float s_p[kAggTile];
  __shared__ uint32_t e_rel[kAggStage];
  __shared__ float e_val[kAggStage];
  __shared__ uint32_t lds[kAggBlock / kWave + 1];
  const uint64_t c0 = (uint64_t)blockIdx.x * kAggWidth;
  const uint64_t c1 = min(c0 + (uint64_t)kAggWidth, d);
  for (uint32_t i = threadIdx.x; i < kAggWidth / 32; i += kAggBlock) touched[i] = 0;
  uint32_t fresh = 0;
  for (uint32_t q0 = 0; q0 < N; q0 += kAggTile) {
    const uint32_t nq = min((uint32_t)kAggTile, N - q0);
    // where each worker of the tile enters and leaves the range
    uint32_t lo = 0, n = 0;
    if (threadIdx.x < nq) {
      if (tab_start != nullptr) {
        const uint64_t at = (uint64_t)blockIdx.x * N + q0 + threadIdx.x;
        lo = tab_start[at];
        const uint32_t hi = tab_end[at];
        n = (hi > lo && hi <= K_up) ? hi - lo : 0u;
        if (MODE != 1 && hi) {                               // leave the table clear
          tab_start[at] = 0;
          tab_end[at] = 0;
        }
      } else {
        const uint32_t* row = up_idx + (uint64_t)(q0 + threadIdx.x) * K_up;
        lo = lower_bound_u32(row, K_up, (uint32_t)c0);
        n = lower_bound_u32(row, K_up, (uint32_t)c1) - lo;   // c1 <= d < 2^32
      }
      s_p[threadIdx.x] = p[q0 + threadIdx.x];
    }
    uint32_t total;
    const uint32_t pref = block_exclusive_scan(n, lds, &total);   // barriers inside
    s_lo[threadIdx.x] = lo;
    s_pref[threadIdx.x] = pref;
    if (threadIdx.x == kAggBlock - 1) s_pref[kAggTile] = total;
    __syncthreads();
    // the tile's pairs in (q, index) order, kAggStage at a time
    uint32_t t_first = 0;                                   // first worker of the stage
    for (uint32_t e0 = 0; e0 < total; e0 += kAggStage) {
      const uint32_t e1 = min(e0 + kAggStage, total);
      for (uint32_t e = e0 + threadIdx.x; e < e1; e += kAggBlock) {
        // worker of pair e: the last t with s_pref[t] <= e
        uint32_t a = 0, b = nq;
        while (b - a > 1) {
          const uint32_t m = (a + b) >> 1;
          if (s_pref[m] <= e) a = m; else b = m;
        }
        const uint64_t src = (uint64_t)(q0 + a) * K_up + s_lo[a] + (e - s_pref[a]);
        const uint32_t i = up_idx[src];
        uint32_t rel = 0xFFFFFFFFu;
        if (i >= c0 && i < c1) {                             // always true for sorted input
          rel = i - (uint32_t)c0;
          const uint32_t bit = 1u << (rel & 31);
          const uint32_t old = atomicOr(&touched[rel >> 5], bit);
          if (!(old & bit)) {                                // first touch: start value
            if (MODE == 0) acc[rel] = dense[i];
            if (MODE == 2) acc[rel] = 0.0f;
            ++fresh;
          }
        }
        if (MODE != 1) {
          e_rel[e - e0] = rel;
          e_val[e - e0] = up_val[src];
        }
      }
      __syncthreads();
      if (MODE != 1) {
        // one round per worker present in the stage, in ascending q
        while (t_first + 1 < nq && s_pref[t_first + 1] <= e0) ++t_first;
        for (uint32_t t = t_first; t < nq && s_pref[t] < e1; ++t) {
          const uint32_t a = max(s_pref[t], e0), b = min(s_pref[t + 1], e1);
          if (b <= a) continue;                              // uniform over the block
          const float pq = s_p[t];
          for (uint32_t e = a + threadIdx.x; e < b; e += kAggBlock) {
            const uint32_t rel = e_rel[e - e0];
            if (rel != 0xFFFFFFFFu) acc[rel] = __fmaf_rn(pq, e_val[e - e0], acc[rel]);
          }
          __syncthreads();                                   // next worker may name the same i
        }
      }
    }
    __syncthreads();
  }
  if (MODE == 0) {
    // write the touched coordinates back
    for (uint32_t w = threadIdx.x; w < kAggWidth / 32; w += kAggBlock) {
      uint32_t bits = touched[w];
      while (bits) {
        const uint32_t t = __ffs(bits) - 1;
        bits &= bits - 1;
        const uint32_t rel = w * 32 + t;
        dense[c0 + rel] = acc[rel];
      }
    }
  }
  if (MODE == 2) {
    // ordered message: rank of a coordinate = set bits below it in the range's bitmap
    static_assert(kAggWidth / 32 <= kAggBlock, "one bitmap word per thread");
    const uint32_t word = threadIdx.x < kAggWidth / 32 ? touched[threadIdx.x] : 0u;
    uint32_t total;
    uint32_t pos = range_off[blockIdx.x] + block_exclusive_scan(__popc(word), lds, &total);
    uint32_t bits = word;
    while (bits) {
      const uint32_t t = __ffs(bits) - 1;
      bits &= bits - 1;
      const uint32_t rel = threadIdx.x * 32 + t;
      const float gt = acc[rel];
      if (msg_idx != nullptr) {
        msg_idx[pos] = (uint32_t)c0 + rel;
        msg_val[pos] = gt;
      }
      if (dense != nullptr) dense[c0 + rel] = __fmaf_rn(neg_alpha, gt, dense[c0 + rel]);
      ++pos;
    }
  }
  if ((MODE == 0 || MODE == 1) && range_nnz != nullptr) {
    uint32_t total;
    (void)block_exclusive_scan(fresh, lds, &total);
    if (threadIdx.x == 0) range_nnz[blockIdx.x] = total;
  }
}

// Exclusive scan of the per-range counts (one block); *total_out receives the sum.
__global__ __launch_bounds__(1024) void k_scan_ranges(const uint32_t* __restrict__ cnt,
                                                      uint32_t* __restrict__ off, uint32_t n,
                                                      uint32_t* __restrict__ total_out) {
  __shared__ uint32_t lds[1024 / kWave + 1];
  const uint32_t per = (n + blockDim.x - 1) / blockDim.x;
  const uint32_t b = min(threadIdx.x * per, n), e = min(b + per, n);
  uint32_t s = 0;
  for (uint32_t i = b; i < e; ++i) s += cnt[i];
  uint32_t total;
  uint32_t run = block_exclusive_scan(s, lds, &total);
  for (uint32_t i = b; i < e; ++i) {
    const uint32_t t = cnt[i];
    off[i] = run;
    run += t;
  }
  if (threadIdx.x == 0 && total_out != nullptr) *total_out = total;
}

// Sum of the per-range counts of distinct coordinates: one block.
__global__ __launch_bounds__(1024) void k_sum_ranges(const uint32_t* __restrict__ v, uint32_t n,
                                                     uint32_t* __restrict__ out) {
  __shared__ uint32_t lds[1024 / kWave + 1];
  uint32_t s = 0;
  for (uint32_t i = threadIdx.x; i < n; i += blockDim.x) s += v[i];
  uint32_t total;
  (void)block_exclusive_scan(s, lds, &total);
  if (threadIdx.x == 0) *out = total;
}

__global__ void k_update(const uint32_t* __restrict__ idx, const float* __restrict__ val,
                         uint32_t K, float neg_alpha, float* __restrict__ w, uint64_t d) {
  const uint32_t j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j < K) {
    const uint32_t i = idx[j];
    if (i < d) w[i] = __fmaf_rn(neg_alpha, val[j], w[i]);
  }
}

}  // namespace

uint32_t aggregate_ranges(uint64_t d) { return (uint32_t)((d + kAggWidth - 1) / kAggWidth); }

hipError_t aggregate(hipStream_t s, const uint32_t* up_idx, const float* up_val, const float* p,
                     uint32_t N, uint32_t K_up, float* delta, uint64_t d, uint32_t* union_nnz,
                     uint32_t* range_scratch, uint32_t* tab_start, uint32_t* tab_end) {
  if (K_up == 0) {
    if (union_nnz != nullptr) return fill_u32(s, union_nnz, 1, 0);
    return hipSuccess;
  }
  const uint32_t ranges = aggregate_ranges(d);
  if (tab_start != nullptr) {
    k_range_bounds<<<dim3((K_up + 255) / 256, N), dim3(256), 0, s>>>(up_idx, N, K_up, d,
                                                                    tab_start, tab_end);
    hipError_t e0 = hipGetLastError();
    if (e0 != hipSuccess) return e0;
  }
  k_aggregate<0><<<dim3(ranges), dim3(kAggBlock), 0, s>>>(
      up_idx, up_val, p, N, K_up, delta, d, union_nnz != nullptr ? range_scratch : nullptr,
      tab_start, tab_end, nullptr, 0.0f, nullptr, nullptr);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || union_nnz == nullptr) return e;
  k_sum_ranges<<<dim3(1), dim3(1024), 0, s>>>(range_scratch, ranges, union_nnz);
  return hipGetLastError();
}

hipError_t aggregate_update_unidirectional(hipStream_t s, const uint32_t* up_idx,
                                           const float* up_val, const float* p, uint32_t N,
                                           uint32_t K_up, float* w, uint64_t d, float alpha_out,
                                           uint32_t* msg_idx, float* msg_val, uint32_t* msg_count,
                                           uint32_t* range_cnt, uint32_t* range_off,
                                           uint32_t* tab_start, uint32_t* tab_end) {
  if (K_up == 0) {
    if (msg_count != nullptr) return fill_u32(s, msg_count, 1, 0);
    return hipSuccess;
  }
  const uint32_t ranges = aggregate_ranges(d);
  if (tab_start != nullptr) {
    k_range_bounds<<<dim3((K_up + 255) / 256, N), dim3(256), 0, s>>>(up_idx, N, K_up, d,
                                                                    tab_start, tab_end);
    hipError_t e0 = hipGetLastError();
    if (e0 != hipSuccess) return e0;
  }
  k_aggregate<1><<<dim3(ranges), dim3(kAggBlock), 0, s>>>(up_idx, up_val, p, N, K_up, nullptr, d,
                                                          range_cnt, tab_start, tab_end, nullptr,
                                                          0.0f, nullptr, nullptr);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  k_scan_ranges<<<dim3(1), dim3(1024), 0, s>>>(range_cnt, range_off, ranges, msg_count);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  k_aggregate<2><<<dim3(ranges), dim3(kAggBlock), 0, s>>>(up_idx, up_val, p, N, K_up, w, d,
                                                          nullptr, tab_start, tab_end, range_off,
                                                          -alpha_out, msg_idx, msg_val);
  return hipGetLastError();
}

hipError_t sgd_update(hipStream_t s, const uint32_t* idx, const float* val, uint32_t K,
                      float alpha_out, float* w, uint64_t d) {
  if (K == 0) return hipSuccess;
  k_update<<<dim3((K + 255) / 256), dim3(256), 0, s>>>(idx, val, K, -alpha_out, w, d);
  return hipGetLastError();
}

}  // namespace bts
