// Server side of Algorithm 2 apart from the compression: the weighted aggregation
//     g_t = sum_q p_q Top_K(a^q) + delta_{t-1}
// and the model update  w_t = w_{t-1} - Top_K(g_t)  on the received pairs.
//
// Aggregation is deterministic without float atomics: the coordinate axis is cut into
// ranges, one workgroup owns a range, and inside it the workers are applied one after
// the other in ascending q (a worker never names a coordinate twice, so the pairs of one
// worker are applied in parallel; a workgroup barrier separates consecutive workers).
// Each worker's pairs that fall into the range are found by binary search in its sorted
// index list.

#include "bts_device.h"

namespace bts {

namespace {

constexpr int kAggBlock = 256;
constexpr int kAggTile = 256;   // workers whose range bounds are held in LDS at a time

__device__ __forceinline__ uint32_t lower_bound_u32(const uint32_t* __restrict__ a, uint32_t n,
                                                    uint32_t key) {
  uint32_t lo = 0, hi = n;
  while (lo < hi) {
    const uint32_t mid = lo + ((hi - lo) >> 1);
    if (a[mid] < key) lo = mid + 1; else hi = mid;
  }
  return lo;
}

__global__ __launch_bounds__(kAggBlock) void k_aggregate(
    const uint32_t* __restrict__ up_idx, const float* __restrict__ up_val,
    const float* __restrict__ p, uint32_t N, uint32_t K_up, float* delta, uint64_t d,
    uint32_t width, uint32_t* __restrict__ union_nnz) {
  extern __shared__ uint32_t touched[];              // width / 32 words
  __shared__ uint32_t s_lo[kAggTile], s_hi[kAggTile];
  __shared__ uint32_t s_new;
  const uint64_t c0 = (uint64_t)blockIdx.x * width;
  const uint64_t c1 = min(c0 + (uint64_t)width, d);
  const uint32_t words = width / 32;
  for (uint32_t i = threadIdx.x; i < words; i += kAggBlock) touched[i] = 0;
  if (threadIdx.x == 0) s_new = 0;
  uint32_t fresh = 0;
  for (uint32_t q0 = 0; q0 < N; q0 += kAggTile) {
    __syncthreads();
    const uint32_t nq = min((uint32_t)kAggTile, N - q0);
    if (threadIdx.x < nq) {
      const uint32_t* row = up_idx + (uint64_t)(q0 + threadIdx.x) * K_up;
      s_lo[threadIdx.x] = lower_bound_u32(row, K_up, (uint32_t)c0);
      // c1 <= d < 2^32 except that c1 == 2^32 cannot occur (d < 2^32)
      s_hi[threadIdx.x] = lower_bound_u32(row, K_up, (uint32_t)c1);
    }
    __syncthreads();
    for (uint32_t t = 0; t < nq; ++t) {
      const uint32_t lo = s_lo[t], hi = s_hi[t];
      if (hi <= lo) continue;                        // uniform over the block
      const uint32_t q = q0 + t;
      const float pq = p[q];
      const uint32_t* row_i = up_idx + (uint64_t)q * K_up;
      const float* row_v = up_val + (uint64_t)q * K_up;
      for (uint32_t j = lo + threadIdx.x; j < hi; j += kAggBlock) {
        const uint32_t i = row_i[j];
        if (i >= c0 && i < c1) {                     // always true for sorted input
          delta[i] = __fmaf_rn(pq, row_v[j], delta[i]);
          const uint32_t rel = i - (uint32_t)c0;
          const uint32_t bit = 1u << (rel & 31);
          const uint32_t old = atomicOr(&touched[rel >> 5], bit);
          fresh += (old & bit) ? 0u : 1u;
        }
      }
      __syncthreads();                               // next worker may name the same i
    }
  }
  if (union_nnz != nullptr) {
    fresh = wave_sum(fresh);
    if (lane_id() == 0 && fresh) atomicAdd(&s_new, fresh);
    __syncthreads();
    if (threadIdx.x == 0 && s_new) atomicAdd(union_nnz, s_new);
  }
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

hipError_t aggregate(hipStream_t s, const uint32_t* up_idx, const float* up_val, const float* p,
                     uint32_t N, uint32_t K_up, float* delta, uint64_t d, uint32_t* union_nnz) {
  if (union_nnz != nullptr) {
    hipError_t e = fill_u32(s, union_nnz, 1, 0);
    if (e != hipSuccess) return e;
  }
  if (K_up == 0) return hipSuccess;
  // Range width: a multiple of 32 coordinates, at most 16384 ranges, at least 1024 wide.
  uint64_t width = (d + 16383) / 16384;
  if (width < 1024) width = 1024;
  width = (width + 31) / 32 * 32;
  const uint32_t ranges = (uint32_t)((d + width - 1) / width);
  const size_t lds = (size_t)(width / 32) * sizeof(uint32_t);
  k_aggregate<<<dim3(ranges), dim3(kAggBlock), lds, s>>>(up_idx, up_val, p, N, K_up, delta, d,
                                                         (uint32_t)width, union_nnz);
  return hipGetLastError();
}

hipError_t sgd_update(hipStream_t s, const uint32_t* idx, const float* val, uint32_t K,
                      float alpha_out, float* w, uint64_t d) {
  if (K == 0) return hipSuccess;
  k_update<<<dim3((K + 255) / 256), dim3(256), 0, s>>>(idx, val, K, -alpha_out, w, d);
  return hipGetLastError();
}

}  // namespace bts
