// Measurement aid: what this part's HBM sustains for the access mixes of the library, with
// the dominant kernel's access shape (one wave per 512 coordinates, two 16-byte non-temporal
// accesses per lane and array in flight, 128-thread workgroups) and nothing else in the
// kernel.  The dominant kernel of the worker stage is priced against the 8 TB/s peak; these
// probes show how much of that peak a plain stream of the same read : write mix reaches.

#include "bts_device.h"

namespace bts {

namespace {

// KIND 0: read src (a word is stored only if a sum of loaded values is NaN, so the loads stay)
// KIND 1: dst = src                                   (1 read : 1 write)
// KIND 2: dst = fma(alpha, src, dst)                  (2 reads : 1 write, the worker stage's mix)
template <int KIND>
__global__ __launch_bounds__(kStreamBlock) void k_probe(const float* __restrict__ src,
                                                        float* __restrict__ dst, uint64_t n,
                                                        float alpha) {
  const uint64_t wc = (uint64_t)blockIdx.x * kStreamWaves + threadIdx.x / kWave;
  const uint64_t base = wc * kWaveChunk;
  if (base + kWaveChunk > n) return;                       // whole chunks only
  const uint64_t e0 = base + (uint64_t)lane_id() * 4;
  f4 a[kUnroll], b[kUnroll];
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const uint64_t e = e0 + (uint64_t)u * (kWave * 4);
    a[u] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(src + e));
    if (KIND == 2) b[u] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(dst + e));
  }
  float sum = 0.0f;
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const uint64_t e = e0 + (uint64_t)u * (kWave * 4);
    if (KIND == 0) sum += a[u].x + a[u].y + a[u].z + a[u].w;
    if (KIND == 1) __builtin_nontemporal_store(a[u], reinterpret_cast<f4*>(dst + e));
    if (KIND == 2) {
      b[u].x = __fmaf_rn(alpha, a[u].x, b[u].x);
      b[u].y = __fmaf_rn(alpha, a[u].y, b[u].y);
      b[u].z = __fmaf_rn(alpha, a[u].z, b[u].z);
      b[u].w = __fmaf_rn(alpha, a[u].w, b[u].w);
      __builtin_nontemporal_store(b[u], reinterpret_cast<f4*>(dst + e));
    }
  }
  if (KIND == 0 && sum != sum) dst[0] = sum;
}

}  // namespace

hipError_t hbm_probe(hipStream_t s, int kind, const float* src, float* dst, uint64_t n,
                     float alpha, int repeats, double* ms_per_launch) {
  const uint64_t chunks = n / kWaveChunk;
  if (chunks == 0 || chunks / kStreamWaves + 1 > 0x7FFFFFFFull) return hipErrorInvalidValue;
  const dim3 grid((unsigned)((chunks + kStreamWaves - 1) / kStreamWaves)), block(kStreamBlock);
  const size_t lds = kind == 2 ? kMixedStreamLds : 0;     // as the dominant kernel is launched
  hipEvent_t e0, e1;
  hipError_t e = hipEventCreate(&e0);
  if (e != hipSuccess) return e;
  e = hipEventCreate(&e1);
  if (e != hipSuccess) {
    (void)hipEventDestroy(e0);
    return e;
  }
  for (int it = -1; it < repeats && e == hipSuccess; ++it) {     // one untimed launch first
    if (it == 0) e = hipEventRecord(e0, s);
    if (e != hipSuccess) break;
    if (kind == 0) k_probe<0><<<grid, block, lds, s>>>(src, dst, n, alpha);
    if (kind == 1) k_probe<1><<<grid, block, lds, s>>>(src, dst, n, alpha);
    if (kind == 2) k_probe<2><<<grid, block, lds, s>>>(src, dst, n, alpha);
    e = hipGetLastError();
  }
  if (e == hipSuccess) e = hipEventRecord(e1, s);
  if (e == hipSuccess) e = hipEventSynchronize(e1);
  float ms = 0.0f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e == hipSuccess) *ms_per_launch = (double)ms / repeats;
  return e;
}

}  // namespace bts
