// libbts_probe: a measurement instrument, not part of libbts.  What this part's HBM sustains
// for the access mixes of the library, with the dominant kernel's access shape (one wave per
// 512 coordinates, two 16-byte non-temporal accesses per lane and array in flight,
// 128-thread workgroups) and nothing else in the kernel.  The dominant kernel of the worker
// stage is priced against the 8 TB/s peak; these probes show how much of that peak a plain
// stream of the same read : write mix reaches, at full occupancy and held to fewer waves
// per compute unit in the two ways a launch can be held (LDS it requests and never touches;
// a register budget set by the waves-per-SIMD attribute).

#include "../../include/bts_probe.h"

#include "bts_device.h"

namespace bts {

namespace {

// KIND 0: read src (a word is stored only if a sum of loaded values is NaN, so the loads stay)
// KIND 1: dst = src                                   (1 read : 1 write)
// KIND 2: dst = fma(alpha, src, dst)                  (2 reads : 1 write, the worker stage's mix)
// CACHED bit 0: plain loads instead of non-temporal ones; bit 1: plain stores.
template <int KIND, int CACHED = 0>
__device__ __forceinline__ void probe_body(const float* __restrict__ src,
                                           float* __restrict__ dst, uint64_t n, float alpha) {
  const uint64_t wc = (uint64_t)blockIdx.x * kStreamWaves + threadIdx.x / kWave;
  const uint64_t base = wc * kWaveChunk;
  if (base + kWaveChunk > n) return;                       // whole chunks only
  const uint64_t e0 = base + (uint64_t)lane_id() * 4;
  f4 a[kUnroll], b[kUnroll];
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const uint64_t e = e0 + (uint64_t)u * (kWave * 4);
    a[u] = (CACHED & 1) ? *reinterpret_cast<const f4*>(src + e)
                        : __builtin_nontemporal_load(reinterpret_cast<const f4*>(src + e));
    if (KIND == 2)
      b[u] = (CACHED & 1) ? *reinterpret_cast<const f4*>(dst + e)
                          : __builtin_nontemporal_load(reinterpret_cast<const f4*>(dst + e));
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
      if (CACHED & 2)
        *reinterpret_cast<f4*>(dst + e) = b[u];
      else
        __builtin_nontemporal_store(b[u], reinterpret_cast<f4*>(dst + e));
    }
  }
  if (KIND == 0 && sum != sum) dst[0] = sum;
}

template <int KIND>
__global__ __launch_bounds__(kStreamBlock) void k_probe(const float* __restrict__ src,
                                                        float* __restrict__ dst, uint64_t n,
                                                        float alpha) {
  probe_body<KIND>(src, dst, n, alpha);
}

// The same stream held to WPS waves per SIMD (4 SIMDs per compute unit) by the compiler:
// it sizes the kernel's register allocation so that no more fit.
template <int KIND, int WPS>
__global__ __launch_bounds__(kStreamBlock) __attribute__((amdgpu_waves_per_eu(1, WPS))) void
k_probe_held(const float* __restrict__ src, float* __restrict__ dst, uint64_t n, float alpha) {
  probe_body<KIND>(src, dst, n, alpha);
}

// The fma-stream at 12 waves per compute unit with plain (cached) loads and/or stores.
template <int CACHED>
__global__ __launch_bounds__(kStreamBlock) __attribute__((amdgpu_waves_per_eu(1, 3))) void
k_probe_cached(const float* __restrict__ src, float* __restrict__ dst, uint64_t n, float alpha) {
  probe_body<2, CACHED>(src, dst, n, alpha);
}

template <int KIND>
void launch(dim3 grid, dim3 block, int waves_per_cu, bool by_registers, hipStream_t s,
            const float* src, float* dst, uint64_t n, float alpha) {
  if (waves_per_cu >= 100) {                 // 101..103: the cached variants of kind 2
    if (waves_per_cu == 101) k_probe_cached<1><<<grid, block, 0, s>>>(src, dst, n, alpha);
    if (waves_per_cu == 102) k_probe_cached<2><<<grid, block, 0, s>>>(src, dst, n, alpha);
    if (waves_per_cu == 103) k_probe_cached<3><<<grid, block, 0, s>>>(src, dst, n, alpha);
  } else if (waves_per_cu == 0) {
    k_probe<KIND><<<grid, block, 0, s>>>(src, dst, n, alpha);
  } else if (by_registers) {
    if (waves_per_cu == 12) k_probe_held<KIND, 3><<<grid, block, 0, s>>>(src, dst, n, alpha);
    if (waves_per_cu == 20) k_probe_held<KIND, 5><<<grid, block, 0, s>>>(src, dst, n, alpha);
    if (waves_per_cu == 24) k_probe_held<KIND, 6><<<grid, block, 0, s>>>(src, dst, n, alpha);
  } else {
    // workgroups of kStreamWaves waves; a compute unit has 160 KB of LDS
    const uint32_t groups = (uint32_t)waves_per_cu / kStreamWaves;
    const uint32_t lds = (163840u / groups) / 512u * 512u;
    k_probe<KIND><<<grid, block, lds, s>>>(src, dst, n, alpha);
  }
}

}  // namespace

}  // namespace bts

using namespace bts;

extern "C" int bts_hbm_probe(void* hip_stream, int kind, const float* src, float* dst,
                             uint64_t n, int waves_per_cu, int by_registers, int repeats,
                             double* ms_per_launch) {
  if (!src || !dst || !ms_per_launch || kind < 0 || kind > 2 || repeats < 1 || n < 512)
    return -1;
  if ((reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(dst) & 15u))
    return -1;
  const bool cached_variant = kind == 2 && waves_per_cu >= 101 && waves_per_cu <= 103;
  if (waves_per_cu != 0 && waves_per_cu != 12 && waves_per_cu != 20 && waves_per_cu != 24 &&
      !cached_variant)
    return -1;
  const uint64_t chunks = n / kWaveChunk;
  if (chunks / kStreamWaves + 1 > 0x7FFFFFFFull) return -1;
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  const dim3 grid((unsigned)((chunks + kStreamWaves - 1) / kStreamWaves)), block(kStreamBlock);
  hipEvent_t e0, e1;
  hipError_t e = hipEventCreate(&e0);
  if (e != hipSuccess) return -1000 - (int)e;
  e = hipEventCreate(&e1);
  if (e != hipSuccess) {
    (void)hipEventDestroy(e0);
    return -1000 - (int)e;
  }
  for (int it = -1; it < repeats && e == hipSuccess; ++it) {     // one untimed launch first
    if (it == 0) e = hipEventRecord(e0, s);
    if (e != hipSuccess) break;
    if (kind == 0) launch<0>(grid, block, waves_per_cu, by_registers != 0, s, src, dst, n, 0.5f);
    if (kind == 1) launch<1>(grid, block, waves_per_cu, by_registers != 0, s, src, dst, n, 0.5f);
    if (kind == 2) launch<2>(grid, block, waves_per_cu, by_registers != 0, s, src, dst, n, 0.5f);
    e = hipGetLastError();
  }
  if (e == hipSuccess) e = hipEventRecord(e1, s);
  if (e == hipSuccess) e = hipEventSynchronize(e1);
  float ms = 0.0f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess) return -1000 - (int)e;
  *ms_per_launch = (double)ms / repeats;
  return 0;
}
