// Device-side helpers for the dense passes (gfx950, wave64).
#pragma once

#include "bts_internal.h"

namespace bts {

using f4 = float __attribute__((ext_vector_type(4)));   // one 16-byte global access

// Magnitude key: fp32 bit pattern with the sign cleared.  Unsigned order on it is the
// order Top_K uses (NaN > Inf > finite > denormal > zero).
__device__ __forceinline__ uint32_t key_of(float x) { return __float_as_uint(x) & 0x7FFFFFFFu; }

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

__device__ __forceinline__ uint64_t lanes_below() {
  return (1ull << lane_id()) - 1ull;
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
  const int l = lane_id();
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    uint32_t t = __shfl_up(v, o, kWave);
    if (l >= o) v += t;
  }
  return v;
}

// Orders this wave's LDS accesses across its lanes (the hardware runs a wave's LDS
// instructions in order; this keeps the compiler from moving them).
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Exclusive prefix over lanes of a per-lane count in 0..7, from three ballots.
__device__ __forceinline__ uint32_t wave_exclusive_small(uint32_t c, uint32_t* total) {
  const uint64_t below = lanes_below();
  uint64_t b0 = __ballot(c & 1u), b1 = __ballot(c & 2u), b2 = __ballot(c & 4u);
  *total = __popcll(b0) + 2u * __popcll(b1) + 4u * __popcll(b2);
  return __popcll(b0 & below) + 2u * __popcll(b1 & below) + 4u * __popcll(b2 & below);
}

// Exclusive scan over the threads of a block (any multiple of 64 up to 1024 threads).
// lds must hold blockDim.x / 64 + 1 words.  Returns the exclusive prefix; *total gets the
// block sum.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* lds,
                                                         uint32_t* total) {
  const int l = lane_id(), w = threadIdx.x / kWave, nw = blockDim.x / kWave;
  uint32_t inc = wave_inclusive_scan(v);
  if (l == kWave - 1) lds[w] = inc;
  __syncthreads();
  if (w == 0) {                                   // the waves' sums, scanned by the first wave
    const uint32_t t = l < nw ? lds[l] : 0u;      // (at most 16 of them)
    const uint32_t s = wave_inclusive_scan(t);
    if (l < nw) lds[l] = s - t;
    if (l == nw - 1) lds[nw] = s;
  }
  __syncthreads();
  uint32_t res = inc - v + lds[w];
  *total = lds[nw];
  __syncthreads();
  return res;
}

// Adds up nparts partial NB-bin histograms (part + b * stride, b < nparts; global memory or
// LDS) and walks the bins from the top to the one holding the `want`-th largest entry;
// *above = entries in higher bins.  All THREADS threads of the block call this; the result is
// returned to every thread.  lds: THREADS / 64 + 1 words, s_out: 2 words.
template <int NB, int THREADS>
__device__ __forceinline__ uint32_t resolve_bins(const uint32_t* part, uint32_t nparts,
                                                 uint32_t stride, uint32_t want, uint32_t* lds,
                                                 uint32_t* s_out, uint32_t* above) {
  static_assert(NB % THREADS == 0, "whole bins per thread");
  constexpr int BPT = NB / THREADS;
  const int top = NB - 1 - (int)threadIdx.x * BPT;       // this thread's highest bin
  uint32_t c[BPT];
#pragma unroll
  for (int i = 0; i < BPT; ++i) c[i] = 0;
  for (uint32_t b = 0; b < nparts; ++b) {
    const uint32_t* h = part + (uint64_t)b * stride;
#pragma unroll
    for (int i = 0; i < BPT; ++i) c[i] += h[top - i];
  }
  uint32_t sum = 0;
#pragma unroll
  for (int i = 0; i < BPT; ++i) sum += c[i];
  uint32_t total;
  const uint32_t excl = block_exclusive_scan(sum, lds, &total);
  if (threadIdx.x == 0) {                                 // want > total: nothing to find
    s_out[0] = 0;
    s_out[1] = 0;
  }
  __syncthreads();
  if (excl < want && want <= excl + sum) {                // exactly one thread
    uint32_t acc = excl;
    int bin = top;
#pragma unroll
    for (int i = 0; i < BPT; ++i) {
      if (acc + c[i] >= want) {
        bin = top - i;
        break;
      }
      acc += c[i];
    }
    s_out[0] = (uint32_t)bin;
    s_out[1] = acc;
  }
  __syncthreads();
  const uint32_t bin = s_out[0];
  *above = s_out[1];
  __syncthreads();
  return bin;
}

// Geometry of one wave-chunk.  Row q covers the absolute element range [lo, hi) of the
// rows x d matrix; wave-chunks are cut at absolute multiples of kWaveChunk so that every
// float4 access is 16-byte aligned whatever d is; the first and last chunk of a row are
// partial and handled element by element.
struct ChunkGeom {
  uint64_t lo, hi, base;
  bool active;   // chunk intersects the row
  bool full;     // chunk lies entirely inside the row
};

__device__ __forceinline__ ChunkGeom wave_chunk(uint64_t d, uint32_t row, uint32_t wc) {
  ChunkGeom c;
  c.lo = (uint64_t)row * d;
  c.hi = c.lo + d;
  c.base = (c.lo / kWaveChunk + wc) * (uint64_t)kWaveChunk;
  c.active = c.base < c.hi;
  c.full = c.base >= c.lo && c.base + kWaveChunk <= c.hi;
  return c;
}

// Visit the wave-chunk in index order.  f(e, v, mask) is called kUnroll times by every
// lane with e = absolute offset of the lane's four consecutive elements, their values and
// a 4-bit mask of those that belong to the row.  With FMA the visited value is
// fma(alpha, g, x) and is stored back to x (each element by exactly one lane).
// streaming (uniform): x is read and written with non-temporal accesses -- the quicker way
// when the rows are far larger than the caches (8.1 against 8.9 ms per dense step at N x d =
// 1.6e9), the slower one when a row that is read again stays cached (rows of a few MB).
template <bool FMA, bool STREAMING, typename F>
__device__ __forceinline__ void visit_chunk_as(const float* __restrict__ g, float* __restrict__ x,
                                               const ChunkGeom& c, float alpha, F&& f) {
  const uint64_t e0 = c.base + (uint64_t)lane_id() * 4;
  if (c.full) {
    f4 xv[kUnroll];
    f4 gv[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint64_t e = e0 + (uint64_t)u * (kWave * 4);
      xv[u] = STREAMING ? __builtin_nontemporal_load(reinterpret_cast<const f4*>(x + e))
                        : *reinterpret_cast<const f4*>(x + e);
      if (FMA) gv[u] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(g + e));
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint64_t e = e0 + (uint64_t)u * (kWave * 4);
      if (FMA) {
        xv[u].x = __fmaf_rn(alpha, gv[u].x, xv[u].x);
        xv[u].y = __fmaf_rn(alpha, gv[u].y, xv[u].y);
        xv[u].z = __fmaf_rn(alpha, gv[u].z, xv[u].z);
        xv[u].w = __fmaf_rn(alpha, gv[u].w, xv[u].w);
        if (STREAMING)
          __builtin_nontemporal_store(xv[u], reinterpret_cast<f4*>(x + e));
        else
          *reinterpret_cast<f4*>(x + e) = xv[u];
      }
      const float v[4] = {xv[u].x, xv[u].y, xv[u].z, xv[u].w};
      f(e, v, 0xFu);
    }
  } else {
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint64_t e = e0 + (uint64_t)u * (kWave * 4);
      float v[4];
      uint32_t mask = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint64_t ee = e + j;
        v[j] = 0.0f;
        if (ee >= c.lo && ee < c.hi) {
          float t = x[ee];
          if (FMA) {
            t = __fmaf_rn(alpha, g[ee], t);
            x[ee] = t;
          }
          v[j] = t;
          mask |= 1u << j;
        }
      }
      f(e, v, mask);
    }
  }
}

template <bool FMA, typename F>
__device__ __forceinline__ void visit_chunk(const float* __restrict__ g, float* __restrict__ x,
                                            const ChunkGeom& c, float alpha, bool streaming,
                                            F&& f) {
  if (streaming)
    visit_chunk_as<FMA, true>(g, x, c, alpha, f);
  else
    visit_chunk_as<FMA, false>(g, x, c, alpha, f);
}

}  // namespace bts
