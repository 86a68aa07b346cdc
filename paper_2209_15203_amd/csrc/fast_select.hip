// Speculative single-pass Top_K select.
//
// The method's floor is one read of g, one read of eps and one write of eps per
// coordinate.  A radix select that histograms first and gathers afterwards reads the row
// again; this path avoids the second read for typical inputs and stays exact:
//
//   1. sample:   a strided sample (256-coordinate slices, every S-th slice) of a = eps +
//                alpha g is histogrammed on the top 13 bits of the magnitude key; a lower
//                bound L is chosen so that about 2K coordinates of the row lie at or above it.
//   2. stream:   the one dense pass computes a, stores it over eps and appends every
//                coordinate with key >= L to the row's candidate list (wave-aggregated
//                atomic append; the order of the list does not matter).
//   3. verify:   if the list holds at least K and at most `cap` entries, the K largest of
//                the row are all in it.  Otherwise the row is flagged and the dense path
//                (which reads the stored a again) redoes it.  The result never depends on L.
//   4. select:   exact radix select of the K-th largest key over the list (three digits),
//                then, if the threshold key is shared by more coordinates than are needed,
//                a radix select of the r-th smallest index among them.
//   5. emit:     kept candidates set one bit each in a per-row bitmap and bump a counter per
//                4096-coordinate bucket; a scan of the bucket counters and a popcount walk of
//                the non-empty buckets writes the message in ascending index order, stores
//                +0 over the kept coordinates and clears the bits again.
//
// Steps 4-5 touch O(K) data.  Used for the worker compression (rows = N, fused with the
// error compensation of Algorithm 2) and for the server compression (one row, no fusion).

#include "bts_device.h"

namespace bts {

namespace {

constexpr int kSampleBits = 13;                       // top bits of the 31-bit key
constexpr int kSampleBins = 1 << kSampleBits;         // 8192
constexpr int kSampleShift = 31 - kSampleBits;        // 18
constexpr uint32_t kSlice = kWave * 4;                // 256 coordinates: one f4 per lane
constexpr int kSliceUnroll = 8;
// The candidate list of a row is kept as kSubLists independent sub-lists, each with its own
// append counter on its own 128-byte line: appends to one address serialise in L2 at a few
// million per second, far too slow for one counter per row.  Wave-chunk wc appends to
// sub-list wc % kSubLists, which spreads even clustered hits evenly.
constexpr uint32_t kSubLists = 64;
constexpr uint32_t kCounterStride = 32;               // words between two counters
constexpr uint32_t kMaxHistBlocks = 32;               // blocks per row in a candidate pass

// ---- 1. sample histogram ------------------------------------------------------------
// Slices are cut at absolute multiples of 256 coordinates (16-byte aligned); only slices
// that lie entirely inside the row are sampled.
template <bool FMA>
__global__ __launch_bounds__(kBlock) void k_sample_hist(const float* __restrict__ g,
                                                        const float* __restrict__ x, uint64_t d,
                                                        float alpha, uint32_t stride,
                                                        uint32_t* __restrict__ shist) {
  __shared__ uint32_t sh[kSampleBins];
  const uint32_t row = blockIdx.y;
  for (int i = threadIdx.x; i < kSampleBins; i += kBlock) sh[i] = 0;
  __syncthreads();
  const uint64_t lo = (uint64_t)row * d, hi = lo + d;
  const uint64_t first = (lo + kSlice - 1) / kSlice;          // first whole slice
  const uint64_t last = hi / kSlice;                          // one past the last whole slice
  const uint64_t n_samp = last > first ? (last - first + stride - 1) / stride : 0;
  const uint32_t wave = blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
  const uint32_t n_waves = gridDim.x * kWavesPerBlock;
  uint32_t bin0 = 0;
  for (uint64_t s0 = (uint64_t)wave * kSliceUnroll; s0 < n_samp;
       s0 += (uint64_t)n_waves * kSliceUnroll) {
    f4 xv[kSliceUnroll], gv[kSliceUnroll];
    bool ok[kSliceUnroll];
#pragma unroll
    for (int u = 0; u < kSliceUnroll; ++u) {
      ok[u] = s0 + u < n_samp;
      const uint64_t e = (first + (s0 + u) * stride) * kSlice + (uint64_t)lane_id() * 4;
      if (ok[u]) {
        xv[u] = *reinterpret_cast<const f4*>(x + e);
        if (FMA) gv[u] = *reinterpret_cast<const f4*>(g + e);
      }
    }
#pragma unroll
    for (int u = 0; u < kSliceUnroll; ++u) {
      if (!ok[u]) continue;
      float v[4] = {xv[u].x, xv[u].y, xv[u].z, xv[u].w};
      if (FMA) {
        v[0] = __fmaf_rn(alpha, gv[u].x, v[0]);
        v[1] = __fmaf_rn(alpha, gv[u].y, v[1]);
        v[2] = __fmaf_rn(alpha, gv[u].z, v[2]);
        v[3] = __fmaf_rn(alpha, gv[u].w, v[3]);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t bin = key_of(v[j]) >> kSampleShift;
        if (bin == 0) ++bin0; else atomicAdd(&sh[bin], 1u);   // sparse rows: see k_hist
      }
    }
  }
  if (bin0) atomicAdd(&sh[0], bin0);
  __syncthreads();
  uint32_t* h = shist + (uint64_t)row * kSampleBins;
  for (int i = threadIdx.x; i < kSampleBins; i += kBlock) {
    const uint32_t v = sh[i];
    if (v) atomicAdd(&h[i], v);
  }
}

// Choose the lower bound: the highest bin edge with at least `target` sampled coordinates
// at or above it (bin 0, i.e. "everything", if the sample is smaller than that).  Clears
// the sample histogram and the row's candidate counter.
__global__ __launch_bounds__(kBlock) void k_pick_bound(uint32_t* __restrict__ shist,
                                                       uint32_t target,
                                                       uint32_t* __restrict__ lower_key,
                                                       uint32_t* __restrict__ cand_cnt) {
  constexpr int BPT = kSampleBins / kBlock;   // 32
  __shared__ uint32_t lds[kBlock / kWave + 1];
  __shared__ uint32_t s_bin;
  const uint32_t row = blockIdx.x;
  uint32_t* h = shist + (uint64_t)row * kSampleBins;
  const int top = kSampleBins - 1 - (int)threadIdx.x * BPT;
  uint32_t s = 0;
  for (int i = 0; i < BPT; ++i) s += h[top - i];
  if (threadIdx.x == 0) s_bin = 0;
  uint32_t total;
  const uint32_t excl = block_exclusive_scan(s, lds, &total);
  if (excl < target && target <= excl + s) {
    uint32_t acc = excl;
    int bin = top;
    for (int i = 0; i < BPT; ++i) {
      acc += h[top - i];
      if (acc >= target) {
        bin = top - i;
        break;
      }
    }
    s_bin = (uint32_t)bin;
  }
  __syncthreads();
  for (int i = 0; i < BPT; ++i) h[top - i] = 0;
  if (threadIdx.x == 0) lower_key[row] = s_bin << kSampleShift;
  if (threadIdx.x < kSubLists)
    cand_cnt[((uint64_t)row * kSubLists + threadIdx.x) * kCounterStride] = 0;
}

// ---- 2. the dense pass ------------------------------------------------------------------
// One wave per kWaveChunk coordinates.  Whole chunks take the fast body: kUnroll 16-byte
// loads per lane and array in flight, fused multiply-add, store, compare against the
// row's lower bound; the lanes' hits (rare) are ranked with one wave scan and appended
// with ONE atomic add per chunk (to the chunk's sub-list).  The partial chunks at the ends of a row go slice by
// slice.
template <bool FMA>
__global__ __launch_bounds__(kStreamBlock) void k_stream_capture(
    const float* __restrict__ g, float* __restrict__ x, uint64_t d, float alpha,
    const uint32_t* __restrict__ lower_key, uint32_t* __restrict__ cand_cnt,
    uint2* __restrict__ cand, uint32_t cap) {
  const uint32_t row = blockIdx.y;
  const uint32_t wc = blockIdx.x * kStreamWaves + threadIdx.x / kWave;
  const ChunkGeom c = wave_chunk(d, row, wc);
  if (!c.active) return;
  const uint32_t L = lower_key[row];
  const uint64_t sub = (uint64_t)row * kSubLists + wc % kSubLists;
  uint2* list = cand + sub * cap;                 // cap = capacity of one sub-list
  uint32_t* counter = cand_cnt + sub * kCounterStride;
  if (c.full) {
    const uint64_t e0 = c.base + (uint64_t)lane_id() * 4;
    f4 xv[kUnroll];
    f4 gv[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint64_t e = e0 + (uint64_t)u * (kWave * 4);
      xv[u] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(x + e));
      if (FMA) gv[u] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(g + e));
    }
    uint32_t flags = 0;                       // bit 4u + j: element j of slice u is a hit
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint64_t e = e0 + (uint64_t)u * (kWave * 4);
      if (FMA) {
        xv[u].x = __fmaf_rn(alpha, gv[u].x, xv[u].x);
        xv[u].y = __fmaf_rn(alpha, gv[u].y, xv[u].y);
        xv[u].z = __fmaf_rn(alpha, gv[u].z, xv[u].z);
        xv[u].w = __fmaf_rn(alpha, gv[u].w, xv[u].w);
        __builtin_nontemporal_store(xv[u], reinterpret_cast<f4*>(x + e));
      }
      flags |= (key_of(xv[u].x) >= L ? 1u : 0u) << (4 * u);
      flags |= (key_of(xv[u].y) >= L ? 2u : 0u) << (4 * u);
      flags |= (key_of(xv[u].z) >= L ? 4u : 0u) << (4 * u);
      flags |= (key_of(xv[u].w) >= L ? 8u : 0u) << (4 * u);
    }
    if (__ballot(flags != 0) == 0) return;
    const uint32_t mine = __popc(flags);
    const uint32_t incl = wave_inclusive_scan(mine);
    const uint32_t total = __shfl(incl, kWave - 1, kWave);
    uint32_t base = 0;
    if (lane_id() == 0) base = atomicAdd(counter, total);
    base = __shfl(base, 0, kWave);
    uint32_t pos = base + incl - mine;
    const uint32_t i0 = (uint32_t)(e0 - c.lo);
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const float v[4] = {xv[u].x, xv[u].y, xv[u].z, xv[u].w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (flags & (1u << (4 * u + j))) {
          if (pos < cap)
            list[pos] = make_uint2(i0 + (uint32_t)u * (kWave * 4) + j, __float_as_uint(v[j]));
          ++pos;
        }
      }
    }
    return;
  }
  visit_chunk<FMA>(g, x, c, alpha, [&](uint64_t e, const float (&v)[4], uint32_t mask) {
    uint32_t flags = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j)
      flags |= ((mask >> j) & 1u) && key_of(v[j]) >= L ? (1u << j) : 0u;
    if (__ballot(flags != 0) == 0) return;
    uint32_t total;
    const uint32_t pre = wave_exclusive_small(__popc(flags), &total);
    uint32_t base = 0;
    if (lane_id() == 0) base = atomicAdd(counter, total);
    base = __shfl(base, 0, kWave);
    uint32_t pos = base + pre;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (flags & (1u << j)) {
        if (pos < cap) list[pos] = make_uint2((uint32_t)(e + j - c.lo), __float_as_uint(v[j]));
        ++pos;
      }
    }
  });
}

// ---- 3 + 4. verify and select on the candidate list ------------------------------------
struct FastSel {
  uint32_t prefix, k_rem;     // key select in progress
  uint32_t T, r, eq_total;    // threshold key, ties to keep, ties present
  uint32_t iprefix, i_rem;    // index select among the ties in progress
  uint32_t I_T;               // ties with index <= I_T are kept
};

// Verify: the single pass succeeded for a row when no sub-list overflowed and the lists
// together hold at least K coordinates (then the K largest of the row are all listed).
__global__ __launch_bounds__(kWave) void k_cand_check(const uint32_t* __restrict__ cand_cnt,
                                                      uint32_t cap, uint32_t K,
                                                      uint32_t* __restrict__ need) {
  const uint32_t row = blockIdx.x;
  const uint32_t c = cand_cnt[((uint64_t)row * kSubLists + threadIdx.x) * kCounterStride];
  const uint32_t total = wave_sum(c);
  const bool over = __ballot(c > cap) != 0;
  if (threadIdx.x == 0) need[row] = (over || total < K) ? 1u : 0u;
}

// PASS 0..2: digits of the key (descending).  PASS 3..5: digits of the index among the
// coordinates whose key equals T (ascending), run only when ties must be split.
// A pass is two kernels: k_cand_hist (a few blocks per row, each histogramming whole
// sub-lists in LDS and storing its partial histogram with plain stores) and k_cand_scan
// (one block per row: adds the partials, walks the bins, advances the row's state).  No
// cross-block atomics or fences: on this part they are served at the memory side and
// same-address traffic serialises.
template <int PASS>
__global__ __launch_bounds__(kBlock) void k_cand_hist(const uint2* __restrict__ cand,
                                                      const uint32_t* __restrict__ cand_cnt,
                                                      uint32_t cap,
                                                      uint32_t* __restrict__ partial,
                                                      const FastSel* __restrict__ sel,
                                                      const uint32_t* __restrict__ need) {
  constexpr int NB = (PASS == 0 || PASS == 3 || PASS == 4) ? 2048 : 1024;
  __shared__ uint32_t sh[NB];
  const uint32_t row = blockIdx.y;
  if (need[row]) return;
  FastSel s;
  if (PASS > 0) s = sel[row];
  if (PASS >= 3 && s.r == s.eq_total) return;         // every tie is kept: nothing to split
  for (int i = threadIdx.x; i < NB; i += kBlock) sh[i] = 0;
  __syncthreads();
  for (uint32_t sl = blockIdx.x; sl < kSubLists; sl += gridDim.x) {
    const uint64_t sub = (uint64_t)row * kSubLists + sl;
    const uint32_t cnt = cand_cnt[sub * kCounterStride];
    const uint2* list = cand + sub * cap;
    for (uint32_t j = threadIdx.x; j < cnt; j += kBlock) {
      const uint2 en = list[j];
      const uint32_t idx = en.x, key = en.y & 0x7FFFFFFFu;
      if (PASS == 0) {
        atomicAdd(&sh[key >> 20], 1u);
      } else if (PASS == 1) {
        if ((key >> 20) == s.prefix) atomicAdd(&sh[(key >> 10) & 1023u], 1u);
      } else if (PASS == 2) {
        if ((key >> 10) == s.prefix) atomicAdd(&sh[key & 1023u], 1u);
      } else if (PASS == 3) {
        if (key == s.T) atomicAdd(&sh[idx >> 21], 1u);
      } else if (PASS == 4) {
        if (key == s.T && (idx >> 21) == s.iprefix) atomicAdd(&sh[(idx >> 10) & 2047u], 1u);
      } else {
        if (key == s.T && (idx >> 10) == s.iprefix) atomicAdd(&sh[idx & 1023u], 1u);
      }
    }
  }
  __syncthreads();
  uint32_t* out = partial + ((uint64_t)row * gridDim.x + blockIdx.x) * 2048;
  for (int i = threadIdx.x; i < NB; i += kBlock) out[i] = sh[i];
}

template <int PASS>
__global__ __launch_bounds__(kBlock) void k_cand_scan(const uint32_t* __restrict__ partial,
                                                      uint32_t nparts, uint32_t K,
                                                      FastSel* __restrict__ sel,
                                                      const uint32_t* __restrict__ need) {
  constexpr bool kOnIndex = PASS >= 3;
  constexpr int NB = (PASS == 0 || PASS == 3 || PASS == 4) ? 2048 : 1024;
  constexpr int BPT = NB / kBlock;
  __shared__ uint32_t lds[kBlock / kWave + 1];
  const uint32_t row = blockIdx.x;
  if (need[row]) return;
  FastSel s;
  if (PASS > 0) s = sel[row];
  if (kOnIndex && s.r == s.eq_total) return;
  const uint32_t want = PASS == 0 ? K : (kOnIndex ? s.i_rem : s.k_rem);
  // thread t owns BPT consecutive bins, walked from the end the select starts at
  const int start = kOnIndex ? (int)threadIdx.x * BPT : NB - 1 - (int)threadIdx.x * BPT;
  const int dir = kOnIndex ? 1 : -1;
  uint32_t c[BPT];
  uint32_t sum = 0;
#pragma unroll
  for (int i = 0; i < BPT; ++i) c[i] = 0;
  for (uint32_t b = 0; b < nparts; ++b) {
    const uint32_t* h = partial + ((uint64_t)row * nparts + b) * 2048;
#pragma unroll
    for (int i = 0; i < BPT; ++i) c[i] += h[start + dir * i];
  }
#pragma unroll
  for (int i = 0; i < BPT; ++i) sum += c[i];
  uint32_t total;
  const uint32_t excl = block_exclusive_scan(sum, lds, &total);
  if (excl < want && want <= excl + sum) {
    uint32_t acc = excl;
    int bin = start;
    uint32_t in_bin = 0;
#pragma unroll
    for (int i = 0; i < BPT; ++i) {
      if (acc + c[i] >= want) {
        bin = start + dir * i;
        in_bin = c[i];
        break;
      }
      acc += c[i];
    }
    const uint32_t b = (uint32_t)bin;
    if (PASS == 0) {
      s.prefix = b;
      s.k_rem = K - acc;
    } else if (PASS == 1) {
      s.prefix = (s.prefix << 10) | b;
      s.k_rem -= acc;
    } else if (PASS == 2) {
      s.T = (s.prefix << 10) | b;
      s.r = s.k_rem - acc;
      s.eq_total = in_bin;
      s.i_rem = s.r;
      s.I_T = 0xFFFFFFFFu;
    } else if (PASS == 3) {
      s.iprefix = b;
      s.i_rem -= acc;
    } else if (PASS == 4) {
      s.iprefix = (s.iprefix << 11) | b;
      s.i_rem -= acc;
    } else {
      s.I_T = (s.iprefix << 10) | b;
    }
    sel[row] = s;
  }
}

// ---- 5. ordered emission through a bitmap ------------------------------------------------
constexpr uint32_t kBucketShift = 12;                       // 4096 coordinates per bucket
constexpr uint32_t kBucketWords = (1u << kBucketShift) / 32; // 128 bitmap words

__global__ __launch_bounds__(kBlock) void k_mark(const uint2* __restrict__ cand,
                                                 const uint32_t* __restrict__ cand_cnt,
                                                 uint32_t cap, const FastSel* __restrict__ sel,
                                                 const uint32_t* __restrict__ need,
                                                 uint32_t* __restrict__ bitmap,
                                                 uint64_t words_per_row,
                                                 uint32_t* __restrict__ bucket_cnt,
                                                 uint32_t nbk) {
  const uint32_t row = blockIdx.y;
  if (need[row]) return;
  const uint32_t T = sel[row].T, I_T = sel[row].I_T;
  const uint64_t sub = (uint64_t)row * kSubLists + blockIdx.x % kSubLists;
  const uint32_t cnt = cand_cnt[sub * kCounterStride];
  const uint2* list = cand + sub * cap;
  const uint32_t part = blockIdx.x / kSubLists, parts = gridDim.x / kSubLists;
  uint32_t* bm = bitmap + (uint64_t)row * words_per_row;
  uint32_t* bc = bucket_cnt + (uint64_t)row * nbk;
  for (uint32_t j = part * kBlock + threadIdx.x; j < cnt; j += parts * kBlock) {
    const uint2 en = list[j];
    const uint32_t idx = en.x, key = en.y & 0x7FFFFFFFu;
    if (key > T || (key == T && idx <= I_T)) {
      atomicOr(&bm[idx >> 5], 1u << (idx & 31u));
      atomicAdd(&bc[idx >> kBucketShift], 1u);
    }
  }
}

__global__ __launch_bounds__(1024) void k_bucket_scan(const uint32_t* __restrict__ bucket_cnt,
                                                      uint32_t* __restrict__ bucket_off,
                                                      uint32_t nbk,
                                                      const uint32_t* __restrict__ need) {
  __shared__ uint32_t lds[1024 / kWave + 1];
  const uint32_t row = blockIdx.x;
  if (need[row]) return;
  const uint32_t per = (nbk + blockDim.x - 1) / blockDim.x;
  const uint32_t b = min(threadIdx.x * per, nbk), e = min(b + per, nbk);
  const uint32_t* c = bucket_cnt + (uint64_t)row * nbk;
  uint32_t* o = bucket_off + (uint64_t)row * nbk;
  uint32_t s = 0;
  for (uint32_t i = b; i < e; ++i) s += c[i];
  uint32_t total;
  uint32_t run = block_exclusive_scan(s, lds, &total);
  for (uint32_t i = b; i < e; ++i) {
    o[i] = run;
    run += c[i];
  }
}

// One wave per group of GROUP consecutive buckets (GROUP = 1, 8 or 64, chosen so that the
// launch has enough waves): the first GROUP lanes fetch the group's counters at once and
// the wave then walks its non-empty buckets; inside a bucket lane l owns bitmap words 2l
// and 2l+1.
template <int GROUP>
__global__ __launch_bounds__(kBlock) void k_emit_bitmap(
    float* __restrict__ x, uint64_t d, uint32_t K, uint32_t* __restrict__ bitmap,
    uint64_t words_per_row, uint32_t* __restrict__ bucket_cnt,
    const uint32_t* __restrict__ bucket_off, uint32_t nbk, const uint32_t* __restrict__ need,
    uint32_t* __restrict__ out_idx, float* __restrict__ out_val) {
  const uint32_t row = blockIdx.y;
  if (need[row]) return;
  const uint32_t group = blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
  const uint32_t bk_mine = group * GROUP + lane_id();
  uint32_t* bc = bucket_cnt + (uint64_t)row * nbk;
  const uint32_t my_cnt = (lane_id() < GROUP && bk_mine < nbk) ? bc[bk_mine] : 0u;
  uint64_t live = __ballot(my_cnt != 0);
  if (live == 0) return;
  const uint32_t my_off = my_cnt ? bucket_off[(uint64_t)row * nbk + bk_mine] : 0u;
  if (my_cnt) bc[bk_mine] = 0;
  uint32_t* bm = bitmap + (uint64_t)row * words_per_row;
  float* xr = x + (uint64_t)row * d;
  uint32_t* oi = out_idx + (uint64_t)row * K;
  float* ov = out_val + (uint64_t)row * K;
  while (live) {
    const int src = __ffsll((unsigned long long)live) - 1;
    live &= live - 1;
    const uint32_t bk = group * GROUP + src;
    const uint64_t w0 = (uint64_t)bk * kBucketWords + 2u * lane_id();
    uint32_t a = 0, b = 0;
    if (w0 < words_per_row) a = bm[w0];
    if (w0 + 1 < words_per_row) b = bm[w0 + 1];
    const uint32_t mine = __popc(a) + __popc(b);
    uint32_t pos = __shfl(my_off, src, kWave) + wave_inclusive_scan(mine) - mine;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      uint32_t bits = half == 0 ? a : b;
      const uint32_t base = (uint32_t)((w0 + half) * 32u);
      while (bits) {
        const uint32_t t = __ffs(bits) - 1;
        bits &= bits - 1;
        const uint32_t idx = base + t;
        if (pos < K && idx < d) {
          oi[pos] = idx;
          ov[pos] = xr[idx];
          xr[idx] = 0.0f;
        }
        ++pos;
      }
    }
    if (a) bm[w0] = 0;
    if (b) bm[w0 + 1] = 0;
  }
}

#define BTS_LAUNCH_CHECK()                       \
  do {                                           \
    hipError_t e_ = hipGetLastError();           \
    if (e_ != hipSuccess) return e_;             \
  } while (0)

}  // namespace

FastPlan fast_plan(uint32_t rows, uint64_t d, uint32_t K) {
  FastPlan p{};
  p.enabled = false;
  p.preferred = false;
  if (K == 0 || d < (1ull << 16) || (uint64_t)K * 64 > d) return p;
  // Below about 16 M coordinates per call the step is bound by kernel launches and the
  // dense path, with fewer launches, is the quicker one.
  p.preferred = (uint64_t)rows * d >= (16ull << 20);
  const uint64_t slices = d / 256;
  uint64_t stride = K / 64;        // about 128 of the sampled coordinates fall in the top 2K
  if (stride < 16) stride = 16;
  if (stride > 4096) stride = 4096;
  if (stride > slices / 64) stride = slices / 64;
  if (stride < 1) stride = 1;
  uint64_t target = (2ull * K + stride - 1) / stride;
  if (target < 48) target = 48;
  // expected list length is 2K..4K (the bound is a histogram bin edge); each of the 64
  // sub-lists gets twice its even share of 4x the target plus slack
  uint64_t cap = (4 * target * stride + 4096) / 64 * 2 + 64;
  p.enabled = true;
  p.stride = (uint32_t)stride;
  p.target = (uint32_t)target;
  p.cap = (uint32_t)cap;
  p.nbk = (uint32_t)((d + 4095) / 4096);
  p.words_per_row = (d + 31) / 32;
  return p;
}

hipError_t fast_select(hipStream_t s, const FastScratch& sc, const FastPlan& pl, const float* g,
                       float* x, uint32_t rows, uint64_t d, uint32_t K, float alpha,
                       uint32_t* out_idx, float* out_val, hipEvent_t ev0, hipEvent_t ev1) {
  const dim3 block(kBlock);
  const uint32_t nwc = (uint32_t)((d + kWaveChunk - 1) / kWaveChunk) + 1;
  const dim3 dense_grid((nwc + kStreamWaves - 1) / kStreamWaves, rows);
  // 1. sample
  const uint64_t n_samp = (d / 256) / pl.stride + 1;
  uint32_t sample_blocks = (uint32_t)((n_samp + kWavesPerBlock * 8 - 1) / (kWavesPerBlock * 8));
  if (sample_blocks > 64) sample_blocks = 64;
  if (sample_blocks < 1) sample_blocks = 1;
  if (g != nullptr)
    k_sample_hist<true><<<dim3(sample_blocks, rows), block, 0, s>>>(g, x, d, alpha, pl.stride,
                                                                   sc.sample_hist);
  else
    k_sample_hist<false><<<dim3(sample_blocks, rows), block, 0, s>>>(nullptr, x, d, 0.0f,
                                                                    pl.stride, sc.sample_hist);
  BTS_LAUNCH_CHECK();
  k_pick_bound<<<dim3(rows), block, 0, s>>>(sc.sample_hist, pl.target, sc.lower_key, sc.cand_cnt);
  BTS_LAUNCH_CHECK();
  // 2. the dense pass
  if (ev0) (void)hipEventRecord(ev0, s);
  if (g != nullptr)
    k_stream_capture<true><<<dense_grid, dim3(kStreamBlock), 0, s>>>(g, x, d, alpha, sc.lower_key, sc.cand_cnt,
                                                        sc.cand, pl.cap);
  else
    k_stream_capture<false><<<dense_grid, dim3(kStreamBlock), 0, s>>>(nullptr, x, d, 0.0f, sc.lower_key,
                                                         sc.cand_cnt, sc.cand, pl.cap);
  BTS_LAUNCH_CHECK();
  if (ev1) (void)hipEventRecord(ev1, s);
  // 3 + 4. verify and select
  // a few blocks per row, each taking whole sub-lists (about 4096 entries per block)
  uint32_t hb = (uint32_t)(((uint64_t)pl.cap * kSubLists / 2 + 4095) / 4096);
  if (hb > kMaxHistBlocks) hb = kMaxHistBlocks;
  if (hb < 1) hb = 1;
  const dim3 hgrid(hb, rows);
  FastSel* sel = reinterpret_cast<FastSel*>(sc.sel);
  k_cand_check<<<dim3(rows), dim3(kWave), 0, s>>>(sc.cand_cnt, pl.cap, K, sc.need);
  BTS_LAUNCH_CHECK();
#define BTS_CAND_PASS(P)                                                                       \
  k_cand_hist<P><<<hgrid, block, 0, s>>>(sc.cand, sc.cand_cnt, pl.cap, sc.hist, sel, sc.need); \
  BTS_LAUNCH_CHECK();                                                                          \
  k_cand_scan<P><<<dim3(rows), block, 0, s>>>(sc.hist, hb, K, sel, sc.need);                   \
  BTS_LAUNCH_CHECK();
  BTS_CAND_PASS(0)
  BTS_CAND_PASS(1)
  BTS_CAND_PASS(2)
  BTS_CAND_PASS(3)
  BTS_CAND_PASS(4)
  BTS_CAND_PASS(5)
#undef BTS_CAND_PASS
  // 5. emit
  uint32_t parts = (pl.cap + 2047) / 2048;            // blocks per sub-list
  if (parts > 4) parts = 4;
  if (parts < 1) parts = 1;
  k_mark<<<dim3(kSubLists * parts, rows), block, 0, s>>>(sc.cand, sc.cand_cnt, pl.cap, sel, sc.need, sc.bitmap,
                                          pl.words_per_row, sc.bucket_cnt, pl.nbk);
  BTS_LAUNCH_CHECK();
  k_bucket_scan<<<dim3(rows), dim3(1024), 0, s>>>(sc.bucket_cnt, sc.bucket_off, pl.nbk, sc.need);
  BTS_LAUNCH_CHECK();
  // enough waves to fill the chip, few enough that empty groups stay cheap
  const uint64_t buckets = (uint64_t)rows * pl.nbk;
  const int group = buckets >= (64ull << 17) ? 64 : (buckets >= (8ull << 17) ? 8 : 1);
  const uint32_t groups = (pl.nbk + group - 1) / group;
  const dim3 egrid((groups + kWavesPerBlock - 1) / kWavesPerBlock, rows);
  if (group == 64)
    k_emit_bitmap<64><<<egrid, block, 0, s>>>(x, d, K, sc.bitmap, pl.words_per_row, sc.bucket_cnt,
                                              sc.bucket_off, pl.nbk, sc.need, out_idx, out_val);
  else if (group == 8)
    k_emit_bitmap<8><<<egrid, block, 0, s>>>(x, d, K, sc.bitmap, pl.words_per_row, sc.bucket_cnt,
                                             sc.bucket_off, pl.nbk, sc.need, out_idx, out_val);
  else
    k_emit_bitmap<1><<<egrid, block, 0, s>>>(x, d, K, sc.bitmap, pl.words_per_row, sc.bucket_cnt,
                                             sc.bucket_off, pl.nbk, sc.need, out_idx, out_val);
  BTS_LAUNCH_CHECK();
  return hipSuccess;
}

size_t fast_sel_bytes() { return sizeof(FastSel); }
uint32_t fast_sublists() { return kSubLists; }
uint32_t fast_counter_stride() { return kCounterStride; }
uint32_t fast_hist_blocks() { return kMaxHistBlocks; }

}  // namespace bts
