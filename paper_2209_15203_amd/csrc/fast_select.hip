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
//                coordinate with key >= L to the row's candidate lists (wave-aggregated
//                atomic append; the order inside a list does not matter).
//   3. verify:   if no list overflowed and the lists hold at least K entries, the K largest
//                of the row are all listed.  Otherwise the row is flagged and the dense path
//                (which reads the stored a again) redoes it.  The result never depends on L.
//   4. select:   exact 11 + 10 + 10 bit radix select of the K-th largest key T over the
//                lists, and r = how many holders of T are kept.
//   5. emit:     candidates above T set a bit in the row's "greater" bitmap, holders of T in
//                its "equal" bitmap, and bump the counter of their 4096-coordinate bucket; a
//                small kernel sums the counters per 2^20-coordinate super-bucket.  One more
//                kernel walks the non-empty buckets in index order: a coordinate is kept if
//                it is greater, or equal with fewer than r equal ones before it (lower index
//                wins); its place in the message is #greater before + min(#equal before, r),
//                which the walk gets from the super-bucket and bucket counters and
//                popcounts.  It writes the indices and clears the bits, then gathers the
//                values from eps in parallel and stores +0 there.
//
// Steps 4-5 touch O(K) data.  Used for the worker compression (rows = N, fused with the
// error compensation of Algorithm 2) and for the server compression (one row, no fusion).
//
// Two facts of this part shaped the kernels: atomics that return a value on one address are
// served at the memory side at a few million per second, and a device-scope fence writes
// back the XCD's L2.  Hence many append counters on separate 128-byte lines, one append per
// wave chunk, per-block partial histograms with plain stores, and kernel boundaries instead
// of last-block-done tickets.

#include "bts_device.h"

namespace bts {

namespace {

constexpr int kSampleBits = 13;                       // top bits of the 31-bit key
constexpr int kSampleBins = 1 << kSampleBits;         // 8192
constexpr int kSampleShift = 31 - kSampleBits;        // 18
constexpr uint32_t kSlice = kWave * 4;                // 256 coordinates: one f4 per lane
constexpr int kSliceUnroll = 8;
// The candidates of a row are kept in kSubLists independent lists, each with its own
// append counter on its own 128-byte line.  Wave-chunk wc appends to list wc % kSubLists,
// which spreads even clustered hits evenly.
constexpr uint32_t kSubLists = 64;
constexpr uint32_t kCounterStride = 32;               // words between two counters
constexpr uint32_t kMaxHistBlocks = 32;               // blocks per row in a candidate pass
constexpr uint32_t kBucketShift = 12;                 // 4096 coordinates per bucket
constexpr uint32_t kBucketWords = (1u << kBucketShift) / 32;   // 128 bitmap words
constexpr uint32_t kSuperShift = 8;                   // 256 buckets per super-bucket

// ---- 1. sample histogram ------------------------------------------------------------
// Slices are cut at absolute multiples of 256 coordinates (16-byte aligned); only slices
// that lie entirely inside the row are sampled.  The kernel also clears the row's bucket
// counters, which the previous call's emission leaves set.
template <bool FMA>
__global__ __launch_bounds__(kBlock) void k_sample_hist(
    const float* __restrict__ g, const float* __restrict__ x, uint64_t d, float alpha,
    uint32_t stride, uint32_t* __restrict__ shist, uint32_t* __restrict__ bucket_cnt,
    uint32_t nbk) {
  __shared__ uint32_t sh[kSampleBins];
  const uint32_t row = blockIdx.y;
  for (int i = threadIdx.x; i < kSampleBins; i += kBlock) sh[i] = 0;
  for (uint32_t i = blockIdx.x * kBlock + threadIdx.x; i < nbk; i += gridDim.x * kBlock)
    bucket_cnt[(uint64_t)row * nbk + i] = 0;
  __syncthreads();
  const uint64_t lo = (uint64_t)row * d, hi = lo + d;
  const uint64_t first = (lo + kSlice - 1) / kSlice;          // first whole slice
  const uint64_t last = hi / kSlice;                          // one past the last whole slice
  const uint64_t n_samp = last > first ? (last - first + stride - 1) / stride : 0;
  const uint32_t wave = blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
  const uint32_t n_waves = gridDim.x * kWavesPerBlock;
  uint32_t bin0 = 0;       // counted per lane: a sparse row would serialise on one LDS word
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
        if (bin == 0) ++bin0; else atomicAdd(&sh[bin], 1u);
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
// the sample histogram and the row's append counters.
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
// with ONE atomic add per chunk (to the chunk's list).  The partial chunks at the ends of
// a row go slice by slice.
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
  uint2* list = cand + sub * cap;                 // cap = capacity of one list
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

// ---- 3 + 4. verify and select on the candidate lists -------------------------------------
struct FastSel {
  uint32_t prefix, k_rem;     // key select in progress
  uint32_t T, r;              // threshold key; how many holders of T are kept
};

// One digit of the select is two kernels: k_cand_hist (a few blocks per row, each
// histogramming whole lists in LDS and storing its partial histogram with plain stores)
// and k_cand_scan (one block per row: adds the partials, walks the bins from the top,
// advances the row's state).  The first histogram kernel also verifies the row: it
// succeeded when no list overflowed and the lists together hold at least K entries.
template <int PASS>
__global__ __launch_bounds__(kBlock) void k_cand_hist(const uint2* __restrict__ cand,
                                                      const uint32_t* __restrict__ cand_cnt,
                                                      uint32_t cap, uint32_t K,
                                                      uint32_t* __restrict__ partial,
                                                      const FastSel* __restrict__ sel,
                                                      uint32_t* __restrict__ need) {
  constexpr int NB = PASS == 0 ? 2048 : 1024;
  __shared__ uint32_t sh[NB];
  __shared__ uint32_t s_need;
  const uint32_t row = blockIdx.y;
  if (PASS == 0) {
    if (threadIdx.x < kWave) {
      const uint32_t c =
          cand_cnt[((uint64_t)row * kSubLists + threadIdx.x) * kCounterStride];
      const uint32_t total = wave_sum(c);
      const bool over = __ballot(c > cap) != 0;
      if (threadIdx.x == 0) {
        s_need = (over || total < K) ? 1u : 0u;
        if (blockIdx.x == 0) need[row] = s_need;
      }
    }
    __syncthreads();
    if (s_need) return;
  } else if (need[row]) {
    return;
  }
  FastSel s{};
  if (PASS > 0) s = sel[row];
  for (int i = threadIdx.x; i < NB; i += kBlock) sh[i] = 0;
  __syncthreads();
  for (uint32_t sl = blockIdx.x; sl < kSubLists; sl += gridDim.x) {
    const uint64_t sub = (uint64_t)row * kSubLists + sl;
    const uint32_t cnt = cand_cnt[sub * kCounterStride];
    const uint2* list = cand + sub * cap;
    for (uint32_t j = threadIdx.x; j < cnt; j += kBlock) {
      const uint32_t key = list[j].y & 0x7FFFFFFFu;
      if (PASS == 0) {
        atomicAdd(&sh[key >> 20], 1u);
      } else if (PASS == 1) {
        if ((key >> 20) == s.prefix) atomicAdd(&sh[(key >> 10) & 1023u], 1u);
      } else {
        if ((key >> 10) == s.prefix) atomicAdd(&sh[key & 1023u], 1u);
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
  constexpr int NB = PASS == 0 ? 2048 : 1024;
  constexpr int BPT = NB / kBlock;
  __shared__ uint32_t lds[kBlock / kWave + 1];
  const uint32_t row = blockIdx.x;
  if (need[row]) return;
  FastSel s{};
  if (PASS > 0) s = sel[row];
  const uint32_t want = PASS == 0 ? K : s.k_rem;
  const int top = NB - 1 - (int)threadIdx.x * BPT;       // this thread's highest bin
  uint32_t c[BPT];
  uint32_t sum = 0;
#pragma unroll
  for (int i = 0; i < BPT; ++i) c[i] = 0;
  for (uint32_t b = 0; b < nparts; ++b) {
    const uint32_t* h = partial + ((uint64_t)row * nparts + b) * 2048;
#pragma unroll
    for (int i = 0; i < BPT; ++i) c[i] += h[top - i];
  }
#pragma unroll
  for (int i = 0; i < BPT; ++i) sum += c[i];
  uint32_t total;
  const uint32_t excl = block_exclusive_scan(sum, lds, &total);
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
    const uint32_t b = (uint32_t)bin;
    if (PASS == 0) {
      s.prefix = b;
      s.k_rem = K - acc;
    } else if (PASS == 1) {
      s.prefix = (s.prefix << 10) | b;
      s.k_rem -= acc;
    } else {
      s.T = (s.prefix << 10) | b;
      s.r = s.k_rem - acc;
    }
    sel[row] = s;
  }
}

// ---- 5. ordered emission through two bitmaps ---------------------------------------------
// Bucket counter: "greater" count in the low 16 bits, "equal" count in the high 16 bits (a
// bucket holds 4096 coordinates, so neither half overflows).  Super-bucket counter: the same
// two counts in the halves of a 64-bit word.
//
// Consecutive entries of a list mostly come from one wave chunk of the dense pass, in index
// order, so neighbouring lanes usually share a bucket: the lanes of a run add their counts
// with one atomic by the run's first lane.
__global__ __launch_bounds__(kBlock) void k_mark(const uint2* __restrict__ cand,
                                                 const uint32_t* __restrict__ cand_cnt,
                                                 uint32_t cap, const FastSel* __restrict__ sel,
                                                 const uint32_t* __restrict__ need,
                                                 uint32_t* __restrict__ bm_gt,
                                                 uint32_t* __restrict__ bm_eq,
                                                 uint64_t words_per_row,
                                                 uint32_t* __restrict__ bucket_cnt,
                                                 uint32_t nbk) {
  const uint32_t row = blockIdx.y;
  if (need[row]) return;
  const uint32_t T = sel[row].T;
  const uint64_t sub = (uint64_t)row * kSubLists + blockIdx.x % kSubLists;
  const uint32_t cnt = cand_cnt[sub * kCounterStride];
  const uint2* list = cand + sub * cap;
  const uint32_t part = blockIdx.x / kSubLists, parts = gridDim.x / kSubLists;
  uint32_t* bc = bucket_cnt + (uint64_t)row * nbk;
  const int lane = lane_id();
  // whole waves stay in the loop together (the run logic uses wave-wide shuffles)
  const uint32_t rounds = (cnt + parts * kBlock - 1) / (parts * kBlock);
  for (uint32_t it = 0; it < rounds; ++it) {
    const uint32_t j = (it * parts + part) * kBlock + threadIdx.x;
    uint32_t bk = 0xFFFFFFFFu, val = 0;
    if (j < cnt) {
      const uint2 en = list[j];
      const uint32_t idx = en.x, key = en.y & 0x7FFFFFFFu;
      if (key >= T) {
        const bool eq = key == T;
        uint32_t* bm = (eq ? bm_eq : bm_gt) + (uint64_t)row * words_per_row;
        atomicOr(&bm[idx >> 5], 1u << (idx & 31u));
        bk = idx >> kBucketShift;
        val = eq ? 0x10000u : 1u;
      }
    }
    const uint32_t prev = __shfl_up(bk, 1, kWave);
    const bool leader = lane == 0 || bk != prev;
    const uint64_t leaders = __ballot(leader);
    const uint32_t incl = wave_inclusive_scan(val);       // a wave holds 64 entries: no carry
    const uint64_t later = lane == kWave - 1 ? 0ull : leaders & ~((2ull << lane) - 1ull);
    const int last = later ? __ffsll((unsigned long long)later) - 2 : kWave - 1;
    const uint32_t run = __shfl(incl, last, kWave) - (incl - val);
    if (leader && bk != 0xFFFFFFFFu) atomicAdd(&bc[bk], run);
  }
}

// Sum of the 256 bucket counters of each super-bucket (one block each), unpacked to 64 bits.
__global__ __launch_bounds__(kBlock) void k_super_sums(const uint32_t* __restrict__ bucket_cnt,
                                                       uint32_t nbk,
                                                       unsigned long long* __restrict__ super_cnt,
                                                       uint32_t nsup,
                                                       const uint32_t* __restrict__ need) {
  static_assert((1u << kSuperShift) == kBlock, "one bucket per thread");
  __shared__ unsigned long long lds[kBlock / kWave];
  const uint32_t row = blockIdx.y;
  if (need[row]) return;
  const uint32_t bk = blockIdx.x * kBlock + threadIdx.x;
  const uint32_t c = bk < nbk ? bucket_cnt[(uint64_t)row * nbk + bk] : 0u;
  unsigned long long v = ((unsigned long long)(c >> 16) << 32) | (c & 0xFFFFu);
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  if (lane_id() == 0) lds[threadIdx.x / kWave] = v;
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned long long t = 0;
    for (int i = 0; i < kBlock / kWave; ++i) t += lds[i];
    super_cnt[(uint64_t)row * nsup + blockIdx.x] = t;
  }
}

__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// One wave per group of GROUP consecutive buckets (GROUP = 1, 8 or 64, chosen so that the
// launch has enough waves; a group never straddles a super-bucket).  The first GROUP lanes
// fetch the group's counters; a wave with a non-empty bucket adds up the super-buckets and
// buckets before its group (its place in the message), then walks its non-empty buckets;
// inside a bucket lane l owns words 2l and 2l+1 of both bitmaps.
template <int GROUP>
__global__ __launch_bounds__(kBlock) void k_emit_bitmap(
    float* __restrict__ x, uint64_t d, uint32_t K, const FastSel* __restrict__ sel,
    uint32_t* __restrict__ bm_gt, uint32_t* __restrict__ bm_eq, uint64_t words_per_row,
    const uint32_t* __restrict__ bucket_cnt, uint32_t nbk,
    const unsigned long long* __restrict__ super_cnt, uint32_t nsup,
    const uint32_t* __restrict__ need, uint32_t* __restrict__ out_idx,
    float* __restrict__ out_val) {
  const uint32_t row = blockIdx.y;
  if (need[row]) return;
  const uint32_t group = blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
  const uint32_t first = group * GROUP;                      // first bucket of the group
  const uint32_t bk_mine = first + lane_id();
  const uint32_t* bc = bucket_cnt + (uint64_t)row * nbk;
  const uint32_t my_cnt = (lane_id() < GROUP && bk_mine < nbk) ? bc[bk_mine] : 0u;
  uint64_t live = __ballot(my_cnt != 0);
  if (live == 0) return;
  const uint32_t r = sel[row].r;
  // counts before the group: whole super-buckets, then the buckets of this super-bucket
  const uint32_t sup = first >> kSuperShift;
  const unsigned long long* sc = super_cnt + (uint64_t)row * nsup;
  unsigned long long before = 0;
  for (uint32_t s = lane_id(); s < sup; s += kWave) before += sc[s];
  for (uint32_t b = (sup << kSuperShift) + lane_id(); b < first; b += kWave) {
    const uint32_t c = bc[b];
    before += ((unsigned long long)(c >> 16) << 32) | (c & 0xFFFFu);
  }
  before = wave_sum_u64(before);
  // exclusive prefix over the buckets of the group (packed: equal << 16 | greater; a group
  // holds at most 64 * 4096 coordinates, so sum the halves separately)
  const uint32_t incl_gt = wave_inclusive_scan(my_cnt & 0xFFFFu);
  const uint32_t incl_eq = wave_inclusive_scan(my_cnt >> 16);
  const uint32_t my_gt0 = (uint32_t)(before & 0xFFFFFFFFull) + incl_gt - (my_cnt & 0xFFFFu);
  const uint32_t my_eq0 = (uint32_t)(before >> 32) + incl_eq - (my_cnt >> 16);
  uint32_t* wg = bm_gt + (uint64_t)row * words_per_row;
  uint32_t* we = bm_eq + (uint64_t)row * words_per_row;
  float* xr = x + (uint64_t)row * d;
  uint32_t* oi = out_idx + (uint64_t)row * K;
  float* ov = out_val + (uint64_t)row * K;
  // the group's slice of the message
  const uint32_t grp_gt0 = __shfl(my_gt0, 0, kWave), grp_eq0 = __shfl(my_eq0, 0, kWave);
  const uint32_t grp_gt1 = grp_gt0 + __shfl(incl_gt, kWave - 1, kWave);
  const uint32_t grp_eq1 = grp_eq0 + __shfl(incl_eq, kWave - 1, kWave);
  const uint32_t p_first = grp_gt0 + min(grp_eq0, r);
  const uint32_t p_end = min(grp_gt1 + min(grp_eq1, r), K);
  // Part one writes the indices only.  The words of up to kBatch buckets are fetched before
  // any of them is walked, so a wave waits for memory once per batch, not once per bucket.
  constexpr int kBatch = GROUP < 8 ? GROUP : 8;
  while (live) {
    int src[kBatch];
#pragma unroll
    for (int b = 0; b < kBatch; ++b) {
      src[b] = live ? __ffsll((unsigned long long)live) - 1 : -1;
      live &= live - 1;
    }
    uint32_t g0[kBatch], g1[kBatch], e0[kBatch], e1[kBatch];
#pragma unroll
    for (int b = 0; b < kBatch; ++b) {
      g0[b] = g1[b] = e0[b] = e1[b] = 0;
      if (src[b] < 0) continue;
      const uint32_t cnt = __shfl(my_cnt, src[b], kWave);
      const uint64_t w0 = (uint64_t)(first + src[b]) * kBucketWords + 2u * lane_id();
      if (cnt & 0xFFFFu) {
        if (w0 < words_per_row) g0[b] = wg[w0];
        if (w0 + 1 < words_per_row) g1[b] = wg[w0 + 1];
      }
      if (cnt >> 16) {
        if (w0 < words_per_row) e0[b] = we[w0];
        if (w0 + 1 < words_per_row) e1[b] = we[w0 + 1];
      }
    }
#pragma unroll
    for (int b = 0; b < kBatch; ++b) {
      if (src[b] < 0) continue;
      const uint64_t w0 = (uint64_t)(first + src[b]) * kBucketWords + 2u * lane_id();
      // per lane at most 64 bits of each kind: the packed scan cannot carry across halves
      const uint32_t mine =
          (__popc(g0[b]) + __popc(g1[b])) | ((__popc(e0[b]) + __popc(e1[b])) << 16);
      const uint32_t pre = wave_inclusive_scan(mine) - mine;
      uint32_t n_gt = __shfl(my_gt0, src[b], kWave) + (pre & 0xFFFFu);   // greater before me
      uint32_t n_eq = __shfl(my_eq0, src[b], kWave) + (pre >> 16);       // equal before me
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const uint32_t gb = half == 0 ? g0[b] : g1[b], eb = half == 0 ? e0[b] : e1[b];
        uint32_t bits = gb | eb;
        const uint32_t base = (uint32_t)((w0 + half) * 32u);
        while (bits) {
          const uint32_t t = __ffs(bits) - 1;
          bits &= bits - 1;
          const bool is_gt = (gb >> t) & 1u;
          if (is_gt || n_eq < r) {
            const uint32_t pos = n_gt + min(n_eq, r);
            if (pos < K) oi[pos] = base + t;
          }
          n_gt += is_gt ? 1u : 0u;
          n_eq += is_gt ? 0u : 1u;
        }
      }
      if (g0[b]) wg[w0] = 0;
      if (g1[b]) wg[w0 + 1] = 0;
      if (e0[b]) we[w0] = 0;
      if (e1[b]) we[w0 + 1] = 0;
    }
  }
  // Part two: the values, one lane per entry of the group's slice.  The indices were stored
  // by this wave; the workgroup-scope fence orders those stores before the loads.
  __threadfence_block();
  for (uint32_t p = p_first + lane_id(); p < p_end; p += kWave) {
    const uint32_t idx = oi[p];
    if (idx < d) {
      ov[p] = xr[idx];
      xr[idx] = 0.0f;
    }
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
  // Below about 25 M coordinates per call the step is bound by kernel launches and the
  // dense path, with fewer launches, is the quicker one (measured: dense ahead at 24 M,
  // single-pass ahead from 25.5 M on).
  p.preferred = (uint64_t)rows * d >= 25000000ull;
  const uint64_t slices = d / 256;
  uint64_t stride = K / 64;        // about 128 of the sampled coordinates fall in the top 2K
  if (stride < 16) stride = 16;
  if (stride > 4096) stride = 4096;
  if (stride > slices / 64) stride = slices / 64;
  if (stride < 1) stride = 1;
  uint64_t target = (2ull * K + stride - 1) / stride;
  if (target < 48) target = 48;
  // expected list length is 2K..4K (the bound is a histogram bin edge); each of the 64
  // lists gets twice its even share of 4x the target plus slack
  uint64_t cap = (4 * target * stride + 4096) / 64 * 2 + 64;
  p.enabled = true;
  p.stride = (uint32_t)stride;
  p.target = (uint32_t)target;
  p.cap = (uint32_t)cap;
  p.nbk = (uint32_t)((d + 4095) / 4096);
  p.nsup = (p.nbk + (1u << kSuperShift) - 1) >> kSuperShift;
  p.words_per_row = (d + 31) / 32;
  return p;
}

hipError_t fast_select(hipStream_t s, const FastScratch& sc, const FastPlan& pl, const float* g,
                       float* x, uint32_t rows, uint64_t d, uint32_t K, float alpha,
                       uint32_t* out_idx, float* out_val, hipEvent_t ev0, hipEvent_t ev1) {
  const dim3 block(kBlock);
  const uint32_t nwc = (uint32_t)((d + kWaveChunk - 1) / kWaveChunk) + 1;
  const dim3 dense_grid((nwc + kStreamWaves - 1) / kStreamWaves, rows);
  unsigned long long* super_cnt = reinterpret_cast<unsigned long long*>(sc.super_cnt);
  if (*sc.dirty) {       // an earlier call failed between marking and emission: clear the bits
    hipError_t e = fill_u32(s, sc.bitmap_gt, (uint64_t)sc.rows * pl.words_per_row, 0);
    if (e == hipSuccess) e = fill_u32(s, sc.bitmap_eq, (uint64_t)sc.rows * pl.words_per_row, 0);
    if (e == hipSuccess) e = fill_u32(s, sc.sample_hist, (uint64_t)sc.rows * kSampleBins, 0);
    if (e != hipSuccess) return e;
  }
  *sc.dirty = true;      // cleared when every launch of this call went out
  // 1. sample
  const uint64_t n_samp = (d / 256) / pl.stride + 1;
  uint32_t sample_blocks = (uint32_t)((n_samp + kWavesPerBlock * 8 - 1) / (kWavesPerBlock * 8));
  if (sample_blocks > 64) sample_blocks = 64;
  if (sample_blocks < 1) sample_blocks = 1;
  if (g != nullptr)
    k_sample_hist<true><<<dim3(sample_blocks, rows), block, 0, s>>>(
        g, x, d, alpha, pl.stride, sc.sample_hist, sc.bucket_cnt, pl.nbk);
  else
    k_sample_hist<false><<<dim3(sample_blocks, rows), block, 0, s>>>(
        nullptr, x, d, 0.0f, pl.stride, sc.sample_hist, sc.bucket_cnt, pl.nbk);
  BTS_LAUNCH_CHECK();
  k_pick_bound<<<dim3(rows), block, 0, s>>>(sc.sample_hist, pl.target, sc.lower_key, sc.cand_cnt);
  BTS_LAUNCH_CHECK();
  // 2. the dense pass
  if (ev0) (void)hipEventRecord(ev0, s);
  if (g != nullptr)
    k_stream_capture<true><<<dense_grid, dim3(kStreamBlock), 0, s>>>(
        g, x, d, alpha, sc.lower_key, sc.cand_cnt, sc.cand, pl.cap);
  else
    k_stream_capture<false><<<dense_grid, dim3(kStreamBlock), 0, s>>>(
        nullptr, x, d, 0.0f, sc.lower_key, sc.cand_cnt, sc.cand, pl.cap);
  BTS_LAUNCH_CHECK();
  if (ev1) (void)hipEventRecord(ev1, s);
  // 3 + 4. verify and select: a few blocks per row, each taking whole lists (about 4096
  // entries per block)
  uint32_t hb = (uint32_t)(((uint64_t)pl.cap * kSubLists / 2 + 4095) / 4096);
  if (hb > kMaxHistBlocks) hb = kMaxHistBlocks;
  if (hb < 1) hb = 1;
  const dim3 hgrid(hb, rows);
  FastSel* sel = reinterpret_cast<FastSel*>(sc.sel);
#define BTS_CAND_PASS(P)                                                                     \
  k_cand_hist<P><<<hgrid, block, 0, s>>>(sc.cand, sc.cand_cnt, pl.cap, K, sc.hist, sel,      \
                                         sc.need);                                           \
  BTS_LAUNCH_CHECK();                                                                        \
  k_cand_scan<P><<<dim3(rows), block, 0, s>>>(sc.hist, hb, K, sel, sc.need);                 \
  BTS_LAUNCH_CHECK();
  BTS_CAND_PASS(0)
  BTS_CAND_PASS(1)
  BTS_CAND_PASS(2)
#undef BTS_CAND_PASS
  // 5. emit
  uint32_t parts = (pl.cap + 2047) / 2048;            // blocks per list
  if (parts > 4) parts = 4;
  if (parts < 1) parts = 1;
  k_mark<<<dim3(kSubLists * parts, rows), block, 0, s>>>(
      sc.cand, sc.cand_cnt, pl.cap, sel, sc.need, sc.bitmap_gt, sc.bitmap_eq, pl.words_per_row,
      sc.bucket_cnt, pl.nbk);
  BTS_LAUNCH_CHECK();
  k_super_sums<<<dim3(pl.nsup, rows), block, 0, s>>>(sc.bucket_cnt, pl.nbk, super_cnt, pl.nsup,
                                                     sc.need);
  BTS_LAUNCH_CHECK();
  // enough waves to fill the chip, few enough that empty groups stay cheap
  const uint64_t buckets = (uint64_t)rows * pl.nbk;
  const int group = buckets >= (64ull << 16) ? 64 : (buckets >= (8ull << 14) ? 8 : 1);
  const uint32_t groups = (pl.nbk + group - 1) / group;
  const dim3 egrid((groups + kWavesPerBlock - 1) / kWavesPerBlock, rows);
#define BTS_EMIT(G)                                                                          \
  k_emit_bitmap<G><<<egrid, block, 0, s>>>(x, d, K, sel, sc.bitmap_gt, sc.bitmap_eq,          \
                                           pl.words_per_row, sc.bucket_cnt, pl.nbk, super_cnt, \
                                           pl.nsup, sc.need, out_idx, out_val)
  if (group == 64)
    BTS_EMIT(64);
  else if (group == 8)
    BTS_EMIT(8);
  else
    BTS_EMIT(1);
#undef BTS_EMIT
  BTS_LAUNCH_CHECK();
  *sc.dirty = false;
  return hipSuccess;
}

size_t fast_sel_bytes() { return sizeof(FastSel); }
uint32_t fast_sublists() { return kSubLists; }
uint32_t fast_counter_stride() { return kCounterStride; }
uint32_t fast_hist_blocks() { return kMaxHistBlocks; }

}  // namespace bts
