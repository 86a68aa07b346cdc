// Speculative single-pass Top_K select.
//
// The method's floor is one read of g, one read of eps and one write of eps per
// coordinate.  A radix select that histograms first and gathers afterwards reads the row
// again; this path avoids the second read for typical inputs and stays exact:
//
//   1. bounds:   on a scratch's first two calls a strided sample (256-coordinate slices,
//                every S-th slice) of a = eps + alpha g is histogrammed on the top 13 bits of
//                the magnitude key; a lower bound L is chosen so that between 1.15 K and 2 K
//                coordinates of the row (by the sample's size) are expected at or above it,
//                and a bound U near the K-th largest key.  Later calls take both from the
//                exact threshold the call before found (cand_finish_body): no sample.
//   2. stream:   the one dense pass computes a, stores it over eps (+0 instead where
//                key >= U: those coordinates are almost surely sent, which spares the
//                emission most of its scattered zero stores) and appends every coordinate
//                with key >= L to the row's candidate lists: the hits of a wave chunk (512
//                coordinates) go, in index order, into one run of one list (one atomic add
//                per chunk with hits), and the chunk notes where its run starts and how long
//                it is in the row's chunk directory.
//   3. verify:   if no list overflowed and the lists hold at least K entries, the K largest
//                of the row are all listed.  Otherwise the row is flagged, gets back the
//                values that step 2 replaced by +0, and the dense path (which reads the
//                stored a again) redoes it.  The result never depends on L or U.
//   4. select:   exact radix select of the K-th largest key T over the lists, on key - L in
//                a 13-bit and a 12-bit digit, and r = how many holders of T are kept (a row
//                whose T lies more than four octaves above L goes to the dense path too).
//   5. emit:     the directory in chunk order names the candidates in index order.  Count
//                the entries greater than / equal to T per tile of 64 chunks, scan the
//                tiles, then walk each tile again: an entry is kept if it is greater, or
//                equal with fewer than r equal ones before it (lower index wins); its place
//                in the message is #greater before + min(#equal before, r).  The pair comes
//                from the list (no second read of eps), +0 is stored to eps there unless
//                step 2 did (and the value goes back where step 2 zeroed a coordinate that
//                is not sent after all), and the directory entries are zeroed for the next
//                call.
//
// Steps 4-5 touch O(K) data.  Used for the worker compression (rows = N, fused with the
// error compensation of Algorithm 2) and for the server compression (one row, no fusion).
//
// Two facts of this part shaped the kernels: atomics that return a value on one address are
// served at the memory side at a few million per second, and a device-scope fence writes
// back the XCD's L2.  Hence many append counters on separate 128-byte lines, one append per
// wave chunk, per-block partial histograms with plain stores, kernel boundaries instead of
// last-block-done tickets, and an emission that needs no atomics at all.

#include "capture_bodies.h"
#include "dense_bodies.h"

namespace bts {

namespace {

constexpr int kSampleBits = 13;                       // top bits of the 31-bit key
constexpr int kSampleBins = 1 << kSampleBits;         // 8192
constexpr int kSampleShift = 31 - kSampleBits;        // 18
constexpr uint32_t kSlice = kWave * 4;                // 256 coordinates: one f4 per lane
constexpr int kSliceUnroll = 8;
// blocks per row in a candidate pass (16 take 2 us off the first pass at 16 x 1.4e5 entries and
// add 5 us to the two kernels that add their partial histograms up)
constexpr uint32_t kMaxHistBlocks = 8;

// ---- 1. sample histogram ------------------------------------------------------------
// Slices are cut at absolute multiples of 256 coordinates (16-byte aligned); only slices
// that lie entirely inside the row are sampled.
template <bool FMA>
__global__ __launch_bounds__(kBlock) void k_sample_hist(
    const float* __restrict__ g, const float* __restrict__ x, uint64_t d, float alpha,
    uint32_t stride, uint32_t* __restrict__ shist) {
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
        xv[u] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(x + e));
        if (FMA) gv[u] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(g + e));
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
//
// target_u != 0: also choose the bound U from which the dense pass stores +0 instead of a
// (see capture_chunk): the bin edge whose count of sampled coordinates at or above it comes
// closest to target_u = K / stride, i.e. closest to K coordinates of the row.  Every
// coordinate between U and the threshold, on either side, costs one scattered store later,
// so the closest edge is the cheapest; no choice of U can make the result wrong.
constexpr uint32_t kNeverKey = 0xFFFFFFFFu;           // above every 31-bit key

__global__ __launch_bounds__(kBlock) void k_pick_bound(uint32_t* __restrict__ shist,
                                                       uint32_t target, uint32_t target_u,
                                                       uint32_t* __restrict__ lower_key,
                                                       uint32_t* __restrict__ upper_key,
                                                       uint32_t* __restrict__ cand_cnt) {
  constexpr int BPT = kSampleBins / kBlock;   // 32
  __shared__ uint32_t lds[kBlock / kWave + 1];
  __shared__ uint32_t s_bin, s_ubin;
  const uint32_t row = blockIdx.x;
  uint32_t* h = shist + (uint64_t)row * kSampleBins;
  const int top = kSampleBins - 1 - (int)threadIdx.x * BPT;
  uint32_t s = 0;
  for (int i = 0; i < BPT; ++i) s += h[top - i];
  if (threadIdx.x == 0) {
    s_bin = 0;
    s_ubin = kSampleBins;                     // no bound found: nothing is zeroed early
  }
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
  if (target_u != 0 && excl < target_u && target_u <= excl + s) {
    uint32_t acc = excl;
    for (int i = 0; i < BPT; ++i) {
      const uint32_t c = h[top - i];
      if (acc + c >= target_u) {
        // at or above bin top - i: acc + c samples; above it: acc
        const bool upper_edge = target_u - acc < acc + c - target_u;
        s_ubin = (uint32_t)(top - i) + (upper_edge ? 1u : 0u);
        break;
      }
      acc += c;
    }
  }
  __syncthreads();
  for (int i = 0; i < BPT; ++i) h[top - i] = 0;
  if (threadIdx.x == 0) {
    lower_key[row] = s_bin << kSampleShift;
    // never below the lower bound (the two targets can land in one bin)
    const uint32_t ub = s_ubin < s_bin ? s_bin : s_ubin;
    upper_key[row] = ub >= (uint32_t)kSampleBins ? kNeverKey : ub << kSampleShift;
  }
  if (threadIdx.x < kSubLists)
    cand_cnt[((uint64_t)row * kSubLists + threadIdx.x) * kCounterStride] = 0;
}


// WPS: the most waves per SIMD (four SIMDs per compute unit) the kernel may run with; the
// compiler sizes the kernel's register allocation so that no more fit (kMaxWavesPerSimd =
// no limit).  A stream of 2 reads : 1 write runs best well below full occupancy, see
// fast_plan.
constexpr int kMaxWavesPerSimd = 8;

template <bool FMA, bool ENERGY, int WPS>
__global__ __launch_bounds__(kStreamBlock) __attribute__((amdgpu_waves_per_eu(1, WPS))) void
k_stream_capture(const float* __restrict__ g, float* __restrict__ x, uint64_t d, float alpha,
                 const uint32_t* __restrict__ lower_key, const uint32_t* __restrict__ upper_key,
                 uint32_t* __restrict__ cand_cnt, uint2* __restrict__ cand, uint32_t cap,
                 uint2* __restrict__ dir, uint32_t nwc_pad, double* __restrict__ energy) {
  const uint32_t row = blockIdx.y;
  capture_chunk<FMA, ENERGY>(row, blockIdx.x * kStreamWaves + threadIdx.x / kWave, lower_key[row],
                             FMA ? upper_key[row] : kNeverKey, g, x, d, alpha, cand_cnt, cand,
                             cap, dir, nwc_pad, energy);
}

// ---- 3 + 4. verify and select on the candidate lists -------------------------------------

// Every candidate has key >= L, and the K-th largest key T usually lies within an octave
// of L, so the select works on off = key - L in two digits: d0 = min(off >> 12, 8191) and
// d1 = off & 4095.  If T falls into the clamped top bin of d0 (T >= L + 2^25 - 2^12, a
// bound sixteen times too low) the row is handed to the dense path instead (need = 2).
//
//   k_cand_hist0:  verifies the row (no list overflowed, at least K entries: then the K
//                  largest of the row are all listed; else need = 1) and histograms d0.
//   k_cand_hist1:  every block resolves d0 from the partial histograms (and, in the same
//                  steps, the bin of the entry at the rank the next call's bound aims at),
//                  then histograms d1 of the entries in d0's bin.
//   k_finish_hist0: one block per row resolves d1: T and r (cand_finish_body), and leaves
//                  the next call's bounds.
//
// A few fat blocks per row, each histogramming its share of the lists in LDS.  The d0
// histograms are stored per block with plain stores (no cross-block atomics, no fences,
// nothing to clear) and added up by the blocks of the next kernel, coarse sums first; the d1
// histogram, which has a few hundred entries at most unless the threshold is a much-repeated
// value, is added to one histogram of the row, which the finishing block zeroes again.
constexpr int kD1Bits = 12;
constexpr int kD0Bins = 8192, kD1Bins = 1 << kD1Bits;
constexpr int kD0Coarse = 256;                        // sums over 32 consecutive d0 bins
constexpr int kD0PerCoarse = kD0Bins / kD0Coarse;
// partial histograms of one block: d0, d1, then the coarse sums of d0
constexpr uint32_t kPartWords = kD0Bins + kD1Bins + kD0Coarse;
constexpr uint32_t kCoarseAt = kD0Bins + kD1Bins;
constexpr int kCandBlock = 1024;                      // threads per block of the histogram kernels
constexpr int kListUnroll = 4;                        // list entries per lane in flight

// How the waves of a row's blocks (gridDim.x blocks of 16 waves) divide the row's 64 lists.
struct ListShare {
  uint32_t first, list_step;     // the wave's lists: first, first + list_step, ...
  uint32_t part, parts;          // of each list, every parts-th group of 256 entries from part
};

__device__ __forceinline__ ListShare list_share() {
  constexpr uint32_t kWavesPerCandBlock = kCandBlock / kWave;
  const uint32_t v = blockIdx.x * kWavesPerCandBlock + threadIdx.x / kWave;
  const uint32_t waves = gridDim.x * kWavesPerCandBlock;
  ListShare ls;
  if (waves >= kSubLists) {              // 64 | waves for every grid the host chooses (4, 8 blocks)
    ls.first = v % kSubLists;
    ls.list_step = kSubLists;
    ls.part = v / kSubLists;
    ls.parts = waves / kSubLists;
  } else {
    ls.first = v;
    ls.list_step = waves;
    ls.part = 0;
    ls.parts = 1;
  }
  return ls;
}

__global__ __launch_bounds__(kCandBlock) void k_cand_hist0(const uint2* __restrict__ cand,
                                                       const uint32_t* __restrict__ cand_cnt,
                                                       uint32_t cap, uint32_t K,
                                                       const uint32_t* __restrict__ lower_key,
                                                       uint32_t* __restrict__ partial,
                                                       uint32_t* __restrict__ need) {
  __shared__ uint32_t sh[kD0Bins];
  __shared__ uint32_t s_need;
  const uint32_t row = blockIdx.y;
  if (threadIdx.x < kWave) {
    const uint32_t c = cand_cnt[((uint64_t)row * kSubLists + threadIdx.x) * kCounterStride];
    const uint32_t total = wave_sum(c);
    const bool over = __ballot(c > cap) != 0;
    if (threadIdx.x == 0) {
      s_need = (over || total < K) ? 1u : 0u;
      if (blockIdx.x == 0) need[row] = s_need;
    }
  }
  for (int i = threadIdx.x; i < kD0Bins; i += kCandBlock) sh[i] = 0;
  __syncthreads();
  if (s_need) return;
  const uint32_t L = lower_key[row];
  // the row's waves share the lists: wave v of the row takes list v % 64 and, where the row
  // has more than 64 waves, every (v / 64)-th group of 256 entries of it; four entries per
  // lane in flight (a list holds thousands of entries where K is a percent of d)
  const ListShare ls = list_share();
  for (uint32_t sl = ls.first; sl < kSubLists; sl += ls.list_step) {
    const uint64_t sub = (uint64_t)row * kSubLists + sl;
    const uint32_t cnt = cand_cnt[sub * kCounterStride];
    const uint2* list = cand + sub * cap;
    for (uint32_t j0 = ls.part * kWave * kListUnroll + lane_id(); j0 < cnt;
         j0 += ls.parts * kWave * kListUnroll) {
      uint32_t key[kListUnroll];
#pragma unroll
      for (int u = 0; u < kListUnroll; ++u) {
        const uint32_t j = j0 + u * kWave;
        key[u] = j < cnt ? list[j].y : 0u;
      }
#pragma unroll
      for (int u = 0; u < kListUnroll; ++u) {
        if (j0 + u * kWave >= cnt) break;
        const uint32_t off = (key[u] & 0x7FFFFFFFu) - L;
        atomicAdd(&sh[min(off >> kD1Bits, (uint32_t)kD0Bins - 1)], 1u);
      }
    }
  }
  __syncthreads();
  uint32_t* out = partial + ((uint64_t)row * gridDim.x + blockIdx.x) * kPartWords;
  for (int i = threadIdx.x; i < kD0Bins; i += kCandBlock) out[i] = sh[i];
  if (threadIdx.x < kD0Coarse) {        // rotated start: no LDS bank conflicts
    uint32_t c = 0;
    for (int i = 0; i < kD0PerCoarse; ++i)
      c += sh[threadIdx.x * kD0PerCoarse + ((i + threadIdx.x) & (kD0PerCoarse - 1))];
    out[kCoarseAt + threadIdx.x] = c;
  }
}

// The d0 bin holding the K-th largest entry from the blocks' partial histograms, coarse sums
// first (256 x nparts words), then the 32 bins of the coarse bin found (32 x nparts words)
// instead of all 8192 x nparts.  *above = entries in higher bins.  In the same steps, with
// the second wave of the block: *bin_next = the bin of the entry at rank `rank_next` (0 if
// the lists hold fewer entries).  All threads call this (at least 256).
__device__ __forceinline__ uint32_t resolve_d0(const uint32_t* __restrict__ part_row,
                                               uint32_t nparts, uint32_t K, uint32_t rank_next,
                                               uint32_t* lds, uint32_t* s_out, uint32_t* above,
                                               uint32_t* bin_next) {
  const int cb = kD0Coarse - 1 - (int)threadIdx.x;        // this thread's coarse bin (if >= 0)
  uint32_t c = 0;
  if (cb >= 0)
    for (uint32_t b = 0; b < nparts; ++b) c += part_row[(uint64_t)b * kPartWords + kCoarseAt + cb];
  uint32_t total;
  const uint32_t excl = block_exclusive_scan(c, lds, &total);
  if (threadIdx.x < 4) s_out[threadIdx.x] = 0;
  __syncthreads();
  if (cb >= 0 && excl < K && K <= excl + c) {
    s_out[0] = (uint32_t)cb;
    s_out[1] = excl;
  }
  if (cb >= 0 && excl < rank_next && rank_next <= excl + c) {
    s_out[2] = (uint32_t)cb;
    s_out[3] = excl;
  }
  __syncthreads();
  const uint32_t which = threadIdx.x / kWave;             // wave 0: K, wave 1: rank_next
  const uint32_t e = s_out[2 * (which & 1u)], above_e = s_out[2 * (which & 1u) + 1];
  const uint32_t want = which == 0 ? K : rank_next;
  __syncthreads();
  if (which < 2) {
    const int fb = kD0PerCoarse - 1 - (int)lane_id();
    uint32_t f = 0;
    if (fb >= 0)
      for (uint32_t b = 0; b < nparts; ++b)
        f += part_row[(uint64_t)b * kPartWords + e * kD0PerCoarse + fb];
    const uint32_t incl = wave_inclusive_scan(f);
    const uint32_t before = above_e + incl - f;
    if (fb >= 0 && before < want && want <= before + f) {
      s_out[2 * which] = e * kD0PerCoarse + (uint32_t)fb;
      s_out[2 * which + 1] = before;
    }
  }
  __syncthreads();
  const uint32_t bin = s_out[0];
  *above = s_out[1];
  *bin_next = s_out[2];
  __syncthreads();
  return bin;
}

// A row that goes to the dense path gets back the values the dense pass replaced by +0 (the
// listed entries with key >= U; a run that did not fit was written back by its own wave).
// The row's blocks walk its lists with the shares of the histogram passes.
__device__ __forceinline__ void restore_early_zeros(uint32_t row, const uint2* __restrict__ cand,
                                                    const uint32_t* __restrict__ cand_cnt,
                                                    uint32_t cap, uint32_t U,
                                                    float* __restrict__ x, uint64_t d) {
  if (U == kNeverKey) return;
  float* xr = x + (uint64_t)row * d;
  const ListShare ls = list_share();
  for (uint32_t sl = ls.first; sl < kSubLists; sl += ls.list_step) {
    const uint64_t sub = (uint64_t)row * kSubLists + sl;
    const uint32_t cnt = min(cand_cnt[sub * kCounterStride], cap);
    const uint2* list = cand + sub * cap;
    for (uint32_t j0 = ls.part * kWave * kListUnroll + lane_id(); j0 < cnt;
         j0 += ls.parts * kWave * kListUnroll) {
#pragma unroll
      for (int u = 0; u < kListUnroll; ++u) {
        const uint32_t j = j0 + u * kWave;
        if (j >= cnt) break;
        const uint2 en = list[j];
        if ((en.y & 0x7FFFFFFFu) >= U && en.x < d) xr[en.x] = __uint_as_float(en.y);
      }
    }
  }
}

__global__ __launch_bounds__(kCandBlock) void k_cand_hist1(const uint2* __restrict__ cand,
                                                       const uint32_t* __restrict__ cand_cnt,
                                                       uint32_t cap, uint32_t K,
                                                       uint32_t rank_next,
                                                       const uint32_t* __restrict__ lower_key,
                                                       const uint32_t* __restrict__ upper_key,
                                                       uint32_t* __restrict__ partial,
                                                       FastSel* __restrict__ sel,
                                                       uint32_t* __restrict__ need,
                                                       float* __restrict__ x, uint64_t d) {
  __shared__ uint32_t sh[kD1Bins];
  __shared__ uint32_t lds[kCandBlock / kWave + 1];
  __shared__ uint32_t s_out[4];
  const uint32_t row = blockIdx.y;
  if (need[row] == 1u) {                   // set by the previous kernel; 2 is set below
    restore_early_zeros(row, cand, cand_cnt, cap, upper_key[row], x, d);
    return;
  }
  uint32_t* part_row = partial + (uint64_t)row * gridDim.x * kPartWords;
  uint32_t above, bin_next;
  const uint32_t b0 = resolve_d0(part_row, gridDim.x, K, rank_next, lds, s_out, &above,
                                 &bin_next);
  if (b0 == (uint32_t)kD0Bins - 1) {       // T is beyond the window: the dense path redoes the row
    if (blockIdx.x == 0 && threadIdx.x == 0) need[row] = 2u;
    restore_early_zeros(row, cand, cand_cnt, cap, upper_key[row], x, d);
    return;
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    sel[row].prefix = b0;
    sel[row].k_rem = K - above;
    sel[row].next_bin = bin_next;
  }
  for (int i = threadIdx.x; i < kD1Bins; i += kCandBlock) sh[i] = 0;
  __syncthreads();
  const uint32_t L = lower_key[row];
  const ListShare ls = list_share();
  for (uint32_t sl = ls.first; sl < kSubLists; sl += ls.list_step) {
    const uint64_t sub = (uint64_t)row * kSubLists + sl;
    const uint32_t cnt = cand_cnt[sub * kCounterStride];
    const uint2* list = cand + sub * cap;
    for (uint32_t j0 = ls.part * kWave * kListUnroll + lane_id(); j0 < cnt;
         j0 += ls.parts * kWave * kListUnroll) {
      uint32_t key[kListUnroll];
#pragma unroll
      for (int u = 0; u < kListUnroll; ++u) {
        const uint32_t j = j0 + u * kWave;
        key[u] = j < cnt ? list[j].y : 0u;
      }
#pragma unroll
      for (int u = 0; u < kListUnroll; ++u) {
        if (j0 + u * kWave >= cnt) break;
        const uint32_t off = (key[u] & 0x7FFFFFFFu) - L;
        if ((off >> kD1Bits) == b0) atomicAdd(&sh[off & (kD1Bins - 1)], 1u);
      }
    }
  }
  __syncthreads();
  // The threshold's bin holds few entries (a few hundred of a row's hundred thousand
  // candidates), so the blocks add their few non-zero counts to ONE histogram of the row (the
  // d1 part of the row's first partial, zero between calls) instead of storing 4096 words each
  // for the next kernel to add up.
  uint32_t* out = part_row + kD0Bins;
  for (int i = threadIdx.x; i < kD1Bins; i += kCandBlock) {
    const uint32_t v = sh[i];
    if (v) atomicAdd(&out[i], v);
  }
}

// Also sets the row's bounds for the NEXT call on this scratch, which then needs no sample:
// the threshold moves little from one step of the training to the next, and this call knows
// it exactly.  The lower bound becomes the key this call found at rank rank_next (a rank
// beyond K, so that about rank_next - K spare candidates are listed), the bound of the early
// zeroing becomes the threshold itself, both moved along with the relative change of the
// threshold over the last call (the residuals of a young run grow from step to step, ever
// more slowly): the zeroing bound by 0.8 of it, which is about unbiased for such a run, the
// lower bound by half of it, which errs towards more candidates.  A wrong guess costs time,
// never the result: the next call verifies its lists like any other and hands a row whose
// lists fall short or overflow to the dense path, whose emission sets the row's bounds from
// its exact threshold instead (k_emit).
__device__ __forceinline__ void cand_finish_body(uint32_t row,
                                                 uint32_t* __restrict__ partial,
                                                 uint32_t nparts, bool early_zero,
                                                 uint32_t* __restrict__ lower_key,
                                                 uint32_t* __restrict__ upper_key,
                                                 uint32_t* __restrict__ prev_T,
                                                 uint32_t* __restrict__ cand_cnt,
                                                 FastSel* __restrict__ sel,
                                                 const uint32_t* __restrict__ need) {
  __shared__ uint32_t lds[kBlock / kWave + 1];
  __shared__ uint32_t s_out[2];
  // the lists are read through the directory from here on: counters clear for the next call
  if (threadIdx.x < kSubLists)
    cand_cnt[((uint64_t)row * kSubLists + threadIdx.x) * kCounterStride] = 0;
  if (need[row]) return;
  const FastSel s = sel[row];
  uint32_t* d1 = partial + (uint64_t)row * nparts * kPartWords + kD0Bins;   // the row's one d1 histogram
  uint32_t above;
  const uint32_t b1 = resolve_bins<kD1Bins, kBlock>(d1, 1, 0, s.k_rem, lds, s_out, &above);
  for (int i = threadIdx.x; i < kD1Bins; i += kBlock)     // zero again for the next call
    if (d1[i]) d1[i] = 0;
  if (threadIdx.x == 0) {
    const uint32_t b_next = s.next_bin;    // first-digit bin of the entry at rank rank_next
    const uint32_t L = lower_key[row];
    const uint32_t T = L + ((s.prefix << kD1Bits) | b1);
    sel[row].T = T;
    sel[row].r = s.k_rem - above;
    sel[row].U = early_zero ? upper_key[row] : kNeverKey;
    uint32_t key_next = L + (b_next << kD1Bits);           // <= T: rank_next > K
    if (key_next > T) key_next = T;
    const uint32_t was = prev_T[row];
    uint32_t L_next = key_next, U_next = T;
    if (T != 0 && T < 0x7F800000u) {                       // finite, non-zero: magnitudes scale
      float change = 0.0f;
      if (was != 0 && was < 0x7F800000u) {
        change = __uint_as_float(T) / __uint_as_float(was) - 1.0f;
        change = fminf(fmaxf(change, -0.2f), 0.5f);
      }
      L_next = __float_as_uint(__uint_as_float(key_next) * (1.0f + 0.5f * change)) & 0x7FFFFFFFu;
      U_next = __float_as_uint(__uint_as_float(T) * (1.0f + 0.8f * change)) & 0x7FFFFFFFu;
      if (L_next > U_next) L_next = U_next;
    }
    lower_key[row] = L_next;
    if (early_zero) upper_key[row] = U_next;
    prev_T[row] = T;
  }
}

// ---- 5. ordered emission through the chunk directory -------------------------------------
// The directory lists a row's runs in chunk order, and a run holds its entries in index
// order, so walking the directory visits the row's candidates in index order; nothing has
// to be sorted and no atomics are needed.  A wave works on a tile of 64 consecutive chunks
// at a time (chunk wc appends to list wc % 64, so lane l's chunk always uses list l): it
// scans the run lengths, then its lanes take the tile's entries round-robin in that order,
// finding an entry's run by bisection on the scanned lengths.
//
//   dir_count_body: per tile, how many entries are greater than T and how many equal T.
//   dir_scan_body:  per row, exclusive prefix of those pairs over the tiles.
//   dir_emit_body:  per tile again: an entry is kept if it is greater, or equal with fewer
//                than r equal ones before it (lower index wins); its place in the message
//                is #greater before + min(#equal before, r).  Writes the pair, stores +0 to
//                x there and zeroes the tile's directory entries (also for rows that the
//                dense path redoes).

template <int TPW>
__device__ __forceinline__ void dir_count_body(
    uint32_t bx, uint32_t row, const uint2* __restrict__ dir, uint32_t nwc_pad,
    const uint2* __restrict__ cand, uint32_t cap, const FastSel* __restrict__ sel,
    const uint32_t* __restrict__ need, unsigned long long* __restrict__ tile_cnt,
    uint32_t ntiles) {
  __shared__ uint32_t s_off[kWavesPerBlock][kTileChunks], s_start[kWavesPerBlock][kTileChunks];
  if (need[row]) return;
  const uint32_t w = threadIdx.x / kWave;
  const uint32_t quarter = (ntiles + TPW - 1) / TPW;
  const uint32_t v = bx * kWavesPerBlock + w;
  if (v >= quarter) return;
  const uint2* dir_row = dir + (uint64_t)row * nwc_pad;
  uint2 ent[TPW];
#pragma unroll
  for (int u = 0; u < TPW; ++u) {
    const uint32_t tile = v + u * quarter;
    ent[u] = tile < ntiles ? dir_row[(uint64_t)tile * kTileChunks + lane_id()] : make_uint2(0u, 0u);
  }
  const uint32_t T = sel[row].T;
  const uint2* cand_row = cand + (uint64_t)row * kSubLists * cap;
#pragma unroll
  for (int u = 0; u < TPW; ++u) {
    const uint32_t tile = v + u * quarter;
    if (tile >= ntiles) break;
    uint32_t gt = 0, eq = 0;
    if (__ballot(ent[u].y != 0) != 0) {
      const TileView t = publish_tile(ent[u], s_off[w], s_start[w]);
      for (uint32_t e0 = 0; e0 < t.total; e0 += kWave * kEmitUnroll) {
        uint32_t key[kEmitUnroll];
#pragma unroll
        for (int k = 0; k < kEmitUnroll; ++k) {
          const uint32_t e = e0 + k * kWave + lane_id();
          key[k] = e < t.total ? tile_entry(t, e, cand_row, cap).y & 0x7FFFFFFFu : 0u;
        }
#pragma unroll
        for (int k = 0; k < kEmitUnroll; ++k) {
          const uint32_t e = e0 + k * kWave + lane_id();
          gt += (e < t.total && key[k] > T) ? 1u : 0u;
          eq += (e < t.total && key[k] == T) ? 1u : 0u;
        }
      }
      gt = wave_sum(gt);
      eq = wave_sum(eq);
    }
    if (lane_id() == 0)
      tile_cnt[(uint64_t)row * ntiles + tile] = ((unsigned long long)eq << 32) | gt;
  }
}

// One block per row; every thread owns a contiguous share of the tiles.
__device__ __forceinline__ void dir_scan_body(uint32_t row,
                                              unsigned long long* __restrict__ tile_cnt,
                                              uint32_t ntiles,
                                              const uint32_t* __restrict__ need) {
  __shared__ uint32_t lds[kBlock / kWave + 1];
  if (need[row]) return;
  unsigned long long* tc = tile_cnt + (uint64_t)row * ntiles;
  const uint32_t per = (ntiles + kBlock - 1) / kBlock;
  const uint32_t lo = min(threadIdx.x * per, ntiles), hi = min(lo + per, ntiles);
  uint32_t gt = 0, eq = 0;
  for (uint32_t i = lo; i < hi; ++i) {
    const unsigned long long v = tc[i];
    gt += (uint32_t)v;
    eq += (uint32_t)(v >> 32);
  }
  uint32_t total;
  uint32_t run_gt = block_exclusive_scan(gt, lds, &total);
  uint32_t run_eq = block_exclusive_scan(eq, lds, &total);
  for (uint32_t i = lo; i < hi; ++i) {
    const unsigned long long v = tc[i];
    tc[i] = ((unsigned long long)run_eq << 32) | run_gt;
    run_gt += (uint32_t)v;
    run_eq += (uint32_t)(v >> 32);
  }
}

// tile_energy (diagnostics only, else null): per tile, the fp64 sum of the squares of the
// tile's entries that are not kept.
template <int TPW>
__device__ __forceinline__ void dir_emit_body(
    uint32_t bx, uint32_t row, uint2* __restrict__ dir, uint32_t nwc_pad,
    const uint2* __restrict__ cand, uint32_t cap, const FastSel* __restrict__ sel,
    const uint32_t* __restrict__ need,
    const unsigned long long* __restrict__ tile_cnt, uint32_t ntiles, float* __restrict__ x,
    uint64_t d, uint32_t K, uint32_t* __restrict__ out_idx, float* __restrict__ out_val,
    double* __restrict__ tile_energy, FusedUpdate upd) {
  __shared__ uint32_t s_off[kWavesPerBlock][kTileChunks], s_start[kWavesPerBlock][kTileChunks];
  const uint32_t w = threadIdx.x / kWave;
  const uint32_t quarter = (ntiles + TPW - 1) / TPW;
  const uint32_t v = bx * kWavesPerBlock + w;
  if (v >= quarter) return;
  uint2* dir_row = dir + (uint64_t)row * nwc_pad;
  uint2 ent[TPW];
#pragma unroll
  for (int u = 0; u < TPW; ++u) {
    const uint32_t tile = v + u * quarter;
    ent[u] = tile < ntiles ? dir_row[(uint64_t)tile * kTileChunks + lane_id()] : make_uint2(0u, 0u);
    if (ent[u].y) dir_row[(uint64_t)tile * kTileChunks + lane_id()] = make_uint2(0u, 0u);
  }
  if (need[row]) return;
  const FastSel s = sel[row];
  const uint32_t U = s.U;                  // the dense pass stored +0 where key >= U
  const uint2* cand_row = cand + (uint64_t)row * kSubLists * cap;
  float* xr = x + (uint64_t)row * d;
  uint32_t* oi = out_idx + (uint64_t)row * K;
  float* ov = out_val + (uint64_t)row * K;
  const uint64_t below = lanes_below();
#pragma unroll
  for (int u = 0; u < TPW; ++u) {
    const uint32_t tile = v + u * quarter;
    if (tile >= ntiles) break;
    if (__ballot(ent[u].y != 0) == 0) {
      if (tile_energy != nullptr && lane_id() == 0)
        tile_energy[(uint64_t)row * ntiles + tile] = 0.0;
      continue;
    }
    double left = 0.0;                           // squares of the entries that stay behind
    const TileView t = publish_tile(ent[u], s_off[w], s_start[w]);
    const unsigned long long before = tile_cnt[(uint64_t)row * ntiles + tile];
    uint32_t run_gt = (uint32_t)before, run_eq = (uint32_t)(before >> 32);
    for (uint32_t e0 = 0; e0 < t.total; e0 += kWave * kEmitUnroll) {
      uint2 en[kEmitUnroll];
#pragma unroll
      for (int k = 0; k < kEmitUnroll; ++k) {
        const uint32_t e = e0 + k * kWave + lane_id();
        en[k] = e < t.total ? tile_entry(t, e, cand_row, cap) : make_uint2(0u, 0u);
      }
#pragma unroll
      for (int k = 0; k < kEmitUnroll; ++k) {
        const uint32_t e = e0 + k * kWave + lane_id();
        const uint32_t key = en[k].y & 0x7FFFFFFFu;
        const bool is_gt = e < t.total && key > s.T;
        const bool is_eq = e < t.total && key == s.T;
        const uint64_t m_gt = __ballot(is_gt), m_eq = __ballot(is_eq);
        const uint32_t n_gt = run_gt + __popcll(m_gt & below);       // greater before me
        const uint32_t n_eq = run_eq + __popcll(m_eq & below);       // equal before me
        if (is_gt || (is_eq && n_eq < s.r)) {
          const uint32_t pos = n_gt + min(n_eq, s.r);
          const uint32_t idx = en[k].x;
          if (pos < K && idx < d) {
            const float val = __uint_as_float(en[k].y);
            oi[pos] = idx;
            ov[pos] = val;
            if (key < U) xr[idx] = 0.0f;
            if (upd.w != nullptr) upd.w[idx] = __fmaf_rn(upd.neg_alpha, val, upd.w[idx]);
          }
        } else if (e < t.total) {
          // stays behind; if the dense pass took it for sent, its value goes back
          if (key >= U && en[k].x < d) xr[en[k].x] = __uint_as_float(en[k].y);
          const double val = (double)__uint_as_float(en[k].y);
          left += val * val;
        }
        run_gt += __popcll(m_gt);
        run_eq += __popcll(m_eq);
      }
    }
    if (tile_energy != nullptr) {
      left = wave_sum_f64(left);
      if (lane_id() == 0) tile_energy[(uint64_t)row * ntiles + tile] = left;
    }
  }
}

// ---- the tail of the select and the gated dense redo in the same launches -----------------
// The rows' flags are final once k_cand_hist1 has run.  The four kernels that remain of the
// single-pass select and the first four of the dense redo of the flagged rows (idle unless
// a row is flagged, but a launch costs 4-5 us either way) do not depend on each other, so
// each pair shares a launch: the first `own` workgroups of the 1-D grid do the select's
// part, the others the dense part on a virtual (gx, rows) grid.  The redo's emission
// follows in a launch of its own, whose workgroups, idle for rows that need no redo, fill
// the aggregation's range tables or apply the model update from the finished messages.
struct DensePart {
  float* x;
  uint64_t d;
  uint32_t K;
  uint32_t* hist;
  SelState* state;
  uint2* cnt;
  uint2* block_sums;
  uint32_t nwc, gx;
  bool streaming;
};

__device__ __forceinline__ VGrid dense_vgrid(uint32_t b, const DensePart& dp) {
  return VGrid{b % dp.gx, b / dp.gx, dp.gx};
}

__global__ __launch_bounds__(kBlock) void k_finish_hist0(uint32_t own, uint32_t* partial,
                                                         uint32_t nparts, bool early_zero,
                                                         uint32_t* lower_key,
                                                         uint32_t* upper_key, uint32_t* prev_T,
                                                         uint32_t* cand_cnt, FastSel* sel,
                                                         const uint32_t* need, DensePart dp) {
  if (blockIdx.x < own)
    cand_finish_body(blockIdx.x, partial, nparts, early_zero, lower_key, upper_key,
                     prev_T, cand_cnt, sel, need);
  else
    hist_body<0, false>(dense_vgrid(blockIdx.x - own, dp), nullptr, dp.x, dp.d, 0.0f, dp.K,
                        dp.hist, dp.nwc, need, dp.streaming);
}

template <int TPW>
__global__ __launch_bounds__(kBlock) void k_dircount_hist1(
    uint32_t own, uint32_t own_gx, const uint2* dir, uint32_t nwc_pad, const uint2* cand,
    uint32_t cap, const FastSel* sel, const uint32_t* need, unsigned long long* tile_cnt,
    uint32_t ntiles, DensePart dp) {
  if (blockIdx.x < own)
    dir_count_body<TPW>(blockIdx.x % own_gx, blockIdx.x / own_gx, dir, nwc_pad, cand, cap, sel,
                        need, tile_cnt, ntiles);
  else
    hist_body<1, false>(dense_vgrid(blockIdx.x - own, dp), nullptr, dp.x, dp.d, 0.0f, dp.K,
                        dp.hist, dp.nwc, need, dp.streaming);
}

__global__ __launch_bounds__(kBlock) void k_dirscan_hist2(uint32_t own,
                                                          unsigned long long* tile_cnt,
                                                          uint32_t ntiles, const uint32_t* need,
                                                          DensePart dp) {
  if (blockIdx.x < own)
    dir_scan_body(blockIdx.x, tile_cnt, ntiles, need);
  else
    hist_body<2, false>(dense_vgrid(blockIdx.x - own, dp), nullptr, dp.x, dp.d, 0.0f, dp.K,
                        dp.hist, dp.nwc, need, dp.streaming);
}

template <int TPW>
__global__ __launch_bounds__(kBlock) void k_diremit_count(
    uint32_t own, uint32_t own_gx, uint2* dir, uint32_t nwc_pad, const uint2* cand, uint32_t cap,
    const FastSel* sel, const uint32_t* need,
    const unsigned long long* tile_cnt, uint32_t ntiles, uint32_t* out_idx, float* out_val,
    double* tile_energy, FusedUpdate upd, DensePart dp) {
  if (blockIdx.x < own)
    dir_emit_body<TPW>(blockIdx.x % own_gx, blockIdx.x / own_gx, dir, nwc_pad, cand, cap, sel,
                       need, tile_cnt, ntiles, dp.x, dp.d, dp.K, out_idx, out_val,
                       tile_energy, upd);
  else
    count_body(dense_vgrid(blockIdx.x - own, dp), dp.x, dp.d, dp.K, dp.hist, dp.state,
               dp.cnt, dp.block_sums, dp.nwc, need, dp.streaming);
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
  // Small calls are bound by kernel launches and the dense path, with fewer launches, is
  // the quicker one.  Measured crossovers: 1.1e7 coordinates per call for several rows (at
  // 1.2e7 the single pass is 8 % ahead, at 2.4e7 21 %; at 8e6 the dense path is 6 % ahead);
  // 8e6 for a single row (per select at K = d / 1000: level at 5e6, 5 us ahead at 7e6, 39 us
  // at 2e7; at K = d / 100: 10 us behind at 5e6, 12 us ahead at 1.1e7).
  p.preferred = rows == 1 ? d >= 8000000ull : (uint64_t)rows * d >= 11000000ull;
  const uint64_t slices = d / 256;
  // Every stride-th slice is sampled: 64 / K of the row, which puts 64 sampled coordinates
  // in the row's top K, or 1 / 171 of the row where that is more (a sample of that size is
  // still bound by the launch, not by its reads, up to rows of about 3e7).
  uint64_t stride = K / 64;
  if (stride > 171) stride = 171;
  // On the largest calls the sample's bytes show (68 us of a 13.7 ms step at 64 x 1.1e8):
  // there every 342nd slice is taken, 32 sampled coordinates in the row's top K, and the
  // bound aims at the rank 2 K (5.7 standard deviations above K).
  if ((uint64_t)rows * d >= 2000000000ull && K / 32 > 171) stride = K / 32 < 342 ? K / 32 : 342;
  if (stride < 16) stride = 16;
  if (stride > slices / 64) stride = slices / 64;
  if (stride < 1) stride = 1;
  // The bound aims at the rank M = K (1 + 7 / sqrt(h)), h = K / stride the sampled
  // coordinates expected in the top K: seven binomial standard deviations above K, between
  // 1.15 K and 2 K.
  const double h = (double)K / (double)stride;
  double over = 7.0 / __builtin_sqrt(h > 1.0 ? h : 1.0);
  if (over > 1.0) over = 1.0;
  if (over < 0.15) over = 0.15;
  const uint64_t M = (uint64_t)((double)K * (1.0 + over)) + 1;
  uint64_t target = (M + stride - 1) / stride;
  if (target < 48) target = 48;
  // expected list length is M..2M (the bound is a histogram bin edge); each of the 64
  // lists gets twice its even share of 4x the target plus slack
  uint64_t cap = (4 * target * stride + 4096) / 64 * 2 + 64;
  p.enabled = true;
  p.stride = (uint32_t)stride;
  p.target = (uint32_t)target;
  p.target_u = (uint32_t)((K + stride / 2) / stride);   // K coordinates of the row, in samples
  if (p.target_u < 1) p.target_u = 1;
  // bounds handed from call to call: a quarter spare candidates, at least 256 (the count at
  // a fixed bound moves by its square root from step to step, and by the drift of the run)
  p.rank_next = K + (K / 4 > 256 ? K / 4 : 256);
  p.cap = (uint32_t)cap;
  // How many waves per SIMD the dense pass is held to (a kernel variant whose register
  // allocation admits no more): a stream of 2 reads : 1 write runs best well below full
  // occupancy, but a wave whose chunk has hits waits for its append, and the more chunks
  // have hits the more waves it takes to hide that.  About 3K candidates over
  // d / kWaveChunk chunks.  Measured per launch: 13.3 against 13.7 ms at 7e9 coordinates
  // (0.15 candidates per chunk, 3 waves per SIMD = 12 per compute unit), 1.545 against
  // 1.58 ms at 8e8 (1.5 per chunk, 5 per SIMD; 3 per SIMD: 1.67 ms), 0.342 against
  // 0.346 ms at 1.8e8 (15 per chunk, 6 per SIMD).
  const uint64_t per_chunk_x10 = 30ull * K * kWaveChunk / d;
  p.stream_waves_per_simd = per_chunk_x10 < 5 ? 3u : (per_chunk_x10 < 50 ? 5u : 6u);
  p.ntiles = (uint32_t)(((d + kWaveChunk - 1) / kWaveChunk + 1 + kTileChunks - 1) / kTileChunks);
  p.nwc_pad = p.ntiles * kTileChunks;
  return p;
}

hipError_t fast_select(hipStream_t s, const FastScratch& sc, const FastPlan& pl, const float* g,
                       float* x, uint32_t rows, uint64_t d, uint32_t K, float alpha,
                       uint32_t* out_idx, float* out_val, hipEvent_t ev0, hipEvent_t ev1,
                       const DenseScratch& dense, bool energy, FusedUpdate upd,
                       MidRanges ranges) {
  const dim3 block(kBlock);
  if (upd.w != nullptr && rows != 1) return hipErrorInvalidValue;
  // the update done by the emitting lanes, or after the emission (see FusedUpdate)
  const FusedUpdate emit_upd = upd.after ? FusedUpdate{nullptr, 0.0f, false} : upd;
  if (energy && (g == nullptr || sc.energy == nullptr || sc.tile_energy == nullptr))
    return hipErrorInvalidValue;
  double* tile_energy = energy ? sc.tile_energy : nullptr;
  const uint32_t nwc = (uint32_t)((d + kWaveChunk - 1) / kWaveChunk) + 1;
  const dim3 dense_grid((nwc + kStreamWaves - 1) / kStreamWaves, rows);
  unsigned long long* tile_cnt = reinterpret_cast<unsigned long long*>(sc.tile_cnt);
  if (*sc.dirty) {       // an earlier call failed before its emission: clear what it left
    hipError_t e = fill_u32(s, reinterpret_cast<uint32_t*>(sc.dir),
                            (uint64_t)sc.rows * pl.nwc_pad * 2, 0);
    if (e == hipSuccess) e = fill_u32(s, sc.sample_hist, (uint64_t)sc.rows * kSampleBins, 0);
    if (e == hipSuccess) e = fill_u32(s, sc.prev_T, sc.rows, 0);
    if (e == hipSuccess) e = fill_u32(s, sc.hist, (uint64_t)sc.rows * fast_hist_words(), 0);
    if (e != hipSuccess) return e;
  }
  // 1. bounds: from a sample on the scratch's first two calls and after a failed one; later
  // calls start from the bounds the call before them left (see cand_finish_body)
  // A row that was redone says so in a pinned host word; the host sees it on a later call (it
  // never waits for it) and samples again for a while: 2 calls, and twice as many after every
  // further redo, up to 64, so that a workload whose threshold cannot be foreseen (the same
  // gradient fed again and again makes it grow by a half, a third, ... per step) ends up
  // sampling almost always, as cheaply as if nothing were handed on; 64 calls without a redo
  // forget the past.
  FastScratch::HostState& hs = *sc.host;
  if (*sc.dirty) hs = FastScratch::HostState{0, 0, 0, 0};
  if (sc.redone_host != nullptr && *sc.redone_host != 0) {
    *sc.redone_host = 0;
    hs.backoff = hs.backoff == 0 ? 2u : (hs.backoff < 64u ? hs.backoff * 2u : 64u);
    hs.cold_left = hs.backoff;
    hs.quiet = 0;
  } else if (++hs.quiet >= 64u) {
    hs.backoff = 0;
  }
  const bool sampled = hs.calls < 2 || hs.cold_left > 0;
  if (hs.cold_left > 0) --hs.cold_left;
  *sc.dirty = true;      // cleared when every launch of this call went out
  if (sampled) {
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
    k_pick_bound<<<dim3(rows), block, 0, s>>>(sc.sample_hist, pl.target,
                                              g != nullptr ? pl.target_u : 0u, sc.lower_key,
                                              sc.upper_key, sc.cand_cnt);
    BTS_LAUNCH_CHECK();
  }
  // 2. the dense pass (a wave of the grid may lie past the row's last chunk, never past
  // the padded directory)
  if (ev0) (void)hipEventRecord(ev0, s);
#define BTS_CAPTURE(FMA, ENERGY, WPS, G, ALPHA, EN)                                        \
  k_stream_capture<FMA, ENERGY, WPS><<<dense_grid, dim3(kStreamBlock), 0, s>>>(            \
      G, x, d, ALPHA, sc.lower_key, sc.upper_key, sc.cand_cnt, sc.cand, pl.cap, sc.dir,      \
      pl.nwc_pad, EN)
  if (g == nullptr) {
    BTS_CAPTURE(false, false, kMaxWavesPerSimd, nullptr, 0.0f, nullptr);
  } else if (energy) {
    if (pl.stream_waves_per_simd == 3) BTS_CAPTURE(true, true, 3, g, alpha, sc.energy);
    else if (pl.stream_waves_per_simd == 5) BTS_CAPTURE(true, true, 5, g, alpha, sc.energy);
    else BTS_CAPTURE(true, true, 6, g, alpha, sc.energy);
  } else {
    if (pl.stream_waves_per_simd == 3) BTS_CAPTURE(true, false, 3, g, alpha, nullptr);
    else if (pl.stream_waves_per_simd == 5) BTS_CAPTURE(true, false, 5, g, alpha, nullptr);
    else BTS_CAPTURE(true, false, 6, g, alpha, nullptr);
  }
#undef BTS_CAPTURE
  BTS_LAUNCH_CHECK();
  if (ev1) (void)hipEventRecord(ev1, s);
  // 3 + 4. verify and select: a few fat blocks per row, each taking whole lists (about 32768
  // entries of capacity per block)
  uint32_t hb = (uint32_t)(((uint64_t)pl.cap * kSubLists / 2 + 32767) / 32768);
  if (hb > 4) hb = kMaxHistBlocks;      // 1-4 blocks (16-64 waves) or 8 (two waves per list)
  if (hb < 1) hb = 1;
  static_assert(kMaxHistBlocks * (kCandBlock / kWave) % kSubLists == 0, "whole waves per list");
  const dim3 hgrid(hb, rows);
  FastSel* sel = reinterpret_cast<FastSel*>(sc.sel);
  k_cand_hist0<<<hgrid, dim3(kCandBlock), 0, s>>>(sc.cand, sc.cand_cnt, pl.cap, K, sc.lower_key,
                                                  sc.hist, sc.need);
  BTS_LAUNCH_CHECK();
  k_cand_hist1<<<hgrid, dim3(kCandBlock), 0, s>>>(sc.cand, sc.cand_cnt, pl.cap, K, pl.rank_next,
                                                  sc.lower_key, sc.upper_key, sc.hist, sel,
                                                  sc.need, x, d);
  BTS_LAUNCH_CHECK();
  // 4 (rest) + 5 + the first four kernels of the gated dense redo, pair by pair
  const DensePlan dpl = dense_plan(dense, rows, d);
  hipError_t e = dense_begin(s, dense);
  if (e != hipSuccess) return e;
  DensePart dp;
  dp.x = x;
  dp.d = d;
  dp.K = K;
  dp.hist = dense.hist;
  dp.state = dense.state;
  dp.cnt = dense.cnt;
  dp.block_sums = dense.block_sums;
  dp.nwc = dpl.nwc;
  dp.gx = dpl.gx;
  dp.streaming = dpl.streaming;
  const uint64_t dense_blocks = (uint64_t)dpl.gx * rows;
  const bool sparse_tiles = 3ull * K < 16ull * pl.ntiles;      // under 16 candidates per tile
  const uint32_t tile_waves = sparse_tiles ? (pl.ntiles + 3) / 4 : pl.ntiles;
  const uint32_t tgx = (tile_waves + kWavesPerBlock - 1) / kWavesPerBlock;
  const uint64_t tile_blocks = (uint64_t)tgx * rows;
  if (tile_blocks + dense_blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
  const dim3 grid_rows((unsigned)(rows + dense_blocks));
  const dim3 grid_tiles((unsigned)(tile_blocks + dense_blocks));
  k_finish_hist0<<<grid_rows, block, 0, s>>>(rows, sc.hist, hb, g != nullptr,
                                             sc.lower_key, sc.upper_key, sc.prev_T, sc.cand_cnt,
                                             sel, sc.need, dp);
  BTS_LAUNCH_CHECK();
  if (sparse_tiles)
    k_dircount_hist1<4><<<grid_tiles, block, 0, s>>>((uint32_t)tile_blocks, tgx, sc.dir,
                                                     pl.nwc_pad, sc.cand, pl.cap, sel, sc.need,
                                                     tile_cnt, pl.ntiles, dp);
  else
    k_dircount_hist1<1><<<grid_tiles, block, 0, s>>>((uint32_t)tile_blocks, tgx, sc.dir,
                                                     pl.nwc_pad, sc.cand, pl.cap, sel, sc.need,
                                                     tile_cnt, pl.ntiles, dp);
  BTS_LAUNCH_CHECK();
  k_dirscan_hist2<<<grid_rows, block, 0, s>>>(rows, tile_cnt, pl.ntiles, sc.need, dp);
  BTS_LAUNCH_CHECK();
  if (sparse_tiles)
    k_diremit_count<4><<<grid_tiles, block, 0, s>>>((uint32_t)tile_blocks, tgx, sc.dir,
                                                    pl.nwc_pad, sc.cand, pl.cap, sel, sc.need,
                                                    tile_cnt, pl.ntiles, out_idx, out_val,
                                                    tile_energy, emit_upd, dp);
  else
    k_diremit_count<1><<<grid_tiles, block, 0, s>>>((uint32_t)tile_blocks, tgx, sc.dir,
                                                    pl.nwc_pad, sc.cand, pl.cap, sel, sc.need,
                                                    tile_cnt, pl.ntiles, out_idx, out_val,
                                                    tile_energy, emit_upd, dp);
  BTS_LAUNCH_CHECK();
  *sc.dirty = false;
  hs.calls += 1;
  // the rest of the redo: emission of the flagged rows, which also sets their next bounds
  return dense_finish(s, dense, dpl, x, rows, d, K, out_idx, out_val, sc.need, upd,
                      NextBounds{sc.lower_key, sc.upper_key, sc.prev_T, g != nullptr,
                                 sc.redone_dev},
                      ranges);
}

size_t fast_sel_bytes() { return sizeof(FastSel); }
uint32_t fast_sublists() { return kSubLists; }
uint32_t fast_counter_stride() { return kCounterStride; }
size_t fast_hist_words() { return (size_t)kMaxHistBlocks * kPartWords; }

}  // namespace bts
