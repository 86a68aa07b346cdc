// Top_K select for rows of middling length and small K, in three launches.
//
// Calls of a few million coordinates are bound by kernel launches: the dense multi-pass
// select needs six of them, the single-pass select with its gated fallback twelve.  Here the
// rows are short enough to stay in the last-level cache between passes, so a second read
// costs little, and the select is cut down to three launches with no fallback at all:
//
//   1. histogram:  one dense pass (with the worker's error compensation a = eps + alpha g
//                  fused in and stored) histograms the top 13 bits of the magnitude key per
//                  row (LDS, flushed with atomics to the row's global histogram, together
//                  with the sums over each exponent's 32 bins).
//   2. capture:    every block finds, from the finished histogram (exponent first, then the
//                  32 bins of that exponent: 1.1 KB to read), the bin b that holds the
//                  row's K-th largest key; then a second pass appends every coordinate with
//                  key >= b << 18 to the row's candidate lists, with the chunk directory of
//                  the single-pass select.  The bound is exact, not sampled: the lists hold
//                  exactly (keys above bin b) + (keys in bin b) >= K entries, and they are
//                  sized so that they cannot overflow (a list can take every coordinate of
//                  the chunks that append to it).  Nothing has to be verified or redone.
//   3. finish:     ONE workgroup per row selects the exact K-th largest key T and the tie
//                  quota r among the candidates of bin b (18 key bits: a 6-bit and a 12-bit
//                  digit in LDS), counts the entries above / on T per directory tile, scans
//                  the tiles, and emits the kept pairs in index order (lower index wins
//                  among equals), stores +0 over them, and leaves histogram, counters and
//                  directory clear for the next call.  For the worker rows it also fills
//                  the aggregation's range table for its row (where the row's sorted
//                  message enters and leaves each range of coordinates).
//
// Typical rows put K + a few hundred candidates on the lists, which one workgroup handles in
// microseconds.  A row whose K-th key sits in a crowded bin (many equal magnitudes, e.g. a
// mostly zero row with K beyond its non-zeros) makes the lists long and the one workgroup slow;
// the result is the same.  The plan therefore allows this path only for K <= 8192,
// K <= d / 64 and rows of at most 2^22 coordinates, and prefers it for K <= 3072 and calls of
// at most 2.4e7 coordinates.

#include "capture_bodies.h"

namespace bts {

namespace {

constexpr int kMidBits = 13;                          // top bits of the 31-bit key
constexpr int kMidBins = 1 << kMidBits;               // 8192
constexpr int kMidShift = 31 - kMidBits;              // 18 key bits below a bin
constexpr int kCoarseBins = 256;                      // the key's top 8 bits (the exponent)
constexpr int kFinePerCoarse = kMidBins / kCoarseBins;   // 32
constexpr int kMidRowHist = kMidBins + kCoarseBins;   // words of histogram per row
constexpr int kMidBlock = 1024;                       // threads of the finishing workgroup
constexpr int kMidWaves = kMidBlock / kWave;
constexpr uint32_t kMidMaxTiles = 256;                // 2^22 coordinates / 32768 per tile (+1)
constexpr int kLoBits = 12, kLoBins = 1 << kLoBits;   // low digit of the key inside the bin
constexpr int kHiBins = 1 << (kMidShift - kLoBits);   // 64: high digit inside the bin

// ---- 1. histogram ---------------------------------------------------------------------------
// Few fat blocks per row (1024 threads, at most 64 blocks per row): every block adds its
// LDS histogram to the row's global one with atomics, and atomics on one address are
// served one after the other at the memory side (about 20 ns each): with 256 blocks per
// row the busiest bin alone costs 5 us, with 64 about 1.
template <bool FMA>
__global__ __launch_bounds__(kMidBlock) void k_mid_hist(const float* __restrict__ g,
                                                        float* __restrict__ x, uint64_t d,
                                                        float alpha, uint32_t* __restrict__ hist,
                                                        uint32_t nwc) {
  __shared__ uint32_t sh[kMidBins];
  const uint32_t row = blockIdx.y;
  for (int i = threadIdx.x; i < kMidBins; i += kMidBlock) sh[i] = 0;
  __syncthreads();
  uint32_t bin0 = 0;       // counted per lane: a sparse row would serialise on one LDS word
  for (uint32_t wc = blockIdx.x * kMidWaves + threadIdx.x / kWave; wc < nwc;
       wc += gridDim.x * kMidWaves) {
    const ChunkGeom c = wave_chunk(d, row, wc);
    if (!c.active) break;
    // plain (cached) accesses: the row is read again by the capture pass
    visit_chunk<FMA>(g, x, c, alpha, false, [&](uint64_t, const float (&v)[4], uint32_t mask) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (mask & (1u << j)) {
          const uint32_t bin = key_of(v[j]) >> kMidShift;
          if (bin == 0) ++bin0; else atomicAdd(&sh[bin], 1u);
        }
      }
    });
  }
  if (bin0) atomicAdd(&sh[0], bin0);
  __syncthreads();
  uint32_t* h = hist + (uint64_t)row * kMidRowHist;
  for (int i = threadIdx.x; i < kMidBins; i += kMidBlock) {
    const uint32_t v = sh[i];
    if (v) atomicAdd(&h[i], v);
  }
  if (threadIdx.x < kCoarseBins) {                    // the sums over each exponent's 32 bins
    uint32_t coarse = 0;
    for (int i = 0; i < kFinePerCoarse; ++i)          // rotated start: no LDS bank conflicts
      coarse += sh[threadIdx.x * kFinePerCoarse + ((i + threadIdx.x) & (kFinePerCoarse - 1))];
    if (coarse) atomicAdd(&h[kMidBins + threadIdx.x], coarse);
  }
}

// The bin holding the row's K-th largest key, from the finished two-level histogram of the
// row: the exponent first (one coarse bin per thread of the 256-thread block), then the 32
// fine bins of that exponent.  *above = keys in higher bins.  All threads call this.
__device__ __forceinline__ uint32_t resolve_two_level(const uint32_t* __restrict__ h, uint32_t K,
                                                      uint32_t* lds, uint32_t* s_out,
                                                      uint32_t* above) {
  const int cb = kCoarseBins - 1 - (int)threadIdx.x;      // this thread's exponent
  const uint32_t c = h[kMidBins + cb];
  uint32_t total;
  const uint32_t excl = block_exclusive_scan(c, lds, &total);
  if (threadIdx.x == 0) {
    s_out[0] = 0;
    s_out[1] = 0;
  }
  __syncthreads();
  if (excl < K && K <= excl + c) {                        // exactly one thread (K <= d)
    s_out[0] = (uint32_t)cb;
    s_out[1] = excl;
  }
  __syncthreads();
  const uint32_t e = s_out[0], above_e = s_out[1];
  __syncthreads();
  if (threadIdx.x < kWave) {                              // the first wave walks the 32 fine bins
    const int fb = kFinePerCoarse - 1 - (int)threadIdx.x;
    const uint32_t f = fb >= 0 ? h[e * kFinePerCoarse + fb] : 0u;
    const uint32_t incl = wave_inclusive_scan(f);
    const uint32_t before = above_e + incl - f;
    if (fb >= 0 && before < K && K <= before + f) {
      s_out[0] = e * kFinePerCoarse + (uint32_t)fb;
      s_out[1] = before;
    }
  }
  __syncthreads();
  const uint32_t b = s_out[0];
  *above = s_out[1];
  __syncthreads();
  return b;
}

// ---- 2. capture -----------------------------------------------------------------------------
struct MidBound {
  uint32_t lower_key;      // b << 18: every candidate has key >= this
  uint32_t above;          // keys in bins above b (all of them among the K largest)
};

__global__ __launch_bounds__(kBlock) void k_mid_capture(
    float* __restrict__ x, uint64_t d, uint32_t K, const uint32_t* __restrict__ hist,
    MidBound* __restrict__ bound, uint32_t* __restrict__ cand_cnt, uint2* __restrict__ cand,
    uint32_t cap, uint2* __restrict__ dir, uint32_t nwc_pad, uint32_t nwc) {
  __shared__ uint32_t lds[kBlock / kWave + 1];
  __shared__ uint32_t s_out[2];
  const uint32_t row = blockIdx.y;
  uint32_t above;
  const uint32_t b = resolve_two_level(hist + (uint64_t)row * kMidRowHist, K, lds, s_out, &above);
  const uint32_t L = b << kMidShift;
  if (blockIdx.x == 0 && threadIdx.x == 0) bound[row] = MidBound{L, above};
  for (uint32_t wc = blockIdx.x * kWavesPerBlock + threadIdx.x / kWave; wc < nwc;
       wc += gridDim.x * kWavesPerBlock)
    capture_chunk<false, false>(row, wc, L, 0xFFFFFFFFu, nullptr, x, d, 0.0f, cand_cnt, cand, cap, dir,
                                nwc_pad, nullptr);
}

// ---- 3. finish: one workgroup per row ---------------------------------------------------------
// Walk an NB-bin LDS histogram (NB <= kMidBlock) from the top bin down to the bin holding
// the want-th largest entry; *above = entries in higher bins.  All threads call this.
template <int NB>
__device__ __forceinline__ uint32_t resolve_small(const uint32_t* sh, uint32_t want,
                                                  uint32_t* lds, uint32_t* s_out,
                                                  uint32_t* above) {
  static_assert(NB <= kMidBlock, "one bin per thread");
  const int bin = NB - 1 - (int)threadIdx.x;             // thread t owns bin NB-1-t
  const uint32_t c = bin >= 0 ? sh[bin] : 0u;
  uint32_t total;
  const uint32_t excl = block_exclusive_scan(c, lds, &total);
  if (threadIdx.x == 0) {
    s_out[0] = 0;
    s_out[1] = 0;
  }
  __syncthreads();
  if (bin >= 0 && excl < want && want <= excl + c) {
    s_out[0] = (uint32_t)bin;
    s_out[1] = excl;
  }
  __syncthreads();
  const uint32_t r = s_out[0];
  *above = s_out[1];
  __syncthreads();
  return r;
}

constexpr uint32_t kLdsEntries = 5120;         // candidates of a row that fit in LDS (40 KB)

template <bool RANGES>
__global__ __launch_bounds__(kMidBlock) void k_mid_finish(
    float* __restrict__ x, uint64_t d, uint32_t K, uint32_t* __restrict__ hist,
    const MidBound* __restrict__ bound, uint32_t* __restrict__ cand_cnt,
    const uint2* __restrict__ cand, uint32_t cap, uint2* __restrict__ dir, uint32_t nwc_pad,
    uint32_t ntiles, uint32_t* __restrict__ out_idx, float* __restrict__ out_val,
    FusedUpdate upd, uint32_t N, uint32_t* __restrict__ tab_start, uint32_t* __restrict__ tab_end,
    uint32_t* __restrict__ tab_any) {
  __shared__ uint32_t sh[kLoBins];
  // either the row's candidates in index order (the usual case), or the per-wave tile views
  // and per-tile counts of the walk over the lists
  __shared__ uint32_t pool[2 * kLdsEntries];
  __shared__ uint32_t lds[kMidWaves + 1];
  __shared__ uint32_t s_out[2];
  __shared__ uint32_t s_wg[kMidWaves], s_we[kMidWaves];
  static_assert(2 * kMidWaves * kTileChunks + 2 * kMidMaxTiles <= 2 * kLdsEntries, "pool");
  const uint32_t row = blockIdx.x, t = threadIdx.x, w = t / kWave;
  const MidBound bd = bound[row];
  const uint32_t L = bd.lower_key;
  const uint2* cand_row = cand + (uint64_t)row * kSubLists * cap;
  const uint32_t* cnt_row = cand_cnt + (uint64_t)row * kSubLists * kCounterStride;
  uint2* dir_row = dir + (uint64_t)row * nwc_pad;
  float* xr = x + (uint64_t)row * d;
  uint32_t* oi = out_idx + (uint64_t)row * K;
  float* ov = out_val + (uint64_t)row * K;
  const uint64_t below = lanes_below();
  uint32_t k_rem = K - bd.above;                   // >= 1: bin b holds the K-th largest key
  // the row's candidates, counted from the directory: thread t owns `per` consecutive chunks
  // (their directory entries stay in registers for the gather below)
  constexpr uint32_t kMaxPer = kMidMaxTiles * kTileChunks / kMidBlock;      // 16
  const uint32_t per = (nwc_pad + kMidBlock - 1) / kMidBlock;
  const uint32_t c0 = min(t * per, nwc_pad), c1 = min(c0 + per, nwc_pad);
  uint2 ent[kMaxPer];
  uint32_t mine = 0;
#pragma unroll
  for (uint32_t u = 0; u < kMaxPer; ++u) {
    ent[u] = c0 + u < c1 ? dir_row[c0 + u] : make_uint2(0u, 0u);
    mine += ent[u].y;
  }
  uint32_t total;
  uint32_t at = block_exclusive_scan(mine, lds, &total);

  if (total <= kLdsEntries) {
    // ---- the candidates fit in LDS: gather them in index order, do the rest there ----------
    uint2* s_ent = reinterpret_cast<uint2*>(pool);
    // the first entry of each of the thread's runs (most runs hold one entry where K is a
    // thousandth of d), loaded together; longer runs after
    {
      uint2 first[kMaxPer];
#pragma unroll
      for (uint32_t u = 0; u < kMaxPer; ++u) {
        first[u] = make_uint2(0u, 0u);
        if (ent[u].y) {
          dir_row[c0 + u] = make_uint2(0u, 0u);    // leave the directory clear
          first[u] = cand_row[(uint64_t)((c0 + u) % kSubLists) * cap + ent[u].x];
        }
      }
#pragma unroll
      for (uint32_t u = 0; u < kMaxPer; ++u) {
        if (ent[u].y == 0) continue;
        if (at < kLdsEntries) s_ent[at] = first[u];
        const uint2* run = cand_row + (uint64_t)((c0 + u) % kSubLists) * cap + ent[u].x;
        for (uint32_t j = 1; j < ent[u].y; ++j)
          if (at + j < kLdsEntries) s_ent[at + j] = run[j];
        at += ent[u].y;
      }
    }
    for (int i = t; i < kHiBins; i += kMidBlock) sh[i] = 0;
    __syncthreads();
    // exact select inside the bin: off = key - L < 2^18 for its entries, more for those above
    for (uint32_t e = t; e < total; e += kMidBlock) {
      const uint32_t off = (s_ent[e].y & 0x7FFFFFFFu) - L;
      if (off < (1u << kMidShift)) atomicAdd(&sh[off >> kLoBits], 1u);
    }
    __syncthreads();
    uint32_t above;
    const uint32_t hi = resolve_small<kHiBins>(sh, k_rem, lds, s_out, &above);
    k_rem -= above;
    for (int i = t; i < kLoBins; i += kMidBlock) sh[i] = 0;
    __syncthreads();
    for (uint32_t e = t; e < total; e += kMidBlock) {
      const uint32_t off = (s_ent[e].y & 0x7FFFFFFFu) - L;
      if ((off >> kLoBits) == hi) atomicAdd(&sh[off & (kLoBins - 1)], 1u);
    }
    __syncthreads();
    const uint32_t lo = resolve_bins<kLoBins, kMidBlock>(sh, 1, 0, k_rem, lds, s_out, &above);
    const uint32_t T = L + ((hi << kLoBits) | lo);   // the exact K-th largest key
    const uint32_t r = k_rem - above;                // holders of T that are kept
    // ordered emission, 1024 entries at a time.  The emitted indices also go to LDS, over
    // the entries already emitted (the message grows no faster than the entries are read:
    // 4 bytes at pos <= e against 8 at e), for the range table below.
    uint32_t* s_idx = pool;
    uint32_t run_gt = 0, run_eq = 0;
    // the model update of the pairs this thread emits: their loads of w go out together after
    // the loop (a load per turn of the loop would be waited for in every turn)
    constexpr uint32_t kEmitTurns = kLdsEntries / kMidBlock;
    static_assert(kEmitTurns * kMidBlock == kLdsEntries, "whole turns");
    uint32_t upd_i[kEmitTurns];
    float upd_v[kEmitTurns];
#pragma unroll
    for (uint32_t turn = 0; turn < kEmitTurns; ++turn) {
      upd_i[turn] = 0xFFFFFFFFu;
      upd_v[turn] = 0.0f;
      const uint32_t e0 = turn * kMidBlock;
      if (e0 >= total) continue;                   // the same for every thread
      const uint32_t e = e0 + t;
      const uint2 en = e < total ? s_ent[e] : make_uint2(0u, 0u);
      const uint32_t key = en.y & 0x7FFFFFFFu;
      const bool is_gt = e < total && key > T, is_eq = e < total && key == T;
      const uint64_t m_gt = __ballot(is_gt), m_eq = __ballot(is_eq);
      if (lane_id() == 0) {
        s_wg[w] = __popcll(m_gt);
        s_we[w] = __popcll(m_eq);
      }
      __syncthreads();
      uint32_t n_gt = run_gt + __popcll(m_gt & below), n_eq = run_eq + __popcll(m_eq & below);
      uint32_t all_gt = 0, all_eq = 0;
#pragma unroll
      for (int v = 0; v < kMidWaves; ++v) {
        const uint32_t a = s_wg[v], b = s_we[v];
        n_gt += v < (int)w ? a : 0u;
        n_eq += v < (int)w ? b : 0u;
        all_gt += a;
        all_eq += b;
      }
      if (is_gt || (is_eq && n_eq < r)) {
        const uint32_t pos = n_gt + min(n_eq, r);
        if (pos < K) s_idx[pos] = en.x;
        if (pos < K && en.x < d) {
          const float val = __uint_as_float(en.y);
          oi[pos] = en.x;
          ov[pos] = val;
          xr[en.x] = 0.0f;
          upd_i[turn] = en.x;
          upd_v[turn] = val;
        }
      }
      run_gt += all_gt;
      run_eq += all_eq;
      __syncthreads();
    }
    if (upd.w != nullptr) {
      float wv[kEmitTurns];
#pragma unroll
      for (uint32_t turn = 0; turn < kEmitTurns; ++turn)
        wv[turn] = upd_i[turn] != 0xFFFFFFFFu ? upd.w[upd_i[turn]] : 0.0f;
#pragma unroll
      for (uint32_t turn = 0; turn < kEmitTurns; ++turn)
        if (upd_i[turn] != 0xFFFFFFFFu)
          upd.w[upd_i[turn]] = __fmaf_rn(upd.neg_alpha, upd_v[turn], wv[turn]);
    }
  } else {
    // ---- long lists (a crowded threshold bin): the same steps from the lists in memory -----
    uint32_t(*s_off)[kTileChunks] = reinterpret_cast<uint32_t(*)[kTileChunks]>(pool);
    uint32_t(*s_start)[kTileChunks] =
        reinterpret_cast<uint32_t(*)[kTileChunks]>(pool + kMidWaves * kTileChunks);
    uint32_t* s_gt = pool + 2 * kMidWaves * kTileChunks;
    uint32_t* s_eq = s_gt + kMidMaxTiles;
    for (int i = t; i < kHiBins; i += kMidBlock) sh[i] = 0;
    __syncthreads();
    for (uint32_t sl = w; sl < kSubLists; sl += kMidWaves) {
      const uint32_t n = cnt_row[sl * kCounterStride];
      const uint2* list = cand_row + (uint64_t)sl * cap;
      for (uint32_t j = lane_id(); j < n; j += kWave) {
        const uint32_t off = (list[j].y & 0x7FFFFFFFu) - L;
        if (off < (1u << kMidShift)) atomicAdd(&sh[off >> kLoBits], 1u);
      }
    }
    __syncthreads();
    uint32_t above;
    const uint32_t hi = resolve_small<kHiBins>(sh, k_rem, lds, s_out, &above);
    k_rem -= above;
    for (int i = t; i < kLoBins; i += kMidBlock) sh[i] = 0;
    __syncthreads();
    for (uint32_t sl = w; sl < kSubLists; sl += kMidWaves) {
      const uint32_t n = cnt_row[sl * kCounterStride];
      const uint2* list = cand_row + (uint64_t)sl * cap;
      for (uint32_t j = lane_id(); j < n; j += kWave) {
        const uint32_t off = (list[j].y & 0x7FFFFFFFu) - L;
        if ((off >> kLoBits) == hi) atomicAdd(&sh[off & (kLoBins - 1)], 1u);
      }
    }
    __syncthreads();
    const uint32_t lo = resolve_bins<kLoBins, kMidBlock>(sh, 1, 0, k_rem, lds, s_out, &above);
    const uint32_t T = L + ((hi << kLoBits) | lo);
    const uint32_t r = k_rem - above;
    // entries above / on T per directory tile (a wave per tile, tiles w, w + 16, ...)
    for (uint32_t tile = w; tile < ntiles; tile += kMidWaves) {
      const uint2 ent = dir_row[(uint64_t)tile * kTileChunks + lane_id()];
      uint32_t gt = 0, eq = 0;
      if (__ballot(ent.y != 0) != 0) {
        const TileView tv = publish_tile(ent, s_off[w], s_start[w]);
        for (uint32_t e0 = 0; e0 < tv.total; e0 += kWave * kEmitUnroll) {
          uint32_t key[kEmitUnroll];
#pragma unroll
          for (int k = 0; k < kEmitUnroll; ++k) {
            const uint32_t e = e0 + k * kWave + lane_id();
            key[k] = e < tv.total ? tile_entry(tv, e, cand_row, cap).y & 0x7FFFFFFFu : 0u;
          }
#pragma unroll
          for (int k = 0; k < kEmitUnroll; ++k) {
            const uint32_t e = e0 + k * kWave + lane_id();
            gt += (e < tv.total && key[k] > T) ? 1u : 0u;
            eq += (e < tv.total && key[k] == T) ? 1u : 0u;
          }
        }
        gt = wave_sum(gt);
        eq = wave_sum(eq);
      }
      if (lane_id() == 0) {
        s_gt[tile] = gt;
        s_eq[tile] = eq;
      }
    }
    __syncthreads();
    {
      static_assert(kMidMaxTiles <= kMidBlock, "one tile per thread in the scan");
      const uint32_t a = t < ntiles ? s_gt[t] : 0u, b = t < ntiles ? s_eq[t] : 0u;
      uint32_t sum;
      const uint32_t ea = block_exclusive_scan(a, lds, &sum);
      const uint32_t eb = block_exclusive_scan(b, lds, &sum);
      if (t < ntiles) {
        s_gt[t] = ea;
        s_eq[t] = eb;
      }
    }
    __syncthreads();
    // ordered emission (and the directory left clear)
    for (uint32_t tile = w; tile < ntiles; tile += kMidWaves) {
      const uint2 ent = dir_row[(uint64_t)tile * kTileChunks + lane_id()];
      if (ent.y) dir_row[(uint64_t)tile * kTileChunks + lane_id()] = make_uint2(0u, 0u);
      if (__ballot(ent.y != 0) == 0) continue;
      const TileView tv = publish_tile(ent, s_off[w], s_start[w]);
      uint32_t run_gt = s_gt[tile], run_eq = s_eq[tile];
      for (uint32_t e0 = 0; e0 < tv.total; e0 += kWave * kEmitUnroll) {
        uint2 en[kEmitUnroll];
#pragma unroll
        for (int k = 0; k < kEmitUnroll; ++k) {
          const uint32_t e = e0 + k * kWave + lane_id();
          en[k] = e < tv.total ? tile_entry(tv, e, cand_row, cap) : make_uint2(0u, 0u);
        }
#pragma unroll
        for (int k = 0; k < kEmitUnroll; ++k) {
          const uint32_t e = e0 + k * kWave + lane_id();
          const uint32_t key = en[k].y & 0x7FFFFFFFu;
          const bool is_gt = e < tv.total && key > T;
          const bool is_eq = e < tv.total && key == T;
          const uint64_t m_gt = __ballot(is_gt), m_eq = __ballot(is_eq);
          const uint32_t n_gt = run_gt + __popcll(m_gt & below);       // greater before me
          const uint32_t n_eq = run_eq + __popcll(m_eq & below);       // equal before me
          if (is_gt || (is_eq && n_eq < r)) {
            const uint32_t pos = n_gt + min(n_eq, r);
            const uint32_t idx = en[k].x;
            if (pos < K && idx < d) {
              const float val = __uint_as_float(en[k].y);
              oi[pos] = idx;
              ov[pos] = val;
              xr[idx] = 0.0f;
              if (upd.w != nullptr) upd.w[idx] = __fmaf_rn(upd.neg_alpha, val, upd.w[idx]);
            }
          }
          run_gt += __popcll(m_gt);
          run_eq += __popcll(m_eq);
        }
      }
    }
  }
  // leave the histogram and the append counters clear for the next call
  uint32_t* h = hist + (uint64_t)row * kMidRowHist;
  for (int i = t; i < kMidRowHist; i += kMidBlock) h[i] = 0;
  if (t < kSubLists) cand_cnt[((uint64_t)row * kSubLists + t) * kCounterStride] = 0;

  if (RANGES) {
    // Where this worker's sorted message enters and leaves each range of coordinates of the
    // aggregation: pair j opens range r if its predecessor lies in another range and closes
    // it if its successor does; the opener also raises the range's flag.  The message was
    // written by this workgroup: after the barrier its own stores are visible to it.
    __syncthreads();
    // the message's indices: from LDS where the emission left them there, else from memory
    const uint32_t* msg = total <= kLdsEntries ? pool : oi;
    for (uint32_t j = t; j < K; j += kMidBlock) {
      const uint32_t i = msg[j];
      if (i >= d) continue;
      const uint32_t rg = i / kAggWidth;
      if (j == 0 || msg[j - 1] / kAggWidth != rg) {
        tab_start[(uint64_t)rg * N + row] = K - j;
        tab_any[rg] = 1u;
      }
      if (j + 1 == K || msg[j + 1] / kAggWidth != rg) tab_end[(uint64_t)rg * N + row] = j + 1;
    }
  }
}

#define BTS_LAUNCH_CHECK()                       \
  do {                                           \
    hipError_t e_ = hipGetLastError();           \
    if (e_ != hipSuccess) return e_;             \
  } while (0)

}  // namespace

MidPlan mid_plan(uint32_t rows, uint64_t d, uint32_t K) {
  MidPlan p{};
  p.enabled = false;
  if (K == 0 || K > 8192 || (uint64_t)K * 64 > d || d <= 8192 || d > (1ull << 22)) return p;
  if ((uint64_t)rows * d > (1ull << 25)) return p;     // lists of rows x d entries: 268 MB at most
  const uint32_t nwc = (uint32_t)((d + kWaveChunk - 1) / kWaveChunk) + 1;
  p.ntiles = (nwc + kTileChunks - 1) / kTileChunks;
  if (p.ntiles > kMidMaxTiles) return p;
  p.nwc_pad = p.ntiles * kTileChunks;
  // list l takes the chunks wc = l mod 64: at most nwc_pad / 64 of them, whole
  p.cap = (p.nwc_pad / kSubLists) * kWaveChunk;
  // a bounded grid of fat blocks that loop over the chunks, as in the dense select
  uint32_t gx = (nwc + kWavesPerBlock - 1) / kWavesPerBlock;
  uint32_t lim = 1024u / rows;
  if (lim < 64u) lim = 64u;
  if (gx > lim) gx = lim;
  p.gx = gx;
  // the histogram pass: 1024-thread blocks, 256 in all but between 1 and 64 per row
  uint32_t gh = 256u / rows;
  if (gh > 64u) gh = 64u;
  if (gh < 1u) gh = 1u;
  const uint32_t most = (nwc + kMidWaves - 1) / kMidWaves;
  p.gx_hist = gh < most ? gh : most;
  p.enabled = true;
  // Measured against the single-pass select (K = d / 1000): ahead by 5-25 % up to 2.4e7
  // coordinates per call (20 x 1.2e6, 50 and 100 x 2.4e5, 8 x 2e6), behind from 3.2e7; and
  // only while a row's candidates (K + the threshold bin's few hundred) fit in LDS.
  p.preferred = (uint64_t)rows * d <= 24000000ull && K <= 3072;
  return p;
}

size_t mid_bound_bytes() { return sizeof(MidBound); }
uint32_t mid_hist_words() { return kMidRowHist; }

hipError_t mid_select(hipStream_t s, const MidScratch& sc, const MidPlan& pl, const float* g,
                      float* x, uint32_t rows, uint64_t d, uint32_t K, float alpha,
                      uint32_t* out_idx, float* out_val, hipEvent_t ev0, hipEvent_t ev1,
                      FusedUpdate upd, const MidRanges& ranges) {
  if (!pl.enabled || rows > sc.rows) return hipErrorInvalidValue;
  if (upd.w != nullptr && rows != 1) return hipErrorInvalidValue;
  const uint32_t nwc = (uint32_t)((d + kWaveChunk - 1) / kWaveChunk) + 1;
  MidBound* bound = reinterpret_cast<MidBound*>(sc.bound);
  if (*sc.dirty) {       // an earlier call failed half way: clear what it may have left
    hipError_t e = fill_u32(s, sc.hist, (uint64_t)sc.rows * kMidRowHist, 0);
    if (e == hipSuccess)
      e = fill_u32(s, sc.cand_cnt, (uint64_t)sc.rows * kSubLists * kCounterStride, 0);
    if (e == hipSuccess)
      e = fill_u32(s, reinterpret_cast<uint32_t*>(sc.dir), (uint64_t)sc.rows * pl.nwc_pad * 2, 0);
    if (e != hipSuccess) return e;
  }
  *sc.dirty = true;      // cleared when every launch of this call went out
  const dim3 grid(pl.gx, rows), block(kBlock);
  const dim3 hgrid(pl.gx_hist, rows), hblock(kMidBlock);
  if (ev0) (void)hipEventRecord(ev0, s);
  if (g != nullptr)
    k_mid_hist<true><<<hgrid, hblock, 0, s>>>(g, x, d, alpha, sc.hist, nwc);
  else
    k_mid_hist<false><<<hgrid, hblock, 0, s>>>(nullptr, x, d, 0.0f, sc.hist, nwc);
  BTS_LAUNCH_CHECK();
  if (ev1) (void)hipEventRecord(ev1, s);
  k_mid_capture<<<grid, block, 0, s>>>(x, d, K, sc.hist, bound, sc.cand_cnt, sc.cand, pl.cap,
                                       sc.dir, pl.nwc_pad, nwc);
  BTS_LAUNCH_CHECK();
  if (ranges.tab_start != nullptr)
    k_mid_finish<true><<<dim3(rows), dim3(kMidBlock), 0, s>>>(
        x, d, K, sc.hist, bound, sc.cand_cnt, sc.cand, pl.cap, sc.dir, pl.nwc_pad, pl.ntiles,
        out_idx, out_val, upd, rows, ranges.tab_start, ranges.tab_end, ranges.any);
  else
    k_mid_finish<false><<<dim3(rows), dim3(kMidBlock), 0, s>>>(
        x, d, K, sc.hist, bound, sc.cand_cnt, sc.cand, pl.cap, sc.dir, pl.nwc_pad, pl.ntiles,
        out_idx, out_val, upd, rows, nullptr, nullptr, nullptr);
  BTS_LAUNCH_CHECK();
  *sc.dirty = false;
  return hipSuccess;
}

}  // namespace bts
