// Dense exact Top_K select: a three-digit (11 + 10 + 10 bit) radix select on the 31-bit
// magnitude key with LDS histograms (each kernel resolves the digits found so far from the
// finished histograms at its start), followed by an ordered emission that needs no
// atomics for placement: per-wave-chunk counts of (key > T) and (key == T), an exclusive
// scan over the chunks of a row, and in-wave ballot/popcount prefix sums.  Ties at the
// threshold go to the lowest indices.  Works for every input and every K in 1..d; it is
// the reference path of the library and the fallback of the speculative single-pass path.
//
// Implements the Top_K operator used on the worker and server compression lines of
// Algorithm 2 (a^q -> Top_K(a^q), eps^q = a^q - Top_K(a^q); g_t -> Top_K(g_t),
// delta_t = g_t - Top_K(g_t)); the first pass can also fuse the worker's error
// compensation a^q = eps^q + alpha g^q.

#include "dense_bodies.h"

namespace bts {

namespace {

template <int DIGIT, bool FMA>
__global__ __launch_bounds__(kBlock) void k_hist(const float* __restrict__ g,
                                                 float* __restrict__ x, uint64_t d, float alpha,
                                                 uint32_t K, uint32_t* __restrict__ hist,
                                                 uint32_t nwc, RowMask need, bool streaming) {
  hist_body<DIGIT, FMA>(VGrid{blockIdx.x, blockIdx.y, gridDim.x}, g, x, d, alpha, K, hist, nwc,
                        need, streaming);
}

__global__ __launch_bounds__(kBlock) void k_count(const float* __restrict__ x, uint64_t d,
                                                  uint32_t K, const uint32_t* __restrict__ hist,
                                                  SelState* __restrict__ st,
                                                  uint32_t* __restrict__ cnt_gt,
                                                  uint32_t* __restrict__ cnt_eq, uint32_t nwc,
                                                  RowMask need, bool streaming) {
  count_body(VGrid{blockIdx.x, blockIdx.y, gridDim.x}, x, d, K, hist, st, cnt_gt, cnt_eq, nwc,
             need, streaming);
}

// Exclusive scan of the per-chunk counts of every row, in place, in two levels: sums of
// tiles of kScanTile chunks, then each tile scanned from the sum of the tiles before it.
constexpr uint32_t kScanTile = 4096;

__global__ __launch_bounds__(1024) void k_tile_sums(const uint32_t* __restrict__ cnt_gt,
                                                    const uint32_t* __restrict__ cnt_eq,
                                                    uint32_t nwc, uint32_t ntiles,
                                                    uint32_t* __restrict__ tile_sums,
                                                    RowMask need) {
  __shared__ uint32_t lds[1024 / kWave + 1];
  const uint32_t row = blockIdx.y, tile = blockIdx.x;
  if (!row_needed(need, row)) return;
  const uint32_t b = tile * kScanTile, e = min(b + kScanTile, nwc);
#pragma unroll 1
  for (int which = 0; which < 2; ++which) {
    const uint32_t* a = (which == 0 ? cnt_gt : cnt_eq) + (uint64_t)row * nwc;
    uint32_t s = 0;
    for (uint32_t i = b + threadIdx.x; i < e; i += blockDim.x) s += a[i];
    uint32_t total;
    (void)block_exclusive_scan(s, lds, &total);
    if (threadIdx.x == 0) tile_sums[((uint64_t)row * 2 + which) * ntiles + tile] = total;
  }
}

__global__ __launch_bounds__(1024) void k_scan_chunks(uint32_t* __restrict__ cnt_gt,
                                                      uint32_t* __restrict__ cnt_eq,
                                                      uint32_t nwc, uint32_t ntiles,
                                                      const uint32_t* __restrict__ tile_sums,
                                                      RowMask need) {
  __shared__ uint32_t lds[1024 / kWave + 1];
  const uint32_t row = blockIdx.y, tile = blockIdx.x;
  if (!row_needed(need, row)) return;
  const uint32_t b = tile * kScanTile, e = min(b + kScanTile, nwc);
  constexpr uint32_t kPer = kScanTile / 1024;        // consecutive chunks per thread
#pragma unroll 1
  for (int which = 0; which < 2; ++which) {
    uint32_t* a = (which == 0 ? cnt_gt : cnt_eq) + (uint64_t)row * nwc;
    const uint32_t* ts = tile_sums + ((uint64_t)row * 2 + which) * ntiles;
    uint32_t before = 0;
    for (uint32_t t = threadIdx.x; t < tile; t += blockDim.x) before += ts[t];
    uint32_t base;
    (void)block_exclusive_scan(before, lds, &base);  // base = sum over the earlier tiles
    uint32_t v[kPer];
    uint32_t s = 0;
    const uint32_t i0 = b + threadIdx.x * kPer;
#pragma unroll
    for (uint32_t k = 0; k < kPer; ++k) {
      v[k] = i0 + k < e ? a[i0 + k] : 0u;
      s += v[k];
    }
    uint32_t total;
    uint32_t run = base + block_exclusive_scan(s, lds, &total);
#pragma unroll
    for (uint32_t k = 0; k < kPer; ++k) {
      if (i0 + k < e) a[i0 + k] = run;
      run += v[k];
    }
  }
}

// Ordered emission.  Every wave re-reads its chunk, ranks its kept coordinates with
// ballots and writes (index, value) to the row's message at
//     #kept before it = #(key > T) before it + min(#(key == T) before it, r),
// then stores +0 over the kept coordinate (the residual).
__global__ __launch_bounds__(kBlock) void k_emit(float* __restrict__ x, uint64_t d, uint32_t K,
                                                 const SelState* __restrict__ st,
                                                 const uint32_t* __restrict__ off_gt,
                                                 const uint32_t* __restrict__ off_eq,
                                                 uint32_t nwc, uint32_t* __restrict__ out_idx,
                                                 float* __restrict__ out_val,
                                                 uint32_t* __restrict__ hist, RowMask need,
                                                 bool streaming) {
  const uint32_t row = blockIdx.y;
  if (!row_needed(need, row)) return;
  if (blockIdx.x == 0)                             // leave the row's histograms clear
    for (int i = threadIdx.x; i < kRowHist; i += kBlock) hist[(uint64_t)row * kRowHist + i] = 0;
  const uint32_t T = st[row].T, r = st[row].r;
  for (uint32_t wc = blockIdx.x * kWavesPerBlock + threadIdx.x / kWave; wc < nwc;
       wc += gridDim.x * kWavesPerBlock) {
  const ChunkGeom c = wave_chunk(d, row, wc);
  if (!c.active) break;
  uint32_t run_gt = off_gt[(uint64_t)row * nwc + wc];   // wave-uniform running counts
  uint32_t run_eq = off_eq[(uint64_t)row * nwc + wc];
  uint32_t* oi = out_idx + (uint64_t)row * K;
  float* ov = out_val + (uint64_t)row * K;
  visit_chunk<false>(nullptr, x, c, 0.0f, streaming,
                     [&](uint64_t e, const float (&v)[4], uint32_t mask) {
    uint32_t fgt = 0, feq = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t key = key_of(v[j]);
      const bool in = mask & (1u << j);
      fgt |= (in && key > T) ? (1u << j) : 0u;
      feq |= (in && key == T) ? (1u << j) : 0u;
    }
    if (__ballot(fgt | feq) == 0) return;     // nothing near the threshold in this slice
    uint32_t tot_gt, tot_eq;
    uint32_t my_gt = run_gt + wave_exclusive_small(__popc(fgt), &tot_gt);
    uint32_t my_eq = run_eq + wave_exclusive_small(__popc(feq), &tot_eq);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bool is_gt = fgt & (1u << j), is_eq = feq & (1u << j);
      if (is_gt || (is_eq && my_eq < r)) {
        const uint32_t pos = my_gt + min(my_eq, r);
        if (pos < K) {
          oi[pos] = (uint32_t)(e + j - c.lo);
          ov[pos] = v[j];
          x[e + j] = 0.0f;
        }
      }
      my_gt += is_gt ? 1u : 0u;
      my_eq += is_eq ? 1u : 0u;
    }
    run_gt += tot_gt;
    run_eq += tot_eq;
  });
  }
}

// x = fma(alpha, g, x) with no selection (K == 0).
__global__ __launch_bounds__(kBlock) void k_axpy(const float* __restrict__ g,
                                                 float* __restrict__ x, uint64_t d,
                                                 float alpha) {
  const uint32_t wc = blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
  const ChunkGeom c = wave_chunk(d, blockIdx.y, wc);
  if (c.active)
    visit_chunk<true>(g, x, c, alpha, true, [](uint64_t, const float (&)[4], uint32_t) {});
}

__global__ void k_fill(uint32_t* p, uint64_t n, uint32_t v) {
  const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

#define BTS_LAUNCH_CHECK()                       \
  do {                                           \
    hipError_t e_ = hipGetLastError();           \
    if (e_ != hipSuccess) return e_;             \
  } while (0)

}  // namespace

uint32_t dense_scan_tiles(uint32_t nwc) { return (nwc + kScanTile - 1) / kScanTile; }

hipError_t fill_u32(hipStream_t s, uint32_t* p, uint64_t n, uint32_t v) {
  if (n == 0) return hipSuccess;
  k_fill<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(p, n, v);
  return hipGetLastError();
}

hipError_t axpy_only(hipStream_t s, const float* g, float* x, uint32_t rows, uint64_t d,
                     float alpha, hipEvent_t ev0, hipEvent_t ev1) {
  const uint32_t nwc = (uint32_t)((d + kWaveChunk - 1) / kWaveChunk) + 1;
  dim3 grid((nwc + kWavesPerBlock - 1) / kWavesPerBlock, rows);
  if (ev0) (void)hipEventRecord(ev0, s);
  k_axpy<<<grid, dim3(kBlock), 0, s>>>(g, x, d, alpha);
  BTS_LAUNCH_CHECK();
  if (ev1) (void)hipEventRecord(ev1, s);
  return hipSuccess;
}

uint32_t dense_row_hist_words() { return kRowHist; }

DensePlan dense_plan(const DenseScratch& sc, uint32_t rows, uint64_t d) {
  DensePlan pl;
  pl.nwc = sc.nwc;
  // A bounded grid whose blocks loop over the chunks: every block flushes its LDS histogram
  // to the row's global histogram with atomics that are served at the memory side and
  // serialise per address, so few fat blocks beat many thin ones; and as a gated fallback
  // most rows leave at once, which keeps idle launches cheap.
  uint32_t gx = (pl.nwc + kWavesPerBlock - 1) / kWavesPerBlock;
  // at least 256 blocks per row, so that a lone row that falls back still streams fast;
  // a single row gets 512 (measured at d = 1.1e7: 512 blocks beat 256 by their streaming,
  // 2048 and 4096 lose 40 and 120 us per select to the flush into the row's histogram)
  uint32_t lim = 512u / rows;
  if (lim < 256u) lim = 256u;
  if (gx > lim) gx = lim;
  pl.gx = gx;
  // rows that are read five times stay in the caches when they are small; beyond the 256 MB
  // of last-level cache they are streamed past it
  pl.streaming = (uint64_t)rows * d * 4 > (256ull << 20);
  return pl;
}

hipError_t dense_begin(hipStream_t s, const DenseScratch& sc) {
  if (*sc.dirty) {                                 // an earlier call failed half way
    hipError_t e = fill_u32(s, sc.hist, (uint64_t)sc.rows * kRowHist, 0);
    if (e != hipSuccess) return e;
  }
  *sc.dirty = true;                                // cleared when every launch went out
  return hipSuccess;
}

hipError_t dense_finish(hipStream_t s, const DenseScratch& sc, const DensePlan& pl, float* x,
                        uint32_t rows, uint64_t d, uint32_t K, uint32_t* out_idx,
                        float* out_val, RowMask need) {
  const uint32_t nwc = pl.nwc;
  const uint32_t ntiles = (nwc + kScanTile - 1) / kScanTile;
  if (ntiles > 1) {                                // a single tile starts from zero
    k_tile_sums<<<dim3(ntiles, rows), dim3(1024), 0, s>>>(sc.cnt_gt, sc.cnt_eq, nwc, ntiles,
                                                          sc.tile_sums, need);
    BTS_LAUNCH_CHECK();
  }
  k_scan_chunks<<<dim3(ntiles, rows), dim3(1024), 0, s>>>(sc.cnt_gt, sc.cnt_eq, nwc, ntiles,
                                                          sc.tile_sums, need);
  BTS_LAUNCH_CHECK();
  k_emit<<<dim3(pl.gx, rows), dim3(kBlock), 0, s>>>(x, d, K, sc.state, sc.cnt_gt, sc.cnt_eq, nwc,
                                                    out_idx, out_val, sc.hist, need,
                                                    pl.streaming);
  BTS_LAUNCH_CHECK();
  *sc.dirty = false;
  return hipSuccess;
}

hipError_t dense_select(hipStream_t s, const DenseScratch& sc, const float* g, float* x,
                        uint32_t rows, uint64_t d, uint32_t K, float alpha, uint32_t* out_idx,
                        float* out_val, RowMask need, bool first_pass_done,
                        hipEvent_t ev0, hipEvent_t ev1) {
  const DensePlan pl = dense_plan(sc, rows, d);
  const uint32_t nwc = pl.nwc;
  const bool streaming = pl.streaming;
  const dim3 grid(pl.gx, rows);
  const dim3 block(kBlock);
  hipError_t e = dense_begin(s, sc);
  if (e != hipSuccess) return e;
  const bool fuse = (g != nullptr) && !first_pass_done;
  if (fuse) {
    if (ev0) (void)hipEventRecord(ev0, s);
    k_hist<0, true><<<grid, block, 0, s>>>(g, x, d, alpha, K, sc.hist, nwc, need, streaming);
    BTS_LAUNCH_CHECK();
    if (ev1) (void)hipEventRecord(ev1, s);
  } else {
    k_hist<0, false><<<grid, block, 0, s>>>(nullptr, x, d, 0.0f, K, sc.hist, nwc, need, streaming);
    BTS_LAUNCH_CHECK();
  }
  k_hist<1, false><<<grid, block, 0, s>>>(nullptr, x, d, 0.0f, K, sc.hist, nwc, need, streaming);
  BTS_LAUNCH_CHECK();
  k_hist<2, false><<<grid, block, 0, s>>>(nullptr, x, d, 0.0f, K, sc.hist, nwc, need, streaming);
  BTS_LAUNCH_CHECK();
  k_count<<<grid, block, 0, s>>>(x, d, K, sc.hist, sc.state, sc.cnt_gt, sc.cnt_eq, nwc, need,
                                 streaming);
  BTS_LAUNCH_CHECK();
  return dense_finish(s, sc, pl, x, rows, d, K, out_idx, out_val, need);
}

}  // namespace bts
