// Dense exact Top_K select: a three-digit (11 + 10 + 10 bit) radix select on the 31-bit
// magnitude key with LDS histograms (each kernel resolves the digits found so far from the
// finished histograms at its start), followed by an ordered emission that needs no
// atomics for placement: the row's chunks are cut into contiguous shares (one per block),
// a pass counts (key > T) and (key == T) per chunk and per share, and the emission finds
// where a share starts from the totals of the shares before it and where a chunk starts
// from a scan of the share's own counts in LDS, then ranks inside the chunk with
// ballot/popcount prefix sums.  Five launches.  Ties at the
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
                                                  uint2* __restrict__ cnt,
                                                  uint2* __restrict__ block_sums, uint32_t nwc,
                                                  RowMask need, bool streaming) {
  count_body(VGrid{blockIdx.x, blockIdx.y, gridDim.x}, x, d, K, hist, st, cnt, block_sums, nwc,
             need, streaming);
}

// Ordered emission.  A block owns the same contiguous share of chunks as in the count.  The
// kept coordinates before the share number the totals of the shares before it; the counts
// of the share's own chunks are scanned in LDS.  The waves then re-read the share's chunks
// side by side, rank their kept coordinates with ballots and write (index, value) to the
// row's message at
//     #kept before it = #(key > T) before it + min(#(key == T) before it, r),
// then store +0 over the kept coordinate (the residual).
__global__ __launch_bounds__(kBlock) void k_emit(float* __restrict__ x, uint64_t d, uint32_t K,
                                                 const SelState* __restrict__ st,
                                                 const uint2* __restrict__ cnt,
                                                 const uint2* __restrict__ block_sums,
                                                 uint32_t nwc, uint32_t* __restrict__ out_idx,
                                                 float* __restrict__ out_val,
                                                 uint32_t* __restrict__ hist, RowMask need,
                                                 bool streaming, FusedUpdate upd,
                                                 NextBounds heal, MidRanges ranges) {
  __shared__ uint32_t lds[kBlock / kWave + 1];
  __shared__ uint32_t s_gt[kMaxShare], s_eq[kMaxShare];
  const uint32_t row = blockIdx.y;
  if (!row_needed(need, row)) {
    if (ranges.tab_start != nullptr) {             // the finished message of a worker row
      const uint32_t* msg = out_idx + (uint64_t)row * K;
      const uint32_t N = gridDim.y;
      for (uint32_t j = blockIdx.x * kBlock + threadIdx.x; j < K; j += gridDim.x * kBlock) {
        const uint32_t i = msg[j];
        if (i >= d) continue;
        const uint32_t rg = i / kAggWidth;
        if (j == 0 || msg[j - 1] / kAggWidth != rg) {
          ranges.tab_start[(uint64_t)rg * N + row] = K - j;
          ranges.any[rg] = 1u;
        }
        if (j + 1 == K || msg[j + 1] / kAggWidth != rg)
          ranges.tab_end[(uint64_t)rg * N + row] = j + 1;
      }
    }
    if (upd.w != nullptr && upd.after) {           // the finished message of a one-row select
      for (uint32_t j = blockIdx.x * kBlock + threadIdx.x; j < K; j += gridDim.x * kBlock) {
        const uint32_t i = out_idx[(uint64_t)row * K + j];
        if (i < d)
          upd.w[i] = __fmaf_rn(upd.neg_alpha, out_val[(uint64_t)row * K + j], upd.w[i]);
      }
    }
    return;
  }
  if (blockIdx.x == 0)                             // leave the row's histograms clear
    for (int i = threadIdx.x; i < kRowHist; i += kBlock) hist[(uint64_t)row * kRowHist + i] = 0;
  const uint32_t T = st[row].T, r = st[row].r;
  if (heal.lower_key != nullptr && blockIdx.x == 0 && threadIdx.x == 0) {
    // a row the single-pass select handed over: its next call starts from the exact
    // threshold, a tenth below it in magnitude (finite, non-zero T; else from zero)
    const bool plain = T != 0 && T < 0x7F800000u;
    heal.lower_key[row] = plain ? __float_as_uint(__uint_as_float(T) * 0.9f) : 0u;
    if (heal.early_zero) heal.upper_key[row] = T ? T : 0xFFFFFFFFu;
    heal.prev_T[row] = 0;                          // no trend across a redo
    if (heal.redone != nullptr) *heal.redone = 1u; // the host samples again on a later call
  }
  const VGrid vg{blockIdx.x, blockIdx.y, gridDim.x};
  const ChunkShare sh = block_share(vg, nwc);
  // kept before this share: every thread adds up some of the earlier shares' totals
  uint32_t a = 0, b = 0;
  const uint2* bs = block_sums + (uint64_t)row * vg.gx;
  for (uint32_t i = threadIdx.x; i < vg.bx; i += kBlock) {
    const uint2 v = bs[i];
    a += v.x;
    b += v.y;
  }
  uint32_t base_gt, base_eq;
  (void)block_exclusive_scan(a, lds, &base_gt);
  (void)block_exclusive_scan(b, lds, &base_eq);
  uint32_t* oi = out_idx + (uint64_t)row * K;
  float* ov = out_val + (uint64_t)row * K;
  // the share in segments of at most kMaxShare chunks (one segment unless the row is
  // longer than 2.7e8 coordinates)
  for (uint32_t seg = sh.begin; seg < sh.end; seg += kMaxShare) {
    const uint32_t n = min(kMaxShare, sh.end - seg);
    // where each chunk of the segment starts: exclusive scan of its counts (a thread owns
    // kMaxShare / kBlock consecutive chunks)
    {
      constexpr uint32_t kPer = kMaxShare / kBlock;
      const uint2* cr = cnt + (uint64_t)row * nwc + seg;
      uint2 v[kPer];
      uint32_t sg = 0, se = 0;
#pragma unroll
      for (uint32_t k = 0; k < kPer; ++k) {
        const uint32_t i = threadIdx.x * kPer + k;
        v[k] = i < n ? cr[i] : make_uint2(0u, 0u);
        sg += v[k].x;
        se += v[k].y;
      }
      uint32_t tot_g, tot_e;
      uint32_t og = base_gt + block_exclusive_scan(sg, lds, &tot_g);
      uint32_t oe = base_eq + block_exclusive_scan(se, lds, &tot_e);
#pragma unroll
      for (uint32_t k = 0; k < kPer; ++k) {
        const uint32_t i = threadIdx.x * kPer + k;
        if (i < n) {
          s_gt[i] = og;
          s_eq[i] = oe;
        }
        og += v[k].x;
        oe += v[k].y;
      }
      base_gt += tot_g;
      base_eq += tot_e;
    }
    __syncthreads();
    for (uint32_t wc = seg + threadIdx.x / kWave; wc < seg + n; wc += kWavesPerBlock) {
      const ChunkGeom c = wave_chunk(d, row, wc);
      if (!c.active) break;
      uint32_t run_gt = s_gt[wc - seg], run_eq = s_eq[wc - seg];   // wave-uniform
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
              const uint32_t i = (uint32_t)(e + j - c.lo);
              oi[pos] = i;
              ov[pos] = v[j];
              x[e + j] = 0.0f;
              if (ranges.tab_start != nullptr) {   // pairs arrive in no order: maxima
                const uint64_t at = (uint64_t)(i / kAggWidth) * gridDim.y + row;
                atomicMax(&ranges.tab_start[at], K - pos);
                atomicMax(&ranges.tab_end[at], pos + 1);
                ranges.any[i / kAggWidth] = 1u;
              }
              if (upd.w != nullptr) upd.w[i] = __fmaf_rn(upd.neg_alpha, v[j], upd.w[i]);
            }
          }
          my_gt += is_gt ? 1u : 0u;
          my_eq += is_eq ? 1u : 0u;
        }
        run_gt += tot_gt;
        run_eq += tot_eq;
      });
    }
    __syncthreads();                              // the next segment reuses the LDS offsets
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

uint32_t dense_max_blocks(uint32_t rows) {
  const uint32_t lim = kDenseMaxGx / (rows ? rows : 1u);
  return lim < 256u ? 256u : lim;
}

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
  const uint32_t lim = dense_max_blocks(rows);
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
                        float* out_val, RowMask need, FusedUpdate upd, NextBounds heal,
                        MidRanges ranges) {
  if (ranges.tab_start != nullptr && need == nullptr) return hipErrorInvalidValue;
  if (upd.w != nullptr && rows != 1) return hipErrorInvalidValue;
  const uint32_t nwc = pl.nwc;
  k_emit<<<dim3(pl.gx, rows), dim3(kBlock), 0, s>>>(x, d, K, sc.state, sc.cnt,
                                                    sc.block_sums, nwc, out_idx, out_val,
                                                    sc.hist, need, pl.streaming, upd, heal,
                                                    ranges);
  BTS_LAUNCH_CHECK();
  *sc.dirty = false;
  return hipSuccess;
}

hipError_t dense_select(hipStream_t s, const DenseScratch& sc, const float* g, float* x,
                        uint32_t rows, uint64_t d, uint32_t K, float alpha, uint32_t* out_idx,
                        float* out_val, RowMask need, bool first_pass_done,
                        hipEvent_t ev0, hipEvent_t ev1, FusedUpdate upd) {
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
  k_count<<<grid, block, 0, s>>>(x, d, K, sc.hist, sc.state, sc.cnt, sc.block_sums, nwc, need,
                                 streaming);
  BTS_LAUNCH_CHECK();
  return dense_finish(s, sc, pl, x, rows, d, K, out_idx, out_val, need, upd);
}

}  // namespace bts
