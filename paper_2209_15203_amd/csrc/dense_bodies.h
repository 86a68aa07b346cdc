// Device bodies of the dense select's first four kernels (three digit histograms and the
// per-chunk counts), shared by dense_select.hip, which launches them as kernels of their
// own, and fast_select.hip, where the gated redo of flagged rows rides in the same launches
// as the tail of the single-pass select.  A body is written against a virtual block index
// (VGrid) instead of the launch's own.
#pragma once

#include "bts_device.h"

namespace bts {

namespace {

struct VGrid {
  uint32_t bx, by, gx;     // block index in x (chunks), in y (row), blocks in x
};

__device__ __forceinline__ bool row_needed(RowMask need, uint32_t row) {
  return need == nullptr || need[row] != 0;
}

// Each row has three global histograms (digit 0: 2048 bins, digits 1 and 2: 1024 bins), all
// zero between calls.  A kernel that needs the digits found so far walks the finished
// histograms itself at its start (every block, redundantly: a few thousand loads), which
// saves a separate launch per digit.
constexpr int kRowHist = kBins0 + 2 * kBinsLo;     // words of histogram per row

// Walk an NB-bin histogram from the top bin down and find the bin holding the `want`-th
// largest key; *above = keys in higher bins.  All threads of the block call this; the result
// is returned to every thread.
template <int NB>
__device__ __forceinline__ uint32_t resolve_digit(const uint32_t* __restrict__ h, uint32_t want,
                                                  uint32_t* lds, uint32_t* s_out,
                                                  uint32_t* above) {
  constexpr int BPT = NB / kBlock;
  const int top = NB - 1 - (int)threadIdx.x * BPT;   // this thread's highest bin
  uint32_t c[BPT];
  uint32_t s = 0;
#pragma unroll
  for (int i = 0; i < BPT; ++i) {
    c[i] = h[top - i];
    s += c[i];
  }
  uint32_t total;
  const uint32_t excl = block_exclusive_scan(s, lds, &total);   // count in higher bins
  if (excl < want && want <= excl + s) {                         // exactly one thread
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

// The digits fixed by the finished histograms of the row: after `digits` of them the key
// prefix (right aligned) and how many of the K wanted keys lie at or below the prefix's bin.
struct Resolved {
  uint32_t prefix, k_rem;
};

template <int DIGITS>
__device__ __forceinline__ Resolved resolve_row(const uint32_t* __restrict__ hist_row, uint32_t K,
                                                uint32_t* lds, uint32_t* s_out) {
  Resolved r{0u, K};
  uint32_t above;
  if (DIGITS >= 1) {
    const uint32_t b = resolve_digit<kBins0>(hist_row, r.k_rem, lds, s_out, &above);
    r.prefix = b;
    r.k_rem -= above;
  }
  if (DIGITS >= 2) {
    const uint32_t b = resolve_digit<kBinsLo>(hist_row + kBins0, r.k_rem, lds, s_out, &above);
    r.prefix = (r.prefix << 10) | b;
    r.k_rem -= above;
  }
  if (DIGITS >= 3) {
    const uint32_t b =
        resolve_digit<kBinsLo>(hist_row + kBins0 + kBinsLo, r.k_rem, lds, s_out, &above);
    r.prefix = (r.prefix << 10) | b;      // the exact K-th largest key T
    r.k_rem -= above;                     // how many holders of T are kept
  }
  return r;
}

// Histogram of one digit of the key over every coordinate of the row whose higher digits
// match the prefix found so far.
template <int DIGIT, bool FMA>
__device__ __forceinline__ void hist_body(const VGrid vg, const float* __restrict__ g,
                                          float* __restrict__ x, uint64_t d, float alpha,
                                          uint32_t K, uint32_t* __restrict__ hist, uint32_t nwc,
                                          RowMask need, bool streaming) {
  constexpr int NB = DIGIT == 0 ? kBins0 : kBinsLo;
  __shared__ uint32_t sh[NB];
  __shared__ uint32_t lds[kBlock / kWave + 1];
  __shared__ uint32_t s_out[2];
  const uint32_t row = vg.by;
  if (!row_needed(need, row)) return;
  uint32_t* hist_row = hist + (uint64_t)row * kRowHist;
  for (int i = threadIdx.x; i < NB; i += kBlock) sh[i] = 0;
  const uint32_t prefix = resolve_row<DIGIT>(hist_row, K, lds, s_out).prefix;
  __syncthreads();
  // Bin 0 is counted per lane: a sparse row (the server's g_t is mostly exact zeros) would
  // otherwise serialise the whole wave on one LDS address.
  uint32_t bin0 = 0;
  for (uint32_t wc = vg.bx * kWavesPerBlock + threadIdx.x / kWave; wc < nwc;
       wc += vg.gx * kWavesPerBlock) {
    const ChunkGeom c = wave_chunk(d, row, wc);
    if (!c.active) break;
    visit_chunk<FMA>(g, x, c, alpha, streaming, [&](uint64_t, const float (&v)[4], uint32_t mask) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (mask & (1u << j)) {
          const uint32_t key = key_of(v[j]);
          uint32_t bin;
          bool hit;
          if (DIGIT == 0) {
            bin = key >> 20;
            hit = true;
          } else if (DIGIT == 1) {
            bin = (key >> 10) & 1023u;
            hit = (key >> 20) == prefix;
          } else {
            bin = key & 1023u;
            hit = (key >> 10) == prefix;
          }
          if (hit) {
            if (bin == 0) ++bin0; else atomicAdd(&sh[bin], 1u);
          }
        }
      }
    });
  }
  if (bin0) atomicAdd(&sh[0], bin0);
  __syncthreads();
  uint32_t* h = hist_row + (DIGIT == 0 ? 0 : (DIGIT == 1 ? kBins0 : kBins0 + kBinsLo));
  for (int i = threadIdx.x; i < NB; i += kBlock) {
    const uint32_t v = sh[i];
    if (v) atomicAdd(&h[i], v);
  }
}

// The count and the emission cut a row's wave chunks into contiguous shares, one per block
// of the (virtual) grid: block bx takes chunks [bx * cpb, (bx + 1) * cpb) and its waves go
// through them side by side (wave w takes the w-th, (w + 4)-th, ... chunk of the share).
// Where a share starts in the row's message follows from the totals of the shares before
// it, and where a chunk starts inside the share from the share's own per-chunk counts: no
// scan over all the chunks, no pass of its own.
constexpr uint32_t kMaxShare = 1024;       // most chunks of one block's share

struct ChunkShare {
  uint32_t begin, end;       // the block's chunks
};

__device__ __forceinline__ ChunkShare block_share(const VGrid vg, uint32_t nwc) {
  const uint32_t cpb = (nwc + vg.gx - 1) / vg.gx;                  // chunks per block
  ChunkShare s;
  s.begin = min(vg.bx * cpb, nwc);
  s.end = min(s.begin + cpb, nwc);
  return s;
}

// Per wave chunk (cnt: rows x nwc pairs) and per block's share (block_sums: rows x gx pairs):
// how many coordinates lie strictly above the threshold key (x), how many on it (y).
__device__ __forceinline__ void count_body(const VGrid vg, const float* __restrict__ x,
                                           uint64_t d, uint32_t K,
                                           const uint32_t* __restrict__ hist,
                                           SelState* __restrict__ st, uint2* __restrict__ cnt,
                                           uint2* __restrict__ block_sums, uint32_t nwc,
                                           RowMask need, bool streaming) {
  __shared__ uint32_t lds[kBlock / kWave + 1];
  __shared__ uint32_t s_out[2];
  __shared__ uint32_t s_gt[kWavesPerBlock], s_eq[kWavesPerBlock];
  const uint32_t row = vg.by;
  if (!row_needed(need, row)) return;
  const Resolved res = resolve_row<3>(hist + (uint64_t)row * kRowHist, K, lds, s_out);
  const uint32_t T = res.prefix;
  if (vg.bx == 0 && threadIdx.x == 0) {            // for the emission kernel
    st[row].T = T;
    st[row].r = res.k_rem;
  }
  const ChunkShare sh = block_share(vg, nwc);
  const uint32_t w = threadIdx.x / kWave;
  uint32_t all_gt = 0, all_eq = 0;
  for (uint32_t wc = sh.begin + w; wc < sh.end; wc += kWavesPerBlock) {
    const ChunkGeom c = wave_chunk(d, row, wc);
    uint32_t gt = 0, eq = 0;
    if (c.active) {
      visit_chunk<false>(nullptr, const_cast<float*>(x), c, 0.0f, streaming,
                         [&](uint64_t, const float (&v)[4], uint32_t mask) {
#pragma unroll
                           for (int j = 0; j < 4; ++j) {
                             const uint32_t key = key_of(v[j]);
                             const bool in = mask & (1u << j);
                             gt += (in && key > T) ? 1u : 0u;
                             eq += (in && key == T) ? 1u : 0u;
                           }
                         });
    }
    gt = wave_sum(gt);
    eq = wave_sum(eq);
    if (lane_id() == 0) cnt[(uint64_t)row * nwc + wc] = make_uint2(gt, eq);
    all_gt += gt;
    all_eq += eq;
  }
  if (lane_id() == 0) {
    s_gt[w] = all_gt;
    s_eq[w] = all_eq;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t a = 0, b = 0;
    for (int i = 0; i < kWavesPerBlock; ++i) {
      a += s_gt[i];
      b += s_eq[i];
    }
    block_sums[(uint64_t)row * vg.gx + vg.bx] = make_uint2(a, b);
  }
}

}  // namespace

}  // namespace bts
