// Device code shared by the selects that capture candidates into per-row lists with a chunk
// directory (fast_select.hip: lower bound from a sample; mid_select.hip: lower bound from an
// exact first-digit histogram): the capture of one wave chunk, and the view of a directory
// tile through which the candidates are read back in index order.
#pragma once

#include "bts_device.h"

namespace bts {

namespace {

// The candidates of a row are kept in kSubLists independent lists, each with its own
// append counter on its own 128-byte line.  Wave-chunk wc appends to list wc % kSubLists,
// which spreads even clustered hits evenly.
constexpr uint32_t kSubLists = 64;
constexpr uint32_t kCounterStride = 32;               // words between two counters

// ---- 2. the dense pass ------------------------------------------------------------------
// One wave per kWaveChunk coordinates.  Whole chunks take the fast body: kUnroll 16-byte
// loads per lane and array in flight, fused multiply-add, store, compare against the
// row's lower bound.  A chunk with hits (rare) ranks them in index order with one wave
// scan, reserves room in its list with ONE atomic add, stores the entries there as one
// run, and records (start of the run, length) in the row's chunk directory.  Chunks
// without hits leave their directory entry alone (it is zero between calls).  The partial
// chunks at the ends of a row load element by element and append the same way.
static_assert(kUnroll == 1 || kUnroll % 2 == 0, "slices are counted in pairs");

// flags: bit 4u + j set = element j of the lane's slice u is a hit; v: the lane's values;
// i0: index in the row of the lane's first element of slice 0 (modulo 2^32 for lanes that
// start before the row).  All lanes of the wave call this together.
// Returns whether the run did not fit into its list (the row is then redone by the dense path).
__device__ __forceinline__ bool append_run(uint32_t flags, const float (&v)[kUnroll][4],
                                           uint32_t i0, uint32_t* counter, uint2* list,
                                           uint32_t cap, uint2* dir_entry) {
  if (__ballot(flags != 0) == 0) return false;
  // index order: slice 0 of every lane, then slice 1, ...  The hits of two slices are
  // counted in the halves of one word (a slice has 256 elements: no carry) and scanned
  // together.
  constexpr int kPairs = (kUnroll + 1) / 2;
  uint32_t excl[kPairs], tot[kPairs];
#pragma unroll
  for (int h = 0; h < kPairs; ++h) {
    uint32_t mine = (uint32_t)__popc((flags >> (8 * h)) & 0xFu);
    if (2 * h + 1 < kUnroll) mine |= (uint32_t)__popc((flags >> (8 * h + 4)) & 0xFu) << 16;
    const uint32_t incl = wave_inclusive_scan(mine);
    tot[h] = __shfl(incl, kWave - 1, kWave);
    excl[h] = incl - mine;
  }
  uint32_t start[kUnroll];                    // hits in the slices before slice u
  uint32_t total = 0;
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    start[u] = total;
    total += (u & 1) ? (tot[u / 2] >> 16) : (tot[u / 2] & 0xFFFFu);
  }
  uint32_t base = 0;
  if (lane_id() == 0) {
    base = atomicAdd(counter, total);
    *dir_entry = make_uint2(base, total);
  }
  base = __shfl(base, 0, kWave);
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    uint32_t pos = base + start[u] + ((u & 1) ? (excl[u / 2] >> 16) : (excl[u / 2] & 0xFFFFu));
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (flags & (1u << (4 * u + j))) {
        if (pos < cap)
          list[pos] = make_uint2(i0 + (uint32_t)u * (kWave * 4) + j, __float_as_uint(v[u][j]));
        ++pos;
      }
    }
  }
  return base + total > cap;
}

// ENERGY (diagnostics only): the wave also sums, in fp64, the squares of its chunk's
// coordinates that are NOT captured and stores the sum at energy[row * nwc_pad + wc]; with
// the squares of the captured-but-not-kept entries (added up by the emission) that is the
// row's residual energy |a - Top_K(a)|^2 without another pass over the row.
__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

//
// U (FMA only; 2^31 and above = never): coordinates with key >= U, a bound U >= L near the
// K-th largest key, are almost surely sent, so +0 instead of a goes to x there with the same
// 16-byte store that writes the chunk -- otherwise the emission would have to zero them with
// K scattered 4-byte stores per row, which cost as much time as a tenth of this pass where K
// is a percent of d.  The value is not lost: it sits in the chunk's run.  Whoever finds out
// that such a coordinate is not sent after all writes it back from there (the emission: the
// few entries between U and the threshold; the select: every such entry of a row that it
// hands to the dense path).  A chunk whose run did not fit into its list has no such copy
// and writes its values back itself, below.
template <bool FMA, bool ENERGY>
__device__ __forceinline__ void capture_chunk(
    uint32_t row, uint32_t wc, uint32_t L, uint32_t U, const float* __restrict__ g,
    float* __restrict__ x, uint64_t d, float alpha, uint32_t* __restrict__ cand_cnt,
    uint2* __restrict__ cand, uint32_t cap, uint2* __restrict__ dir, uint32_t nwc_pad,
    double* __restrict__ energy) {
  const ChunkGeom c = wave_chunk(d, row, wc);
  if (!c.active) return;
  const uint64_t sub = (uint64_t)row * kSubLists + wc % kSubLists;
  uint2* list = cand + sub * cap;                 // cap = capacity of one list
  uint32_t* counter = cand_cnt + sub * kCounterStride;
  uint2* dir_entry = dir + (uint64_t)row * nwc_pad + wc;
  const uint64_t e0 = c.base + (uint64_t)lane_id() * 4;
  const uint32_t i0 = (uint32_t)(e0 - c.lo);
  uint32_t flags = 0;
  uint32_t in_row = 0;                       // ENERGY: which of the lane's elements are the row's
  float v[kUnroll][4];
  if (c.full) {
    in_row = (1u << (4 * kUnroll)) - 1u;
    f4 xv[kUnroll];
    f4 gv[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint64_t e = e0 + (uint64_t)u * (kWave * 4);
      xv[u] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(x + e));
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
      }
      v[u][0] = xv[u].x;
      v[u][1] = xv[u].y;
      v[u][2] = xv[u].z;
      v[u][3] = xv[u].w;
#pragma unroll
      for (int j = 0; j < 4; ++j) flags |= (key_of(v[u][j]) >= L ? 1u : 0u) << (4 * u + j);
      if (FMA) {
        f4 st;
        st.x = key_of(v[u][0]) >= U ? 0.0f : v[u][0];
        st.y = key_of(v[u][1]) >= U ? 0.0f : v[u][1];
        st.z = key_of(v[u][2]) >= U ? 0.0f : v[u][2];
        st.w = key_of(v[u][3]) >= U ? 0.0f : v[u][3];
        __builtin_nontemporal_store(st, reinterpret_cast<f4*>(x + e));
      }
    }
  } else {
    int u = 0;
    visit_chunk<FMA>(g, x, c, alpha, false, [&](uint64_t e, const float (&vv)[4], uint32_t mask) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        v[u][j] = vv[j];
        const bool mine = ((mask >> j) & 1u) != 0;
        flags |= (mine && key_of(vv[j]) >= L ? 1u : 0u) << (4 * u + j);
        if (FMA && mine && key_of(vv[j]) >= U) x[e + j] = 0.0f;    // after the lane's own store of a
      }
      in_row |= mask << (4 * u);
      ++u;
    });
  }
  if (ENERGY) {
    double e = 0.0;
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if ((in_row & ~flags) & (1u << (4 * u + j))) e += (double)v[u][j] * (double)v[u][j];
    e = wave_sum_f64(e);
    if (lane_id() == 0) energy[(uint64_t)row * nwc_pad + wc] = e;
  }
  const bool lost = append_run(flags, v, i0, counter, list, cap, dir_entry);
  if (FMA && lost) {
    // the run did not fit (the bound was far too low for this row): a goes back to x, after
    // the stores above (same lane, same address; the wait makes the order explicit)
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if ((flags & (1u << (4 * u + j))) && key_of(v[u][j]) >= U)
          x[e0 + (uint64_t)u * (kWave * 4) + j] = v[u][j];
  }
}

// Result of the exact select over the candidate lists of a row.
struct FastSel {
  uint32_t prefix, k_rem;     // key select in progress: first digit, keys wanted at or below it
  uint32_t T, r;              // threshold key; how many holders of T are kept
  uint32_t U;                 // the dense pass of this call stored +0 where key >= U
  uint32_t next_bin;          // first-digit bin of the entry at the rank the next call aims at
};

// ---- directory tiles -----------------------------------------------------------------------
constexpr uint32_t kTileChunks = kWave;
constexpr int kEmitUnroll = 4;                // entries per lane in flight

struct TileView {
  uint32_t total;          // entries in the tile
  const uint32_t* off;     // per chunk: entries before it in the tile (LDS, this wave's)
  const uint32_t* start;   // per chunk: start of its run in its list (LDS, this wave's)
};

// Where most tiles are empty (few candidates per tile) a wave takes TPW = 4 tiles, a
// quarter of the row apart (tile v, v + Q, v + 2Q, v + 3Q, so that a run of busy tiles is
// spread over many waves), fetches their directory entries together and skips the empty
// ones without further work; where most tiles are busy a wave takes one.

// Publishes the scanned run lengths of a tile (ent = the lane's directory entry) to the
// wave's part of LDS.
__device__ __forceinline__ TileView publish_tile(uint2 ent, uint32_t* lds_off,
                                                 uint32_t* lds_start) {
  const uint32_t incl = wave_inclusive_scan(ent.y);
  wave_lds_sync();                               // the previous tile's readers are done
  lds_off[lane_id()] = incl - ent.y;
  lds_start[lane_id()] = ent.x;
  wave_lds_sync();
  TileView t;
  t.total = __shfl(incl, kWave - 1, kWave);
  t.off = lds_off;
  t.start = lds_start;
  return t;
}

// Entry e (0 <= e < total) of the tile, in index order.
__device__ __forceinline__ uint2 tile_entry(const TileView& t, uint32_t e,
                                            const uint2* __restrict__ cand_row, uint32_t cap) {
  uint32_t c = 0;                              // the last chunk with off[c] <= e
#pragma unroll
  for (uint32_t s = kTileChunks / 2; s > 0; s >>= 1)
    if (t.off[c + s] <= e) c += s;
  return cand_row[(uint64_t)c * cap + t.start[c] + (e - t.off[c])];
}

}  // namespace

}  // namespace bts
