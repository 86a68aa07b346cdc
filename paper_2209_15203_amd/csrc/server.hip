// Server side of Algorithm 2 apart from the compression: the weighted aggregation
//     g_t = sum_q p_q Top_K(a^q) + delta_{t-1}
// and the model update  w_t = w_{t-1} - Top_K(g_t)  on the received pairs.
//
// Aggregation is deterministic without float atomics: the coordinate axis is cut into
// ranges of kAggWidth coordinates and ONE WAVE owns a range.  It takes the range's pairs
// in (worker, index) order into registers, 256 at a time, gathers the touched part of delta
// into an LDS accumulator, gives every pair its depth (how many earlier pairs name the same
// coordinate) and applies the pairs depth by depth: pairs of one depth name distinct
// coordinates and go in parallel, ascending depths are ascending q for every coordinate.
// Consecutive depths are ordered by the wave's program order alone: no workgroup barrier
// and no HBM latency inside the dependent steps.  Where each worker's sorted list enters
// and leaves each range comes from a table (or from binary searches when the table would be
// too large), and a flag per range lets a wave skip, 64 at a time, the ranges nobody names.

#include "bts_device.h"

namespace bts {

namespace {

constexpr int kAggBlock = 256;
constexpr int kAggWaves = kAggBlock / kWave;
constexpr uint32_t kAggStage = 256;    // pairs a wave holds in registers at a time (4 per lane)
constexpr uint32_t kAggMaxBlocks = 8192;

__device__ __forceinline__ uint32_t lower_bound_u32(const uint32_t* __restrict__ a, uint32_t n,
                                                    uint32_t key) {
  uint32_t lo = 0, hi = n;
  while (lo < hi) {
    const uint32_t mid = lo + ((hi - lo) >> 1);
    if (a[mid] < key) lo = mid + 1; else hi = mid;
  }
  return lo;
}

// Where each worker's sorted index list enters and leaves each range: pair j of worker q
// opens range r if its predecessor lies in another range and closes it if its successor
// does; the opener also raises the range's flag.  Table and flags are all zero between
// calls (the aggregation clears what it reads).
__global__ void k_range_bounds(const uint32_t* __restrict__ up_idx, uint32_t N, uint32_t K_up,
                               uint64_t d, uint32_t* __restrict__ start,
                               uint32_t* __restrict__ end, uint32_t* __restrict__ any) {
  const uint32_t q = blockIdx.y;
  const uint32_t j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= K_up) return;
  const uint32_t* row = up_idx + (uint64_t)q * K_up;
  if (row[j] >= d) return;                       // invalid input never reaches the table
  const uint32_t r = row[j] / kAggWidth;
  if (j == 0 || row[j - 1] / kAggWidth != r) {
    start[(uint64_t)r * N + q] = K_up - j;      // counted down from K_up: zero = none
    any[r] = 1u;
  }
  if (j + 1 == K_up || row[j + 1] / kAggWidth != r) end[(uint64_t)r * N + q] = j + 1;
}

constexpr uint32_t kAggNoRel = 0xFFFFu;
constexpr uint32_t kAggRounds = kAggStage / kWave;     // rounds of 64 pairs in a full stage
constexpr uint32_t kAggNoRange = 0xFFFFFFFFu;

// Where the workers of the first tile enter and leave a range, fetched by the wave while it
// still works on the range before (one entry per lane).
struct AggPrefetch {
  uint32_t lo, hi;
  bool valid;            // wave-uniform
};

struct AggWaveLds {
  float acc[kAggWidth];                 // g_t of the touched coordinates
  uint32_t touched[kAggWidth / 32];
  uint32_t seen[kAggWidth / 4];         // per coordinate, one byte: pairs of the stage so far
  uint32_t lo[kWave];                   // per worker of the tile: first pair in the range
  uint32_t pref[kWave + 1];             // pairs of the tile's earlier workers in the range
  float p[kWave];
};

__device__ __forceinline__ uint32_t seen_byte(const AggWaveLds& L, uint32_t rel) {
  return (L.seen[rel >> 2] >> (8 * (rel & 3))) & 0xFFu;
}

// MODE 0: bidirectional server (Algorithm 2): delta[i] = delta[i] + sum_q p_q v_q[i].
// MODE 1: count the distinct coordinates named in each range and nothing else.
// MODE 2: unidirectional server and update (Algorithm 1): g_t[i] = sum_q p_q v_q[i] from +0,
//         the named coordinates and their g_t written in ascending order to the message at
//         range_off[range] + rank, and w[i] = fma(-alpha_out, g_t[i], w[i]).
// Returns the number of distinct coordinates named in range r (same value in every lane).
//
// The pairs of the range are taken in (worker, index) order, kAggStage at a time (at most
// 64 workers per tile), four per lane, and stay in registers.  The depth of a pair is the number of earlier pairs of the stage on
// the same coordinate; pairs of one depth name distinct coordinates, so they are applied in
// parallel, and going through the depths in ascending order applies each coordinate's
// pairs in ascending q.  Stages and tiles follow each other in ascending q as well.
//
// The loads that depend on each other (table entry -> pair -> start value of delta) are what
// a range costs, so they are issued in batches: the pairs of a stage all at once, the start
// values of a stage all at once, and the table entries of the wave's next range (r_next)
// before the work on this one.
template <int MODE>
__device__ __forceinline__ uint32_t aggregate_range(
    AggWaveLds& L, uint32_t r, uint32_t r_next, AggPrefetch& pf,
    const uint32_t* __restrict__ up_idx,
    const float* __restrict__ up_val, const float* __restrict__ p, uint32_t N, uint32_t K_up,
    float* __restrict__ dense, uint64_t d, uint32_t* __restrict__ tab_start,
    uint32_t* __restrict__ tab_end, const uint32_t* __restrict__ range_off, float neg_alpha,
    uint32_t* __restrict__ msg_idx, float* __restrict__ msg_val) {
  const uint32_t lane = lane_id();
  const uint64_t c0 = (uint64_t)r * kAggWidth;
  const uint64_t c1 = min(c0 + (uint64_t)kAggWidth, d);
  if (lane < kAggWidth / 32) L.touched[lane] = 0;
  wave_lds_sync();
  uint32_t fresh = 0;
  for (uint32_t q0 = 0; q0 < N; q0 += kWave) {
    const uint32_t nq = min((uint32_t)kWave, N - q0);
    // where each worker of the tile enters and leaves the range
    uint32_t lo = 0, n = 0;
    if (lane < nq) {
      if (tab_start != nullptr) {
        const uint64_t at = (uint64_t)r * N + q0 + lane;
        const bool ready = q0 == 0 && pf.valid;
        const uint32_t lo_down = ready ? pf.lo : tab_start[at];   // K_up - first pair, 0 = none
        const uint32_t hi = ready ? pf.hi : tab_end[at];
        lo = K_up - min(lo_down, K_up);
        n = (lo_down != 0 && hi > lo && hi <= K_up) ? hi - lo : 0u;
        if (MODE != 1 && (hi | lo_down)) {                   // leave the table clear
          tab_start[at] = 0;
          tab_end[at] = 0;
        }
      } else {
        const uint32_t* row = up_idx + (uint64_t)(q0 + lane) * K_up;
        lo = lower_bound_u32(row, K_up, (uint32_t)c0);
        n = lower_bound_u32(row, K_up, (uint32_t)c1) - lo;   // c1 <= d < 2^32
      }
      L.p[lane] = p[q0 + lane];
    }
    if (q0 == 0) {                                           // the next range's first tile
      pf.valid = tab_start != nullptr && r_next != kAggNoRange;
      if (pf.valid && lane < nq) {
        const uint64_t at = (uint64_t)r_next * N + lane;
        pf.lo = tab_start[at];
        pf.hi = tab_end[at];
      }
    }
    const uint32_t incl = wave_inclusive_scan(n);
    const uint32_t total = __shfl(incl, kWave - 1, kWave);
    if (total == 0) continue;
    L.lo[lane] = lo;
    L.pref[lane] = incl - n;
    if (lane == kWave - 1) L.pref[kWave] = total;
    wave_lds_sync();
    for (uint32_t e0 = 0; e0 < total; e0 += kAggStage) {
      const uint32_t ne = min(kAggStage, total - e0);        // pairs in the stage
      // 1. fetch the stage's pairs into registers: lane l holds pairs l, l + 64, ... of the
      // stage (independent loads, all issued before the first is used)
      uint32_t rel[kAggRounds];            // coordinate - c0, or kAggNoRel
      float val[kAggRounds], pw[kAggRounds];
      {
        uint32_t pi[kAggRounds], pa[kAggRounds];
#pragma unroll
        for (uint32_t it = 0; it < kAggRounds; ++it) {
          const uint32_t k = it * kWave + lane;
          pi[it] = 0xFFFFFFFFu;
          pa[it] = 0;
          val[it] = 0.0f;
          if (k < ne) {
            const uint32_t e = e0 + k;
            uint32_t a = 0;                                  // the last worker with pref <= e
#pragma unroll
            for (uint32_t st = kWave / 2; st > 0; st >>= 1)
              if (L.pref[a + st] <= e) a += st;
            const uint64_t src = (uint64_t)(q0 + a) * K_up + L.lo[a] + (e - L.pref[a]);
            pi[it] = up_idx[src];
            if (MODE != 1) val[it] = up_val[src];
            pa[it] = a;
          }
        }
#pragma unroll
        for (uint32_t it = 0; it < kAggRounds; ++it) {
          const uint32_t i = pi[it];
          // inside the range for sorted input (never for the slots past the stage's end)
          rel[it] = (i >= c0 && i < c1) ? i - (uint32_t)c0 : kAggNoRel;
          pw[it] = MODE != 1 ? L.p[pa[it]] : 0.0f;
        }
      }
      // 2. first touches fetch the start value (the loads of all rounds are in flight
      // together; the values go to the accumulator after the last round); depth of every pair
      const uint32_t rounds = (ne + kWave - 1) / kWave;
      float sv[kAggRounds];
      bool first[kAggRounds];
      uint32_t depth[kAggRounds];
      const uint64_t below = lanes_below();
#pragma unroll
      for (uint32_t it = 0; it < kAggRounds; ++it) {
        first[it] = false;
        sv[it] = 0.0f;
        depth[it] = 0;
        if (it >= rounds) continue;                          // wave-uniform
        const uint32_t rl = rel[it];
        const bool valid = rl != kAggNoRel;
        uint32_t before = 0;
        if (valid) {
          const uint32_t bit = 1u << (rl & 31);
          const uint32_t old = atomicOr(&L.touched[rl >> 5], bit);
          if (!(old & bit)) {                                // first touch: start value
            first[it] = true;
            if (MODE == 0) sv[it] = dense[c0 + rl];
            ++fresh;
          }
          if (MODE != 1) before = seen_byte(L, rl);
        }
        if (MODE != 1) {
          wave_lds_sync();
          if (valid) atomicAdd(&L.seen[rl >> 2], 1u << (8 * (rl & 3)));
          wave_lds_sync();
          const uint32_t here = valid ? seen_byte(L, rl) - before : 0u;   // of this round
          // rank among the lanes of this round on the same coordinate: one turn of the loop
          // per coordinate that several lanes share (none for uncorrelated workers)
          uint64_t shared = __ballot(here > 1);
          uint32_t rank = 0;
          while (shared) {
            const int j = __ffsll((unsigned long long)shared) - 1;
            const uint32_t rel_j = (uint32_t)__builtin_amdgcn_readlane((int)rl, j);
            const bool same = valid && rl == rel_j;
            const uint64_t grp = __ballot(same);
            if (same) rank = (uint32_t)__popcll(grp & below);
            shared &= ~grp;
          }
          // < 64 when no worker names a coordinate twice; clamped for lists that do
          depth[it] = min(before + rank, (uint32_t)kWave - 1);
        }
      }
      if (MODE != 1) {
        // start values in place, the stage's counts cleaned for the next stage
#pragma unroll
        for (uint32_t it = 0; it < kAggRounds; ++it) {
          if (first[it]) L.acc[rel[it]] = sv[it];            // MODE 2: +0
          if (rel[it] != kAggNoRel) L.seen[rel[it] >> 2] = 0;
        }
        wave_lds_sync();
        // 3. apply, depth by depth: pairs of one depth name distinct coordinates
        for (uint32_t l = 0;; ++l) {
          bool more = false;
#pragma unroll
          for (uint32_t it = 0; it < kAggRounds; ++it) {
            if (rel[it] == kAggNoRel) continue;
            if (depth[it] == l) L.acc[rel[it]] = __fmaf_rn(pw[it], val[it], L.acc[rel[it]]);
            more |= depth[it] > l;
          }
          wave_lds_sync();                                   // the next depth may name the same i
          if (__ballot(more) == 0) break;
        }
      }
    }
  }
  if (MODE == 0) {
    // write the touched coordinates back: a lane takes half a bitmap word
    static_assert(kAggWidth / 16 == kWave, "half a bitmap word per lane");
    uint32_t bits = (L.touched[lane >> 1] >> (16 * (lane & 1))) & 0xFFFFu;
    while (bits) {
      const uint32_t t = __ffs(bits) - 1;
      bits &= bits - 1;
      const uint32_t rel = lane * 16 + t;
      dense[c0 + rel] = L.acc[rel];
    }
  }
  if (MODE == 2) {
    // ordered message: rank of a coordinate = set bits below it in the range's bitmap
    const uint32_t word = lane < kAggWidth / 32 ? L.touched[lane] : 0u;
    const uint32_t pc = __popc(word);
    uint32_t pos = range_off[r] + wave_inclusive_scan(pc) - pc;
    uint32_t bits = word;
    while (bits) {
      const uint32_t t = __ffs(bits) - 1;
      bits &= bits - 1;
      const uint32_t rel = lane * 32 + t;
      const float gt = L.acc[rel];
      if (msg_idx != nullptr) {
        msg_idx[pos] = (uint32_t)c0 + rel;
        msg_val[pos] = gt;
      }
      if (dense != nullptr) dense[c0 + rel] = __fmaf_rn(neg_alpha, gt, dense[c0 + rel]);
      ++pos;
    }
  }
  wave_lds_sync();
  return wave_sum(fresh);
}

// Wave g of the grid takes the ranges g, g + W, g + 2W, ... (W = waves in the grid), so that
// a cluster of busy ranges spreads over the whole chip; it reads the flags of 64 of its
// ranges at a time and visits those that are raised.  any == nullptr: every range is visited.
// MODE 0: nnz_out (nullable) gets one partial sum of distinct coordinates per wave.
// MODE 1: nnz_out gets the count of every range.
template <int MODE>
__global__ __launch_bounds__(kAggBlock) void k_aggregate(
    const uint32_t* __restrict__ up_idx, const float* __restrict__ up_val,
    const float* __restrict__ p, uint32_t N, uint32_t K_up, float* __restrict__ dense,
    uint64_t d, uint32_t ranges, uint32_t* __restrict__ nnz_out, uint32_t* __restrict__ tab_start,
    uint32_t* __restrict__ tab_end, uint32_t* __restrict__ any,
    const uint32_t* __restrict__ range_off, float neg_alpha, uint32_t* __restrict__ msg_idx,
    float* __restrict__ msg_val) {
  __shared__ AggWaveLds lds[kAggWaves];
  AggWaveLds& L = lds[threadIdx.x / kWave];
  const uint32_t lane = lane_id();
  const uint32_t g = blockIdx.x * kAggWaves + threadIdx.x / kWave;
  const uint32_t W = gridDim.x * kAggWaves;
  for (uint32_t i = lane; i < kAggWidth / 4; i += kWave) L.seen[i] = 0;   // every stage cleans up
  uint32_t nnz = 0;
  AggPrefetch pf;
  pf.lo = 0;
  pf.hi = 0;
  pf.valid = false;
  for (uint64_t r0 = g; r0 < ranges; r0 += (uint64_t)W * kWave) {
    const uint64_t mine = r0 + (uint64_t)lane * W;
    bool live = mine < ranges;
    if (live && any != nullptr) {
      live = any[mine] != 0;
      if (live && MODE != 1) any[mine] = 0;                  // leave the flags clear
    }
    if (MODE == 1 && mine < ranges && !live) nnz_out[mine] = 0;
    uint64_t todo = __ballot(live);
    while (todo) {
      const uint32_t src = (uint32_t)__ffsll((unsigned long long)todo) - 1;
      todo &= todo - 1;
      const uint32_t r = (uint32_t)(r0 + (uint64_t)src * W);
      // the wave's next raised range of this batch of 64, if any
      const uint32_t r_next =
          todo ? (uint32_t)(r0 + (uint64_t)((uint32_t)__ffsll((unsigned long long)todo) - 1) * W)
               : kAggNoRange;
      const uint32_t cnt = aggregate_range<MODE>(L, r, r_next, pf, up_idx, up_val, p, N, K_up,
                                                 dense, d,
                                                 tab_start, tab_end, range_off, neg_alpha,
                                                 msg_idx, msg_val);
      if (MODE == 1 && lane == 0) nnz_out[r] = cnt;
      nnz += cnt;
    }
  }
  if (MODE == 0 && nnz_out != nullptr && lane == 0) nnz_out[g] = nnz;
}

// Exclusive scan of the per-range counts (one block of 16 waves); *total_out receives the
// sum.  Each wave owns a contiguous segment (a multiple of 256 counts) and goes through it
// 256 counts at a time, four per lane from one 16-byte load: first for the segment's sum,
// then, from the sum of the segments before it, for the offsets.
__global__ __launch_bounds__(1024) void k_scan_ranges(const uint32_t* __restrict__ cnt,
                                                      uint32_t* __restrict__ off, uint32_t n,
                                                      uint32_t* __restrict__ total_out) {
  constexpr uint32_t kWaves = 1024 / kWave, kStep = kWave * 4;
  __shared__ uint32_t s_tot[kWaves];
  const uint32_t w = threadIdx.x / kWave, lane = lane_id();
  const uint32_t seg = ((n + kWaves - 1) / kWaves + kStep - 1) / kStep * kStep;
  const uint64_t b = (uint64_t)w * seg;
  const uint64_t e = min(b + seg, (uint64_t)n);
  auto load4 = [&](uint64_t i, uint32_t (&v)[4]) {
    if (i + 4 <= e) {
      const uint4 q = *reinterpret_cast<const uint4*>(cnt + i);
      v[0] = q.x, v[1] = q.y, v[2] = q.z, v[3] = q.w;
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) v[j] = i + j < e ? cnt[i + j] : 0u;
    }
  };
  uint32_t sum = 0;
  for (uint64_t i = b + lane * 4; i < e; i += kStep) {
    uint32_t v[4];
    load4(i, v);
    sum += v[0] + v[1] + v[2] + v[3];
  }
  sum = wave_sum(sum);
  if (lane == 0) s_tot[w] = sum;
  __syncthreads();
  uint32_t run = 0, total = 0;
  for (uint32_t i = 0; i < kWaves; ++i) {
    const uint32_t t = s_tot[i];
    if (i < w) run += t;
    total += t;
  }
  for (uint64_t i0 = b; i0 < e; i0 += kStep) {
    const uint64_t i = i0 + lane * 4;
    uint32_t v[4];
    load4(i, v);
    const uint32_t mine = v[0] + v[1] + v[2] + v[3];
    const uint32_t incl = wave_inclusive_scan(mine);
    uint32_t at = run + incl - mine;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (i + j < e) off[i + j] = at;
      at += v[j];
    }
    run += __shfl(incl, kWave - 1, kWave);
  }
  if (threadIdx.x == 0 && total_out != nullptr) *total_out = total;
}

// Sum of the per-range counts of distinct coordinates: one block.
__global__ __launch_bounds__(1024) void k_sum_ranges(const uint32_t* __restrict__ v, uint32_t n,
                                                     uint32_t* __restrict__ out) {
  __shared__ uint32_t lds[1024 / kWave + 1];
  uint32_t s = 0;
  for (uint32_t i = threadIdx.x; i < n; i += blockDim.x) s += v[i];
  uint32_t total;
  (void)block_exclusive_scan(s, lds, &total);
  if (threadIdx.x == 0) *out = total;
}

__global__ void k_update(const uint32_t* __restrict__ idx, const float* __restrict__ val,
                         uint32_t K, float neg_alpha, float* __restrict__ w, uint64_t d) {
  const uint32_t j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j < K) {
    const uint32_t i = idx[j];
    if (i < d) w[i] = __fmaf_rn(neg_alpha, val[j], w[i]);
  }
}

}  // namespace

uint32_t aggregate_ranges(uint64_t d) { return (uint32_t)((d + kAggWidth - 1) / kAggWidth); }

namespace {
// About four ranges to three waves: a wave with a second range fetches its table entries
// while it works on the first, and more waves than that leave each with no second range
// (measured per launch at 10.9 / 25 / 107 thousand ranges: 30.7 / 52 / 25 us, against
// 34 / 55 / 28 us with a wave per range or with three ranges per wave).
// (Up to the 6144 waves the chip holds at once, a wave per range: 5.8 against 8.2 us at 1024.)
uint32_t agg_blocks(uint32_t ranges) {
  uint32_t b = ranges <= 6144u ? (ranges + kAggWaves - 1) / kAggWaves
                               : (uint32_t)(((uint64_t)ranges * 3 + 15) / 16);
  if (b < 1) b = 1;
  return b > kAggMaxBlocks ? kAggMaxBlocks : b;
}
}  // namespace

uint32_t aggregate_scratch_words(uint64_t d) {
  const uint32_t ranges = aggregate_ranges(d);
  const uint32_t waves = agg_blocks(ranges) * kAggWaves;
  return ranges > waves ? ranges : waves;
}

hipError_t aggregate(hipStream_t s, const uint32_t* up_idx, const float* up_val, const float* p,
                     uint32_t N, uint32_t K_up, float* delta, uint64_t d, uint32_t* union_nnz,
                     const AggScratch& sc, bool ranges_ready) {
  if (K_up == 0) {
    if (union_nnz != nullptr) return fill_u32(s, union_nnz, 1, 0);
    return hipSuccess;
  }
  const uint32_t ranges = aggregate_ranges(d);
  const uint32_t blocks = agg_blocks(ranges);
  uint32_t* any = sc.tab_start != nullptr ? sc.any : nullptr;
  if (sc.tab_start != nullptr && !ranges_ready) {
    k_range_bounds<<<dim3((K_up + 255) / 256, N), dim3(256), 0, s>>>(
        up_idx, N, K_up, d, sc.tab_start, sc.tab_end, sc.any);
    hipError_t e0 = hipGetLastError();
    if (e0 != hipSuccess) return e0;
  }
  k_aggregate<0><<<dim3(blocks), dim3(kAggBlock), 0, s>>>(
      up_idx, up_val, p, N, K_up, delta, d, ranges, union_nnz != nullptr ? sc.cnt : nullptr,
      sc.tab_start, sc.tab_end, any, nullptr, 0.0f, nullptr, nullptr);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || union_nnz == nullptr) return e;
  k_sum_ranges<<<dim3(1), dim3(1024), 0, s>>>(sc.cnt, blocks * kAggWaves, union_nnz);
  return hipGetLastError();
}

hipError_t aggregate_update_unidirectional(hipStream_t s, const uint32_t* up_idx,
                                           const float* up_val, const float* p, uint32_t N,
                                           uint32_t K_up, float* w, uint64_t d, float alpha_out,
                                           uint32_t* msg_idx, float* msg_val, uint32_t* msg_count,
                                           const AggScratch& sc, bool ranges_ready) {
  if (K_up == 0) {
    if (msg_count != nullptr) return fill_u32(s, msg_count, 1, 0);
    return hipSuccess;
  }
  const uint32_t ranges = aggregate_ranges(d);
  const uint32_t blocks = agg_blocks(ranges);
  uint32_t* any = sc.tab_start != nullptr ? sc.any : nullptr;
  if (sc.tab_start != nullptr && !ranges_ready) {
    k_range_bounds<<<dim3((K_up + 255) / 256, N), dim3(256), 0, s>>>(
        up_idx, N, K_up, d, sc.tab_start, sc.tab_end, sc.any);
    hipError_t e0 = hipGetLastError();
    if (e0 != hipSuccess) return e0;
  }
  k_aggregate<1><<<dim3(blocks), dim3(kAggBlock), 0, s>>>(
      up_idx, up_val, p, N, K_up, nullptr, d, ranges, sc.cnt, sc.tab_start, sc.tab_end, any,
      nullptr, 0.0f, nullptr, nullptr);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  k_scan_ranges<<<dim3(1), dim3(1024), 0, s>>>(sc.cnt, sc.off, ranges, msg_count);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  k_aggregate<2><<<dim3(blocks), dim3(kAggBlock), 0, s>>>(
      up_idx, up_val, p, N, K_up, w, d, ranges, nullptr, sc.tab_start, sc.tab_end, any, sc.off,
      -alpha_out, msg_idx, msg_val);
  return hipGetLastError();
}

hipError_t sgd_update(hipStream_t s, const uint32_t* idx, const float* val, uint32_t K,
                      float alpha_out, float* w, uint64_t d) {
  if (K == 0) return hipSuccess;
  k_update<<<dim3((K + 255) / 256), dim3(256), 0, s>>>(idx, val, K, -alpha_out, w, d);
  return hipGetLastError();
}

}  // namespace bts
