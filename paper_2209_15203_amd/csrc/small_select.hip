// Top_K select for short rows: one 1024-thread workgroup per row, one launch.
//
// Rows of up to 8192 coordinates (the toy example, small linear models) are bound by kernel
// launches on the multi-kernel paths.  Here a thread keeps
// its share of the row (coordinates t, t + 1024, ..., t + 7168) in registers: the row is read
// once (with the worker's error compensation a = eps + alpha g fused in and stored), the
// three digits of the radix select on the 31-bit magnitude key are histogrammed in LDS from
// the registers, and the ordered emission ranks the kept coordinates with ballots, a
// (slice, wave) count matrix in LDS and one workgroup scan.  Same results as the dense
// path: ascending indices, ties at the threshold to the lowest indices, +0 stored over the
// kept coordinates.

#include "bts_device.h"

namespace bts {

namespace {

constexpr int kRowBlock = 1024;
constexpr int kRowWaves = kRowBlock / kWave;
constexpr int kCopies = 8;
// Coordinates per thread.  One compute unit does all the work on a row, about 70
// instructions per coordinate over the passes, so beyond 8192 coordinates the multi-kernel
// dense path, which spreads a row over the chip, is the quicker one again (measured:
// 17 us against 30 us per select at d = 8192, 35 us against 30 us at d = 29034).
constexpr int kRowSlices = 8;

// A value behind a compiler barrier: a loop that derives its per-slice quantities from its
// own copy recomputes them (an add, a compare) instead of keeping E of them live in
// registers from an earlier loop.
__device__ __forceinline__ uint32_t opaque(uint32_t v) {
  asm volatile("" : "+v"(v));
  return v;
}

// E = coordinates per thread (the row has at most E * 1024).  Sizes for which float[E] is
// not a register-tuple type (8 is fine, 16 and 32 are not) compile without spills.
template <int E, bool FMA>
__global__ __launch_bounds__(kRowBlock) void k_row_select(
    const float* __restrict__ g, float* __restrict__ x, uint32_t d, uint32_t K, float alpha,
    uint32_t* __restrict__ out_idx, float* __restrict__ out_val, FusedUpdate upd) {
  // histogram of the current digit; the first digit (exponent and three mantissa bits: a
  // handful of busy bins) is spread over kCopies copies by lane, or the whole row would
  // serialise on a few LDS words of this one compute unit
  __shared__ uint32_t sh[kCopies * kBins0];
  __shared__ uint32_t cg[E * kRowWaves];             // per (slice, wave): keys above T
  __shared__ uint32_t ce[E * kRowWaves];             // per (slice, wave): keys equal to T
  __shared__ uint32_t lds[kRowWaves + 1];
  __shared__ uint32_t s_out[2];
  const uint32_t row = blockIdx.x, t = threadIdx.x, w = t / kWave;
  float* xr = x + (uint64_t)row * d;
  const float* gr = FMA ? g + (uint64_t)row * d : nullptr;
  float v[E];
  // up to 32 coordinates per thread (and array) in flight at a time
  constexpr int G = E < 32 ? E : 32;
#pragma unroll
  for (int k0 = 0; k0 < E; k0 += G) {
    const uint32_t tl = opaque(t);
    float gv[G];
#pragma unroll
    for (int k = k0; k < k0 + G; ++k) {
      const uint32_t i = (uint32_t)k * kRowBlock + tl;
      v[k] = 0.0f;
      gv[k - k0] = 0.0f;
      if (i < d) {
        v[k] = xr[i];
        if (FMA) gv[k - k0] = gr[i];
      }
    }
    if (FMA) {
#pragma unroll
      for (int k = k0; k < k0 + G; ++k) {
        const uint32_t i = (uint32_t)k * kRowBlock + tl;
        if (i < d) {
          v[k] = __fmaf_rn(alpha, gv[k - k0], v[k]);
          xr[i] = v[k];
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  // Slots past the end of the row hold +0, the smallest key there is, at indices above
  // every real one: with K <= d they change neither the K-th largest key nor which
  // coordinates are kept, so the loops below need no validity test.
  // Exact K-th largest key T and the tie quota r: 11 + 10 + 10 bits
  uint32_t prefix = 0, k_rem = K;
#pragma unroll
  for (int digit = 0; digit < 3; ++digit) {
    const int nb = digit == 0 ? kCopies * kBins0 : kBinsLo;
    for (int i = t; i < nb; i += kRowBlock) sh[i] = 0;
    uint32_t* mine = sh + (digit == 0 ? (t % kCopies) * kBins0 : 0);
    __syncthreads();
    uint32_t bin0 = 0;        // counted per lane: a sparse row would serialise on one LDS word
    const uint32_t mh = opaque(0x7FFFFFFFu);      // per-loop copy of the key mask (see opaque)
#pragma unroll
    for (int k = 0; k < E; ++k) {
      const uint32_t key = __float_as_uint(v[k]) & mh;
      uint32_t bin;
      bool hit = true;
      if (digit == 0) {
        bin = key >> 20;
      } else if (digit == 1) {
        bin = (key >> 10) & 1023u;
        hit = (key >> 20) == prefix;
      } else {
        bin = key & 1023u;
        hit = (key >> 10) == prefix;
      }
      if (hit) {
        if (bin == 0) ++bin0; else atomicAdd(&mine[bin], 1u);
      }
      __builtin_amdgcn_sched_barrier(0);     // keep the slices apart: short live ranges
    }
    if (bin0) atomicAdd(&mine[0], bin0);
    __syncthreads();
    uint32_t above;
    const uint32_t b = digit == 0
                           ? resolve_bins<kBins0, kRowBlock>(sh, kCopies, kBins0, k_rem, lds, s_out,
                                                             &above)
                           : resolve_bins<kBinsLo, kRowBlock>(sh, 1, 0, k_rem, lds, s_out, &above);
    prefix = digit == 0 ? b : ((prefix << 10) | b);
    k_rem -= above;
  }
  const uint32_t T = prefix, r = k_rem;
  // ordered emission: slice k of wave w holds the indices k * 1024 + w * 64 + lane, so the
  // (slice, wave) matrix in row-major order is the index order
  const uint32_t mc = opaque(0x7FFFFFFFu);
#pragma unroll
  for (int k = 0; k < E; ++k) {
    const uint32_t key = __float_as_uint(v[k]) & mc;
    const uint64_t bg = __ballot(key > T), be = __ballot(key == T);
    if (lane_id() == 0) {
      cg[k * kRowWaves + w] = __popcll(bg);
      ce[k * kRowWaves + w] = __popcll(be);
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  __syncthreads();
  {
    const bool mine = t < (uint32_t)(E * kRowWaves);
    const uint32_t a = mine ? cg[t] : 0u, b = mine ? ce[t] : 0u;
    uint32_t total;
    const uint32_t ea = block_exclusive_scan(a, lds, &total);
    const uint32_t eb = block_exclusive_scan(b, lds, &total);
    if (mine) {
      cg[t] = ea;
      ce[t] = eb;
    }
  }
  __syncthreads();
  uint32_t* oi = out_idx + (uint64_t)row * K;
  float* ov = out_val + (uint64_t)row * K;
  const uint64_t below = lanes_below();
  const uint32_t me = opaque(0x7FFFFFFFu);
#pragma unroll
  for (int k = 0; k < E; ++k) {
    const uint32_t key = __float_as_uint(v[k]) & me;
    const bool is_gt = key > T, is_eq = key == T;
    const uint64_t bg = __ballot(is_gt), be = __ballot(is_eq);
    if (bg == 0 && be == 0) continue;                        // uniform over the wave
    const uint32_t n_gt = cg[k * kRowWaves + w] + __popcll(bg & below);   // greater before me
    const uint32_t n_eq = ce[k * kRowWaves + w] + __popcll(be & below);   // equal before me
    if (is_gt || (is_eq && n_eq < r)) {
      const uint32_t pos = n_gt + min(n_eq, r);
      const uint32_t i = (uint32_t)k * kRowBlock + t;
      if (pos < K && i < d) {
        oi[pos] = i;
        ov[pos] = v[k];
        xr[i] = 0.0f;
        if (upd.w != nullptr) upd.w[i] = __fmaf_rn(upd.neg_alpha, v[k], upd.w[i]);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }
}

}  // namespace

bool row_select_fits(uint64_t d) { return d <= (uint64_t)kRowSlices * kRowBlock; }

// Same contract as dense_select without the row mask; d must satisfy row_select_fits.
hipError_t row_select(hipStream_t s, const float* g, float* x, uint32_t rows, uint64_t d,
                      uint32_t K, float alpha, uint32_t* out_idx, float* out_val,
                      hipEvent_t ev0, hipEvent_t ev1, FusedUpdate upd) {
  if (!row_select_fits(d)) return hipErrorInvalidValue;
  if (upd.w != nullptr && rows != 1) return hipErrorInvalidValue;
  const dim3 grid(rows), block(kRowBlock);
  const uint32_t d32 = (uint32_t)d;
  if (ev0) (void)hipEventRecord(ev0, s);
#define BTS_ROW(E)                                                                        \
  do {                                                                                    \
    if (g != nullptr)                                                                     \
      k_row_select<E, true><<<grid, block, 0, s>>>(g, x, d32, K, alpha, out_idx, out_val,   \
                                                   upd);                                  \
    else                                                                                  \
      k_row_select<E, false><<<grid, block, 0, s>>>(nullptr, x, d32, K, 0.0f, out_idx,      \
                                                    out_val, upd);                        \
  } while (0)
  BTS_ROW(kRowSlices);
#undef BTS_ROW
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (ev1) (void)hipEventRecord(ev1, s);
  return hipSuccess;
}

}  // namespace bts
