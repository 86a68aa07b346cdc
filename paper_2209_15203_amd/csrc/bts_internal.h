// Internal declarations shared by the HIP translation units of libbts (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bts {

constexpr int kWave = 64;                 // CDNA wavefront
constexpr int kBlock = 256;               // threads per workgroup in the dense passes
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kUnroll = 2;                // float4 loads in flight per lane and array
constexpr int kStreamBlock = 128;         // threads per workgroup of the dominant kernel
constexpr int kStreamWaves = kStreamBlock / kWave;
// A wave owns kWaveChunk consecutive coordinates (absolute, 16-byte aligned offsets).
constexpr uint32_t kWaveChunk = kWave * 4 * kUnroll;   
constexpr int kBins0 = 2048;              // first digit: key bits 30..20
constexpr int kBinsLo = 1024;             // second and third digit: bits 19..10, 9..0

// Per-row state of the exact radix select on the 31-bit magnitude key.
struct SelState {
  uint32_t T;        // exact K-th largest key
  uint32_t r;        // how many coordinates with key == T are kept (lowest indices first)
};

// Model update line of Algorithm 2 fused into the emission of a ONE-ROW select (the server's
// compression): the lane that writes the pair (i, v) of the message also does
// w[i] = fma(neg_alpha, v, w[i]).  w == nullptr: no update.
// after (single-pass select only): the update is not done by the emitting lanes but from the
// finished message, one pair per thread, in the select's last launch (the emission of the
// gated dense redo, whose workgroups are idle for a row that needs no redo; a row that does
// is updated by the redo's emitting lanes).
struct FusedUpdate {
  float* w;
  float neg_alpha;
  bool after;
};

constexpr uint32_t kAggWidth = 1024;   // coordinates per range of the aggregation

// The aggregation's range tables (ranges x N entries each, all zero between calls), filled
// for the worker rows by the select's last kernel so that the aggregation needs no pass of
// its own over the messages (null: not wanted).  For worker q and range r, tab_start holds
// K - (the first pair of q's message inside r), tab_end one past the last such pair; zero =
// the message does not enter the range.  (The start counts down from K so that both entries
// can be built with atomic maxima on zeroed memory where pairs arrive in no order.)
struct MidRanges {
  uint32_t* tab_start;
  uint32_t* tab_end;
  uint32_t* any;           // per range: somebody names it
};

// Rows that a gated kernel must process (null pointer = all rows).
using RowMask = const uint32_t*;

struct DenseScratch {
  uint32_t* hist;     // rows x dense_row_hist_words(): three digit histograms, zero between calls
  bool* dirty;        // host flag: a call failed half way, clear the histograms first
  uint32_t rows;      // rows the scratch was sized for
  SelState* state;    // rows
  uint2* cnt;         // rows x nwc: per wave chunk, the counts of key > T (x), key == T (y)
  uint2* block_sums;  // rows x dense_max_blocks(1): the same per block's share of chunks
  uint32_t nwc;       // wave-chunks per row (upper bound, same for every row)
};
constexpr uint32_t kDenseMaxGx = 512;     // most blocks per row of a dense pass (a lone row)
uint32_t dense_max_blocks(uint32_t rows);  // most blocks per row when `rows` rows are selected
uint32_t dense_row_hist_words();

// ---- dense exact select (handles any input, any K in 1..d) ----------------------------
// x: rows x d (row stride d).  If g != nullptr the first pass computes
// x = fma(alpha, g, x) and stores it (the worker's error compensation) while it builds
// the first histogram.  On return (stream order) idx/val hold K pairs per row in
// ascending index order and x holds +0 at those positions.
hipError_t dense_select(hipStream_t s, const DenseScratch& sc, const float* g, float* x,
                        uint32_t rows, uint64_t d, uint32_t K, float alpha, uint32_t* out_idx,
                        float* out_val, RowMask need, bool first_pass_done,
                        hipEvent_t ev0, hipEvent_t ev1, FusedUpdate upd = FusedUpdate{nullptr, 0.0f});

// The pieces of dense_select for a caller that runs the first four kernels (three digit
// histograms and the per-chunk counts, see dense_bodies.h) inside launches of its own:
// dense_begin before them, dense_finish (the emission) after them.
struct DensePlan {
  uint32_t nwc;        // wave chunks per row
  uint32_t gx;         // blocks in x of the looping kernels
  bool streaming;      // read x past the caches
};
DensePlan dense_plan(const DenseScratch& sc, uint32_t rows, uint64_t d);
hipError_t dense_begin(hipStream_t s, const DenseScratch& sc);
// heal (all null = none): the single-pass select's bounds for its next call, which the
// emission sets from the exact threshold for the rows it redoes (see cand_finish_body).
struct NextBounds {
  uint32_t* lower_key;
  uint32_t* upper_key;     // written only if early_zero
  uint32_t* prev_T;
  bool early_zero;
  uint32_t* redone;        // pinned host word (device address): set to 1 when a row is redone
};
hipError_t dense_finish(hipStream_t s, const DenseScratch& sc, const DensePlan& pl, float* x,
                        uint32_t rows, uint64_t d, uint32_t K, uint32_t* out_idx,
                        float* out_val, RowMask need, FusedUpdate upd,
                        NextBounds heal = NextBounds{nullptr, nullptr, nullptr, false, nullptr},
                        MidRanges ranges = MidRanges{nullptr, nullptr, nullptr});
// (upd.after: rows that need no redo are updated from their finished message instead;
// ranges, with a row mask only: the emission's launch also fills the range tables, for the
// rows that need no redo from their finished messages, for the others pair by pair)

// x = fma(alpha, g, x) over rows x d and nothing else (K == 0).
hipError_t axpy_only(hipStream_t s, const float* g, float* x, uint32_t rows, uint64_t d,
                     float alpha, hipEvent_t ev0, hipEvent_t ev1);

// ---- short rows: one workgroup per row, one launch (d <= 8192) -------------------------------
bool row_select_fits(uint64_t d);
// Same contract as dense_select without the row mask.
hipError_t row_select(hipStream_t s, const float* g, float* x, uint32_t rows, uint64_t d,
                      uint32_t K, float alpha, uint32_t* out_idx, float* out_val,
                      hipEvent_t ev0, hipEvent_t ev1, FusedUpdate upd = FusedUpdate{nullptr, 0.0f});

// ---- speculative single-pass select (exact; flags rows it cannot finish) -----------------
struct FastPlan {
  bool enabled;            // false: shape is served by the dense path alone (no scratch)
  bool preferred;          // the default choice for this shape
  uint32_t stride;         // every stride-th 256-coordinate slice is sampled
  uint32_t target;         // sampled coordinates wanted at or above the lower bound
  uint32_t target_u;       // K in sampled coordinates: aims the bound of the early zeroing
  uint32_t rank_next;      // the next call's lower bound aims at this rank of the row (> K)
  uint32_t cap;            // capacity of one candidate list
  uint32_t stream_waves_per_simd;   // occupancy the dense pass is held to (3, 5 or 6)
  uint32_t ntiles;         // directory tiles (64 wave chunks) per row
  uint32_t nwc_pad;        // directory entries per row (ntiles * 64)
};

struct FastScratch {
  uint32_t* sample_hist;   // rows x 8192 (zero between calls)
  uint32_t* lower_key;     // rows
  uint32_t* upper_key;     // rows: from which key on the dense pass stores +0 (see capture_chunk)
  uint32_t* prev_T;        // rows: the threshold key the previous call found (0 = none)
  uint32_t* cand_cnt;      // rows x lists, one counter per 128-byte line
  uint2* cand;             // rows x lists x cap (index, value bits)
  uint32_t* hist;          // rows x fast_hist_words() partial histograms
  void* sel;               // rows x fast_sel_bytes()
  uint32_t* need;          // rows: nonzero = the dense path must redo this row
  uint2* dir;              // rows x nwc_pad (zero between calls): per wave chunk the start
                           // of its run in its list and the run's length
  void* tile_cnt;          // rows x ntiles 64-bit words (rewritten by every call)
  bool* dirty;             // host flag: a call failed half way, clear directory and sample first
  // host side of the bounds handed from call to call
  struct HostState {
    uint32_t calls;        // calls since the bounds were last sampled from scratch
    uint32_t cold_left;    // calls that still have to sample (after rows were redone)
    uint32_t backoff;      // how many calls sampled after the last redo (doubles, up to 64)
    uint32_t quiet;        // calls since a redo was last seen
  };
  HostState* host;
  // pinned host word that the redo's emission sets when it redoes a row: the host looks at it,
  // without waiting for anything, at the start of a later call (redone_dev: its device address)
  volatile uint32_t* redone_host;
  uint32_t* redone_dev;
  uint32_t rows;           // rows the scratch was sized for
  // diagnostics only (null otherwise): fp64 sums of squares of what stays behind in the row,
  // per wave chunk (coordinates not captured) and per directory tile (captured, not kept)
  double* energy;          // rows x nwc_pad; slots of chunks outside the row stay zero
  double* tile_energy;     // rows x ntiles
};

FastPlan fast_plan(uint32_t rows, uint64_t d, uint32_t K);
size_t fast_sel_bytes();
uint32_t fast_sublists();
uint32_t fast_counter_stride();
size_t fast_hist_words();
// Same contract as dense_select.  Rows that the single pass cannot finish are flagged and
// redone by the dense path inside this call (its first four kernels share launches with the
// tail of the single-pass select, the rest follows); x holds fma(alpha, g, x) for every row
// before the redo starts.
hipError_t fast_select(hipStream_t s, const FastScratch& sc, const FastPlan& pl, const float* g,
                       float* x, uint32_t rows, uint64_t d, uint32_t K, float alpha,
                       uint32_t* out_idx, float* out_val, hipEvent_t ev0, hipEvent_t ev1,
                       const DenseScratch& dense, bool energy,
                       FusedUpdate upd = FusedUpdate{nullptr, 0.0f},
                       MidRanges ranges = MidRanges{nullptr, nullptr, nullptr});

// ---- middling rows, small K: three launches, no fallback (mid_select.hip) ------------------
struct MidPlan {
  bool enabled;            // false: the shape is served by the other paths
  bool preferred;          // the default choice for this shape
  uint32_t cap;            // capacity of one candidate list (cannot overflow)
  uint32_t ntiles;         // directory tiles (64 wave chunks) per row
  uint32_t nwc_pad;        // directory entries per row (ntiles * 64)
  uint32_t gx;             // blocks per row of the capture pass (256 threads)
  uint32_t gx_hist;        // blocks per row of the histogram pass (1024 threads)
};
struct MidScratch {
  uint32_t* hist;          // rows x mid_hist_words() (zero between calls)
  void* bound;             // rows x mid_bound_bytes(): lower bound and keys above it
  uint32_t* cand_cnt;      // rows x lists, one counter per 128-byte line (zero between calls)
  uint2* cand;             // rows x lists x cap (index, value bits)
  uint2* dir;              // rows x nwc_pad (zero between calls)
  bool* dirty;             // host flag: a call failed half way, clear the scratch first
  uint32_t rows;           // rows the scratch was sized for
};
MidPlan mid_plan(uint32_t rows, uint64_t d, uint32_t K);
size_t mid_bound_bytes();
uint32_t mid_hist_words();
// Same contract as dense_select without the row mask.
hipError_t mid_select(hipStream_t s, const MidScratch& sc, const MidPlan& pl, const float* g,
                      float* x, uint32_t rows, uint64_t d, uint32_t K, float alpha,
                      uint32_t* out_idx, float* out_val, hipEvent_t ev0, hipEvent_t ev1,
                      FusedUpdate upd, const MidRanges& ranges);

// ---- server side ------------------------------------------------------------------------
uint32_t aggregate_ranges(uint64_t d);
uint32_t aggregate_scratch_words(uint64_t d);
struct AggScratch {
  uint32_t* cnt;        // aggregate_scratch_words(d): per-range counts or per-wave partial sums
  uint32_t* off;        // aggregate_scratch_words(d): exclusive scan of the per-range counts
  uint32_t* tab_start;  // optional aggregate_ranges(d) x N tables (all zero between calls) that
  uint32_t* tab_end;    //   replace the per-range binary searches; null = search
  uint32_t* any;        // aggregate_ranges(d) flags (all zero between calls), used with the tables
};
// ranges_ready: the tables and flags of sc were already filled for these messages (by the
// select that wrote them).
hipError_t aggregate(hipStream_t s, const uint32_t* up_idx, const float* up_val, const float* p,
                     uint32_t N, uint32_t K_up, float* delta, uint64_t d, uint32_t* union_nnz,
                     const AggScratch& sc, bool ranges_ready = false);
// Algorithm 1's server and update in one: w -= alpha_out * sum_q p_q Top_K(a^q), the sum
// also returned as a sparse message (named coordinates ascending; msg_idx/msg_val nullable,
// room for N*K_up pairs; msg_count nullable).
hipError_t aggregate_update_unidirectional(hipStream_t s, const uint32_t* up_idx,
                                           const float* up_val, const float* p, uint32_t N,
                                           uint32_t K_up, float* w, uint64_t d, float alpha_out,
                                           uint32_t* msg_idx, float* msg_val, uint32_t* msg_count,
                                           const AggScratch& sc, bool ranges_ready = false);
// ---- per-step diagnostics (rho, rho_hat, 1 - gamma, nnz fraction) -------------------------
struct DiagScratch {
  float* u;          // d: sum_q p_q a^q
  float* v;          // d: delta_{t-1} + sum_q p_q a^q
  double* part;      // diag_part_doubles(N) partial sums
  uint32_t* a_idx;   // K_dn: Top_K(v)
  float* a_val;
  uint32_t* c_idx;   // K_up: Top_K(u)
  float* c_val;
  uint32_t* m_idx;   // N*K_up: sum_q p_q Top_K(a^q), sparse
  float* m_val;
  uint32_t* m_cnt;
};
size_t diag_part_doubles(uint32_t N);
// Residual energies of the worker rows as the single-pass select left them (null chunks:
// not available, every row is summed from eps).
struct RowEnergy {
  const double* chunks;    // rows x nwc_pad
  const double* tiles;     // rows x ntiles
  uint32_t nwc_pad, ntiles;
  const uint32_t* need;    // rows the select handed to the dense path: summed from eps
};
hipError_t diag_before_step(hipStream_t s, const DiagScratch& ds, const float* g,
                            const float* eps, const float* delta, const float* p, uint32_t N,
                            uint64_t d, float alpha);
// A single-pass select for one row of length d (null plan: the dense path does it).
struct OneRowSelect {
  const FastPlan* plan;
  const FastScratch* scratch;
};
hipError_t diag_after_step(hipStream_t s, const DiagScratch& ds, const DenseScratch& dense,
                           const float* eps, const float* delta, const float* p, uint32_t N,
                           uint64_t d, uint32_t K_up, uint32_t K_dn, float alpha,
                           const uint32_t* up_idx, const float* up_val, const uint32_t* dn_idx,
                           const float* dn_val, const AggScratch& agg, const RowEnergy& energy,
                           const OneRowSelect& sel_v, const OneRowSelect& sel_u, double* diag);

hipError_t sgd_update(hipStream_t s, const uint32_t* idx, const float* val, uint32_t K,
                      float alpha_out, float* w, uint64_t d);
hipError_t fill_u32(hipStream_t s, uint32_t* p, uint64_t n, uint32_t v);

}  // namespace bts
