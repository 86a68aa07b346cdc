// C ABI of libbts (see include/bts.h): argument checks, scratch ownership, and the order
// in which the kernels of one step of Algorithm 2 are queued.

#include "../../include/bts.h"
#include "../../include/bts_testing.h"

#include <new>
#include <vector>

#include "bts_internal.h"

using namespace bts;

struct bts_ctx {
  int32_t N;
  uint64_t d;
  uint32_t K_up, K_dn;
  hipStream_t stream;
  int device;
  int last_hip_error;
  DenseScratch dense;
  bool dense_dirty;
  bool fast_up_dirty, fast_dn_dirty;
  FastScratch::HostState fast_up_host, fast_dn_host, fast_diag_u_host, fast_diag_v_host;
  FastPlan plan_up, plan_dn;
  FastScratch fast_up, fast_dn;
  MidPlan mid_plan_up, mid_plan_dn;   // the three-launch select of middling rows with small K
  MidScratch mid_up, mid_dn;
  bool mid_up_dirty, mid_dn_dirty;
  FastPlan plan_diag_u;         // diagnostics: one row of length d with K_up (the select of
  FastScratch fast_diag_u;      //   sum_q p_q a^q); the one with K_dn follows plan_dn with a
  FastScratch fast_diag_v;      //   scratch of its own (a scratch hands its bounds from call
  bool fast_diag_u_dirty;       //   to call, so each sequence of vectors gets one)
  bool fast_diag_v_dirty;
  uint32_t* agg_ranges;         // per-range distinct-coordinate counts of the aggregation
  uint32_t* agg_offsets;        // their exclusive scan (unidirectional message placement)
  uint32_t *agg_start, *agg_end;  // range x worker entry/exit tables (null: binary search)
  uint32_t* agg_any;            // per-range "somebody names it" flags, used with the tables
  bool agg_tables_bad;          // a launch failed while the tables were in use: stop using them
  DiagScratch diag;             // allocated by bts_enable_diagnostics only
  bool diag_ready;
  std::vector<void*> owned;     // every device allocation of the context
  std::vector<void*> owned_host;   // every pinned host allocation of the context
  // timing of the dominant kernel
  bool profile;
  int path_mode;                // 0 = by shape, 1 = dense only, 2 = single-pass where possible,
                                // 3 = the three-launch select where possible
  std::vector<std::pair<hipEvent_t, hipEvent_t>> ev_pool;
  size_t ev_used;
};

namespace {

constexpr size_t kMaxProfileEvents = 4096;   // launches recorded between two bts_profile_read

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int fail_hip(bts_ctx* ctx, hipError_t e) {
  ctx->last_hip_error = (int)e;
  // the aggregation's tables are only clean if every launch that uses them went out
  ctx->agg_tables_bad = true;
  return BTS_EHIP;
}

AggScratch agg_scratch(const bts_ctx* ctx) {
  AggScratch a;
  a.cnt = ctx->agg_ranges;
  a.off = ctx->agg_offsets;
  const bool tables = !ctx->agg_tables_bad && ctx->agg_start != nullptr;
  a.tab_start = tables ? ctx->agg_start : nullptr;
  a.tab_end = tables ? ctx->agg_end : nullptr;
  a.any = tables ? ctx->agg_any : nullptr;
  return a;
}

// Zero-filled device allocation owned by the context.
template <typename T>
bool dev_alloc(bts_ctx* ctx, T** p, size_t count) {
  void* q = nullptr;
  const size_t bytes = count * sizeof(T) + 16;
  if (hipMalloc(&q, bytes) != hipSuccess) return false;
  ctx->owned.push_back(q);
  if (hipMemset(q, 0, bytes) != hipSuccess) return false;
  *p = reinterpret_cast<T*>(q);
  return true;
}

bool alloc_fast(bts_ctx* ctx, const FastPlan& pl, uint32_t rows, FastScratch* sc) {
  if (!pl.enabled) return true;
  uint8_t* sel = nullptr;
  uint64_t* sup = nullptr;
  bool ok = dev_alloc(ctx, &sc->sample_hist, (size_t)rows * 8192) &&
            dev_alloc(ctx, &sc->lower_key, rows) &&
            dev_alloc(ctx, &sc->upper_key, rows) &&
            dev_alloc(ctx, &sc->prev_T, rows) &&
            dev_alloc(ctx, &sc->cand_cnt, (size_t)rows * fast_sublists() * fast_counter_stride()) &&
            dev_alloc(ctx, &sc->cand, (size_t)rows * fast_sublists() * pl.cap) &&
            dev_alloc(ctx, &sc->hist, (size_t)rows * fast_hist_words()) &&
            dev_alloc(ctx, &sel, (size_t)rows * fast_sel_bytes()) &&
            dev_alloc(ctx, &sc->need, rows) &&
            dev_alloc(ctx, &sc->dir, (size_t)rows * pl.nwc_pad) &&
            dev_alloc(ctx, &sup, (size_t)rows * pl.ntiles);
  sc->sel = sel;
  sc->tile_cnt = sup;
  sc->rows = rows;
  // the pinned word through which a redo is reported to the host (see fast_select)
  sc->redone_host = nullptr;
  sc->redone_dev = nullptr;
  void* pinned = nullptr;
  if (ok && hipHostMalloc(&pinned, 64, hipHostMallocMapped) == hipSuccess) {
    ctx->owned_host.push_back(pinned);
    void* dev_ptr = nullptr;
    if (hipHostGetDevicePointer(&dev_ptr, pinned, 0) == hipSuccess) {
      *static_cast<volatile uint32_t*>(pinned) = 0;
      sc->redone_host = static_cast<volatile uint32_t*>(pinned);
      sc->redone_dev = static_cast<uint32_t*>(dev_ptr);
    }
  } else if (ok) {
    (void)hipGetLastError();          // without the word a redo is simply never reported
  }
  return ok;
}

bool alloc_mid(bts_ctx* ctx, const MidPlan& pl, uint32_t rows, MidScratch* sc) {
  if (!pl.enabled) return true;
  uint8_t* bound = nullptr;
  bool ok = dev_alloc(ctx, &sc->hist, (size_t)rows * mid_hist_words()) &&
            dev_alloc(ctx, &bound, (size_t)rows * mid_bound_bytes()) &&
            dev_alloc(ctx, &sc->cand_cnt, (size_t)rows * fast_sublists() * fast_counter_stride()) &&
            dev_alloc(ctx, &sc->cand, (size_t)rows * fast_sublists() * pl.cap) &&
            dev_alloc(ctx, &sc->dir, (size_t)rows * pl.nwc_pad);
  sc->bound = bound;
  sc->rows = rows;
  return ok;
}

// The entry/exit tables pay off when most ranges are empty for most workers; they are
// skipped (binary search instead) when they would be large.
bool alloc_agg_tables(bts_ctx* ctx) {
  const size_t words = (size_t)aggregate_ranges(ctx->d) * (size_t)ctx->N;
  if (ctx->K_up == 0 || words * 8 > (256ull << 20)) return true;
  return dev_alloc(ctx, &ctx->agg_start, words) && dev_alloc(ctx, &ctx->agg_end, words) &&
         dev_alloc(ctx, &ctx->agg_any, (size_t)aggregate_ranges(ctx->d));
}

void release(bts_ctx* ctx) {
  for (void* q : ctx->owned) (void)hipFree(q);
  for (void* q : ctx->owned_host) (void)hipHostFree(q);
  for (auto& pr : ctx->ev_pool) {
    (void)hipEventDestroy(pr.first);
    (void)hipEventDestroy(pr.second);
  }
  delete ctx;
}

// A pair of events for one launch of the dominant kernel, or nulls when not profiling.
void profile_events(bts_ctx* ctx, hipEvent_t* e0, hipEvent_t* e1) {
  *e0 = *e1 = nullptr;
  if (!ctx->profile) return;
  if (ctx->ev_used == kMaxProfileEvents) return;     // unread for too long: stop recording
  if (ctx->ev_used == ctx->ev_pool.size()) {
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess) return;
    if (hipEventCreate(&b) != hipSuccess) {
      (void)hipEventDestroy(a);
      return;
    }
    ctx->ev_pool.emplace_back(a, b);
  }
  *e0 = ctx->ev_pool[ctx->ev_used].first;
  *e1 = ctx->ev_pool[ctx->ev_used].second;
  ctx->ev_used++;
}

// The three-launch select: where the shape allows it and, by default, prefers it (calls
// bound by their launches, not by bytes); it is tried before the single-pass select.
bool use_mid(const bts_ctx* ctx, const MidPlan& mp) {
  if (!mp.enabled || ctx->path_mode == 1 || ctx->path_mode == 2) return false;
  return ctx->path_mode == 3 || mp.preferred;
}

bool use_fast(const bts_ctx* ctx, const FastPlan& pl) {
  if (!pl.enabled || ctx->path_mode == 1 || ctx->path_mode == 3) return false;
  return ctx->path_mode == 2 || pl.preferred;
}

// uplink = true: the N worker rows with the error compensation fused in; false: the one
// server row.  The single-pass path runs first where the plan enables it; rows it flags
// (and every row where it is not enabled) go through the dense path.
// energy (diagnostics, uplink only): the single-pass path also leaves the partial sums of the
// rows' residual energies in its scratch; *energy is cleared if another path ran.
// upd (downlink only): the model update done by the emitting lanes.
// ranges (uplink only, nullable): in: the caller is about to aggregate exactly these
// messages; out: the select has filled the aggregation's range tables for them.
int run_select(bts_ctx* ctx, bool uplink, const float* g, float* x, float alpha, uint32_t* idx,
               float* val, bool* energy = nullptr,
               FusedUpdate upd = FusedUpdate{nullptr, 0.0f}, bool* ranges = nullptr) {
  const uint32_t rows = uplink ? (uint32_t)ctx->N : 1u;
  const uint32_t K = uplink ? ctx->K_up : ctx->K_dn;
  const FastPlan& pl = uplink ? ctx->plan_up : ctx->plan_dn;
  const FastScratch& fs = uplink ? ctx->fast_up : ctx->fast_dn;
  const MidPlan& mp = uplink ? ctx->mid_plan_up : ctx->mid_plan_dn;
  const MidScratch& ms = uplink ? ctx->mid_up : ctx->mid_dn;
  const bool want_ranges = ranges != nullptr && *ranges;
  if (ranges != nullptr) *ranges = false;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (uplink) profile_events(ctx, &e0, &e1);
  hipError_t e;
  const bool want_energy = energy != nullptr && *energy && fs.energy != nullptr;
  if (energy != nullptr) *energy = false;
  if (K == 0) {
    if (g == nullptr) return BTS_OK;
    e = axpy_only(ctx->stream, g, x, rows, ctx->d, alpha, e0, e1);
  } else if (ctx->path_mode == 0 && row_select_fits(ctx->d)) {
    e = row_select(ctx->stream, g, x, rows, ctx->d, K, alpha, idx, val, e0, e1, upd);
  } else if (use_mid(ctx, mp)) {
    MidRanges mr{nullptr, nullptr, nullptr};
    const AggScratch as = agg_scratch(ctx);
    if (want_ranges && as.tab_start != nullptr) {
      mr = MidRanges{as.tab_start, as.tab_end, as.any};
      *ranges = true;
    }
    e = mid_select(ctx->stream, ms, mp, g, x, rows, ctx->d, K, alpha, idx, val, e0, e1, upd, mr);
  } else if (use_fast(ctx, pl)) {
    MidRanges mr{nullptr, nullptr, nullptr};
    const AggScratch as = agg_scratch(ctx);
    if (want_ranges && as.tab_start != nullptr) {
      mr = MidRanges{as.tab_start, as.tab_end, as.any};
      *ranges = true;
    }
    e = fast_select(ctx->stream, fs, pl, g, x, rows, ctx->d, K, alpha, idx, val, e0, e1,
                    ctx->dense, want_energy, upd, mr);
    if (energy != nullptr) *energy = want_energy;
  } else {
    e = dense_select(ctx->stream, ctx->dense, g, x, rows, ctx->d, K, alpha, idx, val, nullptr,
                     false, e0, e1, upd);
  }
  return e == hipSuccess ? BTS_OK : fail_hip(ctx, e);
}

// Server compression and model update lines of Algorithm 2.  For a short message the lane
// that emits a pair also applies it to w (same result as downlink_topk followed by
// sparse_sgd_update, one kernel launch less).  The update reads w at a scattered address, and
// an emitting wave does its pairs one after the other: from a few thousand pairs on, the
// update kernel of its own (one pair per thread, all loads in flight at once) is quicker than
// the launch it costs (at K_dn = 111,740 the fused emission took 43 us against 20 + 6).
int downlink_and_update(bts_ctx* ctx, float* delta, uint32_t* dn_idx, float* dn_val,
                        float alpha_out, float* w) {
  if (ctx->K_dn <= 4096)
    return run_select(ctx, false, nullptr, delta, 0.0f, dn_idx, dn_val, nullptr,
                      FusedUpdate{w, -alpha_out, false});
  // a longer message on the single-pass path: applied, one pair per thread, in the select's
  // last launch, whose workgroups are idle unless the row needs the dense redo
  const bool single_pass = !(ctx->path_mode == 0 && row_select_fits(ctx->d)) &&
                           !use_mid(ctx, ctx->mid_plan_dn) && use_fast(ctx, ctx->plan_dn);
  if (single_pass)
    return run_select(ctx, false, nullptr, delta, 0.0f, dn_idx, dn_val, nullptr,
                      FusedUpdate{w, -alpha_out, true});
  const int rc = run_select(ctx, false, nullptr, delta, 0.0f, dn_idx, dn_val);
  if (rc != BTS_OK) return rc;
  return sparse_sgd_update(ctx, dn_idx, dn_val, ctx->K_dn, alpha_out, w);
}

int aggregate_messages(bts_ctx* ctx, const uint32_t* up_idx, const float* up_val, const float* p,
                       float* delta, uint32_t* union_nnz, bool ranges_ready) {
  hipError_t e = aggregate(ctx->stream, up_idx, up_val, p, (uint32_t)ctx->N, ctx->K_up, delta,
                           ctx->d, union_nnz, agg_scratch(ctx), ranges_ready);
  return e == hipSuccess ? BTS_OK : fail_hip(ctx, e);
}

// Every argument check of a whole step (bidir_step and bidir_step_diag), made before
// anything is queued.
bool step_args_ok(const bts_ctx* ctx, const float* g, const float* eps, const float* delta,
                  const float* w, const float* p, const uint32_t* up_idx, const float* up_val,
                  const uint32_t* dn_idx, const float* dn_val) {
  if (!ctx || !g || !eps || !delta || !w || !p) return false;
  if (!aligned16(g) || !aligned16(eps) || !aligned16(delta)) return false;
  if (ctx->K_up > 0 && (!up_idx || !up_val)) return false;
  if (ctx->K_dn > 0 && (!dn_idx || !dn_val)) return false;
  return true;
}

}  // namespace

extern "C" {

int bts_create(bts_ctx** out, int32_t N, uint64_t d, uint32_t K_up, uint32_t K_dn,
               void* hip_stream) {
  if (out == nullptr) return BTS_EINVAL;
  *out = nullptr;
  if (N <= 0 || N > 65535 || d == 0 || d >= (1ull << 32) || K_up > d || K_dn > d)
    return BTS_EINVAL;
  bts_ctx* ctx = new (std::nothrow) bts_ctx();
  if (ctx == nullptr) return BTS_ENOMEM;
  ctx->N = N;
  ctx->d = d;
  ctx->K_up = K_up;
  ctx->K_dn = K_dn;
  ctx->stream = reinterpret_cast<hipStream_t>(hip_stream);
  ctx->last_hip_error = 0;
  ctx->profile = false;
  ctx->ev_used = 0;
  ctx->path_mode = 0;
  ctx->dense = DenseScratch{};
  ctx->dense_dirty = false;
  ctx->fast_up_dirty = ctx->fast_dn_dirty = ctx->fast_diag_u_dirty = false;
  ctx->fast_diag_v_dirty = false;
  ctx->fast_up_host = ctx->fast_dn_host = FastScratch::HostState{0, 0, 0, 0};
  ctx->fast_diag_u_host = ctx->fast_diag_v_host = FastScratch::HostState{0, 0, 0, 0};
  ctx->fast_up = FastScratch{};
  ctx->fast_dn = FastScratch{};
  ctx->fast_diag_u = FastScratch{};
  ctx->fast_diag_v = FastScratch{};
  ctx->plan_diag_u = FastPlan{};
  ctx->mid_up = MidScratch{};
  ctx->mid_dn = MidScratch{};
  ctx->mid_up_dirty = ctx->mid_dn_dirty = false;
  ctx->agg_ranges = nullptr;
  ctx->diag = DiagScratch{};
  ctx->diag_ready = false;
  ctx->agg_offsets = nullptr;
  ctx->agg_start = ctx->agg_end = ctx->agg_any = nullptr;
  ctx->agg_tables_bad = false;
  if (hipGetDevice(&ctx->device) != hipSuccess) {
    delete ctx;
    return BTS_EHIP;
  }
  const uint32_t rows = (uint32_t)N;
  const uint32_t nwc = (uint32_t)((d + kWaveChunk - 1) / kWaveChunk) + 1;
  ctx->dense.nwc = nwc;
  ctx->dense.rows = rows;
  ctx->dense.dirty = &ctx->dense_dirty;
  ctx->plan_up = fast_plan(rows, d, K_up);
  ctx->plan_dn = fast_plan(1, d, K_dn);
  ctx->mid_plan_up = mid_plan(rows, d, K_up);
  ctx->mid_plan_dn = mid_plan(1, d, K_dn);
  bool ok = dev_alloc(ctx, &ctx->dense.hist, (size_t)rows * dense_row_hist_words()) &&
            dev_alloc(ctx, &ctx->dense.state, (size_t)rows) &&
            dev_alloc(ctx, &ctx->dense.cnt, (size_t)rows * nwc) &&
            dev_alloc(ctx, &ctx->dense.block_sums, (size_t)rows * dense_max_blocks(1)) &&
            dev_alloc(ctx, &ctx->agg_ranges, (size_t)aggregate_scratch_words(d)) &&
            dev_alloc(ctx, &ctx->agg_offsets, (size_t)aggregate_scratch_words(d)) &&
            alloc_agg_tables(ctx);
  if (!ok) {
    (void)hipGetLastError();
    release(ctx);
    return BTS_ENOMEM;
  }
  // The single-pass path is an optimisation: if its scratch does not fit, the dense path
  // serves the shape alone.
  ctx->fast_up.dirty = &ctx->fast_up_dirty;
  ctx->fast_dn.dirty = &ctx->fast_dn_dirty;
  ctx->fast_up.host = &ctx->fast_up_host;
  ctx->fast_dn.host = &ctx->fast_dn_host;
  if (!alloc_fast(ctx, ctx->plan_up, rows, &ctx->fast_up)) {
    (void)hipGetLastError();
    ctx->plan_up.enabled = false;
  }
  if (!alloc_fast(ctx, ctx->plan_dn, 1, &ctx->fast_dn)) {
    (void)hipGetLastError();
    ctx->plan_dn.enabled = false;
  }
  ctx->mid_up.dirty = &ctx->mid_up_dirty;
  ctx->mid_dn.dirty = &ctx->mid_dn_dirty;
  if (!alloc_mid(ctx, ctx->mid_plan_up, rows, &ctx->mid_up)) {
    (void)hipGetLastError();
    ctx->mid_plan_up.enabled = false;
  }
  if (!alloc_mid(ctx, ctx->mid_plan_dn, 1, &ctx->mid_dn)) {
    (void)hipGetLastError();
    ctx->mid_plan_dn.enabled = false;
  }
  // The scratch was cleared with hipMemset on the null stream; the context's stream may be
  // a non-blocking one that does not order itself after it.
  if (hipDeviceSynchronize() != hipSuccess) {
    release(ctx);
    return BTS_EHIP;
  }
  *out = ctx;
  return BTS_OK;
}

void bts_destroy(bts_ctx* ctx) {
  if (ctx == nullptr) return;
  (void)hipStreamSynchronize(ctx->stream);
  release(ctx);
}

int bts_last_hip_error(const bts_ctx* ctx) { return ctx ? ctx->last_hip_error : 0; }

int topk_compress(bts_ctx* ctx, const float* g, float* eps, float alpha_in, uint32_t* up_idx,
                  float* up_val) {
  if (!ctx || !g || !eps || !aligned16(g) || !aligned16(eps)) return BTS_EINVAL;
  if (ctx->K_up > 0 && (!up_idx || !up_val)) return BTS_EINVAL;
  return run_select(ctx, true, g, eps, alpha_in, up_idx, up_val);
}

int sparse_aggregate(bts_ctx* ctx, const uint32_t* up_idx, const float* up_val, const float* p,
                     float* delta, uint32_t* union_nnz) {
  if (!ctx || !p || !delta) return BTS_EINVAL;
  if (ctx->K_up > 0 && (!up_idx || !up_val)) return BTS_EINVAL;
  return aggregate_messages(ctx, up_idx, up_val, p, delta, union_nnz, false);
}

int downlink_topk(bts_ctx* ctx, float* delta, uint32_t* dn_idx, float* dn_val) {
  if (!ctx || !delta || !aligned16(delta)) return BTS_EINVAL;
  if (ctx->K_dn > 0 && (!dn_idx || !dn_val)) return BTS_EINVAL;
  return run_select(ctx, false, nullptr, delta, 0.0f, dn_idx, dn_val);
}

int sparse_sgd_update(bts_ctx* ctx, const uint32_t* idx, const float* val, uint32_t K,
                      float alpha_out, float* w) {
  if (!ctx || !w) return BTS_EINVAL;
  if (K > 0 && (!idx || !val)) return BTS_EINVAL;
  if (K > ctx->d) return BTS_EINVAL;
  hipError_t e = sgd_update(ctx->stream, idx, val, K, alpha_out, w, ctx->d);
  return e == hipSuccess ? BTS_OK : fail_hip(ctx, e);
}

int bidir_step(bts_ctx* ctx, const float* g, float* eps, float* delta, float* w, const float* p,
               float alpha_in, float alpha_out, uint32_t* up_idx, float* up_val,
               uint32_t* dn_idx, float* dn_val, uint32_t* union_nnz) {
  if (!step_args_ok(ctx, g, eps, delta, w, p, up_idx, up_val, dn_idx, dn_val)) return BTS_EINVAL;
  bool ranges = true;       // the aggregation follows on exactly these messages
  int rc = run_select(ctx, true, g, eps, alpha_in, up_idx, up_val, nullptr,
                      FusedUpdate{nullptr, 0.0f}, &ranges);
  if (rc != BTS_OK) return rc;
  rc = aggregate_messages(ctx, up_idx, up_val, p, delta, union_nnz, ranges);
  if (rc != BTS_OK) return rc;
  return downlink_and_update(ctx, delta, dn_idx, dn_val, alpha_out, w);
}

int unidir_step(bts_ctx* ctx, const float* g, float* eps, float* w, const float* p,
                float alpha_in, float alpha_out, uint32_t* up_idx, float* up_val,
                uint32_t* dn_idx, float* dn_val, uint32_t* dn_count) {
  if (!ctx || !g || !eps || !w || !p) return BTS_EINVAL;
  if (!aligned16(g) || !aligned16(eps)) return BTS_EINVAL;
  if (ctx->K_up > 0 && (!up_idx || !up_val)) return BTS_EINVAL;
  if ((dn_idx == nullptr) != (dn_val == nullptr)) return BTS_EINVAL;
  bool ranges = true;
  int rc = run_select(ctx, true, g, eps, alpha_in, up_idx, up_val, nullptr,
                      FusedUpdate{nullptr, 0.0f}, &ranges);
  if (rc != BTS_OK) return rc;
  hipError_t e = aggregate_update_unidirectional(
      ctx->stream, up_idx, up_val, p, (uint32_t)ctx->N, ctx->K_up, w, ctx->d, alpha_out, dn_idx,
      dn_val, dn_count, agg_scratch(ctx), ranges);
  return e == hipSuccess ? BTS_OK : fail_hip(ctx, e);
}

int bts_enable_diagnostics(bts_ctx* ctx) {
  if (!ctx) return BTS_EINVAL;
  if (ctx->diag_ready) return BTS_OK;
  if (ctx->K_up == 0 || ctx->K_dn == 0) return BTS_EINVAL;
  DiagScratch& ds = ctx->diag;
  const size_t nk = (size_t)ctx->N * ctx->K_up;
  bool ok = dev_alloc(ctx, &ds.u, (size_t)ctx->d) && dev_alloc(ctx, &ds.v, (size_t)ctx->d) &&
            dev_alloc(ctx, &ds.part, diag_part_doubles((uint32_t)ctx->N)) &&
            dev_alloc(ctx, &ds.a_idx, (size_t)ctx->K_dn) &&
            dev_alloc(ctx, &ds.a_val, (size_t)ctx->K_dn) &&
            dev_alloc(ctx, &ds.c_idx, (size_t)ctx->K_up) &&
            dev_alloc(ctx, &ds.c_val, (size_t)ctx->K_up) && dev_alloc(ctx, &ds.m_idx, nk) &&
            dev_alloc(ctx, &ds.m_val, nk) && dev_alloc(ctx, &ds.m_cnt, 1);
  if (ok) {                            // the one-row select with K_up (falls back to dense)
    ctx->plan_diag_u = fast_plan(1, ctx->d, ctx->K_up);
    ctx->fast_diag_u.dirty = &ctx->fast_diag_u_dirty;
    ctx->fast_diag_u.host = &ctx->fast_diag_u_host;
    if (!alloc_fast(ctx, ctx->plan_diag_u, 1, &ctx->fast_diag_u)) {
      (void)hipGetLastError();
      ctx->plan_diag_u.enabled = false;
    }
    ctx->fast_diag_v.dirty = &ctx->fast_diag_v_dirty;
    ctx->fast_diag_v.host = &ctx->fast_diag_v_host;
    ok = alloc_fast(ctx, ctx->plan_dn, 1, &ctx->fast_diag_v);
  }
  if (ok && ctx->plan_up.enabled)      // partial sums of the rows' residual energies
    ok = dev_alloc(ctx, &ctx->fast_up.energy, (size_t)ctx->N * ctx->plan_up.nwc_pad) &&
         dev_alloc(ctx, &ctx->fast_up.tile_energy, (size_t)ctx->N * ctx->plan_up.ntiles);
  if (!ok) {
    (void)hipGetLastError();
    return BTS_ENOMEM;
  }
  if (hipDeviceSynchronize() != hipSuccess) return BTS_EHIP;   // see bts_create
  ctx->diag_ready = true;
  return BTS_OK;
}

int bidir_step_diag(bts_ctx* ctx, const float* g, float* eps, float* delta, float* w,
                    const float* p, float alpha_in, float alpha_out, uint32_t* up_idx,
                    float* up_val, uint32_t* dn_idx, float* dn_val, double* diag) {
  if (!diag || !step_args_ok(ctx, g, eps, delta, w, p, up_idx, up_val, dn_idx, dn_val))
    return BTS_EINVAL;
  if (!ctx->diag_ready || ctx->K_up == 0 || ctx->K_dn == 0) return BTS_EINVAL;
  hipError_t e = diag_before_step(ctx->stream, ctx->diag, g, eps, delta, p, (uint32_t)ctx->N,
                                  ctx->d, alpha_in);
  if (e != hipSuccess) return fail_hip(ctx, e);
  // the step itself, with the worker compression also leaving the rows' residual energies
  bool energy = true;
  int rc = run_select(ctx, true, g, eps, alpha_in, up_idx, up_val, &energy);
  if (rc != BTS_OK) return rc;
  rc = sparse_aggregate(ctx, up_idx, up_val, p, delta, nullptr);
  if (rc != BTS_OK) return rc;
  rc = downlink_and_update(ctx, delta, dn_idx, dn_val, alpha_out, w);
  if (rc != BTS_OK) return rc;
  RowEnergy re{};
  if (energy) {
    re.chunks = ctx->fast_up.energy;
    re.tiles = ctx->fast_up.tile_energy;
    re.nwc_pad = ctx->plan_up.nwc_pad;
    re.ntiles = ctx->plan_up.ntiles;
    re.need = ctx->fast_up.need;
  }
  e = diag_after_step(ctx->stream, ctx->diag, ctx->dense, eps, delta, p, (uint32_t)ctx->N, ctx->d,
                      ctx->K_up, ctx->K_dn, alpha_in, up_idx, up_val, dn_idx, dn_val,
                      agg_scratch(ctx), re, OneRowSelect{&ctx->plan_dn, &ctx->fast_diag_v},
                      OneRowSelect{&ctx->plan_diag_u, &ctx->fast_diag_u}, diag);
  return e == hipSuccess ? BTS_OK : fail_hip(ctx, e);
}

int bts_profile_enable(bts_ctx* ctx, int on) {
  if (!ctx) return BTS_EINVAL;
  ctx->profile = on != 0;
  return BTS_OK;
}

int bts_profile_read(bts_ctx* ctx, double* ms_total, uint64_t* launches) {
  if (!ctx || !ms_total || !launches) return BTS_EINVAL;
  double total = 0.0;
  for (size_t i = 0; i < ctx->ev_used; ++i) {
    hipError_t e = hipEventSynchronize(ctx->ev_pool[i].second);
    if (e != hipSuccess) return fail_hip(ctx, e);
    float ms = 0.0f;
    e = hipEventElapsedTime(&ms, ctx->ev_pool[i].first, ctx->ev_pool[i].second);
    if (e != hipSuccess) return fail_hip(ctx, e);
    total += ms;
  }
  *ms_total = total;
  *launches = ctx->ev_used;
  ctx->ev_used = 0;
  return BTS_OK;
}

int bts_last_path(bts_ctx* ctx, int which, uint32_t* rows_fast, uint32_t* rows_dense) {
  if (!ctx || !rows_fast || !rows_dense || (which != 0 && which != 1)) return BTS_EINVAL;
  const uint32_t rows = which == 0 ? (uint32_t)ctx->N : 1u;
  const FastPlan& pl = which == 0 ? ctx->plan_up : ctx->plan_dn;
  const FastScratch& fs = which == 0 ? ctx->fast_up : ctx->fast_dn;
  const uint32_t K = which == 0 ? ctx->K_up : ctx->K_dn;
  *rows_fast = 0;
  *rows_dense = rows;
  const MidPlan& mp = which == 0 ? ctx->mid_plan_up : ctx->mid_plan_dn;
  if (K == 0 || (ctx->path_mode == 0 && row_select_fits(ctx->d)) || use_mid(ctx, mp) ||
      !use_fast(ctx, pl))
    return BTS_OK;
  hipError_t e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return fail_hip(ctx, e);
  std::vector<uint32_t> need(rows);
  e = hipMemcpy(need.data(), fs.need, rows * sizeof(uint32_t), hipMemcpyDeviceToHost);
  if (e != hipSuccess) return fail_hip(ctx, e);
  uint32_t dense = 0;
  for (uint32_t v : need) dense += v ? 1u : 0u;
  *rows_dense = dense;
  *rows_fast = rows - dense;
  return BTS_OK;
}

int bts_testing_plan(uint32_t rows, uint64_t d, uint32_t K, uint32_t* out) {
  if (out == nullptr || rows == 0 || d == 0 || d >= (1ull << 32) || K > d) return BTS_EINVAL;
  const FastPlan fp = fast_plan(rows, d, K);
  const MidPlan mp = mid_plan(rows, d, K);
  uint32_t path = 1;                                          // dense multi-pass
  if (K != 0 && row_select_fits(d)) path = 0;                 // one workgroup per row
  else if (K != 0 && mp.enabled && mp.preferred) path = 3;    // three launches
  else if (K != 0 && fp.enabled && fp.preferred) path = 2;    // single pass
  out[0] = path;
  out[1] = fp.enabled ? 1u : 0u;
  out[2] = fp.cap;
  out[3] = fp.stride;
  out[4] = fp.target;
  out[5] = fp.rank_next;
  out[6] = fp.ntiles;
  out[7] = fp.nwc_pad;
  out[8] = fp.stream_waves_per_simd;
  out[9] = mp.enabled ? 1u : 0u;
  out[10] = mp.cap;
  out[11] = mp.ntiles;
  out[12] = mp.nwc_pad;
  out[13] = mp.gx;
  out[14] = mp.gx_hist;
  out[15] = fast_sublists();
  return BTS_OK;
}

int bts_testing_mark_dirty(bts_ctx* ctx) {
  if (!ctx) return BTS_EINVAL;
  ctx->dense_dirty = true;
  ctx->fast_up_dirty = ctx->fast_dn_dirty = ctx->fast_diag_u_dirty = true;
  ctx->fast_diag_v_dirty = true;
  ctx->mid_up_dirty = ctx->mid_dn_dirty = true;
  ctx->agg_tables_bad = true;
  return BTS_OK;
}

int bts_set_path(bts_ctx* ctx, int mode) {
  if (!ctx || mode < 0 || mode > 3) return BTS_EINVAL;
  ctx->path_mode = mode;
  return BTS_OK;
}

}  // extern "C"
