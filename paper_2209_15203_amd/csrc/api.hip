// C ABI of libbts (see include/bts.h): argument checks, scratch ownership, and the order
// in which the kernels of one step of Algorithm 2 are queued.

#include "../../include/bts.h"

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
  // timing of the dominant kernel
  bool profile;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> ev_pool;
  size_t ev_used;
};

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int fail_hip(bts_ctx* ctx, hipError_t e) {
  ctx->last_hip_error = (int)e;
  return BTS_EHIP;
}

template <typename T>
hipError_t dev_alloc(T** p, size_t count) {
  return hipMalloc(reinterpret_cast<void**>(p), count * sizeof(T) + 16);
}

void release(bts_ctx* ctx) {
  (void)hipFree(ctx->dense.hist);
  (void)hipFree(ctx->dense.state);
  (void)hipFree(ctx->dense.cnt_gt);
  (void)hipFree(ctx->dense.cnt_eq);
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

int run_select(bts_ctx* ctx, const float* g, float* x, uint32_t rows, uint32_t K, float alpha,
               uint32_t* idx, float* val, bool dominant) {
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (dominant) profile_events(ctx, &e0, &e1);
  hipError_t e;
  if (K == 0) {
    if (g == nullptr) return BTS_OK;
    e = axpy_only(ctx->stream, g, x, rows, ctx->d, alpha, e0, e1);
  } else {
    e = dense_select(ctx->stream, ctx->dense, g, x, rows, ctx->d, K, alpha, idx, val, nullptr,
                     false, e0, e1);
  }
  return e == hipSuccess ? BTS_OK : fail_hip(ctx, e);
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
  ctx->dense = DenseScratch{};
  if (hipGetDevice(&ctx->device) != hipSuccess) {
    delete ctx;
    return BTS_EHIP;
  }
  const uint32_t rows = (uint32_t)N;
  const uint32_t nwc = (uint32_t)((d + kWaveChunk - 1) / kWaveChunk) + 1;
  ctx->dense.nwc = nwc;
  bool ok = dev_alloc(&ctx->dense.hist, (size_t)rows * kBins0) == hipSuccess &&
            dev_alloc(&ctx->dense.state, (size_t)rows) == hipSuccess &&
            dev_alloc(&ctx->dense.cnt_gt, (size_t)rows * nwc) == hipSuccess &&
            dev_alloc(&ctx->dense.cnt_eq, (size_t)rows * nwc) == hipSuccess;
  if (!ok) {
    (void)hipGetLastError();
    release(ctx);
    return BTS_ENOMEM;
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
  return run_select(ctx, g, eps, (uint32_t)ctx->N, ctx->K_up, alpha_in, up_idx, up_val, true);
}

int sparse_aggregate(bts_ctx* ctx, const uint32_t* up_idx, const float* up_val, const float* p,
                     float* delta, uint32_t* union_nnz) {
  if (!ctx || !p || !delta) return BTS_EINVAL;
  if (ctx->K_up > 0 && (!up_idx || !up_val)) return BTS_EINVAL;
  hipError_t e = aggregate(ctx->stream, up_idx, up_val, p, (uint32_t)ctx->N, ctx->K_up, delta,
                           ctx->d, union_nnz);
  return e == hipSuccess ? BTS_OK : fail_hip(ctx, e);
}

int downlink_topk(bts_ctx* ctx, float* delta, uint32_t* dn_idx, float* dn_val) {
  if (!ctx || !delta || !aligned16(delta)) return BTS_EINVAL;
  if (ctx->K_dn > 0 && (!dn_idx || !dn_val)) return BTS_EINVAL;
  return run_select(ctx, nullptr, delta, 1, ctx->K_dn, 0.0f, dn_idx, dn_val, false);
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
  if (!ctx || !g || !eps || !delta || !w || !p) return BTS_EINVAL;
  if (!aligned16(g) || !aligned16(eps) || !aligned16(delta)) return BTS_EINVAL;
  if (ctx->K_up > 0 && (!up_idx || !up_val)) return BTS_EINVAL;
  if (ctx->K_dn > 0 && (!dn_idx || !dn_val)) return BTS_EINVAL;
  int rc = topk_compress(ctx, g, eps, alpha_in, up_idx, up_val);
  if (rc != BTS_OK) return rc;
  rc = sparse_aggregate(ctx, up_idx, up_val, p, delta, union_nnz);
  if (rc != BTS_OK) return rc;
  rc = downlink_topk(ctx, delta, dn_idx, dn_val);
  if (rc != BTS_OK) return rc;
  return sparse_sgd_update(ctx, dn_idx, dn_val, ctx->K_dn, alpha_out, w);
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
  *rows_fast = 0;
  *rows_dense = which == 0 ? (uint32_t)ctx->N : 1u;
  return BTS_OK;
}

}  // extern "C"
