/*
 * bts -- one parameter-server step of bidirectional Top_K SGD with error feedback
 * (Algorithm 2 of "Downlink Compression Improves Top_K Sparsification"), simulated on
 * one MI355X for N workers held as an N x d fp32 batch.
 *
 * C ABI.  Unless a parameter is marked "host", every pointer is a DEVICE pointer to
 * memory owned by the caller; the library never frees or reallocates it.  All work is
 * queued on the HIP stream given to bts_create and returns without synchronising the
 * host; results are ready when that stream reaches the end of the queued work.  A
 * context may be used by one host thread at a time and calls on one context must not
 * overlap.  The only allocations the library makes are the scratch buffers owned by
 * the context (made in bts_create, released in bts_destroy).
 *
 * Notation (the paper's): N workers, d coordinates, g^q the gradient of worker q,
 * eps^q its residual, a^q = eps^q + alpha g^q, p_q the worker weights, delta the
 * server residual, g_t the server's error-compensated aggregate, w the model.
 *
 * Top_K(x) keeps the K components of x of largest magnitude and zeroes the rest
 * (abstract and introduction of the paper).  The paper leaves equal magnitudes and
 * special values open; this library orders coordinates by the 31-bit pattern of the
 * fp32 value with the sign cleared (so NaN > Inf > finite > denormal > zero, and +0
 * ties with -0), larger first, and among equal patterns the LOWER index is kept.  A
 * message is the K kept (index, value) pairs in ASCENDING index order, values copied
 * bit for bit; the paper's cost model counts such a message as 2K 32-bit words
 * (communication section).  The residual x - Top_K(x) is x with +0.0f stored at the
 * kept positions.  Denormals are never flushed.  Every multiply-add is one fused,
 * correctly rounded fp32 operation.
 *
 * Return value of every call: BTS_OK, or a negative code.  Arguments are checked
 * before anything is launched; on BTS_EINVAL nothing has been queued.
 *
 * What a context remembers between calls is scratch kept clean and, per direction, where
 * the last call found its rows' thresholds: from its third compression on a context starts
 * its search there instead of sampling the rows (a training run's threshold moves little
 * from step to step; after a call in which that start proved useless it samples again for a
 * few calls).  That only decides how long a call takes, never what it returns:
 * every output of every call is the exact Top_K defined above, whatever the history of the
 * context.
 */
#ifndef BTS_H
#define BTS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BTS_OK 0
#define BTS_EINVAL (-1) /* null required pointer, N <= 0, d == 0, d >= 2^32, K > d,        */
                        /* N > 65535, or a dense buffer (g, eps, delta) not 16-byte aligned */
#define BTS_ENOMEM (-2) /* scratch allocation failed                                       */
#define BTS_EHIP (-3)   /* a HIP call failed; see bts_last_hip_error                       */
#define BTS_ELIMIT (-4) /* shape beyond the fixed scratch of topk_compress_noalloc         */
#define BTS_EHIP_BASE (-1000) /* topk_compress_noalloc only: a HIP call failed with        */
                              /* hipError_t e; the call returns BTS_EHIP_BASE - e           */

typedef struct bts_ctx bts_ctx;

/*
 * Create a context for a fixed problem shape: N workers, d coordinates, K_up kept
 * coordinates per worker on the uplink, K_dn on the downlink (the paper's experiments
 * use K_up == K_dn; its communication section treats them separately).  K == 0 and
 * K == d are legal.  hip_stream is a hipStream_t (host value, borrowed, may be null for
 * the default stream); every later call on the context queues onto it.  Scratch
 * (histograms, per-block counts, candidate lists, chunk directory, selection state) is sized and
 * cleared here once; the call synchronises the device before it returns (of the calls
 * declared here only bts_create, bts_enable_diagnostics and bts_destroy do).
 */
int bts_create(bts_ctx** out, int32_t N, uint64_t d, uint32_t K_up, uint32_t K_dn,
               void* hip_stream);
void bts_destroy(bts_ctx* ctx);

/* HIP error code (hipError_t as int) of the last failed HIP call on this context. */
int bts_last_hip_error(const bts_ctx* ctx);

/*
 * Worker lines of Algorithm 2, for all N workers at once:
 *     a^q = eps^q + alpha_in * g^q ;  send Top_K(a^q) ;  eps^q = a^q - Top_K(a^q).
 * g        N x d row-major fp32, read only (row stride d; d need not be a multiple of 4).
 * eps      N x d row-major fp32, in: eps_{t-1}, out: eps_t.
 * alpha_in host scalar, the step size alpha_{t-1} of the paper.
 * up_idx   N x K_up uint32 out; row q holds worker q's kept coordinates, ascending.
 * up_val   N x K_up fp32 out; the matching values of a^q.
 */
int topk_compress(bts_ctx* ctx, const float* g, float* eps, float alpha_in, uint32_t* up_idx,
                  float* up_val);

/*
 * For callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same operation and same results as
 * topk_compress (g, eps, alpha_in, up_idx, up_val as there), but without a context: the
 * shape travels in the call, the work is queued on hip_stream (a hipStream_t, host value,
 * borrowed, null = the default stream; it must belong to the current device), and the
 * select's scratch lives in a fixed 13 MiB array that each GPU the library runs on holds
 * until the process ends.  The call makes no hipMalloc, hipFree or other allocating call;
 * its first call on a device looks up that device's copy of the array.
 * Limits: N <= 256 and N * (ceil(d / 512) + 1) <= 2^20 (about 5.3e8 coordinates per call);
 * beyond them the call returns BTS_ELIMIT and queues nothing.  A failed HIP call returns
 * BTS_EHIP_BASE - hipError_t.  All calls on one GPU share that GPU's array: calls that
 * overlap on one GPU (two streams, two threads) race and must be serialised by the caller;
 * calls that follow each other on one stream are safe, whatever their shapes.
 */
int topk_compress_noalloc(const float* g, float* eps, int32_t N, uint64_t d, uint32_t K_up,
                          float alpha_in, uint32_t* up_idx, float* up_val, void* hip_stream);

/*
 * Server aggregation line of Algorithm 2:  g_t = sum_q p_q Top_K(a^q) + delta_{t-1}.
 * For every coordinate the accumulator starts at delta_{t-1}[i] and the workers that
 * name i are added in ascending q, one fused multiply-add each, so the result does not
 * depend on scheduling.  Coordinates no worker names keep their bits.
 * up_idx, up_val  as written by topk_compress (each row ascending, all indices < d).
 * p           N fp32 weights (device).
 * delta       d fp32, in: delta_{t-1}, out: g_t.
 * union_nnz   nullable; receives the number of distinct coordinates named by the
 *             uplinks (the "at most K_uplink N non-zero indices" of the paper's
 *             communication section), one uint32 on the device.
 */
int sparse_aggregate(bts_ctx* ctx, const uint32_t* up_idx, const float* up_val, const float* p,
                     float* delta, uint32_t* union_nnz);

/*
 * Server compression lines of Algorithm 2: send Top_K(g_t), keep
 * delta_t = g_t - Top_K(g_t).
 * delta   d fp32, in: g_t, out: delta_t.
 * dn_idx, dn_val   K_dn pairs out, ascending index.
 */
int downlink_topk(bts_ctx* ctx, float* delta, uint32_t* dn_idx, float* dn_val);

/*
 * Model update line of Algorithm 2 on K received pairs: w[idx] -= alpha_out * val (one
 * fused multiply-add per pair).  Indices must be distinct and < d.  The paper folds the
 * step size into a^q and updates with alpha_out = 1.
 */
int sparse_sgd_update(bts_ctx* ctx, const uint32_t* idx, const float* val, uint32_t K,
                      float alpha_out, float* w);

/*
 * One whole iteration of the loop body of Algorithm 2: topk_compress, sparse_aggregate,
 * downlink_topk, sparse_sgd_update, queued in that order; results are identical to
 * making the four calls.  State (eps, delta, w) is updated in place; the uplink and
 * downlink messages are left in the four output buffers.  union_nnz is nullable.
 * Paper form: alpha_in = alpha_{t-1}, alpha_out = 1.
 */
int bidir_step(bts_ctx* ctx, const float* g, float* eps, float* delta, float* w, const float* p,
               float alpha_in, float alpha_out, uint32_t* up_idx, float* up_val,
               uint32_t* dn_idx, float* dn_val, uint32_t* union_nnz);

/*
 * One whole iteration of the loop body of Algorithm 1 (unidirectional Top_K SGD, the
 * paper's baseline): the worker lines are those of Algorithm 2 (topk_compress); the server
 * forms g_t = sum_q p_q Top_K(a^q) (accumulator starts at +0, workers in ascending q, one
 * fused multiply-add each) and sends it uncompressed; the workers apply
 * w -= alpha_out * g_t.  There is no server residual.  g_t is non-zero at most at the
 * coordinates some uplink names (at most K_uplink N of them, communication section), so
 * the message is produced sparse:
 * dn_idx, dn_val  nullable (both or neither); room for N * K_up pairs; receive the named
 *                 coordinates in ascending order and their g_t values.
 * dn_count        nullable; one uint32 on the device: the number of pairs.
 * Same results as bidir_step with K_dn = d and a zero delta.
 */
int unidir_step(bts_ctx* ctx, const float* g, float* eps, float* w, const float* p,
                float alpha_in, float alpha_out, uint32_t* up_idx, float* up_val,
                uint32_t* dn_idx, float* dn_val, uint32_t* dn_count);

/*
 * bidir_step plus the per-step estimates of the constants the paper measures in its section
 * on convergence-bound constants.  bts_enable_diagnostics allocates the extra scratch
 * (2 d floats and O(N K_up) words) once; it is the only other allocation point of the library
 * and needs K_up, K_dn >= 1.  bidir_step_diag queues one extra dense read of g and eps before
 * the step and O(d + N K_up) work after it; state and messages come out exactly as from
 * bidir_step.
 * diag   8 + N doubles on the DEVICE:
 *   [0] rho      = |Top_K(delta_{t-1} + sum_q p_q a^q) - Top_K(g_t)| / |alpha_in sum_q p_q g^q|
 *                  (the two sides of Assumption 5; first Top_K with K_dn)
 *   [1] rho_hat  = |Top_K(sum_q p_q a^q) - sum_q p_q Top_K(a^q)| / |alpha_in sum_q p_q g^q|
 *                  (Assumption 6, the unidirectional counterpart; Top_K with K_up)
 *   [2] max of 1 - gamma = |x - Top_K(x)|^2 / |x|^2 over the step's compressions
 *   [3] |alpha_in sum_q p_q g^q|, [4] numerator of rho, [5] numerator of rho_hat
 *   [6] distinct coordinates named by the uplinks / d (communication section)
 *   [7] 1 - gamma of the server compression, [8 + q] 1 - gamma of worker q.
 * The dense sums are fp32 fused multiply-add chains in ascending q; norms accumulate in fp64.
 */
int bts_enable_diagnostics(bts_ctx* ctx);
int bidir_step_diag(bts_ctx* ctx, const float* g, float* eps, float* delta, float* w,
                    const float* p, float alpha_in, float alpha_out, uint32_t* up_idx,
                    float* up_val, uint32_t* dn_idx, float* dn_val, double* diag);

#ifdef __cplusplus
}
#endif
#endif /* BTS_H */
