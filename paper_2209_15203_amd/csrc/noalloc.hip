// topk_compress_noalloc: the worker lines of Algorithm 2 for callers that cannot allocate
// (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
//
// It runs the dense multi-pass select of dense_select.hip -- the same kernels topk_compress
// uses on its dense path -- with the select's scratch (digit histograms, threshold state,
// per-chunk and per-block counts of the emission) laid out in ONE file-scope device array instead of
// buffers owned by a context.  Every GPU the library runs on holds its own copy of that
// array (kNoallocWords * 4 bytes = 13 MiB) until the process ends.  Nothing here calls
// hipMalloc, hipFree or an allocating library routine.
//
// In host code the array's NAME is only a stand-in for the symbol; its address on a device
// comes from hipGetSymbolAddress, looked up once per device with that device current and
// kept.  Host code below uses that pointer and never the name.

#include "../../include/bts.h"

#include <mutex>

#include "bts_internal.h"

namespace bts {

namespace {

constexpr uint32_t kNoallocMaxRows = 256;              // worker rows per call
constexpr uint64_t kNoallocMaxChunks = 1ull << 20;     // rows x wave chunks per row
// histograms + threshold state + the per-chunk and per-block counts of the emission
constexpr uint64_t kNoallocWords = 3407872;            // 13 MiB

static __device__ __align__(256) uint32_t scratch[kNoallocWords];

constexpr int kMaxDevices = 64;
struct DeviceScratch {
  uint32_t* ptr = nullptr;     // this device's copy of `scratch`
  bool ready = false;
};
DeviceScratch g_scratch[kMaxDevices];
std::mutex g_scratch_mu;

// The current device's copy of the array (first call on a device looks it up).
hipError_t scratch_of_current_device(uint32_t** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  DeviceScratch& ds = g_scratch[dev];
  if (!ds.ready) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    ds.ptr = static_cast<uint32_t*>(p);
    ds.ready = true;
  }
  *out = ds.ptr;
  return hipSuccess;
}

uint64_t round_up_64(uint64_t words) { return (words + 63) / 64 * 64; }   // 256-byte pieces

int hip_code(hipError_t e) { return BTS_EHIP_BASE - (int)e; }

}  // namespace

}  // namespace bts

using namespace bts;

extern "C" int topk_compress_noalloc(const float* g, float* eps, int32_t N, uint64_t d,
                                     uint32_t K_up, float alpha_in, uint32_t* up_idx,
                                     float* up_val, void* hip_stream) {
  if (!g || !eps || N <= 0 || d == 0 || d >= (1ull << 32) || K_up > d) return BTS_EINVAL;
  if ((reinterpret_cast<uintptr_t>(g) & 15u) || (reinterpret_cast<uintptr_t>(eps) & 15u))
    return BTS_EINVAL;
  if (K_up > 0 && (!up_idx || !up_val)) return BTS_EINVAL;
  const uint32_t rows = (uint32_t)N;
  const uint32_t nwc = (uint32_t)((d + kWaveChunk - 1) / kWaveChunk) + 1;
  if (rows > kNoallocMaxRows || (uint64_t)rows * nwc > kNoallocMaxChunks) return BTS_ELIMIT;
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  if (K_up == 0) {
    const hipError_t e = axpy_only(s, g, eps, rows, d, alpha_in, nullptr, nullptr);
    return e == hipSuccess ? BTS_OK : hip_code(e);
  }
  uint32_t* base = nullptr;
  hipError_t e = scratch_of_current_device(&base);
  if (e != hipSuccess) return hip_code(e);
  // carve the array up (the limits above bound every piece)
  const uint64_t w_hist = round_up_64((uint64_t)rows * dense_row_hist_words());
  const uint64_t w_state = round_up_64((uint64_t)rows * (sizeof(SelState) / 4));
  const uint64_t w_cnt = round_up_64((uint64_t)rows * nwc * 2);
  const uint64_t w_blocks = round_up_64((uint64_t)rows * dense_max_blocks(rows) * 2);
  if (w_hist + w_state + w_cnt + w_blocks > kNoallocWords) return BTS_ELIMIT;
  DenseScratch sc{};
  // The array keeps what the last call left (another shape's counts, the histograms of a
  // call that failed half way): `dirty` makes the select clear the histograms, with a fill
  // kernel, before it uses them; every other piece is written before it is read.
  bool dirty = true;
  uint32_t* at = base;
  sc.hist = at;
  at += w_hist;
  sc.state = reinterpret_cast<SelState*>(at);
  at += w_state;
  sc.cnt = reinterpret_cast<uint2*>(at);
  at += w_cnt;
  sc.block_sums = reinterpret_cast<uint2*>(at);
  sc.dirty = &dirty;
  sc.rows = rows;
  sc.nwc = nwc;
  e = dense_select(s, sc, g, eps, rows, d, K_up, alpha_in, up_idx, up_val, nullptr, false,
                   nullptr, nullptr);
  return e == hipSuccess ? BTS_OK : hip_code(e);
}
