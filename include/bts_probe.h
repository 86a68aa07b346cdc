/*
 * bts_probe -- a measurement instrument, built as a library of its own (libbts_probe.so):
 * what this part's HBM sustains for the access mixes of libbts.  Not part of libbts.
 */
#ifndef BTS_PROBE_H
#define BTS_PROBE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * A plain stream over n floats (device pointers, 16-byte aligned, n >= 512; whole 512-float
 * chunks only) with the access shape of libbts's dominant kernel (the dense pass of the
 * worker lines of Algorithm 2) and nothing else:
 * kind 0 reads src, kind 1 copies src to dst, kind 2 does dst = fma(0.5, src, dst) -- the
 * 2 reads : 1 write mix of the worker's error compensation (Algorithm 2, worker line 1).
 * waves_per_cu: 0 = every wave slot may fill; 12, 20 or 24 = the launch is held to that
 * many waves per compute unit, by_registers == 0: through dynamic LDS it requests and
 * never touches; by_registers != 0: through the register allocation of a kernel variant
 * compiled for at most that many waves per SIMD.  With kind 2 only, waves_per_cu = 101, 102,
 * 103: the fma-stream at 12 waves per compute unit with plain instead of non-temporal
 * accesses (101 the loads, 102 the stores, 103 both).
 * Queues one untimed launch and `repeats` timed ones on hip_stream (a hipStream_t, host
 * value, null = default stream), waits for them, and returns the mean time of one launch
 * in milliseconds (host pointer).  kinds 1 and 2 overwrite dst.
 * Returns 0, -1 on bad arguments, or -1000 - hipError_t when a HIP call failed.
 */
int bts_hbm_probe(void* hip_stream, int kind, const float* src, float* dst, uint64_t n,
                  int waves_per_cu, int by_registers, int repeats, double* ms_per_launch);

#ifdef __cplusplus
}
#endif
#endif /* BTS_PROBE_H */
