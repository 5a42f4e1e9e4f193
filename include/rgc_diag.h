/* rgc_diag.h -- diagnostics, test hooks and benchmark timers of the RGC library (see rgc.h for the
 * library itself).  Nothing here changes a result; none of it belongs on a training step's path: every
 * call below except rgc_profile_enable and rgc_stream_yardstick synchronises the stream it is given.
 */
#ifndef RGC_DIAG_H_
#define RGC_DIAG_H_

#include "rgc.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Overwrites the cached threshold hints with deliberately wrong values (mode 0: far too high, 1: far
 * too low, 2: pseudo-random): results must not change, only the path a layer takes (rgc_last_paths
 * then reports 2).  This is how the tests prove that results do not depend on the hints and how the
 * benchmark times a call whose hints miss. */
int rgc_poison_hints(rgc_ctx* ctx, int mode, void* hip_stream);

/* Caps the scratch that compression calls allocate on demand for layers that select a large share of
 * their elements (their candidate lists; see rgc.h, "Stream capture"): a call that would need more than
 * `max_bytes` does not ask for it, as if the device were short of memory, and those layers take the
 * hint-free path.  Results do not change.  A negative value lifts the cap.  Frees what is held beyond
 * the cap (after a device synchronisation). */
int rgc_limit_optional_scratch(rgc_ctx* ctx, int64_t max_bytes);

/* Runs a one-workgroup kernel that checks the wave64 primitives the kernels rely on (DPP
 * prefix scan, ballot ranks) against values computed on the host.  Synchronises `hip_stream`.
 * Returns RGC_OK, RGC_EINTERNAL on a mismatch, or RGC_EHIP. */
int rgc_selftest(rgc_ctx* ctx, void* hip_stream);

/* Copies per-layer path statistics of the LAST compression call into `out` (host memory,
 * int32[num_layers]): 0 = one-pass hinted path, 1 = hint-free multi-pass path, 2 = hinted
 * pass missed and the multi-pass path re-ran on the updated residual.  Synchronises
 * `hip_stream`.  Returns RGC_EINTERNAL if any kernel of an earlier call flagged an internal
 * inconsistency.  A diagnostic for tests and benchmarks. */
int rgc_last_paths(rgc_ctx* ctx, int32_t* out, int32_t num_layers, void* hip_stream);

/* Like rgc_last_paths with more detail: out is int64[num_layers][5] = { path, number of
 * candidates the streaming pass collected (0 on the hint-free path), number of candidates that
 * had to be ranked exactly, magnitude key (float bits, sign cleared) of the k-th entry, number
 * of calls since rgc_create in which this layer slot's hint missed (path 2) }. */
int rgc_last_stats(rgc_ctx* ctx, int64_t* out, int32_t num_layers, void* hip_stream);

/* Kernel timing for benchmarks.  rgc_profile_enable(ctx, 1) makes every later compression and
 * decompression call record HIP events on the caller's stream around its kernels (a few extra
 * microseconds per call); rgc_profile_enable(ctx, 0) stops that.  rgc_profile_read synchronises
 * the recorded events and returns, summed over the calls since the last read, the milliseconds
 * spent in  out_ms[0] the streaming accumulate kernel, out_ms[1] the phase launches after it,
 * out_ms[2] the decompression table kernel, out_ms[3] the decompression tile kernel, and the
 * number of compression / decompression calls in out_calls[0..1].  The record is then cleared. */
int rgc_profile_enable(rgc_ctx* ctx, int enable);
int rgc_profile_read(rgc_ctx* ctx, double* out_ms, int64_t* out_calls);

/* A yardstick for the streaming pass of the compression call (Algorithm 1's accumulate with the momentum
 * correction of Section 2.5): one kernel that reads `grad`, `residual` and `velocity` (device pointers, n fp32
 * elements each, 16-byte aligned, the caller's) and writes  velocity = momentum * velocity + grad,
 * residual = residual + velocity  back in place -- the 20 bytes per element of that pass and none of its
 * selection work, with the same decomposition (one wave per 8192 consecutive elements; `reverse` != 0 walks the
 * tensors from the far end, as every other compression call does).  A benchmark times it to learn what share of
 * the HBM peak this mix of reads and writes reaches on the device at all.  Launches on the current device and
 * `hip_stream`, does not synchronise, needs no context.  RGC_EINVAL: null or misaligned pointer, n < 1. */
int rgc_stream_yardstick(const float* grad, float* residual, float* velocity, int64_t n, float momentum,
                         int reverse, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* RGC_DIAG_H_ */
