/*
 * emc2_probe.h -- measurement probes of the bench (libemc2probe.so), not part of the method: what the part
 * itself sustains for an empty launch, a plain copy and a dense matrix-core loop, so that the hot path's figures
 * can be read against measured ceilings as well as against the published peaks.  No passage of the paper stands
 * behind them.  All pointers are DEVICE pointers owned by the caller; calls enqueue on `stream` (a hipStream_t,
 * NULL = default) and return; the return value is 0 or a hipError_t.
 */
#ifndef EMC2_PROBE_H_
#define EMC2_PROBE_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* n_launches launches of a kernel that does nothing (one 64-thread block each). */
int32_t emc2_probe_empty(int32_t n_launches, void* stream);

/* dst[0 .. bytes) <- src[0 .. bytes): one 16-byte load and store per thread per step, grid-stride; bytes must be
 * a multiple of 16 and both pointers 16-byte aligned.  Moves 2 * bytes through HBM. */
int32_t emc2_probe_copy(void* dst, const void* src, int64_t bytes, void* stream);

/* dst[0 .. bytes) <- a constant pattern, 16 bytes per thread per step: a pure write stream of `bytes`. */
int32_t emc2_probe_fill(void* dst, int64_t bytes, void* stream);

/* n atomic ORs (no return value), one per thread, each on a pseudo-random 4-byte word of d_table[2^log2_words]: the
 * rate at which the memory system retires scattered read-modify-writes. */
int32_t emc2_probe_atomic(uint32_t* d_table, int32_t log2_words, int64_t n, void* stream);

/* Dense fp16 matrix-core loop without memory traffic: `blocks` blocks of 256 threads (4 waves) each issue
 * iters * 8 v_mfma_f32_32x32x16_f16 on eight independent accumulators (2 * 32 * 32 * 16 flop each), then add their
 * accumulators into d_sink[blocks * 256] (fp32) so the loop is not optimised away. */
int32_t emc2_probe_mfma_f16(int64_t iters, int32_t blocks, float* d_sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* EMC2_PROBE_H_ */
