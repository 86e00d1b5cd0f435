/*
 * probes.h -- C ABI of libmquant_probes.so, the benchmark's measurement probes.
 * Not part of the method and not part of libmquant: they measure what this chip
 * attains on the resources the hot path is bound by.  DEVICE calls, asynchronous
 * on `stream`, status codes as in mquant.h.
 */
#ifndef MQUANT_PROBES_H
#define MQUANT_PROBES_H

#include <stdint.h>

#include "mquant.h"

#ifdef __cplusplus
extern "C" {
#endif

/* int8 operations one mqprobe_mfma_i8(iters) launch performs. */
int64_t mqprobe_mfma_i8_ops(int32_t iters);

/*
 * An MFMA-only loop (v_mfma_i32_32x32x32_i8, eight independent accumulators per
 * wave, four waves per SIMD on every CU) whose operands are read once from
 * data_dev (>= 4096 bytes, 16-byte aligned; its contents set the data-dependent
 * matrix clock: zeros, or random bytes as in a real product).  sink_dev: one
 * int32 that is practically never written.
 */
int mqprobe_mfma_i8(int32_t iters, const void *data_dev, int64_t data_bytes, int32_t *sink_dev,
                    mquant_stream_t stream);

/* A read-only stream over data_bytes of data_dev (16-byte aligned), 16 bytes per lane. */
int mqprobe_hbm_read(const void *data_dev, int64_t data_bytes, uint32_t *sink_dev,
                     mquant_stream_t stream);

/* A kernel that does nothing, `groups` work-groups of `threads` threads (a multiple of 64,
 * at most 1024): back to back it gives the launch-to-launch floor. */
int mqprobe_empty(int32_t groups, int32_t threads, mquant_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* MQUANT_PROBES_H */
