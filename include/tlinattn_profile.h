/*
 * libtlinattn - measurement aid, kept apart from the attention interface in tlinattn.h.
 *
 * Per-kernel timing for benchmarks: while enabled, every kernel the library launches is
 * bracketed by a pair of HIP events recorded on the launch stream.  Unlike the attention entry
 * points these two calls create runtime objects (the events, on first use, kept for reuse) and
 * tlin_profile_read synchronises with them.  Leave it off otherwise.
 */
#ifndef TLINATTN_PROFILE_H
#define TLINATTN_PROFILE_H

#include "tlinattn.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Switches the bracketing on (non-zero) or off. */
tlin_status tlin_profile_enable(int32_t enable);

/* Waits for the recorded events, returns the summed durations in milliseconds and the launch
 * counts per kernel class - [0] history partition kernel (in a layer call: the launch that holds
 * the history partitions and the window blocks), [1] window causal kernel, [2] merge kernel -
 * and clears the record. */
tlin_status tlin_profile_read(double ms[3], int64_t launches[3]);

/* Enqueues a kernel that does nothing but read the first bytes (rounded down to a multiple of
 * 32 KiB times the grid) of a device buffer of at least 1 MiB, 16-byte aligned, with plain
 * (nontemporal == 0) or non-temporal loads: timed by the caller, it shows the read rate this GPU
 * delivers to a kernel without any other work, the practical ceiling for the HBM-bound attention
 * shapes.  The buffer is not modified. */
tlin_status tlin_profile_stream_read(const void *buf, size_t bytes, int32_t nontemporal, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TLINATTN_PROFILE_H */
