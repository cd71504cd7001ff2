/*
 * fcv2_diag.h -- diagnostics exported by libfcv2 next to the codec (include/fcv2.h).  Nothing here is part of the method
 * of arxiv 2508.03760; the benchmark uses it as a yardstick.
 */
#ifndef FCV2_DIAG_H
#define FCV2_DIAG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* A plain streaming copy of `bytes` (a multiple of 16) from src_dev to dst_dev (DEVICE pointers, 16-byte aligned),
 * 16 bytes per lane, stores with the non-temporal hint, enqueued on hip_stream.  Returns an FCV2_* status.  Used to
 * measure the practical HBM ceiling next to the codec kernels and to calibrate memory-traffic counters against a
 * transfer of known size. */
int fcv2_stream_copy(const void* src_dev, void* dst_dev, uint64_t bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif
