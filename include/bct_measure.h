/* libbct -- measurement aids.
 *
 * Not part of the decode path: per-launch timing and a plain copy kernel, used by bench.py and the
 * profiles to put numbers beside the path (time of each launch of a decode step; the practical
 * ceiling of a 1:1 read/write stream; a copy of known size to calibrate rocprofv3's HBM counters).
 * Same conventions as bct.h: C ABI, device pointers unless a parameter says host, caller's stream.
 */
#ifndef BCT_MEASURE_H
#define BCT_MEASURE_H

#include "bct.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Per-kernel timing of decode steps with HIP events recorded
 * on the caller's stream around each launch (scores, MV pass, merge).
 * bct_profile_enable(c, n) keeps events for the next n decode steps (n = 0
 * switches it off and releases the events).  bct_profile_read waits for the
 * recorded events, returns how many steps were recorded and the mean
 * duration in milliseconds of each launch (host pointers, any may be NULL),
 * and starts over.  Not for use under graph capture. */
bct_status bct_profile_enable(bct_cache* c, uint32_t n_steps);
bct_status bct_profile_read(bct_cache* c, uint32_t* n_recorded, float* ms_scores, float* ms_mv_pass,
                            float* ms_merge);

/* A plain device-to-device copy kernel (16-byte vectors),
 * n_bytes a multiple of 16, src/dst 16-byte aligned.  Reads n_bytes and
 * writes n_bytes; used to calibrate HBM counters and as the practical ceiling
 * for a 1:1 read/write stream such as the section 3.4 update. */
bct_status bct_stream_copy(void* dst, const void* src, size_t n_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* BCT_MEASURE_H */
