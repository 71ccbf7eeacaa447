/*
 * rh_noalloc.h - an entry point of librh.so that allocates nothing.
 *
 * For callers that cannot call hipMalloc: code under HIP graph capture, tight serving loops,
 * harnesses that forbid allocation.  rh_select_regions needs a context (rh_create allocates its
 * scratch tables); this variant needs none.
 */
#ifndef RH_NOALLOC_H
#define RH_NOALLOC_H

#include "rh.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Most frames one rh_select_regions_noalloc call can take: its per-frame and per-segment tables
 * are a fixed device array of 32 * RH_NOALLOC_MAX_FRAMES bytes (128 KiB) that every GPU the
 * library runs on holds until the process ends. */
#define RH_NOALLOC_MAX_FRAMES 4096

/*
 * Same selection, same outputs and same argument meaning as rh_select_regions (rh.h), for a batch
 * of F frames of mbh x mbw macroblocks, without a context: the work is enqueued on hip_stream
 * (a hipStream_t, NULL = the default stream) of the current device, on which all pointers must
 * live.  Calls no hipMalloc / hipFree and synchronises nothing.
 * Returns RH_E_CAPACITY when F > RH_NOALLOC_MAX_FRAMES, RH_E_SHAPE for non-positive sizes or more
 * than 2^31 - 1 macroblocks, RH_E_INVALID for null pointers, a bad mode or malformed segments
 * (nothing is launched and the outputs are untouched in all these cases), RH_E_DEVICE when a HIP
 * call fails.
 * All calls on one GPU share that GPU's table array, which keeps the last call's contents; a call
 * rewrites every entry it reads before reading it, so calls need no clearing between them, but
 * two calls whose kernels may overlap on one GPU (different streams, no ordering between them)
 * race on the tables and must not be made.
 */
rh_status rh_select_regions_noalloc(const float* importance, int32_t F, int32_t mbh, int32_t mbw,
                                    const rh_segment* segs, int32_t nseg, int32_t mode, uint8_t* mask,
                                    uint32_t* list, uint32_t* n_sel, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* RH_NOALLOC_H */
