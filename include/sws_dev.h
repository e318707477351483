/*
 * sws_dev.h — measurement and test knobs of libsws.  NOT part of the reentrant contract of sws.h:
 * the settings are process-wide, they change which kernel variant or tiling the entry points of
 * sws.h choose (never the result beyond summation order), and a change made while another thread
 * is inside an entry point takes effect at an unspecified launch.  Each knob is a single atomic
 * integer, so concurrent use is a race in policy only, never in memory.  Production callers do
 * not need this header; the parity tests use it to force every kernel variant over the same
 * inputs and the benchmark uses it for A/B timings.
 */
#ifndef SWS_DEV_H
#define SWS_DEV_H

#include "sws.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Known keys: "slide_variant", "pool2d_variant", "conv1d_variant", "conv2d_variant",
 * "copy_variant" (0 = automatic choice), "slide_chunk" (tiling / store-policy bits) and
 * "slide_group" (tiles per work unit).  Returns SWS_ERR_INVALID_ARG for an unknown key. */
sws_status sws_set_option(const char *key, int64_t value);

#ifdef __cplusplus
}
#endif

#endif /* SWS_DEV_H */
