/*
 * dash_profile.h -- measurement instrumentation of libdash.  Not part of the scheme and not needed by a caller of
 * dash.h: the benchmark uses it to time the kernel classes with HIP events on the stream they are launched on.
 */
#ifndef DASH_PROFILE_H
#define DASH_PROFILE_H

#include "dash.h"

#ifdef __cplusplus
extern "C" {
#endif

/* While enabled, every launch of the kernel
 * classes below is bracketed by two HIP events on its stream.  dash_profile_read synchronises,
 * returns the summed kernel time, the number of launches, the units processed (ciphertext rows for
 * GARBLE and for GARBLE_DIGITS, the fused kernel for the digit gates of a sign gadget; gates for EVAL,
 * label-digit MACs for LINEAR) and the algorithmic bytes moved in the
 * one-byte-per-digit layout (GARBLE per gate: input labels + function table + output zero label +
 * p rows; EVAL per gate: input labels + one row + output label), then clears the record. */
enum { DASH_PROF_GARBLE = 0, DASH_PROF_EVAL = 1, DASH_PROF_LINEAR = 2, DASH_PROF_GARBLE_DIGITS = 3, DASH_PROF_KINDS = 4 };
int dash_profile_enable(dash_ctx *ctx, int on);
int dash_profile_read(dash_ctx *ctx, int kind, double *ms, int64_t *launches, double *units, double *alg_bytes);

#ifdef __cplusplus
}
#endif
#endif /* DASH_PROFILE_H */
