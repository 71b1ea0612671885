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

/* AES-128 encryption alone (FIPS-197), in each form the library holds, for measuring them against each other
 * and for checking each against the standard: out[i] = AES_key applied `repeat` times to in[i], i < n_blocks.
 *   variant 0: T-tables in LDS, one 4 KB copy per workgroup (what small gate launches use);
 *   variant 1: T-tables replicated per LDS bank, 64 KB per workgroup (what large gate launches use);
 *   variant 2: bit planes, 32 blocks per lane, no tables; n_blocks must be a multiple of 2048 (DASH_ESIZE).
 *   variant 3: all four T-tables replicated per LDS bank, 128 KB per workgroup (no gate kernel uses it: they run
 *              slower with half the waves per SIMD).
 * key: 16 bytes, host.  in, out: device, 16 bytes per block, may be the same buffer.  Enqueues on `stream`
 * (variant 2 first waits for the stream and copies its key masks into a per-GPU array of the library, so calls
 * of variant 2 that overlap on one GPU race).  Allocates nothing. */
int dash_profile_aes(dash_ctx *ctx, int variant, const uint8_t *key, const void *in, void *out, uint64_t n_blocks,
                     int repeat, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* DASH_PROFILE_H */
