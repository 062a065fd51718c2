/*
 * liec_testing.h -- testing, tuning and measurement aids of the LIEC-SGD library
 * declared in liec.h.  Nothing here is part of the method (Algorithm 1 and
 * Definitions 2-5 of the paper): these calls let the tests reach every path of
 * the threshold search behind top-k and random-k, and let the measurement
 * script time single kernels and calibrate hardware byte counters.  They are
 * exported by the same shared library and follow the same rules: plain
 * pointers, status codes, no exceptions.
 */
#ifndef LIEC_TESTING_H
#define LIEC_TESTING_H

#include "liec.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Testing aid for the threshold search behind top-k (Definition 2) and random-k
 * (Definition 3): makes every such row start the next liec_step's search in the
 * given mode -- 0: filter the band predicted by the previous step, 1: no
 * prediction (first radix digit over the whole row, then filter), 4: the general
 * search over the whole row.  The modes differ in cost only; the kept set is the
 * same in each.  Synchronises the stream.  LIEC_EINVAL for any other mode.
 */
liec_status liec_force_search_mode(liec_ctx *ctx, int32_t mode);

/*
 * Testing and tuning aid: the state the threshold search of row `row` (0 .. N - 1:
 * worker rows, N: the server's vector) is in after the last step, copied to the
 * HOST array `out` of 8 words: out[0] mode the next step starts in (0, 1 or 4 as
 * above), out[1] / out[2] lower / upper end of the band of keys predicted for the
 * next step, out[3] candidates the last step listed, out[4] steps so far whose
 * predicted band failed, out[5] the predictor's current swing (an eighth of the
 * band's half width unless a floor or the last change of the threshold decides),
 * out[6] 1 if the last step took the general search, out[7] reserved (0).
 * Synchronises the stream.  LIEC_EINVAL for a row out of range or one whose
 * operator has no threshold search.
 */
liec_status liec_get_search_state(liec_ctx *ctx, int32_t row, uint32_t *out);

/*
 * Testing aid for the general search (mode 4 above, also what constant or
 * mostly-zero rows fall to): several thread blocks share a row and wait for one
 * another between its phases; `polls` bounds each wait (default 65536, about 0.2 s).
 * A wait that runs out is not an error: one block then repeats the search on its
 * own, with the same result.  0 makes every wait run out at once, which is how the
 * tests reach that path.  LIEC_EINVAL for a negative value.
 */
liec_status liec_set_search_wait(liec_ctx *ctx, int32_t polls);

/*
 * Testing and tuning aid for top-k workers: the form of the candidate bitmap that
 * the threshold search leaves for the aggregation -- 0: one bit per 4 columns,
 * 1: one bit per 64-byte line (16 columns).  liec_create* picks it from d (the
 * second form from 4e7 columns up, where it measured faster); results do not
 * depend on it.  Takes effect with the next step.  LIEC_EINVAL for another value
 * or when the workers' operator is not top-k.
 */
liec_status liec_set_group_bitmap(liec_ctx *ctx, int32_t per_line);

/*
 * Testing and tuning aid for top-k workers: how the aggregation (Algorithm 1,
 * v = e + mean p^i) fetches the rows' candidates -- 0: row after row, 1: the
 * candidates of 8 rows requested together, then added in worker order.
 * liec_create* picks the second for rows under 2^23 columns, where the kernel is
 * bound by the latency of its dependent loads and it measured a third faster (it
 * is a fifth to a half slower on the long rows of the DNN-shaped workloads);
 * results do not depend on it.  Takes effect with the next step.  LIEC_EINVAL for
 * another value or when the workers' operator is not top-k.
 */
liec_status liec_set_gather_batching(liec_ctx *ctx, int32_t on);

/*
 * Per-kernel timing with HIP events on the context's stream, for measurement.
 * liec_profile_begin(ctx, max_steps, update_only) makes every following
 * liec_step record an event before and after each kernel it launches, or, with
 * update_only != 0, around the update kernel alone (the kernel that moves most
 * of the bytes; two events per step disturb the step least).  At most
 * max_steps steps are recorded, later ones run unrecorded.  liec_profile_end
 * synchronises, stops recording and fills HOST arrays: names[s] (static
 * strings), total_ms[s] and launches[s] for s < *n_slots (in: capacity of the
 * arrays, out: slots used).
 */
liec_status liec_profile_begin(liec_ctx *ctx, int32_t max_steps, int32_t update_only);
liec_status liec_profile_end(liec_ctx *ctx, int32_t *n_slots, const char **names, double *total_ms,
                             int64_t *launches);

/*
 * Measurement aid, not part of the method: a plain 128-bit device-to-device
 * copy kernel enqueued on `hip_stream` (hipStream_t as void*, NULL = null
 * stream).  dst and src are DEVICE pointers, 16-byte aligned, non-overlapping;
 * bytes must be a multiple of 16.  It gives the achievable streaming bandwidth
 * to quote next to the step's kernels and calibrates hardware byte counters.
 */
liec_status liec_device_copy(void *dst, const void *src, int64_t bytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* LIEC_TESTING_H */
