/*
 * liec.h -- C ABI of the MI355X (gfx950) implementation of one compressed
 * iteration of LIEC-SGD (Algorithm 1 of the paper, the branches taken when the
 * iteration is not an averaging iteration), with N simulated workers batched
 * as the rows of an [N, d] fp32 tensor on one GPU.
 *
 * Per call of liec_step, for worker i = 0..N-1 and column j = 0..d-1:
 *   p^i  = C_w(g_i)                           worker compression (Alg. 1, worker part)
 *   v    = e + (1/N) sum_i p^i                server compensation
 *   p    = C_s(v)                             server compression, broadcast
 *   e   <- v - p                              global error update
 *   x^i <- x^i - lr * (p + (g_i - p^i))       local immediate error compensation
 * C_w / C_s are the scaled-sign operator (Definition 4), its blockwise form
 * (Definition 5), top-k (Definition 2), random-k (Definition 3) or the identity.
 * Conventions the definitions leave open:
 *   - scaled sign: scale = fp32(sum_j |v_j| / d) with the sum carried in fp64;
 *     sign is binary, v >= 0 (both zeros included) -> +scale, v < 0 -> -scale;
 *   - top-k: magnitudes compare through the integer key (bits & 0x7fffffff);
 *     among equal keys the lower index wins; exactly k entries are kept;
 *   - random-k: the k-subset of a draw is the k indices of highest priority under
 *     a counter-based generator keyed by (seed, draw, row) -- see liec_set_random;
 *   - the N messages are added in worker order in fp32, then one fused
 *     multiply-add by 1/N adds e; the update is one fused multiply-add by -lr.
 *
 * All tensor arguments are DEVICE pointers to fp32, contiguous, row-major and
 * owned by the caller; nothing here takes or returns torch types.  The library
 * owns only scratch memory (allocated by liec_create*, released by
 * liec_destroy).  No entry point throws; every failure is a status code.
 * A context serves one caller thread at a time.
 */
#ifndef LIEC_H
#define LIEC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct liec_ctx liec_ctx; /* opaque */

typedef enum {
    LIEC_OK = 0,
    LIEC_EINVAL = 1,     /* bad argument (null pointer, size, k, lr, overlap)   */
    LIEC_ENOMEM = 2,     /* host or device allocation failed                    */
    LIEC_EDEVICE = 3,    /* a HIP call failed; sticky until liec_destroy        */
    LIEC_ENONFINITE = 4  /* liec_get_info only: last step saw a NaN or Inf      */
} liec_status;

typedef enum {
    LIEC_COMP_IDENTITY = 0, /* C(v) = v; with it on both sides the step is P-SGD */
    LIEC_COMP_SIGN = 1,     /* Definition 4 */
    LIEC_COMP_TOPK = 2,     /* Definition 2 */
    LIEC_COMP_BLOCKSIGN = 3, /* Definition 5: Definition 4 on each block of liec_set_blocks */
    LIEC_COMP_RANDK = 4     /* Definition 3: k coordinates drawn uniformly, see liec_set_random */
} liec_comp;

/* Scalars describing the LAST completed step (filled by liec_get_info). */
typedef struct {
    int32_t N;
    int64_t d;
    int32_t worker_comp, server_comp;
    int64_t worker_k, server_k;
    float lr;
    int64_t steps_done;
    float server_scale;       /* scaled sign on the server: ||v||_1 / d            */
    double server_l1;         /* scaled sign on the server: ||v||_1 (fp64 sum)     */
    uint32_t server_tau_key;  /* top-k on the server: magnitude key of k-th entry
                                 (random-k: priority of the k-th kept index)       */
    int64_t server_cutoff;    /* top-k / random-k on the server: largest kept index
                                 among entries whose key equals server_tau_key     */
    int32_t nonfinite;        /* 1 if a NaN/Inf reached an L1 sum or a top-k key   */
    int32_t slow_rows;        /* top-k / random-k: rows (workers + server) whose last
                                 threshold search fell to the general single-block
                                 search -- constant or near-constant rows; results are
                                 exact either way, such rows only take much longer   */
    int64_t band_misses;      /* top-k: row-steps, since the context was created, whose
                                 threshold fell outside the band predicted from the
                                 previous steps, so that the row needed two more passes
                                 (steps without a prediction, such as the first, do not
                                 count); results are exact either way               */
} liec_info;

/*
 * liec_create: same operator C and same k on the worker and the server side
 * (the form Algorithm 1 is written in), launching on the default (null) stream.
 *   out         receives the context (host pointer to a host pointer)
 *   1 <= N <= 65535   number of simulated workers (rows)
 *   1 <= d < 2^31 - 2^20   model dimension (columns); also N * (d / 1024 + 4097) < 2^31
 *   k           kept entries for LIEC_COMP_TOPK / LIEC_COMP_RANDK, 1 <= k <= d; ignored otherwise
 *   lr          learning rate eta, finite
 * Allocates the context's device scratch: 4d bytes for v; N * d / 8 for sign or
 * random-k bitmaps; with top-k or random-k on either side also (N + 1) * 8 *
 * (min(d / 16, 8 k) + 4096) for the candidate lists, N * d / 32 for the group bitmap and about
 * 50 KiB per row of histograms and short lists; d / 8 for the server's sign bits or d / 32 for its
 * group bitmap (liec_scratch_bytes reports the total).  The
 * context belongs to the HIP device that is current at this call: every later call
 * on it makes that device current for its own duration and puts the caller's back.
 */
liec_status liec_create(liec_ctx **out, int32_t N, int64_t d, liec_comp compressor, int64_t k,
                        float lr);

/*
 * liec_create_ex: different operators / k on the two sides, and the HIP stream
 * (a hipStream_t passed as void*, NULL = null stream) all work is enqueued on.
 * The stream must belong to the device current at this call and outlive the context.
 */
liec_status liec_create_ex(liec_ctx **out, int32_t N, int64_t d, liec_comp worker_comp,
                           int64_t worker_k, liec_comp server_comp, int64_t server_k, float lr,
                           void *hip_stream);

/*
 * liec_step: one compressed iteration of Algorithm 1 as stated at the top.
 *   grads      [N, d] device, read only   stochastic gradients g_i of this iteration
 *   x          [N, d] device, in/out      local models x^i (they differ between workers)
 *   server_err [d]    device, in/out      global error e_t on entry, e_{t+1} on return
 * The three buffers must not overlap.  Any alignment is accepted; rows that are
 * 16-byte aligned (base pointers 16-byte aligned and d % 4 == 0) take the
 * 128-bit load path, anything else a slower element-wise path.
 * Asynchronous: work is enqueued on the context's stream and the call returns
 * without synchronising, allocating or copying to the host.  Inputs must be
 * finite; otherwise results are unspecified and liec_get_info reports it.
 */
liec_status liec_step(liec_ctx *ctx, const float *grads, float *x, float *server_err);

/*
 * liec_step_sync: the averaging iteration of Algorithm 1 (taken when (t+1) is a
 * multiple of the averaging period, which the caller keeps): gradients and
 * models are exchanged uncompressed, so
 *   v = e + (1/N) sum_i g_i ;  e <- v - v = 0 ;  x^i <- (1/N) sum_i x^i - lr * v  for every i.
 * Same buffers, layout, alignment rules, ownership, asynchrony and errors as
 * liec_step; the context's operators play no part.  Both sums add in worker
 * order in fp32.
 */
liec_status liec_step_sync(liec_ctx *ctx, const float *grads, float *x, float *server_err);

/*
 * liec_iteration: iteration t (0-based) of Algorithm 1 as a whole: the averaging
 * iteration (liec_step_sync) when period >= 2 and (t + 1) is a multiple of
 * period, the compressed iteration (liec_step) otherwise; period = 0 means no
 * averaging iterations.  The paper sets the period to floor(1 / delta) and uses
 * 32 and 100 in its experiments.  LIEC_EINVAL for t < 0, period < 0 or period = 1;
 * otherwise as the call it forwards to.
 */
liec_status liec_iteration(liec_ctx *ctx, int64_t t, int64_t period, const float *grads, float *x,
                           float *server_err);

/*
 * liec_set_blocks: the block table of Blockwise-SignSGD (Definition 5), needed
 * before the first liec_step of a context that uses LIEC_COMP_BLOCKSIGN on
 * either side (liec_step returns LIEC_EINVAL without it).
 *   offsets  HOST array of nblocks + 1 column offsets, offsets[0] = 0,
 *            offsets[nblocks] = d, strictly increasing (block b is the columns
 *            offsets[b] .. offsets[b+1]-1 and has its own length d_b)
 *   nblocks  1 .. 65536 (one block gives Definition 4)
 * Synchronises the stream, replaces any earlier table and allocates
 * O((N + 1) * (d / 4096 + nblocks)) bytes of device scratch.
 */
liec_status liec_set_blocks(liec_ctx *ctx, const int64_t *offsets, int32_t nblocks);

/*
 * Synchronises the stream and copies the per-block scales of the last step to
 * HOST arrays: worker_scales [N * nblocks] (row-major) and server_scales
 * [nblocks]; either may be NULL; a side that does not use LIEC_COMP_BLOCKSIGN
 * gets zeros.  LIEC_EINVAL without a block table.
 */
liec_status liec_get_block_scales(liec_ctx *ctx, float *worker_scales, float *server_scales);

/*
 * Bytes of one message C(v) on the wire, as the paper counts communication
 * (one bit per element for the sign operators, "32x"): identity 4d; scaled sign
 * ceil(d/8) + 4 (bits + scale); blockwise ceil(d/8) + 4*nblocks; top-k and
 * random-k 8k (32-bit index + fp32 value per kept entry; a receiver that shares
 * the seed could rebuild random-k's indices itself, which is not counted here).
 * -1 for bad arguments.  Host only.
 */
int64_t liec_message_bytes(liec_comp comp, int64_t d, int64_t k, int32_t nblocks);

/*
 * Average bytes moved per iteration of Algorithm 1 (the quantity of the paper's
 * communication-cost table): a compressed iteration moves N worker messages up
 * and the server message down to each of the N workers; every period-th
 * iteration is an averaging iteration that moves N full gradients up and N full
 * vectors down, plus the N models each way when count_model_exchange != 0 (the
 * paper's table leaves them out).  period = 0 means compressed iterations only;
 * period = 1 is rejected.  Host arithmetic only; writes *bytes_per_iteration.
 */
liec_status liec_comm_cost(int32_t N, int64_t d, liec_comp worker_comp, int64_t worker_k,
                           liec_comp server_comp, int64_t server_k, int32_t nblocks, int32_t period,
                           int32_t count_model_exchange, double *bytes_per_iteration);

/*
 * Wire bits of worker `worker`'s (blockwise) scaled-sign message of the last
 * step: ceil(d/8) bytes written to the DEVICE buffer `out`, bit j % 8 of byte
 * j / 8 set when g_j < 0, unused bits zero.  Enqueued on the context's stream.
 * The scale(s) that complete the message come from liec_get_worker_desc /
 * liec_get_block_scales.  LIEC_EINVAL unless the worker operator is a sign
 * operator and a step has run.
 */
liec_status liec_pack_sign_bits(liec_ctx *ctx, int32_t worker, uint8_t *out);

/*
 * Decompression of such a message into the dense vector p (DEVICE, [d]):
 * p_j = -s or +s, with s = scales[0] (blockwise == 0) or the scale of the block
 * holding j (blockwise != 0; scales has nblocks entries, the context's block
 * table applies).  bits: DEVICE, ceil(d/8) bytes.  scales: HOST, read before
 * the call returns.  Enqueued on the context's stream; with blockwise == 0 the
 * call neither copies nor synchronises (the scale travels with the launch), with
 * blockwise != 0 the scales are first copied to the device synchronously.
 */
liec_status liec_unpack_sign_message(liec_ctx *ctx, const uint8_t *bits, const float *scales,
                                     int32_t blockwise, float *p_out);

/*
 * Wire form of worker `worker`'s top-k (Definition 2) or random-k (Definition 3)
 * message of the last step:
 * its worker_k kept entries as (index, value) pairs in increasing index order,
 * written to the DEVICE arrays idx_out / val_out (worker_k entries each, 8k
 * bytes in all).  `grads` must be the [N, d] DEVICE tensor the last liec_step
 * was given (the library does not keep it).  Enqueued on the context's stream;
 * the first call allocates a small scratch array.
 */
liec_status liec_pack_topk_message(liec_ctx *ctx, const float *grads, int32_t worker, uint32_t *idx_out,
                                   float *val_out);

/*
 * Decompression of such a message: p_out (DEVICE, [d]) is zero except
 * p_out[idx[r]] = val[r] for r < k.  idx / val: DEVICE arrays of k entries with
 * distinct indices below d.
 */
liec_status liec_unpack_topk_message(liec_ctx *ctx, const uint32_t *idx, const float *val, int64_t k,
                                     float *p_out);

/*
 * Telemetry: the l2 norm of a DEVICE vector of n fp32 values, e.g. of server_err:
 * the norm of the error variable is what Lemma 1 bounds and what the paper plots
 * to show the effect of immediate compensation.  Summed in fp64 in a fixed order
 * on the context's stream (after the work already enqueued there, using the
 * context's scratch: do not call it between liec_step's kernels from another
 * thread), then the stream is synchronised and the norm written to the HOST
 * double *norm_out.  Not part of the step.
 */
liec_status liec_l2_norm(liec_ctx *ctx, const float *vec, int64_t n, double *norm_out);

/*
 * liec_l2_norm_static: liec_l2_norm for callers that cannot allocate device
 * memory or wait for the device -- code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  It needs no context, allocates
 * nothing, copies nothing to the host and does not synchronise: two kernels are
 * enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = null stream) of
 * the current device, and the norm is written to the DEVICE double *norm_out
 * (8-byte aligned) when they have run.
 *   vec   DEVICE, n fp32 values, 4-byte aligned, read only
 *   n     1 .. LIEC_L2_STATIC_MAX_N; anything else is LIEC_EINVAL
 * The block partials live in a 32 KiB array that is part of the library's image
 * on every GPU it runs on (held until the process ends); its address on a device
 * is looked up at the first call on that device, which therefore should be made
 * outside a capture.  All calls on one GPU share that array: calls that may
 * overlap there (two streams, two threads) race and must be serialised by the
 * caller.  The sum of squares is carried in fp64 in a fixed order; the result
 * can differ from liec_l2_norm's in the last bits (the number of partials
 * differs), not more.
 */
#define LIEC_L2_STATIC_MAX_N ((int64_t)1 << 32)
liec_status liec_l2_norm_static(const float *vec, int64_t n, double *norm_out, void *hip_stream);

/* Learning-rate schedules (the paper decays eta during training): takes effect
 * from the next liec_step. */
liec_status liec_set_lr(liec_ctx *ctx, float lr);

/*
 * Random-k (Definition 3: keep the coordinates of a set S drawn uniformly from
 * the k-element subsets of [d]).  The draw of row r (worker index, or N for the
 * server) in the compressed iteration number `draw` under `seed` is made by a
 * counter-based generator, so that it can be reproduced anywhere:
 *   mix(z): z = (z ^ z >> 30) * 0xBF58476D1CE4E5B9; z = (z ^ z >> 27) * 0x94D049BB133111EB; z ^ z >> 31
 *   G = 0x9E3779B97F4A7C15;  s = mix(mix(mix(seed + G) + draw + G) + r + G)        (64-bit, wrapping)
 *   h = j ^ low32(s); h ^= h >> 16; h *= 0x85EBCA6B; h ^= h >> 13; h += high32(s);
 *   h *= 0xC2B2AE35; h ^= h >> 16;  priority(j) = h >> 1                            (32-bit, wrapping)
 * S = the k indices of highest priority, equal priorities (at most pairs) to the
 * lower index.  liec_set_random sets the seed and the number of the next draw
 * (both 0 in a new context); every liec_step uses one draw number and then
 * advances it by one (liec_step_sync does not).  Both live in device memory and
 * the step advances the number on the device, so a liec_step captured into a HIP
 * graph makes a new draw at every replay.  liec_get_random reads them back, e.g.
 * for a checkpoint; both calls synchronise the context's stream.  The gradients are not read to make a draw, so
 * non-finite inputs are not reported for this operator.
 */
liec_status liec_set_random(liec_ctx *ctx, uint64_t seed, uint64_t draw);
liec_status liec_get_random(liec_ctx *ctx, uint64_t *seed, uint64_t *draw);

/* Synchronises the stream and copies the scalars of the last step to the host
 * struct `info`.  Returns LIEC_ENONFINITE (with `info` filled) if that step met
 * a NaN or Inf. */
liec_status liec_get_info(liec_ctx *ctx, liec_info *info);

/*
 * Synchronises the stream and copies the per-worker message descriptors of the
 * last step into HOST arrays of length N; any pointer may be NULL.
 *   scales  scaled sign: ||g_i||_1 / d
 *   l1      scaled sign: ||g_i||_1 as summed in fp64
 *   tau     top-k: magnitude key of the k-th kept entry of g_i (random-k: its priority)
 *   cutoff  top-k / random-k: largest kept index among entries of g_i whose key equals tau
 * Arrays that do not apply to the worker operator are zero-filled.
 */
liec_status liec_get_worker_desc(liec_ctx *ctx, float *scales, double *l1, uint32_t *tau,
                                 int64_t *cutoff);

/* Releases the scratch memory and the context.  NULL is accepted. */
void liec_destroy(liec_ctx *ctx);

/* Static description of a status code. */
const char *liec_status_string(liec_status s);

/* Bytes of device scratch the context holds. */
int64_t liec_scratch_bytes(const liec_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* LIEC_H */
