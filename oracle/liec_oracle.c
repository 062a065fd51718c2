/*
 * liec_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow CPU statement (single-threaded unless built with -fopenmp, which only spreads
 * the independent workers of a step over threads) of one compressed iteration of
 * LIEC-SGD (Algorithm 1, the ELSE branches), of its averaging iteration (the IF
 * branches) and of the compression operators it uses (Definition 2 top-k,
 * Definition 4 scaled sign, Definition 5 blockwise scaled sign, and the identity
 * operator that the uncompressed branch of Algorithm 1 amounts to).
 *
 * Nothing here is shared with the HIP library: no header, constant, helper or
 * table is common to both.  Only tests, the smoke check and the bench's CPU
 * baseline leg may call into this file.
 *
 * Build with -O2 -ffp-contract=off and never -ffast-math: every fp32
 * expression below is meant to be one IEEE-754 operation, exactly as written.
 *
 * Readings taken where the paper leaves a choice (each is also listed in the
 * design notes of the repository):
 *   - Definition 4: the L1 norm is summed in extended precision (x86 long
 *     double, 64-bit significand), rounded to fp64, divided by d in fp64 and
 *     rounded once to fp32.  sign(.) is binary: v >= 0 (including both zeros)
 *     maps to +1, v < 0 to -1, so that the message really is one bit per
 *     element and ||C(v)||_1 = d * scale holds without exception.
 *   - Definition 2: the permutation pi is not unique when magnitudes tie; the
 *     lower index wins, and exactly k entries are kept even if some are zero.
 *     Magnitudes are compared through the integer key (bits & 0x7fffffff),
 *     which orders finite fp32 magnitudes exactly as |.| does.
 *   - Definition 3: the k-subset S is drawn by giving every index a priority
 *     from a counter-based generator keyed by (seed, draw, row) and keeping the
 *     k indices of highest priority (ties, at most pairs, to the lower index).
 *     `draw` counts the compressed iterations, `row` is the worker index, or N
 *     for the server.  The generator is stated below; the HIP library carries
 *     its own statement of it.
 *   - Algorithm 1, server average: the N messages are added in worker order
 *     in fp32 starting from +0, then one fused multiply-add with 1/N adds the
 *     global error.
 *   - Algorithm 1, worker update: the cached local error g - p^i is formed
 *     first and then added to the broadcast p (the order the prose after the
 *     algorithm describes), then one fused multiply-add with -eta.
 *
 * Parity pins for every function in this file live in tests/test_oracle_*.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_IDENTITY = 0, ORACLE_SIGN = 1, ORACLE_TOPK = 2, ORACLE_BLOCKSIGN = 3, ORACLE_RANDK = 4 };

/* What a compressed message consists of besides the per-element part. */
typedef struct {
    float scale;          /* scaled sign: ||v||_1 / d                         */
    double l1;            /* scaled sign: ||v||_1 rounded to fp64              */
    uint32_t tau_key;     /* top-k: magnitude key of the k-th kept entry       */
    int64_t cutoff;       /* top-k: index of the k-th kept entry (largest kept
                             index among entries whose key equals tau_key)    */
    int64_t count_above;  /* top-k: number of entries with key > tau_key       */
} oracle_desc;

static uint32_t abs_key(float v)
{
    uint32_t u;
    memcpy(&u, &v, sizeof u);
    return u & 0x7fffffffu;
}

/* Definition 4 (scaled sign). p may be NULL when only the scale is wanted. */
static void compress_sign(const float *v, int64_t d, float *p, oracle_desc *desc)
{
    long double sum = 0.0L;
    for (int64_t j = 0; j < d; ++j)
        sum += fabsl((long double)v[j]);
    double l1 = (double)sum;
    float scale = (float)(l1 / (double)d);
    if (p)
        for (int64_t j = 0; j < d; ++j)
            p[j] = (v[j] < 0.0f) ? -scale : scale;
    desc->scale = scale;
    desc->l1 = l1;
}

static int cmp_u64_desc(const void *a, const void *b)
{
    uint64_t x = *(const uint64_t *)a, y = *(const uint64_t *)b;
    return (x < y) - (x > y);
}

/* Definition 2 (top-k), ties to the lower index.  Sort every index by
 * (magnitude key descending, index ascending) and keep the first k. */
static int compress_topk(const float *v, int64_t d, int64_t k, float *p, oracle_desc *desc)
{
    if (k < 1 || k > d || d > (int64_t)0x7fffffff)
        return 1;
    uint64_t *order = (uint64_t *)malloc((size_t)d * sizeof *order);
    if (!order)
        return 2;
    for (int64_t j = 0; j < d; ++j)
        order[j] = ((uint64_t)abs_key(v[j]) << 32) | (uint64_t)(0xffffffffu - (uint32_t)j);
    qsort(order, (size_t)d, sizeof *order, cmp_u64_desc);
    if (p) {
        for (int64_t j = 0; j < d; ++j)
            p[j] = 0.0f;
        for (int64_t r = 0; r < k; ++r) {
            int64_t j = (int64_t)(0xffffffffu - (uint32_t)(order[r] & 0xffffffffu));
            p[j] = v[j];
        }
    }
    uint32_t tau = (uint32_t)(order[k - 1] >> 32);
    int64_t above = 0;
    while (above < k && (uint32_t)(order[above] >> 32) > tau)
        ++above;
    desc->tau_key = tau;
    desc->cutoff = (int64_t)(0xffffffffu - (uint32_t)(order[k - 1] & 0xffffffffu));
    desc->count_above = above;
    free(order);
    return 0;
}

/* Definition 3 (random-k): the generator behind "S is sampled uniformly from the k-element
 * subsets".  One 64-bit stream word per (seed, draw, row) through three rounds of a 64-bit
 * multiply-xorshift finalizer (the SplitMix64 output function with its additive constant), then
 * per index j a keyed 32-bit multiply-xorshift permutation of j (two odd multipliers, the
 * stream's low word mixed in before the first and its high word between the two).  Every step
 * of the 32-bit part is a bijection of 32-bit words, so distinct indices get distinct 32-bit
 * words; the priority is that word without its lowest bit (31 bits, like a magnitude key). */
static uint64_t mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

uint64_t liec_oracle_randk_stream(uint64_t seed, uint64_t draw, uint32_t row)
{
    const uint64_t gamma = 0x9E3779B97F4A7C15ull;
    uint64_t z = mix64(seed + gamma);
    z = mix64(z + draw + gamma);
    z = mix64(z + (uint64_t)row + gamma);
    return z;
}

uint32_t liec_oracle_randk_priority(uint64_t stream, uint32_t j)
{
    uint32_t h = j ^ (uint32_t)(stream & 0xffffffffu);
    h ^= h >> 16;
    h *= 0x85EBCA6Bu;
    h ^= h >> 13;
    h += (uint32_t)(stream >> 32);
    h *= 0xC2B2AE35u;
    h ^= h >> 16;
    return h >> 1;
}

/* Priorities of the indices 0 .. d-1 in one draw (for tests of the generator). */
void liec_oracle_randk_priorities(uint64_t seed, uint64_t draw, uint32_t row, int64_t d, uint32_t *out)
{
    const uint64_t stream = liec_oracle_randk_stream(seed, draw, row);
    for (int64_t j = 0; j < d; ++j)
        out[j] = liec_oracle_randk_priority(stream, (uint32_t)j);
}

/* Definition 3: keep the k indices of highest priority (priority descending, index ascending),
 * zero elsewhere.  The descriptor carries the priority of the k-th kept index and that index. */
static int compress_randk(const float *v, int64_t d, int64_t k, uint64_t seed, uint64_t draw,
                          uint32_t row, float *p, oracle_desc *desc)
{
    if (k < 1 || k > d || d > (int64_t)0x7fffffff)
        return 1;
    uint64_t *order = (uint64_t *)malloc((size_t)d * sizeof *order);
    if (!order)
        return 2;
    const uint64_t stream = liec_oracle_randk_stream(seed, draw, row);
    for (int64_t j = 0; j < d; ++j)
        order[j] = ((uint64_t)liec_oracle_randk_priority(stream, (uint32_t)j) << 32) |
                   (uint64_t)(0xffffffffu - (uint32_t)j);
    qsort(order, (size_t)d, sizeof *order, cmp_u64_desc);
    if (p) {
        for (int64_t j = 0; j < d; ++j)
            p[j] = 0.0f;
        for (int64_t r = 0; r < k; ++r) {
            int64_t j = (int64_t)(0xffffffffu - (uint32_t)(order[r] & 0xffffffffu));
            p[j] = v[j];
        }
    }
    uint32_t tau = (uint32_t)(order[k - 1] >> 32);
    int64_t above = 0;
    while (above < k && (uint32_t)(order[above] >> 32) > tau)
        ++above;
    desc->tau_key = tau;
    desc->cutoff = (int64_t)(0xffffffffu - (uint32_t)(order[k - 1] & 0xffffffffu));
    desc->count_above = above;
    free(order);
    return 0;
}

/* Definition 5 (Blockwise-SignSGD): Definition 4 applied independently to each of the B consecutive
 * blocks [off[b], off[b+1]) of v, each with its own length d_b = off[b+1] - off[b] (off[0] = 0,
 * off[B] = d, strictly increasing).  scales [B] receives the per-block scales. */
static int compress_blocksign(const float *v, int64_t d, const int64_t *off, int32_t B, float *p,
                              float *scales)
{
    if (!off || B < 1 || off[0] != 0 || off[B] != d)
        return 1;
    for (int32_t b = 0; b < B; ++b) {
        if (off[b + 1] <= off[b])
            return 1;
        oracle_desc blk;
        compress_sign(v + off[b], off[b + 1] - off[b], p ? p + off[b] : NULL, &blk);
        if (scales)
            scales[b] = blk.scale;
    }
    return 0;
}

/* p = C(v) for the chosen operator.  Returns 0 on success.  (seed, draw, row) name the random
 * draw of Definition 3 and are ignored by the other operators. */
int liec_oracle_compress_rng(int comp, const float *v, int64_t d, int64_t k, const int64_t *off,
                             int32_t B, uint64_t seed, uint64_t draw, uint32_t row, float *p,
                             oracle_desc *desc, float *block_scales);

int liec_oracle_compress_ex(int comp, const float *v, int64_t d, int64_t k, const int64_t *off,
                            int32_t B, float *p, oracle_desc *desc, float *block_scales)
{
    return liec_oracle_compress_rng(comp, v, d, k, off, B, 0, 0, 0, p, desc, block_scales);
}

int liec_oracle_compress(int comp, const float *v, int64_t d, int64_t k, float *p,
                         oracle_desc *desc)
{
    return liec_oracle_compress_ex(comp, v, d, k, NULL, 0, p, desc, NULL);
}

int liec_oracle_compress_rng(int comp, const float *v, int64_t d, int64_t k, const int64_t *off,
                             int32_t B, uint64_t seed, uint64_t draw, uint32_t row, float *p,
                             oracle_desc *desc, float *block_scales)
{
    oracle_desc local;
    if (!desc)
        desc = &local;
    memset(desc, 0, sizeof *desc);
    if (!v || d < 1)
        return 1;
    switch (comp) {
    case ORACLE_IDENTITY:
        if (p)
            for (int64_t j = 0; j < d; ++j)
                p[j] = v[j];
        return 0;
    case ORACLE_SIGN:
        compress_sign(v, d, p, desc);
        return 0;
    case ORACLE_TOPK:
        return compress_topk(v, d, k, p, desc);
    case ORACLE_BLOCKSIGN:
        return compress_blocksign(v, d, off, B, p, block_scales);
    case ORACLE_RANDK:
        return compress_randk(v, d, k, seed, draw, row, p, desc);
    default:
        return 1;
    }
}

/* Algorithm 1, server compensation: v = e + (1/N) sum_i p^i.
 * P is [N, d] row-major (the N uplink messages, decompressed). */
void liec_oracle_server_average(const float *P, int32_t N, int64_t d, const float *e, float *v)
{
    const float inv_n = 1.0f / (float)N;
    for (int64_t j = 0; j < d; ++j) {
        float acc = 0.0f;
        for (int32_t i = 0; i < N; ++i)
            acc = acc + P[(size_t)i * (size_t)d + (size_t)j];
        v[j] = fmaf(acc, inv_n, e[j]);
    }
}

/* Algorithm 1, global error update: e_{t+1} = v_t - p_t. */
void liec_oracle_error_update(const float *v, const float *p, int64_t d, float *e_next)
{
    for (int64_t j = 0; j < d; ++j)
        e_next[j] = v[j] - p[j];
}

/* Algorithm 1, worker update with local immediate compensation, one worker:
 * x^i <- x^i - eta * (p + (g_i - p^i)). */
void liec_oracle_worker_update(const float *g_i, const float *p_i, const float *p, int64_t d,
                               float lr, float *x_i)
{
    for (int64_t j = 0; j < d; ++j) {
        float local_err = g_i[j] - p_i[j];
        float u = p[j] + local_err;
        x_i[j] = fmaf(-lr, u, x_i[j]);
    }
}

/* One compressed iteration of Algorithm 1 for all N workers and the server.
 *   g [N,d] gradients (read only), x [N,d] local models (in/out),
 *   e [d] global error (in/out).  Optional outputs (may be NULL):
 *   wdesc [N], sdesc [1], v_out [d] (compensated average), p_out [d] (broadcast),
 *   P_out [N,d] (uplink messages, decompressed).
 * Returns 0 on success, 1 on bad arguments, 2 when out of memory. */
int liec_oracle_step_rng(int32_t N, int64_t d, int worker_comp, int64_t worker_k, int server_comp,
                         int64_t server_k, float lr, const float *g, float *x, float *e,
                         const int64_t *off, int32_t B, uint64_t seed, uint64_t draw,
                         oracle_desc *wdesc, oracle_desc *sdesc, float *wscales, float *sscales,
                         float *v_out, float *p_out, float *P_out);

int liec_oracle_step_ex(int32_t N, int64_t d, int worker_comp, int64_t worker_k, int server_comp,
                        int64_t server_k, float lr, const float *g, float *x, float *e,
                        const int64_t *off, int32_t B, oracle_desc *wdesc, oracle_desc *sdesc,
                        float *wscales, float *sscales, float *v_out, float *p_out, float *P_out)
{
    return liec_oracle_step_rng(N, d, worker_comp, worker_k, server_comp, server_k, lr, g, x, e, off, B,
                                0, 0, wdesc, sdesc, wscales, sscales, v_out, p_out, P_out);
}

int liec_oracle_step(int32_t N, int64_t d, int worker_comp, int64_t worker_k, int server_comp,
                     int64_t server_k, float lr, const float *g, float *x, float *e,
                     oracle_desc *wdesc, oracle_desc *sdesc, float *v_out, float *p_out,
                     float *P_out)
{
    return liec_oracle_step_ex(N, d, worker_comp, worker_k, server_comp, server_k, lr, g, x, e, NULL, 0,
                               wdesc, sdesc, NULL, NULL, v_out, p_out, P_out);
}

/* The same iteration with the block table of Definition 5 available to either side
 * (off [B+1], used where the operator is the blockwise scaled sign); wscales [N*B] and sscales [B]
 * optionally receive the per-block scales.  (seed, draw) name this iteration's random draws of
 * Definition 3: worker i draws with row i, the server with row N. */
int liec_oracle_step_rng(int32_t N, int64_t d, int worker_comp, int64_t worker_k, int server_comp,
                         int64_t server_k, float lr, const float *g, float *x, float *e,
                         const int64_t *off, int32_t B, uint64_t seed, uint64_t draw,
                         oracle_desc *wdesc, oracle_desc *sdesc, float *wscales, float *sscales,
                         float *v_out, float *p_out, float *P_out)
{
    if (N < 1 || d < 1 || !g || !x || !e)
        return 1;
    size_t nd = (size_t)N * (size_t)d;
    float *P = P_out ? P_out : (float *)malloc(nd * sizeof(float));
    float *v = v_out ? v_out : (float *)malloc((size_t)d * sizeof(float));
    float *p = p_out ? p_out : (float *)malloc((size_t)d * sizeof(float));
    int rc = (!P || !v || !p) ? 2 : 0;

    /* worker i: p^i = C(g_i).  The workers are independent of one another: a build with -fopenmp
     * (the "all host cores" timing of the bench) runs them on several threads, each worker's
     * arithmetic unchanged and single-threaded; the plain build runs them in order. */
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1)
#endif
    for (int32_t i = 0; i < N; ++i) {
        int failed;
#ifdef _OPENMP
#pragma omp atomic read
#endif
        failed = rc;
        if (failed != 0)
            continue;
        int r = liec_oracle_compress_rng(worker_comp, g + (size_t)i * (size_t)d, d, worker_k, off, B,
                                         seed, draw, (uint32_t)i, P + (size_t)i * (size_t)d,
                                         wdesc ? &wdesc[i] : NULL,
                                         wscales ? wscales + (size_t)i * (size_t)B : NULL);
        if (r != 0) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            rc = r;
        }
    }
    if (rc == 0) {
        /* server: v = e + mean_i p^i ; p = C(v) ; e <- v - p */
        liec_oracle_server_average(P, N, d, e, v);
        rc = liec_oracle_compress_rng(server_comp, v, d, server_k, off, B, seed, draw, (uint32_t)N, p,
                                      sdesc, sscales);
    }
    if (rc == 0) {
        liec_oracle_error_update(v, p, d, e);
        /* worker i: x^i <- x^i - eta (p - p^i + g_i) */
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1)
#endif
        for (int32_t i = 0; i < N; ++i)
            liec_oracle_worker_update(g + (size_t)i * (size_t)d, P + (size_t)i * (size_t)d, p, d,
                                      lr, x + (size_t)i * (size_t)d);
    }
    if (!P_out) free(P);
    if (!v_out) free(v);
    if (!p_out) free(p);
    return rc;
}

/* The averaging iteration of Algorithm 1 (the branches taken when (t+1) is a multiple of the
 * averaging period): workers send the uncompressed gradient and their model, the server
 * compensates v = e + mean_i g_i and sends it uncompressed together with the mean model, so the
 * global error becomes v - v = 0 and every worker restarts from the same point
 *   x^i <- mean_i x^i - eta * (p - p^i + g_i)  with p = v, p^i = g_i.
 * Readings: both means add in worker order in fp32 from +0; the gradient mean enters v through one
 * fused multiply-add with 1/N (as in the compressed iteration), the model mean is one multiply by
 * 1/N; the cached local error g_i - p^i is formed first (it is exactly 0), then added to p, then one
 * fused multiply-add with -eta onto the mean model.
 *   g [N,d] (read only), x [N,d] (in/out), e [d] (in/out), v_out [d] optional. */
int liec_oracle_step_sync(int32_t N, int64_t d, float lr, const float *g, float *x, float *e,
                          float *v_out)
{
    if (N < 1 || d < 1 || !g || !x || !e)
        return 1;
    const float inv_n = 1.0f / (float)N;
    for (int64_t j = 0; j < d; ++j) {
        float acc_g = 0.0f, acc_x = 0.0f;
        for (int32_t i = 0; i < N; ++i) {
            acc_g = acc_g + g[(size_t)i * (size_t)d + (size_t)j];
            acc_x = acc_x + x[(size_t)i * (size_t)d + (size_t)j];
        }
        const float v = fmaf(acc_g, inv_n, e[j]);
        const float p = v;                       /* sent uncompressed */
        const float x_mean = acc_x * inv_n;
        e[j] = v - p;
        if (v_out)
            v_out[j] = v;
        for (int32_t i = 0; i < N; ++i) {
            const float g_ij = g[(size_t)i * (size_t)d + (size_t)j];
            const float local_err = g_ij - g_ij;  /* p^i = g_i */
            const float u = p + local_err;
            x[(size_t)i * (size_t)d + (size_t)j] = fmaf(-lr, u, x_mean);
        }
    }
    return 0;
}

/* Wire form of a scaled-sign message (Definition 4; the paper counts it as one bit per element):
 * bit (j mod 8) of byte (j div 8) is 1 when v_j < 0; unused bits of the last byte are 0. */
void liec_oracle_pack_sign(const float *v, int64_t d, uint8_t *bytes)
{
    for (int64_t b = 0; b < (d + 7) / 8; ++b)
        bytes[b] = 0;
    for (int64_t j = 0; j < d; ++j)
        if (v[j] < 0.0f)
            bytes[j / 8] |= (uint8_t)(1u << (j % 8));
}

/* Decompression of that message: p_j = -scale or +scale; with a block table (Definition 5) the scale
 * of the block holding j.  off == NULL means one block. */
void liec_oracle_unpack_sign(const uint8_t *bytes, int64_t d, const float *scales, const int64_t *off,
                             int32_t B, float *p)
{
    int32_t b = 0;
    for (int64_t j = 0; j < d; ++j) {
        if (off)
            while (b + 1 < B && j >= off[b + 1])
                ++b;
        const float s = scales[off ? b : 0];
        p[j] = ((bytes[j / 8] >> (j % 8)) & 1u) ? -s : s;
    }
}

static int cmp_u32_asc(const void *a, const void *b)
{
    uint32_t x = *(const uint32_t *)a, y = *(const uint32_t *)b;
    return (x > y) - (x < y);
}

/* Wire form of a top-k message (Definition 2): the k kept entries as (index, value) pairs in
 * increasing index order; 8k bytes.  Kept entries may be zero when zeros had to be admitted. */
int liec_oracle_pack_topk(const float *v, int64_t d, int64_t k, uint32_t *idx, float *val)
{
    if (k < 1 || k > d || d > (int64_t)0x7fffffff)
        return 1;
    uint64_t *order = (uint64_t *)malloc((size_t)d * sizeof *order);
    if (!order)
        return 2;
    for (int64_t j = 0; j < d; ++j)
        order[j] = ((uint64_t)abs_key(v[j]) << 32) | (uint64_t)(0xffffffffu - (uint32_t)j);
    qsort(order, (size_t)d, sizeof *order, cmp_u64_desc);
    for (int64_t r = 0; r < k; ++r)
        idx[r] = 0xffffffffu - (uint32_t)(order[r] & 0xffffffffu);
    free(order);
    qsort(idx, (size_t)k, sizeof *idx, cmp_u32_asc);
    for (int64_t r = 0; r < k; ++r)
        val[r] = v[idx[r]];
    return 0;
}

/* Wire form of a random-k message (Definition 3): the k kept entries as (index, value) pairs in
 * increasing index order, as for top-k. */
int liec_oracle_pack_randk(const float *v, int64_t d, int64_t k, uint64_t seed, uint64_t draw,
                           uint32_t row, uint32_t *idx, float *val)
{
    if (k < 1 || k > d || d > (int64_t)0x7fffffff)
        return 1;
    uint64_t *order = (uint64_t *)malloc((size_t)d * sizeof *order);
    if (!order)
        return 2;
    const uint64_t stream = liec_oracle_randk_stream(seed, draw, row);
    for (int64_t j = 0; j < d; ++j)
        order[j] = ((uint64_t)liec_oracle_randk_priority(stream, (uint32_t)j) << 32) |
                   (uint64_t)(0xffffffffu - (uint32_t)j);
    qsort(order, (size_t)d, sizeof *order, cmp_u64_desc);
    for (int64_t r = 0; r < k; ++r)
        idx[r] = 0xffffffffu - (uint32_t)(order[r] & 0xffffffffu);
    free(order);
    qsort(idx, (size_t)k, sizeof *idx, cmp_u32_asc);
    for (int64_t r = 0; r < k; ++r)
        val[r] = v[idx[r]];
    return 0;
}

/* Decompression: zeros everywhere except the listed entries. */
void liec_oracle_unpack_topk(const uint32_t *idx, const float *val, int64_t k, int64_t d, float *p)
{
    for (int64_t j = 0; j < d; ++j)
        p[j] = 0.0f;
    for (int64_t r = 0; r < k; ++r)
        p[idx[r]] = val[r];
}

int liec_oracle_desc_size(void) { return (int)sizeof(oracle_desc); }

/* Threads a step's per-worker loops may use: 1 in the plain build. */
int liec_oracle_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
