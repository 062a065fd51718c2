/*
 * selftest.c -- TEST INFRASTRUCTURE.  Drives every entry point of liec_oracle.c on small inputs so
 * that the file can be run under AddressSanitizer / UndefinedBehaviorSanitizer on the host
 * (tests/test_oracle_sanitizers.py builds and runs it).  It checks only what can be stated without
 * repeating the oracle's arithmetic: exit status, counts and the invariants of the operators.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "liec_oracle.c"

static float frand(uint32_t *s)
{
    *s = *s * 1664525u + 1013904223u;
    return ((int32_t)(*s >> 8) - (1 << 23)) / (float)(1 << 20);
}

int main(void)
{
    uint32_t seed = 7;
    const int32_t N = 3;
    const int64_t sizes[] = {1, 5, 64, 257, 1000};
    for (size_t z = 0; z < sizeof sizes / sizeof sizes[0]; ++z) {
        const int64_t d = sizes[z];
        float *g = malloc((size_t)N * d * sizeof *g), *x = calloc((size_t)N * d, sizeof *x);
        float *e = calloc((size_t)d, sizeof *e), *p = malloc((size_t)d * sizeof *p);
        uint8_t *bits = malloc((size_t)(d + 7) / 8);
        uint32_t *idx = malloc((size_t)d * sizeof *idx);
        float *val = malloc((size_t)d * sizeof *val);
        if (!g || !x || !e || !p || !bits || !idx || !val) return 2;
        for (int64_t q = 0; q < N * d; ++q) g[q] = (q % 7 == 0) ? 0.0f : frand(&seed);
        const int64_t k = d / 3 + 1;
        int64_t off[4] = {0, d > 2 ? d / 3 : d, d > 2 ? d / 3 + 1 : d, d};
        const int32_t B = d > 2 ? 3 : 1;
        if (B == 1) off[1] = d;
        oracle_desc wd[3], sd;
        float ws[9], ss[3];
        for (int wc = 0; wc < 5; ++wc)
            for (int sc = 0; sc < 5; ++sc)
                if (liec_oracle_step_rng(N, d, wc, k, sc, k, 0.1f, g, x, e, off, B, 5, (uint64_t)z, wd, &sd, ws, ss,
                                         NULL, NULL, NULL)) return 3;
        if (liec_oracle_step_sync(N, d, 0.1f, g, x, e, NULL)) return 4;
        for (int64_t j = 0; j < d; ++j) if (e[j] != 0.0f) return 5;
        if (liec_oracle_compress(ORACLE_TOPK, g, d, k, p, &sd)) return 6;
        int64_t kept = 0;
        for (int64_t j = 0; j < d; ++j) {
            const uint32_t key = abs_key(g[j]);
            kept += key > sd.tau_key || (key == sd.tau_key && j <= sd.cutoff);
        }
        if (kept != k) return 7;
        if (liec_oracle_pack_topk(g, d, k, idx, val)) return 8;
        liec_oracle_unpack_topk(idx, val, k, d, p);
        liec_oracle_pack_sign(g, d, bits);
        liec_oracle_unpack_sign(bits, d, ss, off, B, p);
        for (int64_t j = 0; j < d; ++j) if ((p[j] < 0.0f) != (g[j] < 0.0f) && p[j] != 0.0f) return 9;
        if (liec_oracle_compress(ORACLE_TOPK, g, d, 0, p, &sd) == 0) return 10;      /* bad k must be refused */
        if (liec_oracle_pack_randk(g, d, k, 1, 2, 3, idx, val)) return 11;
        for (int64_t r = 1; r < k; ++r) if (idx[r] <= idx[r - 1] || idx[r] >= (uint32_t)d) return 12;
        liec_oracle_randk_priorities(1, 2, 3, d, idx);
        if (liec_oracle_compress_rng(ORACLE_RANDK, g, d, d + 1, NULL, 0, 1, 2, 3, p, &sd, NULL) == 0) return 13;
        free(g); free(x); free(e); free(p); free(bits); free(idx); free(val);
    }
    puts("oracle selftest ok");
    return 0;
}
