/* Driver for a sanitizer build of the oracle (see test_oracle_sanitizers.py): every entry point on
 * every storage kind, with each array allocated at exactly the size the interface states, so that
 * AddressSanitizer sees any access past an end and UBSan any shift or conversion out of range. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "mpo_ref.h"

static uint32_t lcg(uint32_t *s) { *s = *s * 1664525u + 1013904223u; return *s; }

static void *exact(size_t bytes) { return malloc(bytes ? bytes : 1); }

static int run(uint64_t n, int fmt, int res_bits, int packed, int round)
{
    uint32_t s = (uint32_t)(n * 2654435761u) ^ (uint32_t)(fmt * 977 + res_bits * 131 + packed * 17 + round);
    const uint64_t rb = mpo_ref_res_bytes(n, fmt, res_bits, packed);
    float *w = exact(n * 4), *back = exact(n * 4), *m = exact(n * 4), *v = exact(n * 4);
    uint16_t *hi = exact(n * 2), *g = exact(n * 2);
    uint8_t *res = exact(rb);
    memset(res, 0, rb);
    memset(m, 0, n * 4);
    memset(v, 0, n * 4);
    for (uint64_t i = 0; i < n; ++i) {
        uint32_t bits = lcg(&s);
        if (i % 3 == 0) bits = (bits & 0x807FFFFFu) | 0x3C000000u;      /* model-like magnitudes */
        memcpy(&w[i], &bits, 4);
        g[i] = (uint16_t)(lcg(&s) >> 16);
    }
    mpo_ref_split(w, hi, res, n, fmt, res_bits, packed, round, 99, 3, 0);
    mpo_ref_merge(hi, res, back, n, fmt, res_bits, packed, round);
    mpo_ref_adam_cfg a = {1e-3, 0.9, 0.999, 1e-8, 0.01, 1, 1.0, fmt, fmt, res_bits, packed, round, 99, 0.5};
    mpo_ref_sgd_cfg q = {1e-2, 0.9, 1e-4, 128.0, fmt, fmt, res_bits, packed, round, 99, 0.0};
    for (uint64_t t = 1; t <= 2; ++t) {
        mpo_ref_adam_step(hi, res, g, m, v, n, &a, t, 3, 0);
        mpo_ref_sgd_step(hi, res, g, m, n, &q, t, 3, 0);
    }
    q.momentum = 0.0;
    mpo_ref_sgd_step(hi, res, g, NULL, n, &q, 3, 3, 0);
    mpo_ref_merge(hi, res, back, n, fmt, res_bits, packed, round);
    free(w); free(back); free(m); free(v); free(hi); free(g); free(res);
    return 1;
}

int main(void)
{
    static const uint64_t sizes[] = {0, 1, 2, 3, 5, 7, 8, 9, 15, 16, 17, 31, 33, 63, 65, 127, 129, 4095, 4097};
    int cases = 0;
    for (unsigned k = 0; k < sizeof sizes / sizeof sizes[0]; ++k)
        for (int fmt = 0; fmt <= 1; ++fmt) {
            const int full = fmt == MPO_REF_FP16 ? 13 : 16;
            for (int round = 0; round <= 2; ++round) {
                /* slots: all bits, a cut 16-bit slot, byte slots (stochastic needs room for its flag) */
                cases += run(sizes[k], fmt, 0, 0, round);
                cases += run(sizes[k], fmt, 11, 0, round);
                cases += run(sizes[k], fmt, round == MPO_REF_STOCHASTIC ? 7 : 8, 0, round);
                cases += run(sizes[k], fmt, 1, 0, round);
                /* planes: every stored width that leaves 1..full kept bits */
                for (int S = 1; S <= 15; ++S) {
                    const int kept = S - (round == MPO_REF_STOCHASTIC ? 1 : 0);
                    if (kept >= 1 && kept <= full) cases += run(sizes[k], fmt, S, 1, round);
                }
            }
        }
    uint32_t c[4] = {1, 2, 3, 4}, key[2] = {5, 6}, out[4];
    mpo_ref_philox4x32_10(c, key, out);
    float f = mpo_ref_cvt16(0x3C00, MPO_REF_FP16);
    printf("%d cases, %u %g\n", cases, out[0], (double)f);
    return 0;
}
