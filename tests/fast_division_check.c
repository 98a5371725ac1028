/*
 * Host-side check of the division-free quotient the activation-quantization kernel uses:
 *     r = RN(1 / s);  q = x * r;  q = fma(fma(-s, q, x), r, q)
 * against true IEEE binary32 division, over every bf16 input for many scales, over random
 * binary32 inputs including constructed near-ties, and (mode "edge") over the scales whose
 * significand is all ones or nearly, where RN(1 / s) is least accurate.  The arithmetic is retyped here on purpose
 * (it shares no code with the GPU kernel): this validates the algorithm, the GPU parity
 * tests validate the implementation.  Prints "pairs quotient_mismatches_that_matter
 * code_mismatches"; quotient mismatches are only tolerated below 2^-30, where every code is 0.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

static float fast_quotient(float x, float s, float r) {
    float q = x * r;
    q = fmaf(fmaf(-s, q, x), r, q);
    return q;
}
static float qmax = 127.f;
static float code_of(float q) { return fminf(fmaxf(rintf(q), -qmax), qmax); }

static uint64_t state = 88172645463325252ULL;
static uint64_t next(void) { state ^= state << 13; state ^= state >> 7; state ^= state << 17; return state; }

/* The asymmetric quantizer (unsigned codes, zero point per row) uses the same quotient for
 * x / s and for min / s, with quotients far above the code range when a row lies far from
 * zero.  Rows [lo, hi] of either sign with |lo| / (hi - lo) up to 2^20; x anywhere in the row,
 * its ends included, half of them truncated to bf16.  Counts rows * samples, rounded quotients
 * that differ, and final codes that differ. */
static int asym_main(long rows, long per_row, float levels) {
    long pairs = 0, bad_round = 0, bad_code = 0;
    for (long it = 0; it < rows; ++it) {
        uint32_t ab = (uint32_t)(next() & 0x7fffffff);
        float range, lo;
        memcpy(&range, &ab, 4);
        if (!(range > 0x1p-40f && range < 0x1p40f)) continue;
        float ratio = ldexpf((float)(next() & 0xffff) / 65536.0f, (int)(next() % 22) - 1);
        lo = range * ratio * ((next() & 1) ? 1.0f : -1.0f) - ((next() & 2) ? range * 0.5f : 0.0f);
        if (it & 4) { uint32_t u; memcpy(&u, &lo, 4); u &= 0xffff0000u; memcpy(&lo, &u, 4); }
        float hi = lo + range;
        float span = hi - lo;
        if (!(span > 0.0f)) continue;
        float s = span / levels, r = 1.0f / s;
        float z_true = -rintf(lo / s), z_fast = -rintf(fast_quotient(lo, s, r));
        if (z_true != z_fast) ++bad_round;
        for (long j = 0; j < per_row; ++j) {
            float x;
            if (j == 0) x = lo;
            else if (j == 1) x = hi;
            else x = lo + span * ((float)(next() & 0xffffff) / 16777215.0f);
            if (j & 1) { uint32_t u; memcpy(&u, &x, 4); u &= 0xffff0000u; memcpy(&x, &u, 4); }
            if (!(x >= lo && x <= hi)) continue;
            float a = rintf(x / s), b = rintf(fast_quotient(x, s, r));
            ++pairs;
            if (a != b) ++bad_round;
            float ca = fminf(fmaxf(a + z_true, 0.0f), levels), cb = fminf(fmaxf(b + z_fast, 0.0f), levels);
            if (ca != cb) ++bad_code;
        }
    }
    printf("%ld %ld %ld\n", pairs, bad_round, bad_code);
    return 0;
}

/* Scales with significand 0x7FFFF0 .. 0x7FFFFF over 140 exponents; x a (half-)integer or
 * random multiple of s within +-255 steps, nudged by up to 3 ulps, half of them cut to bf16. */
static int edge_main(long per_scale) {
    long pairs = 0, bad_q = 0, bad_round = 0;
    for (int e = 60; e < 200; ++e)
        for (uint32_t m = 0x7FFFF0u; m <= 0x7FFFFFu; ++m) {
            uint32_t sb = ((uint32_t)e << 23) | m, xb;
            float s, x;
            memcpy(&s, &sb, 4);
            const float r = 1.0f / s;
            for (long it = 0; it < per_scale; ++it) {
                float k = (float)((int)(next() % 511) - 255) +
                          ((it & 1) ? 0.5f : (float)(next() & 0xffff) / 65536.0f);
                x = k * s;
                memcpy(&xb, &x, 4);
                xb += (uint32_t)(next() % 7) - 3;
                if (it & 2) xb &= 0xffff0000u;
                memcpy(&x, &xb, 4);
                float q = x / s, f = fast_quotient(x, s, r);
                ++pairs;
                if (memcmp(&q, &f, 4) != 0 && fabsf(q) > 0x1p-30f) ++bad_q;
                if (rintf(q) != rintf(f)) ++bad_round;
            }
        }
    printf("%ld %ld %ld\n", pairs, bad_q, bad_round);
    return 0;
}

int main(int argc, char **argv) {
    long scales = argc > 1 ? atol(argv[1]) : 400, randoms = argc > 2 ? atol(argv[2]) : 20000000;
    if (argc > 3) qmax = (float)atof(argv[3]);
    if (argc > 4 && strcmp(argv[4], "edge") == 0) return edge_main(scales);
    if (argc > 4 && strcmp(argv[4], "asym") == 0) return asym_main(scales, randoms, qmax);
    long pairs = 0, bad_q = 0, bad_code = 0;
    for (long si = 0; si < scales; ++si) {
        uint32_t ab = (uint32_t)(next() & 0x7fffffff);
        float a;
        memcpy(&a, &ab, 4);
        if (!(a > 0x1p-60f && a < 0x1p100f)) continue;
        if (si % 2) { ab &= 0xffff0000u; memcpy(&a, &ab, 4); }
        float s = a / qmax, r = 1.0f / s;
        for (uint32_t hb = 0; hb < 65536; ++hb) {
            uint32_t u = hb << 16;
            float x;
            memcpy(&x, &u, 4);
            if (!(fabsf(x) <= a)) continue;
            float q = x / s, f = fast_quotient(x, s, r);
            ++pairs;
            if (memcmp(&q, &f, 4) != 0 && fabsf(q) > 0x1p-30f) ++bad_q;
            if (code_of(q) != code_of(f)) ++bad_code;
        }
    }
    for (long it = 0; it < randoms; ++it) {
        uint32_t ab = (uint32_t)(next() & 0x7fffffff);
        float a, x;
        memcpy(&a, &ab, 4);
        if (!(a > 0x1p-60f && a < 0x1p100f)) continue;
        float s = a / qmax, r = 1.0f / s;
        if (it & 1) {
            x = a * ((float)(next() & 0xffffff) / 8388608.0f - 1.0f);
        } else { /* a half-integer multiple of s, nudged by a few ulps */
            float k = (float)((int)(next() % (2 * (int)qmax + 1)) - (int)qmax) + 0.5f;
            uint32_t xb;
            x = k * s;
            memcpy(&xb, &x, 4);
            xb += (uint32_t)(next() % 5) - 2;
            memcpy(&x, &xb, 4);
        }
        if (!(fabsf(x) <= a)) continue;
        float q = x / s, f = fast_quotient(x, s, r);
        ++pairs;
        if (memcmp(&q, &f, 4) != 0 && fabsf(q) > 0x1p-30f) ++bad_q;
        if (code_of(q) != code_of(f)) ++bad_code;
    }
    printf("%ld %ld %ld\n", pairs, bad_q, bad_code);
    return 0;
}
