/*
 * CPU oracle for the static skip statistics -- TEST INFRASTRUCTURE ONLY.
 *
 * Sec. III-C: a step of Alg. 3 whose score difference s_i - s_{i-1} lies at or below -6
 * has a weight of (almost) 0 and may be skipped (the output is kept); at or above 11 the
 * weight is (almost) 1 and the output becomes v_i.  Table I reports how often that happens.
 * This file counts, over every query row and every step i >= 2 of its visible keys,
 *     steps, steps with s_i - s_{i-1} <= lo, steps with s_i - s_{i-1} >= hi.
 *
 * The comparison decides an integer, so the arithmetic that feeds it is fixed here exactly
 * (the paper states no accumulator width; fp32 is this build's reading):
 *     acc = 0;  acc = fma(q[t], k[t], acc) for t = 0 .. d-1 in this order (fp32, one
 *     rounding per step);  s = acc * scale (fp32);  diff = s_i - s_{i-1} (fp32).
 * Inputs arrive as float (an exact container for fp32, fp16 and bf16 storage values).
 * Same layout, head mapping and causal rule as attn_oracle.c.
 */
#include <math.h>
#include <stddef.h>

int oracle_skip_stats(const float *q, const float *k, int B, int Hq, int Hkv, int Lq, int Lk,
                      int d, int causal, float scale, float lo, float hi,
                      unsigned long long *counts)
{
    if (!q || !k || !counts || B < 1 || Hq < 1 || Hkv < 1 || Lq < 1 || Lk < 1 || d < 1 ||
        Hq % Hkv != 0)
        return -1;
    const int g = Hq / Hkv;
    unsigned long long steps = 0, low = 0, high = 0;
#pragma omp parallel for collapse(2) reduction(+ : steps, low, high) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hq; ++h) {
            const float *kh = k + ((size_t)b * Hkv + h / g) * (size_t)Lk * d;
            for (int i = 0; i < Lq; ++i) {
                const float *qrow = q + (((size_t)b * Hq + h) * Lq + i) * (size_t)d;
                long nvis = Lk;
                if (causal) {
                    nvis = (long)i + ((long)Lk - (long)Lq) + 1;
                    if (nvis < 0) nvis = 0;
                    if (nvis > Lk) nvis = Lk;
                }
                float prev = 0.0f;
                for (long j = 0; j < nvis; ++j) {
                    const float *krow = kh + (size_t)j * d;
                    float acc = 0.0f;
                    for (int t = 0; t < d; ++t) acc = fmaf(qrow[t], krow[t], acc);
                    const float s = acc * scale;
                    if (j > 0) {
                        const float diff = s - prev;
                        ++steps;
                        if (diff <= lo) ++low;
                        if (diff >= hi) ++high;
                    }
                    prev = s;
                }
            }
        }
    counts[0] = steps;
    counts[1] = low;
    counts[2] = high;
    return 0;
}
