/*
 * CPU oracle for attention over a chunk of keys with the state of Alg. 3 handed in and
 * out -- TEST INFRASTRUCTURE ONLY.
 *
 * Alg. 3 taken literally, in fp64 (Sec. III-C): the state after a run of keys is
 * (o, s_last, ln w_last).  With a state handed in, the first key of this call is an
 * ordinary later step of the recurrence, w = sigma(s - s_last + ln w_last) (boxed weight
 * equation of Sec. III-B, plus sign); without one, or when the state is that of a row that
 * has seen no key (s_last = -inf), the first visible key starts the run with w = 1.
 * The state written out is the literal (o, s_last, ln w_last), not a normalised form.
 *
 * Layout: q: [B][Hq][Lq][d]; k, v: [B][Hkv][Lk][d]; states: [B][Hq][Lq][d + 2] doubles,
 * (o[0..d), s, ln w) per query row.  causal: key j of this call is visible to query i iff
 * j <= i + shift.  s_j = scale * dot(q, k_j), scale widened from fp32.
 */
#include <math.h>
#include <stddef.h>

int oracle_attn_state(const float *q, const float *k, const float *v, const double *state_in,
                      double *state_out, int B, int Hq, int Hkv, int Lq, int Lk, int d, int causal,
                      int shift, float scale)
{
    if (!q || !k || !v || !state_out || B < 1 || Hq < 1 || Hkv < 1 || Lq < 1 || Lk < 1 || d < 1 ||
        Hq % Hkv != 0)
        return -1;
    const int g = Hq / Hkv;
    const double sc = (double)scale;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hq; ++h) {
            const float *kh = k + ((size_t)b * Hkv + h / g) * (size_t)Lk * d;
            const float *vh = v + ((size_t)b * Hkv + h / g) * (size_t)Lk * d;
            for (int i = 0; i < Lq; ++i) {
                const size_t row = ((size_t)b * Hq + h) * Lq + i;
                const float *qrow = q + row * (size_t)d;
                double *out = state_out + row * (size_t)(d + 2);
                double s_prev = -INFINITY, lnw = 0.0;
                int started = 0;
                for (int t = 0; t < d; ++t) out[t] = 0.0;
                if (state_in) {
                    const double *in = state_in + row * (size_t)(d + 2);
                    if (in[d] != -INFINITY) {
                        for (int t = 0; t < d; ++t) out[t] = in[t];
                        s_prev = in[d];
                        lnw = in[d + 1];
                        started = 1;
                    }
                }
                long nvis = Lk;
                if (causal) {
                    nvis = (long)i + (long)shift + 1;
                    if (nvis < 0) nvis = 0;
                    if (nvis > Lk) nvis = Lk;
                }
                for (long j = 0; j < nvis; ++j) {
                    const float *krow = kh + (size_t)j * d;
                    const float *vrow = vh + (size_t)j * d;
                    double dot = 0.0;
                    for (int t = 0; t < d; ++t) dot += (double)qrow[t] * (double)krow[t];
                    const double s = sc * dot;
                    if (!started) {
                        for (int t = 0; t < d; ++t) out[t] = (double)vrow[t];
                        lnw = 0.0;
                        started = 1;
                    } else {
                        const double x = s - s_prev + lnw;
                        double w, lw;
                        if (x >= 0.0) {
                            const double e = exp(-x);
                            w = 1.0 / (1.0 + e);
                            lw = -log1p(e);
                        } else {
                            const double e = exp(x);
                            w = e / (1.0 + e);
                            lw = x - log1p(e);
                        }
                        for (int t = 0; t < d; ++t) out[t] += ((double)vrow[t] - out[t]) * w;
                        lnw = lw;
                    }
                    s_prev = s;
                }
                out[d] = s_prev;
                out[d + 1] = lnw;
            }
        }
    return 0;
}
