/*
 * Driver for the AddressSanitizer / UndefinedBehaviorSanitizer build of the C oracle
 * (test infrastructure).  Every buffer is a heap block of exactly the size the oracle's
 * interface states, so a read or write past an end stops the program.  Inputs come from an
 * integer hash (values k / 8192, exact in fp32) that the Python test repeats; every result is
 * printed as a hexadecimal double for that test to compare with the ordinary build.
 */
#include <stdio.h>
#include <stdlib.h>

int oracle_attn(int algo, const float *q, const float *k, const float *v, double *o, int B,
                int Hq, int Hkv, int Lq, int Lk, int d, int causal, float scale, const int *rows,
                long nrows);
int oracle_attn_state(const float *q, const float *k, const float *v, const double *state_in,
                      double *state_out, int B, int Hq, int Hkv, int Lq, int Lk, int d, int causal,
                      int shift, float scale);
int oracle_skip_stats(const float *q, const float *k, int B, int Hq, int Hkv, int Lq, int Lk,
                      int d, int causal, float scale, float lo, float hi,
                      unsigned long long *counts);

static float gen(unsigned idx, unsigned salt)
{
    unsigned x = idx * 2654435761u + salt * 40503u;
    x ^= x >> 15;
    x *= 2246822519u;
    x ^= x >> 13;
    return (float)((int)((x >> 8) & 0xffffu) - 32768) / 8192.0f;
}

static float *make(size_t n, unsigned salt)
{
    float *p = (float *)malloc(n * sizeof(float));
    if (!p) exit(3);
    for (size_t i = 0; i < n; ++i) p[i] = gen((unsigned)i, salt);
    return p;
}

static void dump(const char *tag, int c, const double *x, size_t n)
{
    for (size_t i = 0; i < n; ++i) printf("%s %d %zu %a\n", tag, c, i, x[i]);
}

typedef struct { int B, Hq, Hkv, Lq, Lk, d, causal; } shape_t;

int main(void)
{
    static const shape_t shapes[] = {
        {1, 1, 1, 1, 1, 1, 0}, {2, 4, 2, 5, 9, 8, 1}, {1, 2, 1, 9, 5, 4, 1},
        {1, 3, 3, 7, 7, 16, 0}, {1, 2, 2, 3, 70, 2, 1}};
    const int ns = (int)(sizeof(shapes) / sizeof(shapes[0]));
    for (int c = 0; c < ns; ++c) {
        const shape_t s = shapes[c];
        const size_t nq = (size_t)s.B * s.Hq * s.Lq * s.d, nk = (size_t)s.B * s.Hkv * s.Lk * s.d;
        float *q = make(nq, 3u * c + 1), *k = make(nk, 3u * c + 2), *v = make(nk, 3u * c + 3);
        const float scale = 0.75f;
        double *o = (double *)malloc(nq * sizeof(double));
        for (int algo = 0; algo < 4; ++algo) {
            if (oracle_attn(algo, q, k, v, o, s.B, s.Hq, s.Hkv, s.Lq, s.Lk, s.d, s.causal, scale,
                            NULL, 0) != 0)
                return 4;
            char tag[16];
            snprintf(tag, sizeof tag, "attn%d", algo);
            dump(tag, c, o, nq);
        }
        /* a subset of rows: first and last row of the last head */
        int *rows = (int *)malloc(2 * 3 * sizeof(int));
        rows[0] = s.B - 1; rows[1] = s.Hq - 1; rows[2] = 0;
        rows[3] = s.B - 1; rows[4] = s.Hq - 1; rows[5] = s.Lq - 1;
        double *orow = (double *)malloc(2 * (size_t)s.d * sizeof(double));
        if (oracle_attn(0, q, k, v, orow, s.B, s.Hq, s.Hkv, s.Lq, s.Lk, s.d, s.causal, scale, rows,
                        2) != 0)
            return 5;
        dump("rows", c, orow, 2 * (size_t)s.d);
        /* two chunks of keys with the state handed on (the second chunk may be empty-handed) */
        const size_t nst = (size_t)s.B * s.Hq * s.Lq * (s.d + 2);
        double *st1 = (double *)malloc(nst * sizeof(double)), *st2 = (double *)malloc(nst * sizeof(double));
        const int cut = s.Lk > 1 ? s.Lk / 2 : 1;
        /* chunk 1 holds keys [0, cut) of every kv head: copy them out contiguously */
        const size_t nk1 = (size_t)s.B * s.Hkv * cut * s.d;
        float *k1 = (float *)malloc(nk1 * sizeof(float)), *v1 = (float *)malloc(nk1 * sizeof(float));
        for (int u = 0; u < s.B * s.Hkv; ++u)
            for (int j = 0; j < cut; ++j)
                for (int t = 0; t < s.d; ++t) {
                    k1[((size_t)u * cut + j) * s.d + t] = k[((size_t)u * s.Lk + j) * s.d + t];
                    v1[((size_t)u * cut + j) * s.d + t] = v[((size_t)u * s.Lk + j) * s.d + t];
                }
        if (oracle_attn_state(q, k1, v1, NULL, st1, s.B, s.Hq, s.Hkv, s.Lq, cut, s.d, s.causal,
                              s.Lk - s.Lq, scale) != 0)
            return 6;
        dump("state1", c, st1, nst);
        if (s.Lk - cut >= 1) {
            const int rest = s.Lk - cut;
            const size_t nk2 = (size_t)s.B * s.Hkv * rest * s.d;
            float *k2 = (float *)malloc(nk2 * sizeof(float)), *v2 = (float *)malloc(nk2 * sizeof(float));
            for (int u = 0; u < s.B * s.Hkv; ++u)
                for (int j = 0; j < rest; ++j)
                    for (int t = 0; t < s.d; ++t) {
                        k2[((size_t)u * rest + j) * s.d + t] = k[((size_t)u * s.Lk + cut + j) * s.d + t];
                        v2[((size_t)u * rest + j) * s.d + t] = v[((size_t)u * s.Lk + cut + j) * s.d + t];
                    }
            if (oracle_attn_state(q, k2, v2, st1, st2, s.B, s.Hq, s.Hkv, s.Lq, rest, s.d, s.causal,
                                  s.Lk - s.Lq - cut, scale) != 0)
                return 7;
            dump("state2", c, st2, nst);
            free(k2); free(v2);
        }
        unsigned long long *counts = (unsigned long long *)malloc(3 * sizeof(unsigned long long));
        if (oracle_skip_stats(q, k, s.B, s.Hq, s.Hkv, s.Lq, s.Lk, s.d, s.causal, scale, -1.0f, 1.5f,
                              counts) != 0)
            return 8;
        printf("skip %d %llu %llu %llu\n", c, counts[0], counts[1], counts[2]);
        free(counts); free(k1); free(v1); free(st1); free(st2); free(orow); free(rows);
        free(o); free(q); free(k); free(v);
    }
    /* argument errors must be refused, not acted on */
    if (oracle_attn(0, NULL, NULL, NULL, NULL, 1, 1, 1, 1, 1, 1, 0, 1.0f, NULL, 0) == 0) return 9;
    printf("done\n");
    return 0;
}
