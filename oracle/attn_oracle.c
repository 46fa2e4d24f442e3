/*
 * CPU oracle for the attention forward pass -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, fp64.  Nothing in the product path may call this file; it
 * exists so the HIP kernels can be compared with something that shares no
 * code with them.  Inputs arrive as float (an exact container for fp32, fp16
 * and bf16 storage values) and every arithmetic step is done in double.
 *
 * Four evaluations of the same quantity, selected by `algo`:
 *   0  the definition (Sec. II-A): s_j = dot(q,k_j), f_j = e^{s_j}/sum e^{s},
 *      Attn = sum f_j v_j, evaluated with the safe-softmax max subtraction
 *      the same section describes;
 *   1  Alg. 1 (baseline FlashAttention, division inside the loop);
 *   2  Alg. 2 (FlashAttention2, one division at the end);
 *   3  Alg. 3 (FLASH-D): w_1 = 1, w_i = sigma(s_i - s_{i-1} + ln w_{i-1})
 *      (boxed weight equation of Sec. III-B, with the + sign of that equation
 *      and of its derivation; the algorithm box prints a minus, which
 *      contradicts both), o_i = o_{i-1} + (v_i - o_{i-1}) w_i (Sec. IV-A).
 *
 * Readings the paper leaves open (same for all four):
 *   - s_j = scale * dot(q, k_j); the paper's dot has no scale factor.
 *   - heads and batches are independent repeats (Sec. II, single head
 *     without loss of generality); query head h reads kv head h / (Hq/Hkv).
 *   - causal: key j is visible to query i iff j <= i + (Lk - Lq); a masked
 *     key is not an iteration of the loop; a row with no visible key is zero.
 *   - initial state of Alg. 1/2: m_0 = -inf, l_0 = 0, o_0 = 0.
 *
 * Layout: q, o: [B][Hq][Lq][d]; k, v: [B][Hkv][Lk][d], row-major.
 * If `rows` is NULL every row is computed and `o` is the full [B][Hq][Lq][d]
 * tensor; otherwise `rows` holds nrows triples (b, h, i) and `o` is
 * [nrows][d].  Returns 0, or -1 on a bad argument.
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>

#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    const float *q, *k, *v;
    int B, Hq, Hkv, Lq, Lk, d, causal;
    double scale;
} problem_t;

/* number of keys visible to query row i: keys 0 .. nvis-1 */
static long visible_count(const problem_t *p, int i)
{
    long n = p->Lk;
    if (p->causal) {
        n = (long)i + ((long)p->Lk - (long)p->Lq) + 1;
        if (n < 0) n = 0;
        if (n > p->Lk) n = p->Lk;
    }
    return n;
}

static double score(const problem_t *p, const float *qrow, const float *krow)
{
    double acc = 0.0;
    for (int t = 0; t < p->d; ++t) acc += (double)qrow[t] * (double)krow[t];
    return p->scale * acc;
}

/* Sec. II-A definition with the safe-softmax shift of the same section. */
static void row_definition(const problem_t *p, const float *qrow, const float *K,
                           const float *V, long n, double *s, double *out)
{
    int d = p->d;
    for (int t = 0; t < d; ++t) out[t] = 0.0;
    if (n == 0) return;
    double mx = -INFINITY;
    for (long j = 0; j < n; ++j) {
        s[j] = score(p, qrow, K + (size_t)j * d);
        if (s[j] > mx) mx = s[j];
    }
    double den = 0.0;
    for (long j = 0; j < n; ++j) den += exp(s[j] - mx);
    for (long j = 0; j < n; ++j) {
        double f = exp(s[j] - mx) / den;
        const float *vr = V + (size_t)j * d;
        for (int t = 0; t < d; ++t) out[t] += f * (double)vr[t];
    }
}

/* Alg. 1: state (m, l, o), division by l_i inside the loop. */
static void row_alg1(const problem_t *p, const float *qrow, const float *K,
                     const float *V, long n, double *out)
{
    int d = p->d;
    double m = -INFINITY, l = 0.0;
    for (int t = 0; t < d; ++t) out[t] = 0.0;
    for (long j = 0; j < n; ++j) {
        double sj = score(p, qrow, K + (size_t)j * d);
        double mn = sj > m ? sj : m;
        double carry = l * exp(m - mn);          /* l_{i-1} e^{m_{i-1}-m_i} */
        double fresh = exp(sj - mn);             /* e^{s_i - m_i}           */
        double ln = carry + fresh;
        const float *vr = V + (size_t)j * d;
        for (int t = 0; t < d; ++t)
            out[t] = out[t] * (carry / ln) + (double)vr[t] * (fresh / ln);
        m = mn;
        l = ln;
    }
}

/* Alg. 2: same state, output left unnormalised, one division at the end. */
static void row_alg2(const problem_t *p, const float *qrow, const float *K,
                     const float *V, long n, double *out)
{
    int d = p->d;
    double m = -INFINITY, l = 0.0;
    for (int t = 0; t < d; ++t) out[t] = 0.0;
    for (long j = 0; j < n; ++j) {
        double sj = score(p, qrow, K + (size_t)j * d);
        double mn = sj > m ? sj : m;
        double resc = exp(m - mn);
        double fresh = exp(sj - mn);
        const float *vr = V + (size_t)j * d;
        l = l * resc + fresh;
        for (int t = 0; t < d; ++t) out[t] = out[t] * resc + (double)vr[t] * fresh;
        m = mn;
    }
    if (n > 0)
        for (int t = 0; t < d; ++t) out[t] /= l;
}

/* sigma(x) and ln sigma(x), each evaluated on the side where e^{-|x|} <= 1 */
static double sigmoid(double x)
{
    if (x >= 0.0) return 1.0 / (1.0 + exp(-x));
    double e = exp(x);
    return e / (1.0 + e);
}

static double log_sigmoid(double x)
{
    if (x >= 0.0) return -log1p(exp(-x));
    return x - log1p(exp(x));
}

/* Alg. 3: state (s_{i-1}, ln w_{i-1}, o_{i-1}); no max, no l, no division. */
static void row_alg3(const problem_t *p, const float *qrow, const float *K,
                     const float *V, long n, double *out)
{
    int d = p->d;
    double s_prev = 0.0, lnw = 0.0;
    for (int t = 0; t < d; ++t) out[t] = 0.0;
    for (long j = 0; j < n; ++j) {
        double sj = score(p, qrow, K + (size_t)j * d);
        const float *vr = V + (size_t)j * d;
        double w;
        if (j == 0) {
            w = 1.0;
            lnw = 0.0;
        } else {
            double x = sj - s_prev + lnw;
            w = sigmoid(x);
            lnw = log_sigmoid(x);   /* ln w_i taken from x, not from the rounded w_i */
        }
        for (int t = 0; t < d; ++t) out[t] += ((double)vr[t] - out[t]) * w;
        s_prev = sj;
    }
}

int oracle_attn(int algo, const float *q, const float *k, const float *v, double *o,
                int B, int Hq, int Hkv, int Lq, int Lk, int d, int causal, float scale,
                const int *rows, long nrows)
{
    if (!q || !k || !v || !o) return -1;
    if (B < 1 || Hq < 1 || Hkv < 1 || Lq < 1 || Lk < 1 || d < 1) return -1;
    if (Hq % Hkv != 0 || algo < 0 || algo > 3) return -1;
    problem_t p = {q, k, v, B, Hq, Hkv, Lq, Lk, d, causal != 0, (double)scale};
    long total = rows ? nrows : (long)B * Hq * Lq;
    int g = Hq / Hkv;
    int bad = 0;

#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)Lk);
#pragma omp for schedule(dynamic, 16)
        for (long r = 0; r < total; ++r) {
            int b, h, i;
            if (rows) {
                b = rows[3 * r]; h = rows[3 * r + 1]; i = rows[3 * r + 2];
                if (b < 0 || b >= B || h < 0 || h >= Hq || i < 0 || i >= Lq) {
#pragma omp atomic write
                    bad = 1;
                    continue;
                }
            } else {
                i = (int)(r % Lq);
                h = (int)((r / Lq) % Hq);
                b = (int)(r / ((long)Lq * Hq));
            }
            const float *qrow = q + (((size_t)b * Hq + h) * Lq + i) * d;
            const float *K = k + ((size_t)b * Hkv + h / g) * (size_t)Lk * d;
            const float *V = v + ((size_t)b * Hkv + h / g) * (size_t)Lk * d;
            double *out = o + (size_t)r * d;
            long n = visible_count(&p, i);
            switch (algo) {
            case 0: row_definition(&p, qrow, K, V, n, s, out); break;
            case 1: row_alg1(&p, qrow, K, V, n, out); break;
            case 2: row_alg2(&p, qrow, K, V, n, out); break;
            default: row_alg3(&p, qrow, K, V, n, out); break;
            }
        }
        free(s);
    }
    return bad ? -1 : 0;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
