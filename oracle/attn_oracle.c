/*
 * TEST INFRASTRUCTURE -- NOT THE PRODUCT.
 *
 * Plain, slow, fp64 CPU definition of incremental-prefill attention.  It exists only so
 * that tests, the smoke check and the benchmark's CPU-baseline leg can compare the GPU
 * library against something obviously correct.  Nothing in the product path may call it.
 *
 * What it computes (paper Section 3, "System Overview": a prefill task has a history of
 * l_hist cached tokens and l_incr new tokens, an initial prefill being the l_hist = 0 case;
 * after the prefill the decode worker holds the KV of every token and decoding continues
 * one token at a time, Section 1).  The paper never writes the attention formula out; the
 * reading taken here is ordinary scaled-dot-product softmax attention, with the new query
 * i (0-based, absolute position C+i) seeing keys 0..C+i -- the only alignment under which
 * an incremental prefill over a cache equals a from-scratch prefill of the concatenation.
 * Query head hq reads KV head hq / (Hq/Hkv) (consecutive query heads share a KV head).
 *
 *   s_j  = scale * <q[i,hq,:], K[j,kvh,:]>         j = 0 .. C+i
 *   p_j  = exp(s_j - max_j s_j) / sum_j exp(s_j - max_j s_j)
 *   o[i,hq,:] = sum_j p_j V[j,kvh,:]
 *
 * No blocking, no online softmax, no reordering: three passes per (query, head).
 * K and V are contiguous [T][Hkv][d] copies (T = C+L), the paging having been undone by
 * the caller with a plain gather.
 */
#include <math.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* rows == NULL: compute all L new queries (nrows must equal L).
 * out  [nrows][Hq][d]; psum [nrows][Hq] (sum of the normalised probabilities; may be NULL).
 * Returns 0, or -1 on a bad argument / allocation failure. */
int ampd_oracle_attn(const double *q, const double *K, const double *V,
                     int C, int L, int Hq, int Hkv, int d, double scale,
                     const int *rows, int nrows, double *out, double *psum)
{
    if (C < 0 || L < 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || Hq % Hkv != 0 || nrows < 0) return -1;
    if (!rows && nrows != L) return -1;
    const int G = Hq / Hkv;
    int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int ri = 0; ri < nrows; ++ri) {
        for (int hq = 0; hq < Hq; ++hq) {
            const int i = rows ? rows[ri] : ri;
            if (i < 0 || i >= L) { fail = 1; continue; }
            const int kvh = hq / G;
            const int n = C + i + 1;                         /* visible keys */
            double *s = (double *)malloc(sizeof(double) * (size_t)n);
            if (!s) { fail = 1; continue; }
            const double *qv = q + ((size_t)i * Hq + hq) * d;
            double smax = -INFINITY;
            for (int j = 0; j < n; ++j) {
                const double *kv = K + ((size_t)j * Hkv + kvh) * d;
                double dot = 0.0;
                for (int x = 0; x < d; ++x) dot += qv[x] * kv[x];
                s[j] = scale * dot;
                if (s[j] > smax) smax = s[j];
            }
            double denom = 0.0;
            for (int j = 0; j < n; ++j) { s[j] = exp(s[j] - smax); denom += s[j]; }
            double *o = out + ((size_t)ri * Hq + hq) * d;
            for (int x = 0; x < d; ++x) o[x] = 0.0;
            double ps = 0.0;
            for (int j = 0; j < n; ++j) {
                const double p = s[j] / denom;
                ps += p;
                const double *vv = V + ((size_t)j * Hkv + kvh) * d;
                for (int x = 0; x < d; ++x) o[x] += p * vv[x];
            }
            if (psum) psum[(size_t)ri * Hq + hq] = ps;
            free(s);
        }
    }
    return fail ? -1 : 0;
}

/* The normalised probabilities of ONE (query i, head hq): p[0..C+i].  Used by the pins. */
int ampd_oracle_probs(const double *q, const double *K, int C, int L, int Hq, int Hkv, int d,
                      double scale, int i, int hq, double *p)
{
    if (i < 0 || i >= L || hq < 0 || hq >= Hq || Hq % Hkv != 0) return -1;
    const int kvh = hq / (Hq / Hkv);
    const int n = C + i + 1;
    const double *qv = q + ((size_t)i * Hq + hq) * d;
    double smax = -INFINITY;
    for (int j = 0; j < n; ++j) {
        const double *kv = K + ((size_t)j * Hkv + kvh) * d;
        double dot = 0.0;
        for (int x = 0; x < d; ++x) dot += qv[x] * kv[x];
        p[j] = scale * dot;
        if (p[j] > smax) smax = p[j];
    }
    double denom = 0.0;
    for (int j = 0; j < n; ++j) { p[j] = exp(p[j] - smax); denom += p[j]; }
    for (int j = 0; j < n; ++j) p[j] /= denom;
    return 0;
}

int ampd_oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
