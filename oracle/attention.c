/*
 * CPU oracle for batched causal attention with grouped-query heads.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP kernels are checked against; the product path never calls it.
 *
 * What it computes (paper Sec. 2.1 for prefill/decode, Sec. 3 "lossless
 * attention semantics", Sec. 3.2 for prefix + suffix KV): for every request
 * i, query head h and query row t, with ctx = Lkv_i - Lq_i,
 *
 *     s[j]   = scale * sum_c q[t,h,c] * k[j,g(h),c]      for 0 <= j <= ctx + t
 *     p[j]   = exp(s[j] - max_j s[j]) / sum_j exp(s[j] - max_j s[j])
 *     o[t,h] = sum_j p[j] * v[j,g(h),:]
 *
 * with g(h) = h / (Hq / Hkv).  Decode is the case Lq_i = 1.  The function
 * knows nothing about groups, pages, tiles or splits: it works on the logical
 * per-request tensors.  Inputs are fp32 (bf16 inputs are up-cast by the
 * caller); every sum is accumulated in fp64.
 *
 * Readings of points the paper leaves open: scale is passed in (1/sqrt(d) in
 * all configurations); query rows are the LAST Lq positions of the request
 * (bottom-right aligned causal mask); a decode query attends to all Lkv keys.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* One query row against keys 0..nkeys-1 of one KV head.
 * k, v point at token 0 of that head; consecutive tokens are kv_stride apart.
 * Writes d outputs; if lse_out != NULL also the natural-log sum-exp of the
 * scaled scores.  scores is scratch of nkeys doubles. */
static void attend_row(const float *q, const float *k, const float *v,
                       int64_t nkeys, int64_t kv_stride, int d, double scale,
                       double *scores, double *acc, float *out, double *lse_out)
{
    double m = -INFINITY;
    for (int64_t j = 0; j < nkeys; ++j) {
        const float *kj = k + j * kv_stride;
        double s = 0.0;
        for (int c = 0; c < d; ++c) s += (double)q[c] * (double)kj[c];
        s *= scale;
        scores[j] = s;
        if (s > m) m = s;
    }
    double denom = 0.0;
    for (int c = 0; c < d; ++c) acc[c] = 0.0;
    for (int64_t j = 0; j < nkeys; ++j) {
        double p = exp(scores[j] - m);
        denom += p;
        const float *vj = v + j * kv_stride;
        for (int c = 0; c < d; ++c) acc[c] += p * (double)vj[c];
    }
    for (int c = 0; c < d; ++c) out[c] = (float)(acc[c] / denom);
    if (lse_out) *lse_out = m + log(denom);
}

/*
 * Ragged batch.  q: [sum Lq, Hq, d], k and v: [sum Lkv, Hkv, d], out like q.
 * q_start, kv_start: n+1 cumulative row offsets.  rows: optional list of
 * nrows (request, head, t) triples; when NULL every row of every request and
 * head is computed into `out` (full layout); otherwise out is [nrows, d].
 * lse (optional) has one double per computed row, in the same order.
 * Returns the number of threads used, or -1 on a bad argument.
 */
int oracle_attention_ragged(const float *q, const float *k, const float *v,
                            const int64_t *q_start, const int64_t *kv_start,
                            int n, int Hq, int Hkv, int d, double scale,
                            const int32_t *rows, int64_t nrows,
                            float *out, double *lse, int nthreads)
{
    if (n < 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || Hq % Hkv != 0) return -1;
    const int r = Hq / Hkv;
    int64_t max_kv = 0;
    for (int i = 0; i < n; ++i) {
        int64_t lq = q_start[i + 1] - q_start[i], lkv = kv_start[i + 1] - kv_start[i];
        if (lq < 0 || lkv < lq) return -1;
        if (lkv > max_kv) max_kv = lkv;
    }
    int64_t total;
    int64_t *row_base = NULL;           /* full mode: first flat row of request i */
    if (rows == NULL) {
        row_base = (int64_t *)malloc((size_t)(n + 1) * sizeof(int64_t));
        row_base[0] = 0;
        for (int i = 0; i < n; ++i)
            row_base[i + 1] = row_base[i] + (q_start[i + 1] - q_start[i]) * Hq;
        total = row_base[n];
    } else {
        total = nrows;
    }
    int used = 1;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
    used = omp_get_max_threads();
#endif
    int bad = 0;
#pragma omp parallel
    {
        double *scores = (double *)malloc((size_t)(max_kv + 1) * sizeof(double));
        double *acc = (double *)malloc((size_t)d * sizeof(double));
#pragma omp for schedule(dynamic, 16)
        for (int64_t w = 0; w < total; ++w) {
            int i, h; int64_t t;
            if (rows) {
                i = rows[3 * w]; h = rows[3 * w + 1]; t = rows[3 * w + 2];
            } else {
                int lo = 0, hi = n;            /* request owning flat row w */
                while (hi - lo > 1) { int mid = (lo + hi) / 2; if (row_base[mid] <= w) lo = mid; else hi = mid; }
                i = lo;
                int64_t rem = w - row_base[i];
                t = rem / Hq; h = (int)(rem % Hq);
            }
            int64_t lq = 0, lkv = 0;
            if (i >= 0 && i < n) { lq = q_start[i + 1] - q_start[i]; lkv = kv_start[i + 1] - kv_start[i]; }
            if (i < 0 || i >= n || h < 0 || h >= Hq || t < 0 || t >= lq) { bad = 1; continue; }
            const int64_t ctx = lkv - lq;
            const int g = h / r;
            const float *qr = q + ((q_start[i] + t) * Hq + h) * (int64_t)d;
            const float *kb = k + (kv_start[i] * Hkv + g) * (int64_t)d;
            const float *vb = v + (kv_start[i] * Hkv + g) * (int64_t)d;
            float *o = rows ? out + w * d : out + ((q_start[i] + t) * Hq + h) * (int64_t)d;
            int64_t li = rows ? w : (q_start[i] + t) * Hq + h;
            attend_row(qr, kb, vb, ctx + t + 1, (int64_t)Hkv * d, d, scale,
                       scores, acc, o, lse ? lse + li : NULL);
        }
        free(scores); free(acc);
    }
    free(row_base);
    return bad ? -1 : used;
}
