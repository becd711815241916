/* hc_oracle.c -- CPU oracle, see hc_oracle.h.  TEST INFRASTRUCTURE ONLY. */
#include "hc_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double bf16_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* softmax(q K^T / sqrt(D)) V for one query head over the resident set (Algorithm 1, ModelForward). */
static int attn_one(const hc_ref_job* job, int g, int D)
{
    const int n = job->n;
    const uint16_t* q = job->q + (size_t)g * D;
    double* logit = job->logits ? job->logits + (size_t)g * n : (double*)malloc(sizeof(double) * (size_t)n);
    double* out = job->out + (size_t)g * D;
    int bad = 0;
    if (!logit) return -1;

    const double scale = 1.0 / sqrt((double)D);
    double m = -INFINITY;
    for (int t = 0; t < n; ++t) {
        const size_t j = job->idx ? (size_t)job->idx[t] : (size_t)t;
        const uint16_t* k = job->K + j * D;
        double dot = 0.0;
        for (int d = 0; d < D; ++d) dot += bf16_to_double(q[d]) * bf16_to_double(k[d]);
        logit[t] = dot * scale;
        if (!isfinite(logit[t])) bad = 1;
        if (logit[t] > m) m = logit[t];
    }
    double Z = 0.0;
    for (int d = 0; d < D; ++d) out[d] = 0.0;
    for (int t = 0; t < n; ++t) {
        const size_t j = job->idx ? (size_t)job->idx[t] : (size_t)t;
        const uint16_t* v = job->V + j * D;
        const double w = exp(logit[t] - m);
        Z += w;
        for (int d = 0; d < D; ++d) out[d] += w * bf16_to_double(v[d]);
    }
    for (int d = 0; d < D; ++d) {
        out[d] /= Z;
        if (!isfinite(out[d])) bad = 1;
    }
    job->lse[g] = m + log(Z);
    if (!job->logits) free(logit);
    return bad ? -1 : 0;
}

int hc_ref_attn_jobs(const hc_ref_job* jobs, int32_t njobs, int32_t G, int32_t D)
{
    int err = 0;
    if (!jobs || njobs < 0 || G < 1 || D < 1) return -1;
    for (int i = 0; i < njobs; ++i)
        if (jobs[i].n < 1 || !jobs[i].q || !jobs[i].K || !jobs[i].V || !jobs[i].out || !jobs[i].lse) return -1;
#pragma omp parallel for collapse(2) schedule(dynamic, 1) reduction(| : err)
    for (int i = 0; i < njobs; ++i)
        for (int g = 0; g < G; ++g)
            if (attn_one(&jobs[i], g, D) != 0) err |= 1;
    return err ? -1 : 0;
}

int hc_ref_scores(const double* logits, const double* lse, int32_t G, int32_t N, int32_t agg, double* s)
{
    if (!logits || !s || G < 1 || N < 0 || (agg == 0 && !lse)) return -1;
    for (int j = 0; j < N; ++j) {
        double acc = 0.0;
        for (int g = 0; g < G; ++g) {
            const double l = logits[(size_t)g * N + j];
            acc += (agg == 0) ? exp(l - lse[g]) : l;
        }
        s[j] = acc / (double)G;
    }
    return 0;
}

typedef struct { float s; int32_t j; } scored;

static int by_score_desc_index_asc(const void* a, const void* b)
{
    const scored* x = (const scored*)a;
    const scored* y = (const scored*)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->j > y->j) - (x->j < y->j);   /* equal scores (also -0 == +0): lowest index first */
}

static int by_int_asc(const void* a, const void* b)
{
    const int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
    return (x > y) - (x < y);
}

int hc_ref_topk(const float* s, int32_t lo, int32_t hi, int32_t k, int32_t* out)
{
    if (!s || !out || lo < 0 || hi < lo || k < 0 || k > hi - lo) return -1;
    const int n = hi - lo;
    scored* a = (scored*)malloc(sizeof(scored) * (size_t)(n > 0 ? n : 1));
    if (!a) return -1;
    for (int t = 0; t < n; ++t) {
        if (isnan(s[lo + t])) { free(a); return -1; }
        a[t].s = s[lo + t];
        a[t].j = lo + t;
    }
    qsort(a, (size_t)n, sizeof(scored), by_score_desc_index_asc);
    for (int t = 0; t < k; ++t) out[t] = a[t].j;
    qsort(out, (size_t)k, sizeof(int32_t), by_int_asc);
    free(a);
    return 0;
}

int32_t hc_ref_intersect(const int32_t* a, int32_t na, const int32_t* b, int32_t nb)
{
    int32_t c = 0;
    for (int i = 0; i < na; ++i) {
        if (a[i] < 0) continue;
        for (int j = 0; j < nb; ++j)
            if (a[i] == b[j]) { ++c; break; }
    }
    return c;
}

int32_t hc_ref_trigger(const int32_t* window_inter, int32_t W, int32_t k, int32_t metric,
                       int32_t tau_num, int32_t tau_den)
{
    if (!window_inter || W < 1 || k < 1 || tau_den < 1) return -1;
    int32_t* w = (int32_t*)malloc(sizeof(int32_t) * (size_t)W);
    if (!w) return -1;
    memcpy(w, window_inter, sizeof(int32_t) * (size_t)W);
    qsort(w, (size_t)W, sizeof(int32_t), by_int_asc);
    const int64_t med = w[(W - 1) / 2];          /* lower middle for even W */
    free(w);
    if (metric == 0)                              /* med/k < num/den */
        return med * (int64_t)tau_den < (int64_t)tau_num * (int64_t)k;
    /* Jaccard of two k-sets: med/(2k-med) < num/den */
    return med * (int64_t)tau_den < (int64_t)tau_num * (2 * (int64_t)k - med);
}

int32_t hc_ref_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
