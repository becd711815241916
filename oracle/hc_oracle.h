/* hc_oracle.h -- CPU oracle for the HeteroCache decode hot path (TEST INFRASTRUCTURE ONLY).
 *
 * Plain, slow, fp64 C written from the paper's definitions (Sec. 4.3, Eq. 1, 9, 10,
 * Algorithm 1 stage 3, App. C.1).  It shares no code, header, table or constant with the
 * HIP library and must never be linked or imported by the product path: only the tests,
 * the smoke check and the benchmark's cpu_baseline leg may use it.
 *
 * All pointers are HOST pointers.  bf16 values are passed as their 16-bit patterns and
 * are widened exactly to double before any arithmetic.
 *
 * Pins (tests/test_oracle_*.py): dense fp64 attention of a library routine, closed forms
 * (identical keys, dominant key, LSE merge of any partition, permutation invariance),
 * brute force on tiny inputs, stable-argsort top-k, hand-derived integer thresholds of the
 * drift test, a bivariate-normal expectation of the overlap after a query rotation.
 * The paper prints no worked numeric example for this path, so parity with the authors'
 * own prototype is unpinned; parity is to the definitions.
 */
#ifndef HC_ORACLE_H
#define HC_ORACLE_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* One KV head's attention for its G query heads (Algorithm 1, ModelForward over C_GPU;
 * the resident set is defined in Sec. 4.3). */
typedef struct {
    const uint16_t* q;      /* bf16 [G][D]: the query heads that share this KV head          */
    const uint16_t* K;      /* bf16 [N][D]: master (full-length) keys of this KV head        */
    const uint16_t* V;      /* bf16 [N][D]: master values                                    */
    const int32_t*  idx;    /* resident positions, n entries; NULL means 0..n-1              */
    int32_t         n;      /* number of resident tokens (>= 1)                              */
    double*         out;    /* [G][D]  softmax(qK^T/sqrt(D)) V                               */
    double*         lse;    /* [G]     log-sum-exp of the scaled logits                      */
    double*         logits; /* [G][n]  scaled logits in resident order, or NULL              */
} hc_ref_job;

/* Runs every job.  Returns 0, or -1 if a non-finite input or an empty job is found. */
int hc_ref_attn_jobs(const hc_ref_job* jobs, int32_t njobs, int32_t G, int32_t D);

/* GQA-aggregated score of every position (App. C.1: mean of the group's attention weights):
 *   agg = 0:  s[j] = (1/G) sum_g exp(logits[g][j] - lse[g])
 *   agg = 1:  s[j] = (1/G) sum_g logits[g][j]                  (test mode)                   */
int hc_ref_scores(const double* logits, const double* lse, int32_t G, int32_t N, int32_t agg, double* s);

/* TopIndices_k (Algorithm 1): the k candidates of [lo,hi) that come first under the total
 * order (score descending, index ascending), returned as an ascending index list.  The scores
 * are fp32 because that is the precision the decision is taken in.  Returns 0, -1 on bad args. */
int hc_ref_topk(const float* s, int32_t lo, int32_t hi, int32_t k, int32_t* out);

/* |A ∩ B| for two index lists without repeated entries (negative entries never match). */
int32_t hc_ref_intersect(const int32_t* a, int32_t na, const int32_t* b, int32_t nb);

/* Retrieval signal r_t (Eq. 10) from the last W intersection sizes (all against sets of size k):
 * lower median of the window, then the exact integer form of  statistic < tau_num/tau_den  with
 *   metric 0 (overlap, Eq. 9):  inter/k            metric 1 (Jaccard):  inter/(2k - inter).   */
int32_t hc_ref_trigger(const int32_t* window_inter, int32_t W, int32_t k, int32_t metric,
                       int32_t tau_num, int32_t tau_den);

/* Threads the jobs loop will use (for reporting). */
int32_t hc_ref_threads(void);

#ifdef __cplusplus
}
#endif
#endif
