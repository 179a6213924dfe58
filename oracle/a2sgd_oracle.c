/*
 * TEST INFRASTRUCTURE — not part of the product.
 *
 * Plain, slow, scalar CPU oracle of one A2SGD step (two-level gradient averaging), written from the paper's
 * definitions.  It shares no code, header, table or helper with the HIP library; only tests, the smoke check
 * and the benchmark's cpu_baseline leg may call it.  Build: gcc -O2 -ffp-contract=off (no fast-math), so
 * every float expression below is the IEEE-754 operation it looks like.
 *
 * What it follows:
 *   - mu_+(v): mean of v_i over {i : v_i >= 0}; mu_-(v): mean of |v_i| over {i : v_i < 0}   (Sec. 3.1, the
 *     two definitions before Eq. 2).  Zeros belong to the ">= 0" group.
 *   - enc(v) = pos(v)*mu_+(v) - neg(v)*mu_-(v)                                               (Eq. 2)
 *   - Algorithm 1, line 3 (local means), line 4 (error = v - enc(v)), line 5 (global means = plain average
 *     of the workers' means), line 6 (rebuild from the global means), line 7 (w <- w - eta * update).
 *   - The update of all P workers is averaged as in Eq. 1, because one shared w stands for the P replicas.
 *
 * Readings where the paper is silent or at odds with itself:
 *   - Retained-error mode (default): the vector that is encoded is v = fl32(g + e_old); the new error
 *     v - enc(v) is stored for the next step and only the global-mean vector is applied (abstract and
 *     Sec. 3: the local errors are kept, error feedback through a local error vector).
 *   - Algorithm-1-literal mode: the error is added back in the same step, update = error + global-mean vector
 *     (Algorithm 1 lines 4-7 as printed; this is Theorem 1's g + grad-mu form).
 *   - Empty group: its mean is 0 and enters the global average as 0.
 *   - Each worker's message is two fp32 numbers (Sec. 4.3: 64 bits), so the local means are rounded to fp32
 *     before they are averaged; the global means are rounded to fp32 as well.
 *   - NaN belongs to neither group: counted in n_nan, added to no sum, propagates to its own e and w.
 *
 * Precision: the fold v = g + e is one fp32 round-to-nearest add (it is part of the definition, since the
 * sign of v decides the group).  Sums are accumulated in long double (x86 80-bit, 64-bit significand), whose
 * worst-case relative error n * 2^-64 is below 1e-10 for every n used here.  Elementwise results are
 * evaluated in double and rounded once to fp32.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

typedef struct {
    long double s_pos; /* sum of v_i over v_i >= 0 */
    long double s_neg; /* sum of |v_i| over v_i < 0 */
    uint64_t n_pos, n_neg, n_zero, n_nan;
} a2sgd_oracle_acc_t;

enum { A2SGD_ORACLE_RETAINED_ERROR = 0, A2SGD_ORACLE_ALG1_LITERAL = 1 };

/* The vector that gets encoded.  e == NULL means "no retained error": v = g. */
static float fold(const float *g, const float *e, uint64_t i)
{
    if (e == NULL)
        return g[i];
    float v = g[i] + e[i]; /* fp32 add, round to nearest even */
    return v;
}

void a2sgd_oracle_acc_init(a2sgd_oracle_acc_t *acc)
{
    acc->s_pos = 0.0L;
    acc->s_neg = 0.0L;
    acc->n_pos = acc->n_neg = acc->n_zero = acc->n_nan = 0;
}

/* Algorithm 1 line 3, first half: one traversal of a chunk of one worker's vector, adding to the running
 * sums and counts of the two groups.  Chunks may be fed in any split; the order of chunks is the order of
 * summation. */
void a2sgd_oracle_accumulate(const float *g, const float *e, uint64_t m, a2sgd_oracle_acc_t *acc)
{
    for (uint64_t i = 0; i < m; ++i) {
        float v = fold(g, e, i);
        if (v >= 0.0f) {
            acc->n_pos += 1;
            acc->s_pos += (long double)v;
            if (v == 0.0f)
                acc->n_zero += 1;
        } else if (v < 0.0f) {
            acc->n_neg += 1;
            acc->s_neg += -(long double)v;
        } else {
            acc->n_nan += 1;
        }
    }
}

/* Algorithm 1 line 3, second half: the two local means, each rounded to the fp32 that is transmitted. */
void a2sgd_oracle_local_means(const a2sgd_oracle_acc_t *acc, float *mu_pos, float *mu_neg)
{
    *mu_pos = acc->n_pos ? (float)(acc->s_pos / (long double)acc->n_pos) : 0.0f;
    *mu_neg = acc->n_neg ? (float)(acc->s_neg / (long double)acc->n_neg) : 0.0f;
}

/* Algorithm 1 line 5: Allreduce(average) of the P workers' pairs, p ascending, unweighted. */
void a2sgd_oracle_global_means(const float *mu_pos, const float *mu_neg, uint32_t P, float *gmu_pos, float *gmu_neg)
{
    double sp = 0.0, sn = 0.0;
    for (uint32_t p = 0; p < P; ++p) {
        sp += (double)mu_pos[p];
        sn += (double)mu_neg[p];
    }
    *gmu_pos = (float)(sp / (double)P);
    *gmu_neg = (float)(sn / (double)P);
}

/* Algorithm 1 lines 4, 6 and 7 on a chunk of m elements, for all P workers.
 *   g[p], e[p]   : worker p's chunk (e may be NULL, or e[p] may be NULL: no retained error)
 *   e_new[p]     : out, the new local error of worker p (line 4)
 *   mask[p]      : out (may be NULL), 1 where v_i >= 0, else 0: pos(v)
 *   w -> w_new   : line 7 with the update averaged over the workers (Eq. 1)
 */
void a2sgd_oracle_apply_chunk(const float *const *g, const float *const *e, uint32_t P, uint64_t m,
                              const float *mu_pos, const float *mu_neg, float gmu_pos, float gmu_neg, float eta,
                              int mode, float *const *e_new, const float *w, float *w_new, uint8_t *const *mask)
{
    for (uint64_t i = 0; i < m; ++i) {
        double usum = 0.0;
        for (uint32_t p = 0; p < P; ++p) {
            float v = fold(g[p], e ? e[p] : NULL, i);
            double err, glob;
            if (v >= 0.0f) {
                err = (double)v - (double)mu_pos[p]; /* v - enc(v) where pos(v) = 1 */
                glob = (double)gmu_pos;
            } else if (v < 0.0f) {
                err = (double)v + (double)mu_neg[p]; /* v - enc(v) where neg(v) = 1 */
                glob = -(double)gmu_neg;
            } else { /* NaN: in neither group, enc = 0 */
                err = (double)v;
                glob = (double)v;
            }
            e_new[p][i] = (float)err;
            if (mask && mask[p])
                mask[p][i] = (uint8_t)(v >= 0.0f);
            usum += (mode == A2SGD_ORACLE_ALG1_LITERAL) ? err + glob : glob;
        }
        double U = usum / (double)P;
        w_new[i] = (float)((double)w[i] - (double)eta * U);
    }
}

/* Final synchronisation step of Algorithm 1 (lines 9-10) and the dense-SGD update of Eq. 1:
 * w <- w - eta * (1/P) sum_p g^p. */
void a2sgd_oracle_dense_step(const float *const *g, uint32_t P, uint64_t m, float eta, const float *w, float *w_new)
{
    for (uint64_t i = 0; i < m; ++i) {
        double s = 0.0;
        for (uint32_t p = 0; p < P; ++p)
            s += (double)g[p][i];
        w_new[i] = (float)((double)w[i] - (double)eta * (s / (double)P));
    }
}

/* Algorithm 1 lines 4, 6 and 7 as each worker runs them on its OWN replica of the model: the same error and
 * rebuilt gradient as a2sgd_oracle_apply_chunk, but w[p] <- w[p] - eta * u^p per worker, with no averaging over
 * the workers (line 7 as printed; the replicas drift apart, which is why the algorithm ends with a
 * synchronisation step). */
void a2sgd_oracle_apply_chunk_replicas(const float *const *g, const float *const *e, uint32_t P, uint64_t m,
                                       const float *mu_pos, const float *mu_neg, float gmu_pos, float gmu_neg,
                                       float eta, int mode, float *const *e_new, const float *const *w,
                                       float *const *w_new)
{
    for (uint32_t p = 0; p < P; ++p) {
        for (uint64_t i = 0; i < m; ++i) {
            float v = fold(g[p], e ? e[p] : NULL, i);
            double err, glob;
            if (v >= 0.0f) {
                err = (double)v - (double)mu_pos[p];
                glob = (double)gmu_pos;
            } else if (v < 0.0f) {
                err = (double)v + (double)mu_neg[p];
                glob = -(double)gmu_neg;
            } else {
                err = (double)v;
                glob = (double)v;
            }
            e_new[p][i] = (float)err;
            double u = (mode == A2SGD_ORACLE_ALG1_LITERAL) ? err + glob : glob;
            w_new[p][i] = (float)((double)w[p][i] - (double)eta * u);
        }
    }
}

/* Final synchronisation on replicas (Algorithm 1 lines 9-10): every replica takes the same dense averaged
 * gradient, w[p] <- w[p] - eta * (1/P) sum_q g^q. */
void a2sgd_oracle_dense_step_replicas(const float *const *g, uint32_t P, uint64_t m, float eta,
                                      const float *const *w, float *const *w_new)
{
    for (uint64_t i = 0; i < m; ++i) {
        double s = 0.0;
        for (uint32_t p = 0; p < P; ++p)
            s += (double)g[p][i];
        for (uint32_t p = 0; p < P; ++p)
            w_new[p][i] = (float)((double)w[p][i] - (double)eta * (s / (double)P));
    }
}

/* How far the replicas have drifted: with wbar_i = (1/P) sum_p w[p][i], per worker the largest |w[p][i] - wbar_i|
 * and the sum of squares of those deviations, accumulated over chunks (max_abs[p] and sum_sq[p] are updated in
 * place; start them at 0). */
void a2sgd_oracle_replica_drift(const float *const *w, uint32_t P, uint64_t m, double *max_abs, long double *sum_sq)
{
    for (uint64_t i = 0; i < m; ++i) {
        double s = 0.0;
        for (uint32_t p = 0; p < P; ++p)
            s += (double)w[p][i];
        double mean = s / (double)P;
        for (uint32_t p = 0; p < P; ++p) {
            double d = (double)w[p][i] - mean;
            double a = fabs(d);
            if (a > max_abs[p] || a != a)
                max_abs[p] = a;
            sum_sq[p] += (long double)d * (long double)d;
        }
    }
}
