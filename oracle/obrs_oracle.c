/*
 * OBRS oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, float64 CPU statement of what the Jackpot / OBRS hot path
 * computes, written from the paper's definitions.  Only the test-suite, the
 * smoke check and the benchmark's cpu_baseline leg may call it.  It shares no
 * code, header, table or helper with the HIP library and neither side
 * includes the other.
 *
 * Notation (paper Sec. 3.1 / Sec. 4.1): q = softmax(actor logits) is the
 * rollout ("inference") distribution p_inf, p = softmax(policy logits) is the
 * target distribution p_target, lambda > 0 the rejection threshold, x the
 * token that was sampled from q.
 *
 * Every function below is pinned by tests that do not call it to produce
 * their expected value (closed forms, brute force on tiny vocabularies,
 * library routines, theorems of Sec. 3.3 / App. A).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { JPO_F32 = 0, JPO_BF16 = 1, JPO_F64 = 2 };

/* Per-row results.  Field order is mirrored by the ctypes binding. */
typedef struct {
    double lse_q, lse_p;        /* log-sum-exp of the two logit rows            */
    double logq_x, logp_x;      /* log q(x), log p(x) of the sampled token      */
    double logratio;            /* log p(x) - log q(x)                          */
    double accept;              /* a(x) = min(1, p(x) / (lambda q(x)))          */
    double z_approx;            /* sum over V_k of min(q, p/lambda)             */
    double z_exact;             /* sum over the vocabulary of min(q, p/lambda)  */
    double kl_p_q;              /* KL(p || q)                                   */
    double kl_p_qtilde;         /* KL(p || q~), q~ = min(q, p/lambda)/Z         */
    int32_t mask;               /* 1 iff u < a(x)                               */
    int32_t union_size;         /* |V_k|                                        */
    int32_t valid;              /* 0 for a padding row (x < 0)                  */
    int32_t pad_;
} jpo_row_out;

/* Batch results (Sec. 4.4.2). */
typedef struct {
    int64_t n_valid;            /* proposed tokens B                            */
    int64_t n_accept;           /* accepted tokens                              */
    double alpha_hat;           /* n_accept / n_valid                           */
    double mean_z_approx;       /* (1/B) sum_i Z_approx^(i)                     */
    double kappa;               /* alpha_hat / mean_z_approx                    */
    double mean_z_exact;
    double mean_accept;         /* (1/B) sum_i a(x_i)                           */
    double mean_kl_p_q;         /* (1/B) sum_i KL(p_i || q_i): the distillation loss value
                                   of Sec. 4.2 (3), Eq. distill_loss                 */
} jpo_batch_out;

/* ---- exact widening of stored logits ---------------------------------- */

static double bf16_to_double(uint16_t h)
{
    /* bfloat16 is the upper half of an IEEE binary32. */
    uint32_t w = (uint32_t)h << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

void jpo_widen_row(const void *src, int dtype, int64_t V, double *dst)
{
    if (dtype == JPO_F32) {
        const float *s = (const float *)src;
        for (int64_t v = 0; v < V; ++v) dst[v] = (double)s[v];
    } else if (dtype == JPO_BF16) {
        const uint16_t *s = (const uint16_t *)src;
        for (int64_t v = 0; v < V; ++v) dst[v] = bf16_to_double(s[v]);
    } else {
        memcpy(dst, src, (size_t)V * sizeof(double));
    }
}

/* ---- softmax in the log domain ----------------------------------------
 * The distribution of a language model is the softmax of its logits
 * (Sec. 2).  log softmax(l)_v = l_v - LSE(l),
 * LSE(l) = m + log sum_v exp(l_v - m), m = max_v l_v.               */
double jpo_logsumexp(const double *l, int64_t V)
{
    double m = -INFINITY;
    for (int64_t v = 0; v < V; ++v)
        if (l[v] > m) m = l[v];
    if (!(m > -INFINITY)) return m;          /* all -inf (or empty) */
    double s = 0.0;
    for (int64_t v = 0; v < V; ++v) s += exp(l[v] - m);
    return m + log(s);
}

/* ---- top-k(p): the k most probable tokens (Sec. 4.4.1) ----------------
 * Selection is on the logits (softmax is monotone).  Equal values are
 * ordered by the lowest token id first.  The whole id list is sorted and
 * the first k entries are returned, in that order.                    */
static const double *g_sort_key;
#ifdef _OPENMP
#pragma omp threadprivate(g_sort_key)
#endif

static int cmp_desc_value_asc_id(const void *a, const void *b)
{
    int32_t ia = *(const int32_t *)a, ib = *(const int32_t *)b;
    double va = g_sort_key[ia], vb = g_sort_key[ib];
    if (va > vb) return -1;
    if (va < vb) return 1;
    return (ia > ib) - (ia < ib);
}

void jpo_topk(const double *l, int64_t V, int32_t k, int32_t *ids_out)
{
    int32_t *ids = (int32_t *)malloc((size_t)V * sizeof(int32_t));
    for (int64_t v = 0; v < V; ++v) ids[v] = (int32_t)v;
    g_sort_key = l;
    qsort(ids, (size_t)V, sizeof(int32_t), cmp_desc_value_asc_id);
    for (int32_t j = 0; j < k; ++j) ids_out[j] = ids[j];
    free(ids);
}

/* min(q_v, p_v / lambda): the un-normalised post-rejection mass of token v
 * (Eq. obrs_dist; App. A.1). */
static double kept_mass(double logq_v, double logp_v, double lambda)
{
    double qv = exp(logq_v);
    double pv = exp(logp_v) / lambda;
    return qv < pv ? qv : pv;
}

/* From log q(x) and log p(x) already in `out`: their difference, the acceptance probability and
 * the Bernoulli draw (shared by the two-tensor and the stored-actor form of a row).             */
static void accept_and_mask(jpo_row_out *out, double u, double lambda)
{
    out->logratio = out->logp_x - out->logq_x;

    /* Eq. obrs_accept: a(x) = min(1, p(x) / (lambda q(x))) */
    double r = exp(out->logratio) / lambda;
    out->accept = r < 1.0 ? r : 1.0;

    /* Mask(x) ~ Bernoulli(a(x)), realised as U(0,1) < a  (Alg. 2) */
    out->mask = (u < out->accept) ? 1 : 0;
}

/* ---- one token position ------------------------------------------------
 * lq, lp: logits of the rollout and the target model over V tokens.
 * x: sampled token (x < 0 marks a padding row; x >= V is no token of the vocabulary: the row is
 * left out like a padding row, with NaN results), u: uniform in [0,1).
 * topk_q / topk_p (each k ids) may be NULL.                              */
void jpo_row(const double *lq, const double *lp, int64_t V, int32_t x, double u,
             double lambda, int32_t k, jpo_row_out *out, int32_t *topk_q, int32_t *topk_p)
{
    memset(out, 0, sizeof *out);
    if (x < 0) return;
    if ((int64_t)x >= V) {                  /* not a token of this vocabulary: no part of the batch */
        out->lse_q = out->lse_p = out->logq_x = out->logp_x = out->logratio = out->accept = NAN;
        out->z_approx = out->z_exact = out->kl_p_q = out->kl_p_qtilde = NAN;
        return;
    }
    out->valid = 1;

    double lse_q = jpo_logsumexp(lq, V);
    double lse_p = jpo_logsumexp(lp, V);
    out->lse_q = lse_q;
    out->lse_p = lse_p;

    /* log-probabilities of the sampled token */
    out->logq_x = lq[x] - lse_q;
    out->logp_x = lp[x] - lse_p;
    accept_and_mask(out, u, lambda);

    /* V_k = top-k(q) U top-k(p), a set (Sec. 4.4.1) */
    int32_t *kq = (int32_t *)malloc((size_t)k * sizeof(int32_t));
    int32_t *kp = (int32_t *)malloc((size_t)k * sizeof(int32_t));
    jpo_topk(lq, V, k, kq);
    jpo_topk(lp, V, k, kp);
    unsigned char *in_union = (unsigned char *)calloc((size_t)V, 1);
    for (int32_t j = 0; j < k; ++j) in_union[kq[j]] = 1;
    for (int32_t j = 0; j < k; ++j) in_union[kp[j]] = 1;

    /* Z_approx over V_k, Z over the whole vocabulary, both in id order */
    double z_approx = 0.0, z_exact = 0.0;
    int32_t usize = 0;
    for (int64_t v = 0; v < V; ++v) {
        double t = kept_mass(lq[v] - lse_q, lp[v] - lse_p, lambda);
        z_exact += t;
        if (in_union[v]) {
            z_approx += t;
            ++usize;
        }
    }
    out->z_approx = z_approx;
    out->z_exact = z_exact;
    out->union_size = usize;

    /* diagnostics used only by the oracle's own pins: KL(p||q), KL(p||q~) */
    double kl_pq = 0.0, kl_pqt = 0.0;
    for (int64_t v = 0; v < V; ++v) {
        double logp_v = lp[v] - lse_p, logq_v = lq[v] - lse_q;
        double pv = exp(logp_v);
        if (pv > 0.0) {
            double qt = kept_mass(logq_v, logp_v, lambda) / z_exact;
            kl_pq += pv * (logp_v - logq_v);
            kl_pqt += pv * (logp_v - log(qt));
        }
    }
    out->kl_p_q = kl_pq;
    out->kl_p_qtilde = kl_pqt;

    if (topk_q) memcpy(topk_q, kq, (size_t)k * sizeof(int32_t));
    if (topk_p) memcpy(topk_p, kp, (size_t)k * sizeof(int32_t));
    free(in_union);
    free(kp);
    free(kq);
}

/* ---- one token position with the actor side as the rollout phase stored it --------------
 * Alg. 1, Phase 1 keeps, per position, the sampled token's probability p_inf(a_t) and the top-k
 * log-probabilities TopK_inf of the rollout model, not its logits; Phase 2 has the target
 * model's full logits.  So here: lp[V] target logits; ids_q[nq], logq_ids[nq] the stored list
 * (an id < 0 marks an unused slot, a repeated id counts once); logq_x = log q(x).
 *   a(x), mask: as in jpo_row, from logq_x and log p(x).
 *   V_k = stored ids U top-k(p)                                     (Alg. 1 step 2)
 *   Z_approx = sum_{v in stored} min(q_v, p_v/lambda) + sum_{v in top-k(p), not stored} min(qhat, p_v/lambda)
 * The paper does not say what q_v is for a token of TopK_new that TopK_inf does not hold.  qhat is
 * a stated rule: 0 = such tokens contribute nothing; 1 = the smallest stored probability (an
 * upper bound of q_v, since v is not among the k largest); 2 = the probability mass the stored
 * list leaves, spread evenly over the other V - n tokens, capped by rule 1's bound.
 * z_exact, kl_* are not available in this form (NaN).                                         */
enum { JPO_TAIL_DROP = 0, JPO_TAIL_KTH = 1, JPO_TAIL_REST = 2 };

void jpo_row_stored(const double *lp, int64_t V, const int32_t *ids_q, const double *logq_ids,
                    int32_t nq, double logq_x, int32_t x, double u, double lambda, int32_t k,
                    int tail_rule, jpo_row_out *out, int32_t *topk_p)
{
    memset(out, 0, sizeof *out);
    if (x < 0) return;
    if ((int64_t)x >= V) {                  /* not a token of this vocabulary: no part of the batch */
        out->lse_q = out->lse_p = out->logq_x = out->logp_x = out->logratio = out->accept = NAN;
        out->z_approx = out->z_exact = out->kl_p_q = out->kl_p_qtilde = NAN;
        return;
    }
    out->valid = 1;
    double lse_p = jpo_logsumexp(lp, V);
    out->lse_q = 0.0;
    out->lse_p = lse_p;
    out->logq_x = logq_x;
    out->logp_x = lp[x] - lse_p;
    accept_and_mask(out, u, lambda);

    /* the stored list: first occurrence of every valid id */
    double *qlog = (double *)malloc((size_t)V * sizeof(double));
    unsigned char *stored = (unsigned char *)calloc((size_t)V, 1);
    int64_t n = 0;
    double kth = 0.0, mass = 0.0;          /* smallest stored log-probability, stored probability mass */
    for (int32_t j = 0; j < nq; ++j) {
        int32_t v = ids_q[j];
        if (v < 0 || v >= V || stored[v]) continue;
        stored[v] = 1;
        qlog[v] = logq_ids[j];
        if (n == 0 || logq_ids[j] < kth) kth = logq_ids[j];
        mass += exp(logq_ids[j]);
        ++n;
    }
    double tail;                            /* log qhat */
    if (tail_rule == JPO_TAIL_DROP || n == V) {
        tail = -INFINITY;
    } else if (tail_rule == JPO_TAIL_KTH) {
        tail = kth;                         /* log 1 = 0 when nothing is stored */
    } else {
        double rest = 1.0 - mass;
        if (rest < 0.0) rest = 0.0;
        double share = rest / (double)(V - n);
        tail = log(share);
        if (tail > kth) tail = kth;
    }

    int32_t *kp = (int32_t *)malloc((size_t)k * sizeof(int32_t));
    jpo_topk(lp, V, k, kp);
    unsigned char *in_p = (unsigned char *)calloc((size_t)V, 1);
    for (int32_t j = 0; j < k; ++j) in_p[kp[j]] = 1;
    double z = 0.0;
    int32_t usize = 0;
    for (int64_t v = 0; v < V; ++v) {
        if (stored[v]) {
            z += kept_mass(qlog[v], lp[v] - lse_p, lambda);
            ++usize;
        } else if (in_p[v]) {
            z += kept_mass(tail, lp[v] - lse_p, lambda);
            ++usize;
        }
    }
    out->z_approx = z;
    out->union_size = usize;
    out->z_exact = NAN;
    out->kl_p_q = NAN;
    out->kl_p_qtilde = NAN;
    if (topk_p) memcpy(topk_p, kp, (size_t)k * sizeof(int32_t));
    free(in_p);
    free(kp);
    free(stored);
    free(qlog);
}

/* The same for a batch: target logits in their storage dtype, the stored actor side as the
 * rollout phase would hand it over (int32 ids, float32 log-probabilities).  Returns threads used. */
int jpo_rows_stored(const void *policy, int dtype, int64_t T, int64_t V, int64_t row_stride,
                    const int32_t *ids_q, const float *logq_ids, const float *logq_x,
                    const int32_t *x, const float *u, double lambda, int32_t k, int tail_rule,
                    jpo_row_out *out, int32_t *topk_p, int n_threads)
{
    size_t esz = dtype == JPO_F32 ? 4 : dtype == JPO_BF16 ? 2 : 8;
    int used = 1;
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
#else
    {
#endif
        double *lp = (double *)malloc((size_t)V * sizeof(double));
        double *lq = (double *)malloc((size_t)k * sizeof(double));
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 1)
#endif
        for (int64_t t = 0; t < T; ++t) {
            jpo_widen_row((const char *)policy + (size_t)t * (size_t)row_stride * esz, dtype, V, lp);
            for (int32_t j = 0; j < k; ++j) lq[j] = (double)logq_ids[(size_t)t * k + j];
            jpo_row_stored(lp, V, ids_q + (size_t)t * k, lq, k, (double)logq_x[t], x[t],
                           u ? (double)u[t] : 2.0, lambda, k, tail_rule, &out[t],
                           topk_p ? topk_p + (size_t)t * k : NULL);
        }
        free(lq);
        free(lp);
    }
    return used;
}

/* Post-rejection distribution q~_v = min(q_v, p_v/lambda) / Z for one row
 * (Eq. obrs_dist), written to qt[V]; returns Z. */
double jpo_post_rejection(const double *lq, const double *lp, int64_t V, double lambda, double *qt)
{
    double lse_q = jpo_logsumexp(lq, V), lse_p = jpo_logsumexp(lp, V);
    double z = 0.0;
    for (int64_t v = 0; v < V; ++v) {
        qt[v] = kept_mass(lq[v] - lse_q, lp[v] - lse_p, lambda);
        z += qt[v];
    }
    for (int64_t v = 0; v < V; ++v) qt[v] /= z;
    return z;
}

/* ---- a batch of rows stored in their input dtype -----------------------
 * actor / policy: [T, V] row-major with row_stride elements between rows.
 * Rows are independent, so they may be computed by several threads; each
 * row is computed exactly as jpo_row does.  Returns the threads used.   */
int jpo_rows(const void *actor, const void *policy, int dtype, int64_t T, int64_t V,
             int64_t row_stride, const int32_t *x, const float *u, double lambda, int32_t k,
             jpo_row_out *out, int32_t *topk_q, int32_t *topk_p, int n_threads)
{
    size_t esz = dtype == JPO_F32 ? 4 : dtype == JPO_BF16 ? 2 : 8;
    int used = 1;
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
#else
    {
#endif
        double *lq = (double *)malloc((size_t)V * sizeof(double));
        double *lp = (double *)malloc((size_t)V * sizeof(double));
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 1)
#endif
        for (int64_t t = 0; t < T; ++t) {
            const char *ra = (const char *)actor + (size_t)t * (size_t)row_stride * esz;
            const char *rp = (const char *)policy + (size_t)t * (size_t)row_stride * esz;
            jpo_widen_row(ra, dtype, V, lq);
            jpo_widen_row(rp, dtype, V, lp);
            jpo_row(lq, lp, V, x[t], u ? (double)u[t] : 2.0, lambda, k, &out[t],
                    topk_q ? topk_q + (size_t)t * k : NULL, topk_p ? topk_p + (size_t)t * k : NULL);
        }
        free(lp);
        free(lq);
    }
    return used;
}

/* ---- gradient of the distillation term (Sec. 4.2 (3), Eq. distill_loss) --
 * The loss per token is KL(SG(p) || q) = sum_v p_v (log p_v - log q_v) with
 * p held fixed, q = softmax(lq).  Since d log q_u / d lq_v = [u = v] - q_v,
 *   d KL / d lq_v = -p_v + q_v sum_u p_u = q_v - p_v.
 * out[v] = weight * (q_v - p_v).                                          */
void jpo_distill_grad_row(const double *lq, const double *lp, int64_t V, double weight, double *out)
{
    const double lse_q = jpo_logsumexp(lq, V), lse_p = jpo_logsumexp(lp, V);
    for (int64_t v = 0; v < V; ++v) out[v] = weight * (exp(lq[v] - lse_q) - exp(lp[v] - lse_p));
}

/* The same for a batch stored in its input dtype.  Padding rows (x[t] < 0), rows whose
 * sampled id is outside the vocabulary and rows with a non-finite log-sum-exp get zeros
 * (they take no part in the loss).  weight_t = scale * (row_scale ? row_scale[t] : 1).  */
void jpo_distill_grad(const void *actor, const void *policy, int dtype, int64_t T, int64_t V,
                      int64_t row_stride, const int32_t *x, const float *row_scale, double scale,
                      double *out /* [T, V] */)
{
    size_t esz = dtype == JPO_F32 ? 4 : dtype == JPO_BF16 ? 2 : 8;
    double *lq = (double *)malloc((size_t)V * sizeof(double));
    double *lp = (double *)malloc((size_t)V * sizeof(double));
    for (int64_t t = 0; t < T; ++t) {
        double *o = out + (size_t)t * (size_t)V;
        jpo_widen_row((const char *)actor + (size_t)t * (size_t)row_stride * esz, dtype, V, lq);
        jpo_widen_row((const char *)policy + (size_t)t * (size_t)row_stride * esz, dtype, V, lp);
        const double lse_q = jpo_logsumexp(lq, V), lse_p = jpo_logsumexp(lp, V);
        if (x[t] < 0 || x[t] >= V || !isfinite(lse_q) || !isfinite(lse_p)) {
            for (int64_t v = 0; v < V; ++v) o[v] = 0.0;
            continue;
        }
        jpo_distill_grad_row(lq, lp, V, scale * (row_scale ? (double)row_scale[t] : 1.0), o);
    }
    free(lp);
    free(lq);
}

/* ---- the scaling factor for a given acceptance budget (Sec. 3.3, Theorem 2) -----------------
 * For a budget abar in (0, 1] there is a lambda with sum_v q_v min(1, p_v / (lambda q_v)) = abar.
 * The left side is Z(lambda) = sum_{r_v > lambda} q_v + (1/lambda) sum_{r_v <= lambda} p_v with
 * r_v = p_v / q_v: continuous, equal to 1 up to min_v r_v, strictly decreasing after it, and
 * piecewise of the form A + B / lambda between consecutive ratios.  So: sort the ratios, find the
 * piece on which Z crosses abar, solve A + B / lambda = abar there.  For abar = 1 every
 * lambda <= min r_v does; the largest of them is returned (lambda = sup{ l : Z(l) >= abar }).
 * Tokens with q_v = 0 or p_v = 0 keep nothing whatever lambda is and are left out.
 * Returns NaN for abar outside (0, 1].                                                         */
typedef struct { double r, q, p; } jpo_ratio;

static int cmp_ratio(const void *a, const void *b)
{
    double ra = ((const jpo_ratio *)a)->r, rb = ((const jpo_ratio *)b)->r;
    return (ra > rb) - (ra < rb);
}

/* Sort the n (ratio, q-mass, p-mass) entries and solve Z(lambda) = abar on the piece where Z crosses it. */
static double solve_budget(jpo_ratio *e, int64_t n, double abar)
{
    if (n == 0) return NAN;
    qsort(e, (size_t)n, sizeof(jpo_ratio), cmp_ratio);
    /* A = mass of q on ratios above the piece, B = mass of p on ratios at or below it */
    double A = 0.0, B = 0.0, lambda = NAN;
    for (int64_t i = 0; i < n; ++i) A += e[i].q;
    /* piece 0 is lambda <= r_(1): Z = A (all of q that can be kept); it holds the budget only if abar >= A */
    if (abar >= A) { lambda = e[0].r; return lambda; }
    for (int64_t i = 0; i < n; ++i) {
        A -= e[i].q;
        B += e[i].p;
        /* piece i+1: r_(i+1) <= lambda < r_(i+2) (the last piece is unbounded above) */
        double upper = (i + 1 < n) ? e[i + 1].r : INFINITY;
        double z_upper = (i + 1 < n) ? A + B / upper : 0.0;
        if (abar > z_upper || i + 1 == n) {
            lambda = B / (abar - A);
            break;
        }
    }
    return lambda;
}

double jpo_lambda_for_budget(const double *lq, const double *lp, int64_t V, double abar)
{
    if (!(abar > 0.0) || abar > 1.0) return NAN;
    double lse_q = jpo_logsumexp(lq, V), lse_p = jpo_logsumexp(lp, V);
    jpo_ratio *e = (jpo_ratio *)malloc((size_t)V * sizeof(jpo_ratio));
    int64_t n = 0;
    for (int64_t v = 0; v < V; ++v) {
        double q = exp(lq[v] - lse_q), p = exp(lp[v] - lse_p);
        if (!(q > 0.0) || !(p > 0.0)) continue;
        e[n].r = exp((lp[v] - lse_p) - (lq[v] - lse_q));
        e[n].q = q;
        e[n].p = p;
        ++n;
    }
    double lambda = solve_budget(e, n, abar);
    free(e);
    return lambda;
}

void jpo_lambda_for_budget_rows(const void *actor, const void *policy, int dtype, int64_t T, int64_t V,
                                int64_t row_stride, const int32_t *x, const float *row_target,
                                double target, double *out)
{
    size_t esz = dtype == JPO_F32 ? 4 : dtype == JPO_BF16 ? 2 : 8;
    double *lq = (double *)malloc((size_t)V * sizeof(double));
    double *lp = (double *)malloc((size_t)V * sizeof(double));
    for (int64_t t = 0; t < T; ++t) {
        if (x[t] < 0) { out[t] = 0.0; continue; }
        jpo_widen_row((const char *)actor + (size_t)t * (size_t)row_stride * esz, dtype, V, lq);
        jpo_widen_row((const char *)policy + (size_t)t * (size_t)row_stride * esz, dtype, V, lp);
        out[t] = jpo_lambda_for_budget(lq, lp, V, row_target ? (double)row_target[t] : target);
    }
    free(lp);
    free(lq);
}

/* One lambda for a whole batch: (1/n) sum_t Z_t(lambda) = abar over the n valid rows.  The mean
 * of the rows' Z functions has the same shape as one of them (sum of the q-masses above lambda
 * plus 1/lambda times the p-masses at or below it, every row weighted 1/n), so the same
 * sort-and-solve applies to the pooled ratios.  Padding rows (x < 0) are left out.  Returns NaN for
 * abar outside (0, 1] or an empty batch.                                                       */
double jpo_lambda_for_budget_batch(const void *actor, const void *policy, int dtype, int64_t T,
                                   int64_t V, int64_t row_stride, const int32_t *x, double abar)
{
    if (!(abar > 0.0) || abar > 1.0) return NAN;
    size_t esz = dtype == JPO_F32 ? 4 : dtype == JPO_BF16 ? 2 : 8;
    int64_t n_rows = 0;
    for (int64_t t = 0; t < T; ++t) n_rows += x[t] >= 0 ? 1 : 0;
    if (n_rows == 0) return NAN;
    double *lq = (double *)malloc((size_t)V * sizeof(double));
    double *lp = (double *)malloc((size_t)V * sizeof(double));
    jpo_ratio *e = (jpo_ratio *)malloc((size_t)n_rows * (size_t)V * sizeof(jpo_ratio));
    int64_t n = 0;
    for (int64_t t = 0; t < T; ++t) {
        if (x[t] < 0) continue;
        jpo_widen_row((const char *)actor + (size_t)t * (size_t)row_stride * esz, dtype, V, lq);
        jpo_widen_row((const char *)policy + (size_t)t * (size_t)row_stride * esz, dtype, V, lp);
        double lse_q = jpo_logsumexp(lq, V), lse_p = jpo_logsumexp(lp, V);
        for (int64_t v = 0; v < V; ++v) {
            double q = exp(lq[v] - lse_q), p = exp(lp[v] - lse_p);
            if (!(q > 0.0) || !(p > 0.0)) continue;
            e[n].r = exp((lp[v] - lse_p) - (lq[v] - lse_q));
            e[n].q = q / (double)n_rows;
            e[n].p = p / (double)n_rows;
            ++n;
        }
    }
    free(lp);
    free(lq);
    double lambda = solve_budget(e, n, abar);
    free(e);
    return lambda;
}

/* The adjustment function F of the importance weight (Sec. 2, related work; Eq. obrs_ppo applies it
 * to p_target / p'_inf):  0 = truncation F(w) = min(w, c1) (TIS; the paper's choice, Alg. 1 step 3),
 * 1 = identity F(w) = w,  2 = two-sided truncation F(w) = w if lo <= w <= hi, else 0.             */
enum { JPO_F_TRUNCATE = 0, JPO_F_IDENTITY = 1, JPO_F_BAND = 2 };

double jpo_adjust(double w, int f_mode, double c1, double lo, double hi)
{
    if (f_mode == JPO_F_IDENTITY) return w;
    if (f_mode == JPO_F_BAND) return (w >= lo && w <= hi) ? w : 0.0;
    return w < c1 ? w : c1;
}

/* ---- batch-level bias correction and weights (Sec. 4.4.2, Alg. 1 step 2-3)
 * mask[t] is taken as given (the Bernoulli draw is an input of this stage).
 * alpha_hat = accepted / proposed;  kappa = alpha_hat / mean(Z_approx);
 * Z_t = kappa Z_approx;  w = Z_t max(lambda, p(x)/q(x));
 * rho = F(w) * min(p_ref(x)/p(x), c2)   (second factor 1 if no ref; F by f_mode).
 * use_expected_alpha != 0 replaces alpha_hat by the mean of a(x).        */
void jpo_batch_f(const jpo_row_out *rows, const int32_t *mask, int64_t T, double lambda,
                 int f_mode, double c1, double f_lo, double f_hi, double c2,
                 const double *ref_logprob, int use_expected_alpha,
                 jpo_batch_out *b, double *w_out, double *rho_out)
{
    memset(b, 0, sizeof *b);
    double sz = 0.0, sze = 0.0, sa = 0.0, skl = 0.0;
    for (int64_t t = 0; t < T; ++t) {
        if (!rows[t].valid) continue;
        b->n_valid += 1;
        b->n_accept += mask[t] ? 1 : 0;
        sz += rows[t].z_approx;
        sze += rows[t].z_exact;
        sa += rows[t].accept;
        skl += rows[t].kl_p_q;
    }
    double n = (double)b->n_valid;
    b->alpha_hat = (double)b->n_accept / n;
    b->mean_z_approx = sz / n;
    b->mean_z_exact = sze / n;
    b->mean_accept = sa / n;
    b->mean_kl_p_q = skl / n;
    double alpha = use_expected_alpha ? b->mean_accept : b->alpha_hat;
    b->kappa = alpha / b->mean_z_approx;

    for (int64_t t = 0; t < T; ++t) {
        if (!rows[t].valid) {
            if (w_out) w_out[t] = 0.0;
            if (rho_out) rho_out[t] = 0.0;
            continue;
        }
        double z_t = b->kappa * rows[t].z_approx;
        double ratio = exp(rows[t].logratio);
        double w = z_t * (lambda > ratio ? lambda : ratio);
        double rho = jpo_adjust(w, f_mode, c1, f_lo, f_hi);
        if (ref_logprob) {
            double rr = exp(ref_logprob[t] - rows[t].logp_x);
            rho *= rr < c2 ? rr : c2;
        }
        if (w_out) w_out[t] = w;
        if (rho_out) rho_out[t] = rho;
    }
}

void jpo_batch(const jpo_row_out *rows, const int32_t *mask, int64_t T, double lambda,
               double c1, double c2, const double *ref_logprob, int use_expected_alpha,
               jpo_batch_out *b, double *w_out, double *rho_out)
{
    jpo_batch_f(rows, mask, T, lambda, JPO_F_TRUNCATE, c1, 0.0, 0.0, c2, ref_logprob,
                use_expected_alpha, b, w_out, rho_out);
}

/* ---- log-probability of one token per row under one logit tensor ---------------------------
 * log softmax(l_t)[x_t] = l_t[x_t] - LSE(l_t): how log p_ref(a_t) (Alg. 1, Phase 2 step 1) is read
 * off a third logit tensor.  Padding rows (x < 0) give 0, ids outside the vocabulary NaN.      */
void jpo_token_logprob(const void *logits, int dtype, int64_t T, int64_t V, int64_t row_stride,
                       const int32_t *x, double *out)
{
    size_t esz = dtype == JPO_F32 ? 4 : dtype == JPO_BF16 ? 2 : 8;
    double *l = (double *)malloc((size_t)V * sizeof(double));
    for (int64_t t = 0; t < T; ++t) {
        if (x[t] < 0) { out[t] = 0.0; continue; }
        if (x[t] >= V) { out[t] = NAN; continue; }
        jpo_widen_row((const char *)logits + (size_t)t * (size_t)row_stride * esz, dtype, V, l);
        out[t] = l[x[t]] - jpo_logsumexp(l, V);
    }
    free(l);
}

int jpo_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
