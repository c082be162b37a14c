/*
 * jp_obrs.h -- C ABI of the MI355X (gfx950) OBRS hot path of Jackpot.
 *
 * Per token position t, from the rollout-model ("actor", p_inf, written q) logits and the
 * target-model ("policy", p_target, written p) logits over the whole vocabulary:
 *
 *   a_t        = min(1, p(x_t) / (lambda q(x_t)))                     Sec. 4.1, Eq. obrs_accept
 *   mask_t     = (u_t < a_t)                                          Sec. 4.2 (1); App. A Alg. 2
 *   V_k        = top-k(q) U top-k(p)  (a set)                         Sec. 4.4.1
 *   Z_approx,t = sum_{v in V_k} min(q(v), p(v)/lambda)                Sec. 4.4.1; Alg. 1 step 2
 *   Z_t (diagnostic) = sum_{v in V} min(q(v), p(v)/lambda)            Sec. 4.1, Eq. obrs_dist
 *   alpha_hat  = accepted / proposed,  kappa = alpha_hat / mean_t Z_approx,t      Sec. 4.4.2
 *   w_t        = kappa Z_approx,t max(lambda, p(x_t)/q(x_t))          Alg. 1 step 3
 *   rho_t      = F(w_t) min(p_ref(x_t)/p(x_t), c2), F(w) = min(w, c1)  Alg. 1 step 3; Sec. 2 for other F
 *   KL_t (optional) = sum_v p(v) (log p(v) - log q(v))                Sec. 4.2 (3), Eq. distill_loss
 *
 * Conventions
 *   - Every pointer argument is a DEVICE pointer unless it is a params / outputs struct
 *     (those are host structs read during the call).  The caller owns all buffers for the
 *     lifetime of the enqueued work.  Inputs are never written.
 *   - The library allocates nothing and never synchronises: all work is enqueued on `stream`
 *     (a hipStream_t passed as void*; NULL is the default stream).
 *   - Logit tensors are [T, V] row-major with `row_stride` ELEMENTS between consecutive rows
 *     (row_stride >= V).  Base pointers must be 16-byte aligned and row_stride * sizeof(element)
 *     must be a multiple of 16.
 *   - top-k lists are ordered by (logit descending, token id ascending); ties therefore go to
 *     the lowest id.
 *   - A row with sampled_ids[t] < 0 is padding: it is skipped, its outputs are 0 (top-k ids
 *     -1) and it is not counted in the batch statistics.
 *   - Errors the host can see return a status before anything is launched.  Errors only the
 *     device can see (sampled id >= V, non-finite log-sum-exp, no valid row) set bits in
 *     jp_obrs_stats.error_flags and put NaN in the affected outputs.
 *   - Re-entrant.  Calls that share a workspace must be ordered by the caller.  The library keeps
 *     two pieces of process-wide state, both written once per device through atomics: whether the
 *     GEMM kernel of the lm_head forms has been allowed its 160 KB of LDS on that device (one
 *     hipFuncSetAttribute on the first lm_head call there, which therefore must not run under
 *     stream capture), and the address of the static scratch of jp_obrs_forward_static.
 */
#ifndef JP_OBRS_H
#define JP_OBRS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define JP_K_MAX 256            /* largest supported top-k count per distribution */
#define JP_STATIC_MAX_T 131072  /* most token positions jp_obrs_forward_static takes     */

typedef enum jp_status {
    JP_OK = 0,
    JP_ERR_NULL = 1,            /* a required pointer is NULL                          */
    JP_ERR_SHAPE = 2,           /* T < 0, V <= 0, row_stride < V, sizes out of range   */
    JP_ERR_PARAM = 3,           /* lambda / c1 / c2 not positive or NaN, k < 1, k > V  */
    JP_ERR_ALIGN = 4,           /* pointer or row pitch not 16-byte aligned            */
    JP_ERR_WORKSPACE = 5,       /* workspace NULL or smaller than jp_obrs_workspace_bytes */
    JP_ERR_UNSUPPORTED = 6,     /* k > JP_K_MAX, unknown dtype or flag                 */
    JP_ERR_HIP = 7,             /* a HIP launch failed                                 */
    JP_ERR_TOO_LARGE = 8        /* jp_obrs_forward_static only: T > JP_STATIC_MAX_T    */
} jp_status;

/* Element type of a logit tensor.  The argument is a plain 32-bit integer on both sides of the
 * boundary, so a value outside the list is an error the library reports (JP_ERR_UNSUPPORTED) and not an
 * out-of-range enumeration value, which a C++ callee could not even inspect without undefined
 * behaviour.  jp_tail_rule below is declared the same way for the same reason. */
typedef int32_t jp_dtype;
enum { JP_F32 = 0, JP_BF16 = 1 };

enum {
    JP_FLAG_EXACT_Z = 1,        /* also compute Z over the whole vocabulary (second sweep)  */
    JP_FLAG_TOPK_LOGPROBS = 2,  /* also write log-probabilities of the two top-k lists      */
    JP_FLAG_ALPHA_EXPECTED = 4, /* alpha_hat := mean_t a_t instead of accepted/proposed     */
    JP_FLAG_DISTILL_KL = 8,     /* also compute the per-token distillation term KL(p || q)   */
    JP_FLAG_W_VOCAB_MAJOR = 16, /* jp_obrs_forward_lmhead only: W_* are [V, d] (one row per token
                                   of the vocabulary, the layout of an output embedding) instead
                                   of [d, V]; no transpose is then needed                     */
    JP_FLAG_ONE_WAVE_PER_ROW = 32 /* never split a row over several wavefronts (the library does
                                   so by itself for small batches, T <= 1792, in the two-tensor,
                                   stored-actor and lm_head forms; the index lists are the same either way, floats agree
                                   to rounding of the log-sum-exp; the exact-normaliser sweep
                                   follows the row stage; jp_obrs_token_logprob and
                                   jp_obrs_lambda_for_budget, which take no flags, always
                                   split by that rule)                                       */
};

enum {                          /* bits of jp_obrs_stats.error_flags */
    JP_DATA_ERR_ID_RANGE = 1,   /* some sampled id >= V                      */
    JP_DATA_ERR_NONFINITE = 2,  /* some row had a NaN / +inf log-sum-exp     */
    JP_DATA_ERR_EMPTY = 4       /* no valid row: kappa is NaN                */
};

/* Adjustment function F applied to w_t = p_target(x_t)/p'_inf(x_t) in rho_t (Eq. obrs_ppo; the
 * choices are those of Sec. 2): the truncation min(w, c1) that Alg. 1 step 3 uses (TIS), the
 * identity, or the two-sided truncation that keeps w inside [f_lo, f_hi] and zeroes it outside. */
typedef enum jp_adjust { JP_F_TRUNCATE = 0, JP_F_IDENTITY = 1, JP_F_BAND = 2 } jp_adjust;

typedef struct jp_obrs_params {
    float lambda;               /* rejection threshold, > 0 (paper default 1.0)            */
    int32_t k;                  /* top-k count per distribution, 1 <= k <= min(V, JP_K_MAX) */
    float c1;                   /* clip of w_OBRS, > 0 (+inf disables)                     */
    float c2;                   /* clip of p_ref/p, > 0 (+inf disables)                    */
    uint32_t flags;             /* JP_FLAG_*                                               */
    uint32_t f_mode;            /* jp_adjust; 0 = the paper's truncation                   */
    float f_lo, f_hi;           /* JP_F_BAND only: 0 <= f_lo <= f_hi                       */
} jp_obrs_params;

/* Batch statistics, written to device memory by the finalize stage (Sec. 4.4.2). */
typedef struct jp_obrs_stats {
    int64_t n_valid;            /* proposed tokens B (non-padding, error-free rows) */
    int64_t n_accept;           /* sum_t mask_t                                     */
    double alpha_hat;           /* n_accept / n_valid (or mean a_t, see flags)      */
    double mean_z_approx;       /* (1/B) sum_t Z_approx,t                           */
    double kappa;               /* alpha_hat / mean_z_approx                        */
    double mean_z_exact;        /* (1/B) sum_t Z_t, NaN without JP_FLAG_EXACT_Z     */
    double mean_accept;         /* (1/B) sum_t a_t                                  */
    uint32_t error_flags;       /* JP_DATA_ERR_*                                    */
    uint32_t reserved;
    double mean_distill_kl;     /* (1/B) sum_t KL(p_t || q_t), NaN without JP_FLAG_DISTILL_KL */
} jp_obrs_stats;

/* Output pointers (device memory, caller-owned).  NULL = not wanted. */
typedef struct jp_obrs_outputs {
    float *accept_prob;         /* [T]   a_t                                               */
    uint8_t *mask;              /* [T]   1 = accepted (needs uniforms)                     */
    float *logq;                /* [T]   log q(x_t)                                        */
    float *logp;                /* [T]   log p(x_t)                                        */
    float *logratio;            /* [T]   log p(x_t) - log q(x_t)                           */
    float *z_approx;            /* [T]                                                     */
    float *z_exact;             /* [T]   required with JP_FLAG_EXACT_Z                     */
    float *w_obrs;              /* [T]   un-clipped w_t (not multiplied by the mask)       */
    float *rho;                 /* [T]   rho_t          (not multiplied by the mask)       */
    int32_t *union_size;        /* [T]   |V_k|                                             */
    int32_t *topk_actor;        /* [T,k] ids of top-k(q)                                   */
    int32_t *topk_policy;       /* [T,k] ids of top-k(p)                                   */
    float *topk_actor_logq;     /* [T,k] log q of topk_actor,  with JP_FLAG_TOPK_LOGPROBS  */
    float *topk_policy_logp;    /* [T,k] log p of topk_policy, with JP_FLAG_TOPK_LOGPROBS  */
    jp_obrs_stats *stats;       /* one struct, written by the finalize stage               */
    float *distill_kl;          /* [T]   KL(p_t || q_t) = sum_v p(v) (log p(v) - log q(v)), the
                                         per-token on-policy distillation term of Sec. 4.2 (3),
                                         Eq. distill_loss; with JP_FLAG_DISTILL_KL            */
} jp_obrs_outputs;

/* Bytes of device scratch the calls below need for these sizes (0 on invalid sizes). */
size_t jp_obrs_workspace_bytes(int64_t T, int64_t V, int32_t k, jp_dtype dt, uint32_t flags);

/*
 * The whole hot path: row stage (log-sum-exp of both rows, sampled-token log-probs, both top-k
 * lists, a_t, mask_t, Z_approx,t [, Z_t]) followed by the batch stage (alpha_hat, kappa, w_t,
 * rho_t).  uniforms == NULL implies JP_FLAG_ALPHA_EXPECTED and no mask; ref_logprob == NULL
 * makes the p_ref/p factor 1.  T == 0 is valid and does nothing but write the stats.
 */
jp_status jp_obrs_forward(const void *actor_logits, const void *policy_logits,
                          int64_t T, int64_t V, int64_t row_stride, jp_dtype dt,
                          const int32_t *sampled_ids,   /* [T] x_t                       */
                          const float *uniforms,        /* [T] u_t in [0,1), or NULL     */
                          const float *ref_logprob,     /* [T] log p_ref(x_t), or NULL   */
                          const jp_obrs_params *prm, const jp_obrs_outputs *out,
                          void *workspace, size_t workspace_bytes, void *stream);

/*
 * jp_obrs_forward for callers that cannot allocate device memory and have no workspace to hand
 * over: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * scratch that jp_obrs_forward takes as `workspace` (the per-token scalars kept between the row
 * stage and the batch stage, ~46 bytes per token) is here a static device array inside the library,
 * sized for T <= JP_STATIC_MAX_T (5.75 MiB; every GPU the library runs on holds it until the process
 * ends).  Same kernels, same results bit for bit; no hipMalloc, hipFree or allocating library call.
 *   - T > JP_STATIC_MAX_T returns JP_ERR_TOO_LARGE and launches nothing.
 *   - The GPU whose stream is passed must be the current device of the calling thread.  The first
 *     call on a device looks the array's address up (hipGetSymbolAddress) and must be made outside
 *     stream capture; later calls only launch.
 *   - All calls on one GPU share the one array: calls whose enqueued work may overlap in time (two
 *     streams, two threads) race on it and must be ordered by the caller; jp_obrs_forward with
 *     separate workspaces has no such limit.  Nothing in the array needs clearing between calls:
 *     the row stage writes every entry of the first T positions before the batch stage reads them,
 *     whatever an earlier, larger call left behind.
 * Inputs, outputs and every other convention as jp_obrs_forward.
 */
jp_status jp_obrs_forward_static(const void *actor_logits, const void *policy_logits,
                                 int64_t T, int64_t V, int64_t row_stride, jp_dtype dt,
                                 const int32_t *sampled_ids, const float *uniforms,
                                 const float *ref_logprob, const jp_obrs_params *prm,
                                 const jp_obrs_outputs *out, void *stream);

/* Row stage only (everything of jp_obrs_forward that needs no batch statistic). */
jp_status jp_obrs_rows(const void *actor_logits, const void *policy_logits,
                       int64_t T, int64_t V, int64_t row_stride, jp_dtype dt,
                       const int32_t *sampled_ids, const float *uniforms,
                       const jp_obrs_params *prm, const jp_obrs_outputs *out,
                       void *workspace, size_t workspace_bytes, void *stream);

/*
 * Batch stage only (Sec. 4.4.2 and Alg. 1 step 3) over the per-row results that a preceding
 * jp_obrs_rows call with the SAME workspace, T and outputs struct left behind.
 * This call cannot see whether the row stage was given uniforms: if it ran with uniforms == NULL
 * (no Bernoulli draw, every mask 0), set JP_FLAG_ALPHA_EXPECTED here, otherwise alpha_hat and with
 * it kappa, w_t and rho_t come out 0.
 */
jp_status jp_obrs_finalize(int64_t T, const int32_t *sampled_ids, const float *ref_logprob,
                           const jp_obrs_params *prm, const jp_obrs_outputs *out,
                           void *workspace, size_t workspace_bytes, void *stream);

/*
 * Fused lm_head form of jp_obrs_forward: the logits are not given but computed on the matrix
 * cores, lq = H_actor x W_actor and lp = H_policy x W_policy (bf16 inputs, fp32 accumulation,
 * no rounding of the logits), one vocabulary chunk at a time, and consumed by the same row
 * stage without ever materialising [T, V].  Everything else (Sec. 4.1, 4.4.1, 4.4.2, Alg. 1
 * steps 2-3) is as in jp_obrs_forward.
 *   H_actor  [T, d_actor]  bf16 row-major, contiguous, 16-byte aligned; d_actor  % 64 == 0
 *   W_actor  [d_actor, V]  bf16 row-major, contiguous; with JP_FLAG_W_VOCAB_MAJOR [V, d_actor]
 *            row-major, contiguous, 16-byte aligned
 *   H_policy [T, d_policy], W_policy [d_policy, V] (or [V, d_policy]) likewise
 *   vocab_chunk: columns per chunk (rounded up to a multiple of 256); 0 = chosen from T
 *            (4096 for T > 6144, 8192 down to T = 1537, 16384 down to T = 769, 65536 below)
 * JP_FLAG_EXACT_Z is not available here (JP_ERR_UNSUPPORTED): the logits are gone after one pass.
 * Workspace: jp_obrs_lmhead_workspace_bytes (two fp32 logit buffers [T, 4 chunk]: the row stage
 * runs once per four chunks; the transposed weight chunks, a per-row record of ~1.6 KB at
 * k <= 64, plus the jp_obrs_forward workspace; 2.2 GB at T = 16384 and no more than that at any
 * smaller T with the default chunk, V = 151936, d = 2048 + 4096).
 */
size_t jp_obrs_lmhead_workspace_bytes(int64_t T, int64_t V, int64_t d_actor, int64_t d_policy,
                                      int32_t k, int64_t vocab_chunk);
jp_status jp_obrs_forward_lmhead(const void *H_actor, int64_t d_actor, const void *W_actor,
                                 const void *H_policy, int64_t d_policy, const void *W_policy,
                                 int64_t T, int64_t V, int64_t vocab_chunk,
                                 const int32_t *sampled_ids, const float *uniforms,
                                 const float *ref_logprob, const jp_obrs_params *prm,
                                 const jp_obrs_outputs *out, void *workspace,
                                 size_t workspace_bytes, void *stream);

/*
 * The whole hot path with the actor side in the form the rollout phase stores it (Alg. 1,
 * Phase 1): per position the sampled token's log-probability log p_inf(a_t) and the k ids and
 * log-probabilities of TopK_inf, instead of a [T, V] actor logit tensor.  Only the target model's
 * logits are swept, so the bytes moved per token are halved.
 *   a_t, mask_t: from actor_logprob_x[t] and log p(x_t)                  Eq. obrs_accept
 *   V_k = TopK_inf U top-k(p)                                            Alg. 1 step 2
 *   Z_approx,t = sum_{v in TopK_inf} min(q(v), p(v)/lambda)
 *              + sum_{v in top-k(p), not in TopK_inf} min(qhat_t, p(v)/lambda)
 * The paper does not say what q(v) is for a token of top-k(p) that TopK_inf does not hold; qhat_t
 * is chosen by tail_rule:
 *   JP_TAIL_DROP  such tokens contribute nothing (a lower bound of the two-tensor Z_approx)
 *   JP_TAIL_KTH   the smallest stored probability (v is not among the k largest, so q(v) cannot
 *                 exceed it: an upper bound of the two-tensor Z_approx)
 *   JP_TAIL_REST  the mass the stored list leaves, 1 - sum of the stored probabilities, spread
 *                 evenly over the other V - n tokens, capped by the JP_TAIL_KTH bound
 * Batch stage (alpha_hat, kappa, w_t, rho_t) and every other convention as in jp_obrs_forward.
 *   actor_topk_ids      device [T, k] int32; an id outside [0, V) marks an unused slot, of a
 *                       repeated id the first occurrence counts; any order
 *   actor_topk_logprob  device [T, k] fp32, log q of those ids
 *   actor_logprob_x     device [T] fp32, log q(x_t)
 * Outputs: logq is a copy of actor_logprob_x; topk_actor / topk_actor_logq are not written (they
 * are inputs here).  JP_FLAG_EXACT_Z and JP_FLAG_DISTILL_KL need the actor row: JP_ERR_UNSUPPORTED.
 * Workspace: jp_obrs_workspace_bytes.
 */
typedef int32_t jp_tail_rule;
enum { JP_TAIL_DROP = 0, JP_TAIL_KTH = 1, JP_TAIL_REST = 2 };
jp_status jp_obrs_forward_stored(const void *policy_logits, int64_t T, int64_t V, int64_t row_stride,
                                 jp_dtype dt, const int32_t *actor_topk_ids,
                                 const float *actor_topk_logprob, const float *actor_logprob_x,
                                 const int32_t *sampled_ids, const float *uniforms,
                                 const float *ref_logprob, const jp_obrs_params *prm,
                                 jp_tail_rule tail_rule, const jp_obrs_outputs *out,
                                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * Alg. 1 as a trainer runs it: the target logits lp = H_policy x W_policy come from the matrix
 * cores one vocabulary chunk at a time (as in jp_obrs_forward_lmhead, never materialised) and the
 * actor side is what the rollout phase stored (as in jp_obrs_forward_stored).  One head instead of
 * two, no [T, V] tensor at all.  The target logit of a stored id is picked up when its chunk
 * passes.  Arguments, outputs, tail rules and flags as in those two entry points; the near-tie
 * remark of the lm_head form applies to top-k(p).
 * Workspace: jp_obrs_lmhead_stored_workspace_bytes (one fp32 logit buffer [T, 2 chunk], one
 * transposed weight chunk, the per-row record, plus the jp_obrs_forward workspace).
 */
size_t jp_obrs_lmhead_stored_workspace_bytes(int64_t T, int64_t V, int64_t d_policy, int32_t k,
                                             int64_t vocab_chunk);
jp_status jp_obrs_forward_lmhead_stored(const void *H_policy, int64_t d_policy, const void *W_policy,
                                        int64_t T, int64_t V, int64_t vocab_chunk,
                                        const int32_t *actor_topk_ids, const float *actor_topk_logprob,
                                        const float *actor_logprob_x, const int32_t *sampled_ids,
                                        const float *uniforms, const float *ref_logprob,
                                        const jp_obrs_params *prm, jp_tail_rule tail_rule,
                                        const jp_obrs_outputs *out, void *workspace,
                                        size_t workspace_bytes, void *stream);

/*
 * log-probability of the sampled token under one more logit tensor,
 *   out[t] = logits[t, x_t] - log sum_v exp(logits[t, v]),
 * e.g. log p_ref(a_t) of Alg. 1 (Phase 2, step 1) when p_ref and p_new are separate tensors: its
 * result is the ref_logprob argument of jp_obrs_forward.  One sweep of the tensor.  Padding rows
 * (x_t < 0) give 0; an id >= V or a non-finite log-sum-exp gives NaN.  No workspace.
 */
jp_status jp_obrs_token_logprob(const void *logits, int64_t T, int64_t V, int64_t row_stride,
                                jp_dtype dt, const int32_t *sampled_ids, float *out_logprob,
                                void *stream);

/*
 * The three-distribution form of Eq. obrs_ppo / Alg. 1: rollout logits (p_inf), the updated
 * policy's logits (p_new) and the reference policy's logits (p_ref) as separate tensors, with the
 * OBRS target chosen by `target_is_ref` (Sec. 4.3: either may serve as p_target).
 *   target_is_ref == 0: p_target = p_new; the factor p_ref(x)/p_target(x) of rho_t is computed from
 *                       a sweep of policy_ref (jp_obrs_token_logprob into the workspace)
 *   target_is_ref != 0: p_target = p_ref; that factor is 1 and policy_new is not read (may be NULL)
 * Everything else as jp_obrs_forward on (actor, p_target).  Workspace:
 * jp_obrs_workspace_bytes(...) + 4 T rounded up to 256 bytes (jp_obrs_forward3_workspace_bytes).
 */
size_t jp_obrs_forward3_workspace_bytes(int64_t T, int64_t V, int32_t k, jp_dtype dt, uint32_t flags);
jp_status jp_obrs_forward3(const void *actor_logits, const void *policy_new_logits,
                           const void *policy_ref_logits, int32_t target_is_ref,
                           int64_t T, int64_t V, int64_t row_stride, jp_dtype dt,
                           const int32_t *sampled_ids, const float *uniforms,
                           const jp_obrs_params *prm, const jp_obrs_outputs *out,
                           void *workspace, size_t workspace_bytes, void *stream);

/*
 * The scaling factor for an acceptance budget (Sec. 3.3, Theorem 2): for every row the lambda_t with
 *   sum_v q_t(v) min(1, p_t(v) / (lambda_t q_t(v))) = abar_t,   abar_t = row_target ? row_target[t] : target,
 * i.e. the threshold at which the OBRS rule accepts exactly the fraction abar_t of the proposals.
 * For abar_t = 1 (every lambda up to min_v p/q accepts everything) the largest such lambda is
 * returned.  The log-sum-exps and the row status come from `workspace`, where a preceding
 * jp_obrs_rows / jp_obrs_forward call on the SAME tensors and T left them.
 * Cost: two sweeps of the two logit tensors on ordinary rows (one that locates the crossing to
 * 3/16 in log2 lambda from an approximate histogram, one exact over 256 bins of that bracket), up
 * to six on degenerate ones (the crossing outside the resolved ratios 2^-16 .. 2^16, a single
 * token that carries a visible part of the budget next to the crossing, abar at the keepable mass).
 * Accuracy: the last step is the closed form lambda = B / (abar - A) on the crossing bin, exact up
 * to the tokens inside that bin; the search ends when their q-mass times (2^bin width - 1) is
 * below 1e-4 abar (bf16 logits) or 1e-6 abar (fp32), or the bin is narrower than 1e-6, so the
 * budget is met to the float tolerance of the other outputs; lambda itself is only as well
 * determined as the budget determines it (near abar = 1 it is not).  Ratios are searched over
 * [2^-64, 2^64].
 *   out_lambda: device [T] fp32; padding rows 0; rows with data errors, or a budget outside (0, 1], NaN.
 * target is checked on the host (JP_ERR_PARAM) when row_target is NULL.
 */
jp_status jp_obrs_lambda_for_budget(const void *actor_logits, const void *policy_logits,
                                    int64_t T, int64_t V, int64_t row_stride, jp_dtype dt,
                                    const float *row_target, float target, float *out_lambda,
                                    const void *workspace, size_t workspace_bytes, void *stream);

/*
 * One scaling factor for a whole batch: the lambda with (1/n) sum_t Z_t(lambda) = target over the n
 * valid rows (the mean acceptance of the batch under one global lambda, which is how Sec. 4 uses
 * lambda).  Same search as jp_obrs_lambda_for_budget with the histogram bins summed over the rows
 * in device memory (64-bit fixed point: the sums do not depend on the order of the rows) and a
 * one-wave kernel between the sweeps that picks the next bracket; nothing passes through the host.
 * The launch sequence is fixed (six sweep kernels and the smallest-ratio sweep, each of which
 * returns at once when the search has ended), so the call can be captured.
 *   out_lambda: device, one fp32 (NaN if the batch has no valid row)
 *   scratch:    device, jp_obrs_budget_scratch_bytes() bytes, 16-byte aligned, contents irrelevant
 * workspace as for jp_obrs_lambda_for_budget.
 */
size_t jp_obrs_budget_scratch_bytes(void);
jp_status jp_obrs_lambda_for_budget_batch(const void *actor_logits, const void *policy_logits,
                                          int64_t T, int64_t V, int64_t row_stride, jp_dtype dt,
                                          float target, float *out_lambda,
                                          const void *workspace, size_t workspace_bytes,
                                          void *scratch, size_t scratch_bytes, void *stream);

/*
 * Gradient of the on-policy distillation term of Sec. 4.2 (3), Eq. distill_loss, with respect to
 * the actor logits.  The term per token is KL(SG(p_t) || q_t) with the target p_t held fixed and
 * q_t = softmax(actor logits), so d/d lq_t[v] = q_t(v) - p_t(v).  This call writes
 *   grad_actor[t, v] = scale * (row_scale ? row_scale[t] : 1) * (q_t(v) - p_t(v))
 * (e.g. scale = lambda_distill / B for the batch mean of the joint objective, Eq. sys_joint_obj).
 * It is a second streaming pass over the two logit tensors that takes the two log-sum-exps and the
 * row status from `workspace`, where a preceding jp_obrs_rows / jp_obrs_forward call on the SAME
 * tensors, T and workspace left them.  Rows that were padding, had a sampled id outside the
 * vocabulary or a non-finite log-sum-exp get zeros.
 *   grad_actor: device [T, V], grad_row_stride elements between rows (>= V), dtype grad_dt
 *               (JP_F32, or JP_BF16 rounded to nearest even); 16-byte aligned base and row pitch.
 *   row_scale:  device [T] or NULL.
 * Status codes as for jp_obrs_forward; scale must be finite.  Nothing else is read or written.
 */
jp_status jp_obrs_distill_grad(const void *actor_logits, const void *policy_logits,
                               int64_t T, int64_t V, int64_t row_stride, jp_dtype dt,
                               const float *row_scale, float scale,
                               void *grad_actor, int64_t grad_row_stride, jp_dtype grad_dt,
                               const void *workspace, size_t workspace_bytes, void *stream);

/* Text for a status code (a static string; any other integer gives "unknown status"). */
const char *jp_status_string(int32_t status);

/* ABI version of this header (bumped on incompatible change). */
int jp_obrs_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* JP_OBRS_H */
