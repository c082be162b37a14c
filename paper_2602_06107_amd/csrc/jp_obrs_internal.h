// Internal interface between the C-ABI entry points and the kernel launchers.
#ifndef JP_OBRS_INTERNAL_H
#define JP_OBRS_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "jp_obrs.h"

namespace jp {

// Per-row status byte kept in the workspace between the row stage and the batch stage.
enum : uint8_t { ROW_OK = 0, ROW_PADDING = 1, ROW_BAD_ID = 2, ROW_NONFINITE = 3 };

struct RowArgs {
    const void *actor, *policy;       // [T, V] logits
    int64_t T, V, stride;             // stride in elements
    const int32_t *ids;               // [T]
    const float *uni;                 // [T] or nullptr
    float lambda;
    double ln_lambda;                 // log(lambda), taken on the host
    int k;
    int waves;                        // wavefronts per row (1, 2 or 4)
    // per-row results: never nullptr (user buffer or workspace)
    float *accept, *logq, *logp, *logratio, *zapprox;
    float *kl;                        // KL(p || q) per token (distill != 0 only)
    int distill;
    double *lse_q, *lse_p;
    uint8_t *mask, *rowflag;
    // optional user outputs
    int32_t *usize, *topk_a, *topk_p;
    float *topk_a_lq, *topk_p_lp;
    // vocabulary-chunked form only: this launch covers ids [id_base, id_base + V) of V_total
    int64_t V_total, id_base;
    int carry_in, carry_out;          // a row record is read before / written after this chunk
    unsigned char *state;             // [T] records of state_stride bytes (carry_state_bytes(k))
    int64_t state_stride;
    // stored-actor form only: the actor side as ids + log-probabilities instead of a logit tensor
    const int32_t *stored_ids;        // [T, k]
    const float *stored_logq;         // [T, k]
    const float *stored_logq_x;       // [T]
    int tail_rule;
};

// Row record carried from one vocabulary chunk to the next, followed by the two top-k lists as
// [2][3][KC] 32-bit words (ids, own logits, the other tensor's logits).
struct CarryHeader {
    float M2[2];                      // exponent references (log2 domain) of actor / policy
    int nl[2];                        // entries in the two lists
    double S[2];                      // sums of 2^(l log2e - M2)
    float x_logit[2];                 // logits of the sampled token, once its chunk has passed
    int have_x, pad;
    double D;                         // sum of 2^(lp log2e - M2) (lp - lq), for the distillation term
    unsigned char reserve[8];
};
static_assert(sizeof(CarryHeader) == 64, "carry header is 64 bytes");
inline int carry_kc(int k) { return k <= 64 ? 64 : (k <= 128 ? 128 : 256); }
inline size_t carry_state_bytes(int k) { return sizeof(CarryHeader) + (size_t)24 * carry_kc(k); }

struct ZExactArgs {
    const void *actor, *policy;
    int64_t T, V, stride;
    const double *lse_q, *lse_p;
    const uint8_t *rowflag;
    float lambda;
    float *zexact;
    int waves;                        // wavefronts per row: 4 or 1 (as the row stage chose)
};

struct FinalizeArgs {
    int64_t T;
    const uint8_t *rowflag, *mask;
    const float *accept, *zapprox, *zexact, *logratio, *logp, *ref_logprob;
    const float *kl;                  // nullptr unless the distillation term was requested
    float lambda, c1, c2;
    int f_mode;                       // JP_F_*
    float f_lo, f_hi;
    int alpha_expected;
    jp_obrs_stats *stats;
    float *w, *rho;
};

struct GradArgs {
    const void *actor, *policy;       // [T, V] logits, `stride` elements between rows
    int64_t T, V, stride;
    const double *lse_q, *lse_p;      // [T] from the row stage
    const uint8_t *rowflag;           // [T] from the row stage
    const float *row_scale;           // [T] or nullptr
    float scale;
    void *grad;                       // [T, V], `grad_stride` elements between rows
    int64_t grad_stride;
    uint32_t seg_chunks, segs;        // set by the launcher: pieces per workgroup, workgroups per row
};

struct LogprobArgs {
    const void *logits;               // [T, V]
    int64_t T, V, stride;
    const int32_t *ids;               // [T]
    float *out;                       // [T]
};

struct BudgetArgs {
    const void *actor, *policy;       // [T, V] logits
    int64_t T, V, stride;
    const double *lse_q, *lse_p;      // [T] from the row stage
    const uint8_t *rowflag;           // [T] from the row stage
    const float *row_target;          // [T] or nullptr
    float target;
    float *lambda_out;                // [T]
    float eps_rel;                    // error of Z, relative to the budget, below which the search stops
};

// Device-resident state of the per-batch budget search (in the caller's scratch buffer).
struct BudgetBatchState {
    float lo, hi;                     // current bracket, log2 of the ratio
    int done, dmin_ord;               // finished flag; smallest log2 ratio as an order-preserving int
    double lambda;
    unsigned long long n_rows, above, below;   // valid rows; mass outside the bracket (2^-32 units)
    unsigned long long coarse[512];            // first sweep: q-mass per coarse bin over all rows (2^-31 units)
    unsigned long long fq[256], fp[256];       // exact sweeps: q- and p-mass per fine bin over all rows (2^-32 units)
};

// Small batches: one wave per row leaves most of the chip idle, and a single wave needs ~0.14 ms for
// a row of 152 k logits whatever else runs.  Up to T = 1792 a row is split over four waves (two when
// it is short), provided every wave still gets at least two sweep iterations of 64 16-byte pieces;
// measured on V = 151936, k = 64: 2.2x at T = 256, 1.9x at 512, 1.2x at 1024, 1.1x at 1536, and a
// loss from T = 2048 on, where one wave per row already fills the chip.
inline int waves_per_row(int64_t T, int64_t V, int elem_bytes)
{
    const int64_t iterations = V / (16 / elem_bytes) / 64;
    if (T > 1792) return 1;
    return iterations >= 8 ? 4 : (iterations >= 4 ? 2 : 1);
}

hipError_t launch_budget(const BudgetArgs &a, int dtype, hipStream_t st);
hipError_t launch_budget_batch(const BudgetArgs &a, int dtype, BudgetBatchState *S, float *out_lambda, hipStream_t st);
hipError_t launch_token_logprob(const LogprobArgs &a, int dtype, hipStream_t st);
hipError_t launch_rows(const RowArgs &a, int dtype, hipStream_t st);
hipError_t launch_rows_stored(const RowArgs &a, int dtype, hipStream_t st);   // a.actor unused
hipError_t launch_rows_carry_stored(const RowArgs &a, hipStream_t st);        // chunked fp32 policy logits + stored actor side
hipError_t launch_distill_grad(const GradArgs &a, int dtype, int grad_dtype, hipStream_t st);
// Two independent TN GEMMs sharing M, N and ldc (policy head and actor head of one vocabulary chunk).
struct GemmArgs {
    const void *A[2];                 // [M, K] bf16
    const void *Bt[2];                // [N, K] bf16 (N padded to a multiple of 256 with zero rows)
    float *C[2];                      // [M, ldc] fp32
    int K[2];
    int M, N, nproblems;
    int64_t ldc;
};
constexpr int LMHEAD_N_ALIGN = 256;   // GEMM column tile

hipError_t launch_transpose_chunk(const void *W, int64_t ldw, int d, int64_t v0, int ncols, int npad,
                                  void *Wt, hipStream_t st);
hipError_t launch_copy_rows_chunk(const void *W, int d, int64_t v0, int ncols, int npad, void *Wt, hipStream_t st);
hipError_t launch_touch_rows(const void *W, int64_t bytes, void *sink, hipStream_t st);   // read and drop: warms the caches
hipError_t launch_gemm_pair(const GemmArgs &g, hipStream_t st);
hipError_t launch_rows_carry(const RowArgs &a, hipStream_t st);   // fp32 logits chunk, carried state
hipError_t launch_zexact(const ZExactArgs &a, int dtype, hipStream_t st);
hipError_t launch_finalize(const FinalizeArgs &a, hipStream_t st);

}  // namespace jp
#endif
