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
    // per-row results: never nullptr (user buffer or workspace)
    float *accept, *logq, *logp, *logratio, *zapprox;
    double *lse_q, *lse_p;
    uint8_t *mask, *rowflag;
    // optional user outputs
    int32_t *usize, *topk_a, *topk_p;
    float *topk_a_lq, *topk_p_lp;
};

struct ZExactArgs {
    const void *actor, *policy;
    int64_t T, V, stride;
    const double *lse_q, *lse_p;
    const uint8_t *rowflag;
    float lambda;
    float *zexact;
};

struct FinalizeArgs {
    int64_t T;
    const uint8_t *rowflag, *mask;
    const float *accept, *zapprox, *zexact, *logratio, *logp, *ref_logprob;
    float lambda, c1, c2;
    int alpha_expected;
    jp_obrs_stats *stats;
    float *w, *rho;
};

hipError_t launch_rows(const RowArgs &a, int dtype, hipStream_t st);
hipError_t launch_zexact(const ZExactArgs &a, int dtype, hipStream_t st);
hipError_t launch_finalize(const FinalizeArgs &a, hipStream_t st);

}  // namespace jp
#endif
