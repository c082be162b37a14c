// C-ABI entry points: argument validation, workspace carving, launches.  No allocation, no sync.
#include <math.h>
#include <stdint.h>

#include <atomic>

#include "jp_obrs_internal.h"

namespace {

constexpr uint32_t KNOWN_FLAGS = JP_FLAG_EXACT_Z | JP_FLAG_TOPK_LOGPROBS | JP_FLAG_ALPHA_EXPECTED | JP_FLAG_DISTILL_KL |
                                 JP_FLAG_W_VOCAB_MAJOR | JP_FLAG_ONE_WAVE_PER_ROW;
constexpr size_t ALIGN = 256;

size_t round_up(size_t n) { return (n + ALIGN - 1) / ALIGN * ALIGN; }

// Scratch kept between the row stage and the batch stage (user buffers replace the float
// arrays when the caller asked for those outputs).
struct Workspace {
    float *accept, *logq, *logp, *logratio, *zapprox, *zexact, *kl;
    double *lse_q, *lse_p;
    uint8_t *mask, *rowflag;
    jp_obrs_stats *stats;
    size_t bytes;
};

Workspace carve(void *base, int64_t T)
{
    Workspace w;
    char *p = (char *)base;
    size_t off = 0;
    const size_t n = (size_t)(T > 0 ? T : 0);
    auto take = [&](size_t bytes) { char *r = p ? p + off : nullptr; off += round_up(bytes); return r; };
    w.accept = (float *)take(n * 4);
    w.logq = (float *)take(n * 4);
    w.logp = (float *)take(n * 4);
    w.logratio = (float *)take(n * 4);
    w.zapprox = (float *)take(n * 4);
    w.zexact = (float *)take(n * 4);
    w.kl = (float *)take(n * 4);
    w.lse_q = (double *)take(n * 8);
    w.lse_p = (double *)take(n * 8);
    w.mask = (uint8_t *)take(n);
    w.rowflag = (uint8_t *)take(n);
    w.stats = (jp_obrs_stats *)take(sizeof(jp_obrs_stats));
    w.bytes = off;
    return w;
}

bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

// ---- static scratch of the entry point that allocates nothing ------------------------------------
// The same layout carve() gives a caller's workspace, for up to JP_STATIC_MAX_T token positions, in
// a device array that every GPU the library runs on holds until the process ends (5.75 MiB).
constexpr size_t round_up_c(size_t n) { return (n + ALIGN - 1) / ALIGN * ALIGN; }
constexpr size_t static_scratch_bytes(size_t n)
{
    return 7 * round_up_c(n * 4) + 2 * round_up_c(n * 8) + 2 * round_up_c(n) + round_up_c(sizeof(jp_obrs_stats));
}
constexpr size_t STATIC_SCRATCH_BYTES = static_scratch_bytes(JP_STATIC_MAX_T);
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

// Device address of `scratch` on each GPU (the array's name is only a host-side handle; every GPU
// holds its own copy at its own address).  Looked up once per device, with that device current.
constexpr int MAX_DEVICES = 64;
std::atomic<void *> scratch_ptr[MAX_DEVICES];

jp_status static_scratch(void **ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return JP_ERR_HIP;
    void *p = scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return JP_ERR_HIP;
        scratch_ptr[dev].store(p, std::memory_order_release);   // two threads racing here store the same address
    }
    *ptr = p;
    return JP_OK;
}

jp_status check_params(const jp_obrs_params *prm, int64_t V, bool need_clips)
{
    if (!prm) return JP_ERR_NULL;
    if (prm->flags & ~KNOWN_FLAGS) return JP_ERR_UNSUPPORTED;
    if (!(prm->lambda > 0.f) || !isfinite(prm->lambda)) return JP_ERR_PARAM;
    if (need_clips && (!(prm->c1 > 0.f) || !(prm->c2 > 0.f))) return JP_ERR_PARAM;
    if (prm->f_mode > JP_F_BAND) return JP_ERR_UNSUPPORTED;
    if (prm->f_mode == JP_F_BAND && !(prm->f_lo >= 0.f && prm->f_lo <= prm->f_hi)) return JP_ERR_PARAM;
    if (prm->k < 1 || (int64_t)prm->k > V) return JP_ERR_PARAM;
    if (prm->k > JP_K_MAX) return JP_ERR_UNSUPPORTED;
    return JP_OK;
}

jp_status check_shape(int64_t T, int64_t V, int64_t row_stride, jp_dtype dt)
{
    if (dt != JP_F32 && dt != JP_BF16) return JP_ERR_UNSUPPORTED;
    if (T < 0 || T > 0x7fffffffLL || V <= 0 || V > 0x7fffffffLL || row_stride < V) return JP_ERR_SHAPE;
    return JP_OK;
}

jp_status rows_impl(const void *actor, const void *policy, int64_t T, int64_t V, int64_t row_stride,
                    jp_dtype dt, const int32_t *ids, const float *uni, const jp_obrs_params *prm,
                    const jp_obrs_outputs *out, void *workspace, size_t workspace_bytes,
                    hipStream_t st, bool need_clips)
{
    if (!prm || !out) return JP_ERR_NULL;
    jp_status s = check_shape(T, V, row_stride, dt);
    if (s != JP_OK) return s;
    s = check_params(prm, V, need_clips);
    if (s != JP_OK) return s;
    if (T > 0 && (!actor || !policy || !ids)) return JP_ERR_NULL;
    const size_t esz = dt == JP_BF16 ? 2 : 4;
    if (!aligned16(actor) || !aligned16(policy) || ((size_t)row_stride * esz) % 16 != 0) return JP_ERR_ALIGN;
    if (!workspace || workspace_bytes < jp_obrs_workspace_bytes(T, V, prm->k, dt, prm->flags)) return JP_ERR_WORKSPACE;
    if (((uintptr_t)workspace & (ALIGN - 1)) != 0) return JP_ERR_ALIGN;
    if (T == 0) return JP_OK;

    const Workspace w = carve(workspace, T);
    jp::RowArgs a{};
    a.actor = actor; a.policy = policy; a.T = T; a.V = V; a.stride = row_stride;
    a.ids = ids; a.uni = uni; a.lambda = prm->lambda; a.ln_lambda = log((double)prm->lambda); a.k = prm->k;
    a.accept = out->accept_prob ? out->accept_prob : w.accept;
    a.logq = out->logq ? out->logq : w.logq;
    a.logp = out->logp ? out->logp : w.logp;
    a.logratio = out->logratio ? out->logratio : w.logratio;
    a.zapprox = out->z_approx ? out->z_approx : w.zapprox;
    a.distill = (prm->flags & JP_FLAG_DISTILL_KL) ? 1 : 0;
    a.kl = out->distill_kl ? out->distill_kl : w.kl;
    a.lse_q = w.lse_q; a.lse_p = w.lse_p;
    a.mask = out->mask ? out->mask : w.mask;
    a.rowflag = w.rowflag;
    a.usize = out->union_size;
    a.topk_a = out->topk_actor; a.topk_p = out->topk_policy;
    const bool lp = (prm->flags & JP_FLAG_TOPK_LOGPROBS) != 0;
    a.topk_a_lq = lp ? out->topk_actor_logq : nullptr;
    a.topk_p_lp = lp ? out->topk_policy_logp : nullptr;
    a.waves = (prm->flags & JP_FLAG_ONE_WAVE_PER_ROW) ? 1 : jp::waves_per_row(T, V, (int)esz);
    if (jp::launch_rows(a, (int)dt, st) != hipSuccess) return JP_ERR_HIP;

    if (prm->flags & JP_FLAG_EXACT_Z) {
        jp::ZExactArgs z{};
        z.actor = actor; z.policy = policy; z.T = T; z.V = V; z.stride = row_stride;
        z.lse_q = w.lse_q; z.lse_p = w.lse_p; z.rowflag = w.rowflag; z.lambda = prm->lambda;
        z.zexact = out->z_exact ? out->z_exact : w.zexact;
        z.waves = a.waves;
        if (jp::launch_zexact(z, (int)dt, st) != hipSuccess) return JP_ERR_HIP;
    }
    return JP_OK;
}

jp_status finalize_impl(int64_t T, const int32_t *ids, const float *uni_given, const float *ref_logprob,
                        const jp_obrs_params *prm, const jp_obrs_outputs *out, void *workspace,
                        size_t workspace_bytes, hipStream_t st, bool have_uniforms)
{
    (void)ids; (void)uni_given;
    if (!prm || !out) return JP_ERR_NULL;
    if (T < 0 || T > 0x7fffffffLL) return JP_ERR_SHAPE;
    if (prm->flags & ~KNOWN_FLAGS) return JP_ERR_UNSUPPORTED;
    if (!(prm->lambda > 0.f) || !isfinite(prm->lambda) || !(prm->c1 > 0.f) || !(prm->c2 > 0.f)) return JP_ERR_PARAM;
    if (prm->f_mode > JP_F_BAND) return JP_ERR_UNSUPPORTED;
    if (prm->f_mode == JP_F_BAND && !(prm->f_lo >= 0.f && prm->f_lo <= prm->f_hi)) return JP_ERR_PARAM;
    const Workspace w = carve(workspace, T);
    if (!workspace || workspace_bytes < w.bytes) return JP_ERR_WORKSPACE;
    if (((uintptr_t)workspace & (ALIGN - 1)) != 0) return JP_ERR_ALIGN;

    jp::FinalizeArgs f{};
    f.T = T;
    f.rowflag = w.rowflag;
    f.mask = out->mask ? out->mask : w.mask;
    f.accept = out->accept_prob ? out->accept_prob : w.accept;
    f.zapprox = out->z_approx ? out->z_approx : w.zapprox;
    f.zexact = (prm->flags & JP_FLAG_EXACT_Z) ? (out->z_exact ? out->z_exact : w.zexact) : nullptr;
    f.logratio = out->logratio ? out->logratio : w.logratio;
    f.logp = out->logp ? out->logp : w.logp;
    f.ref_logprob = ref_logprob;
    f.kl = (prm->flags & JP_FLAG_DISTILL_KL) ? (out->distill_kl ? out->distill_kl : w.kl) : nullptr;
    f.lambda = prm->lambda; f.c1 = prm->c1; f.c2 = prm->c2;
    f.f_mode = (int)prm->f_mode; f.f_lo = prm->f_lo; f.f_hi = prm->f_hi;
    f.alpha_expected = ((prm->flags & JP_FLAG_ALPHA_EXPECTED) || !have_uniforms) ? 1 : 0;
    f.stats = out->stats ? out->stats : w.stats;
    f.w = out->w_obrs; f.rho = out->rho;
    if (jp::launch_finalize(f, st) != hipSuccess) return JP_ERR_HIP;
    return JP_OK;
}

// ---- fused lm_head path ------------------------------------------------------------------------

constexpr int64_t LM_GROUP = 4;

struct LmheadPlan {
    int64_t group, ldc;
    int64_t chunk, npad, nchunks;
    size_t off_state, off_wt_p, off_wt_a, off_lp, off_lq, bytes;
    size_t state_stride;
};

// d_actor == 0: the stored-actor form, which has no actor head (no weight chunk, no logit buffer for it)
bool plan_lmhead(int64_t T, int64_t V, int64_t d_actor, int64_t d_policy, int32_t k, int64_t vocab_chunk,
                 LmheadPlan &p)
{
    if (T < 0 || T > 0x7fffffffLL || V <= 0 || V > 0x7fffffffLL || k < 1) return false;
    if (d_actor < 0 || d_policy <= 0 || d_actor % 64 || d_policy % 64 || d_actor > (1 << 20) || d_policy > (1 << 20)) return false;
    // Default width: a chunk of 4096 columns keeps the logit buffers of a large batch in the caches
    // between the GEMM and the row stage; a small batch has few row tiles, and needs wider chunks for
    // its GEMM launches to fill the chip, in two generations of workgroups at least, so that the short
    // tiles of the actor head fill in behind the policy head's (T = 256: 4.5 ms per call at 4096
    // columns, 1.7 at 65536).
    const int64_t by_batch = T <= 768 ? 65536 : (T <= 1536 ? 16384 : (T <= 6144 ? 8192 : 4096));
    int64_t c = vocab_chunk > 0 ? vocab_chunk : by_batch;
    c = (c + jp::LMHEAD_N_ALIGN - 1) / jp::LMHEAD_N_ALIGN * jp::LMHEAD_N_ALIGN;
    const int64_t vpad = (V + jp::LMHEAD_N_ALIGN - 1) / jp::LMHEAD_N_ALIGN * jp::LMHEAD_N_ALIGN;
    if (c > vpad) c = vpad;
    p.chunk = c; p.npad = c; p.nchunks = (V + c - 1) / c;
    p.state_stride = jp::carry_state_bytes(k);
    size_t off = carve(nullptr, T).bytes;
    const size_t n = (size_t)(T > 0 ? T : 0);
    p.off_state = off; off += round_up(n * p.state_stride);
    p.off_wt_p = off; off += round_up((size_t)c * (size_t)d_policy * 2);
    p.off_wt_a = off; off += round_up((size_t)c * (size_t)d_actor * 2);
    // the logit buffers hold LM_GROUP chunks side by side: the row stage runs once per group, which
    // spreads its per-row fixed cost (record read/write, list merge) over more columns
    p.group = p.nchunks < LM_GROUP ? p.nchunks : LM_GROUP;
    p.ldc = c * p.group;
    p.off_lp = off; off += round_up(n * (size_t)p.ldc * 4);
    p.off_lq = off; off += d_actor > 0 ? round_up(n * (size_t)p.ldc * 4) : 0;
    p.bytes = off;
    return true;
}

}  // namespace

extern "C" {

size_t jp_obrs_lmhead_workspace_bytes(int64_t T, int64_t V, int64_t d_actor, int64_t d_policy, int32_t k,
                                      int64_t vocab_chunk)
{
    LmheadPlan p;
    return d_actor > 0 && plan_lmhead(T, V, d_actor, d_policy, k, vocab_chunk, p) ? p.bytes : 0;
}

size_t jp_obrs_lmhead_stored_workspace_bytes(int64_t T, int64_t V, int64_t d_policy, int32_t k, int64_t vocab_chunk)
{
    LmheadPlan p;
    return plan_lmhead(T, V, 0, d_policy, k, vocab_chunk, p) ? p.bytes : 0;
}

/* Target logits from the matrix cores chunk by chunk, actor side as the rollout phase stored it. */
jp_status jp_obrs_forward_lmhead_stored(const void *H_policy, int64_t d_policy, const void *W_policy, int64_t T,
                                        int64_t V, int64_t vocab_chunk, const int32_t *actor_topk_ids,
                                        const float *actor_topk_logprob, const float *actor_logprob_x,
                                        const int32_t *sampled_ids, const float *uniforms,
                                        const float *ref_logprob, const jp_obrs_params *prm,
                                        jp_tail_rule tail_rule, const jp_obrs_outputs *out, void *workspace,
                                        size_t workspace_bytes, void *stream)
{
    if (!prm || !out) return JP_ERR_NULL;
    LmheadPlan pl;
    if (!plan_lmhead(T, V, 0, d_policy, prm->k, vocab_chunk, pl)) {
        if (prm->k < 1) return JP_ERR_PARAM;
        return JP_ERR_SHAPE;
    }
    jp_status s = check_params(prm, V, true);
    if (s != JP_OK) return s;
    if (prm->flags & (JP_FLAG_EXACT_Z | JP_FLAG_DISTILL_KL)) return JP_ERR_UNSUPPORTED;   // need the actor row
    if (tail_rule != JP_TAIL_DROP && tail_rule != JP_TAIL_KTH && tail_rule != JP_TAIL_REST) return JP_ERR_PARAM;
    if (T > 0 && (!H_policy || !W_policy || !sampled_ids || !actor_topk_ids || !actor_topk_logprob || !actor_logprob_x))
        return JP_ERR_NULL;
    if (!aligned16(H_policy) || ((uintptr_t)W_policy & 1)) return JP_ERR_ALIGN;
    const bool vmajor = (prm->flags & JP_FLAG_W_VOCAB_MAJOR) != 0;
    if (vmajor && !aligned16(W_policy)) return JP_ERR_ALIGN;
    if (!workspace || workspace_bytes < pl.bytes) return JP_ERR_WORKSPACE;
    if (((uintptr_t)workspace & (ALIGN - 1)) != 0) return JP_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;

    if (T > 0) {
        const Workspace w = carve(workspace, T);
        char *base = (char *)workspace;
        jp::RowArgs a{};
        a.actor = nullptr; a.policy = base + pl.off_lp;
        a.T = T; a.stride = pl.ldc; a.ids = sampled_ids; a.uni = uniforms;
        a.lambda = prm->lambda; a.ln_lambda = log((double)prm->lambda); a.k = prm->k;
        a.accept = out->accept_prob ? out->accept_prob : w.accept;
        a.logq = out->logq ? out->logq : w.logq;
        a.logp = out->logp ? out->logp : w.logp;
        a.logratio = out->logratio ? out->logratio : w.logratio;
        a.zapprox = out->z_approx ? out->z_approx : w.zapprox;
        a.kl = w.kl;
        a.lse_q = w.lse_q; a.lse_p = w.lse_p;
        a.mask = out->mask ? out->mask : w.mask;
        a.rowflag = w.rowflag;
        a.usize = out->union_size;
        a.topk_a = nullptr; a.topk_p = out->topk_policy;
        a.topk_a_lq = nullptr;
        a.topk_p_lp = (prm->flags & JP_FLAG_TOPK_LOGPROBS) ? out->topk_policy_logp : nullptr;
        a.V_total = V; a.state = (unsigned char *)base + pl.off_state; a.state_stride = (int64_t)pl.state_stride;
        a.stored_ids = actor_topk_ids; a.stored_logq = actor_topk_logprob; a.stored_logq_x = actor_logprob_x;
        a.tail_rule = (int)tail_rule;

        jp::GemmArgs g{};
        g.A[0] = H_policy; g.Bt[0] = base + pl.off_wt_p; g.K[0] = (int)d_policy;
        g.M = (int)T; g.nproblems = 1; g.ldc = pl.ldc;
        float *const c_policy = (float *)(base + pl.off_lp);
        int64_t group_base = 0, group_cols = 0, groups_done = 0;
        for (int64_t j = 0; j < pl.nchunks; ++j) {
            const int64_t v0 = j * pl.chunk;
            const int ncols = (int)((V - v0) < pl.chunk ? (V - v0) : pl.chunk);
            const int nthis = (ncols + jp::LMHEAD_N_ALIGN - 1) / jp::LMHEAD_N_ALIGN * jp::LMHEAD_N_ALIGN;
            g.N = nthis;
            const int64_t slot = j % pl.group;
            g.C[0] = c_policy + slot * pl.chunk;
            if (slot == 0) { group_base = v0; group_cols = 0; }
            group_cols += ncols;
            if (!vmajor) {
                if (jp::launch_transpose_chunk(W_policy, V, (int)d_policy, v0, ncols, nthis, base + pl.off_wt_p, st) != hipSuccess) return JP_ERR_HIP;
                g.Bt[0] = base + pl.off_wt_p;
            } else if (ncols == nthis) {
                g.Bt[0] = (const char *)W_policy + (size_t)v0 * (size_t)d_policy * 2;
                if (jp::launch_touch_rows(g.Bt[0], (int64_t)nthis * d_policy * 2, base + pl.off_wt_p, st) != hipSuccess) return JP_ERR_HIP;
            } else {
                if (jp::launch_copy_rows_chunk(W_policy, (int)d_policy, v0, ncols, nthis, base + pl.off_wt_p, st) != hipSuccess) return JP_ERR_HIP;
                g.Bt[0] = base + pl.off_wt_p;
            }
            if (jp::launch_gemm_pair(g, st) != hipSuccess) return JP_ERR_HIP;
            const bool last = j + 1 == pl.nchunks;
            if (slot + 1 == pl.group || last) {
                a.V = group_cols; a.id_base = group_base; a.carry_in = groups_done > 0; a.carry_out = !last;
                a.waves = (prm->flags & JP_FLAG_ONE_WAVE_PER_ROW) ? 1 : jp::waves_per_row(T, group_cols, 4);
                if (jp::launch_rows_carry_stored(a, st) != hipSuccess) return JP_ERR_HIP;
                ++groups_done;
            }
        }
    }
    return finalize_impl(T, sampled_ids, uniforms, ref_logprob, prm, out, workspace, workspace_bytes, st,
                         uniforms != nullptr);
}

jp_status jp_obrs_forward_lmhead(const void *H_actor, int64_t d_actor, const void *W_actor,
                                 const void *H_policy, int64_t d_policy, const void *W_policy,
                                 int64_t T, int64_t V, int64_t vocab_chunk, const int32_t *sampled_ids,
                                 const float *uniforms, const float *ref_logprob,
                                 const jp_obrs_params *prm, const jp_obrs_outputs *out, void *workspace,
                                 size_t workspace_bytes, void *stream)
{
    if (!prm || !out) return JP_ERR_NULL;
    LmheadPlan pl;
    if (d_actor <= 0 || !plan_lmhead(T, V, d_actor, d_policy, prm->k, vocab_chunk, pl)) {
        if (prm->k < 1) return JP_ERR_PARAM;
        return JP_ERR_SHAPE;
    }
    jp_status s = check_params(prm, V, true);
    if (s != JP_OK) return s;
    if (prm->flags & JP_FLAG_EXACT_Z) return JP_ERR_UNSUPPORTED;   // needs a second pass over logits that are gone
    if (T > 0 && (!H_actor || !W_actor || !H_policy || !W_policy || !sampled_ids)) return JP_ERR_NULL;
    if (!aligned16(H_actor) || !aligned16(H_policy) || ((uintptr_t)W_actor & 1) || ((uintptr_t)W_policy & 1)) return JP_ERR_ALIGN;
    const bool vmajor = (prm->flags & JP_FLAG_W_VOCAB_MAJOR) != 0;
    if (vmajor && (!aligned16(W_actor) || !aligned16(W_policy))) return JP_ERR_ALIGN;
    if (!workspace || workspace_bytes < pl.bytes) return JP_ERR_WORKSPACE;
    if (((uintptr_t)workspace & (ALIGN - 1)) != 0) return JP_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;

    if (T > 0) {
        const Workspace w = carve(workspace, T);
        char *base = (char *)workspace;
        jp::RowArgs a{};
        a.actor = base + pl.off_lq; a.policy = base + pl.off_lp;
        a.T = T; a.stride = pl.ldc; a.ids = sampled_ids; a.uni = uniforms;
        a.lambda = prm->lambda; a.ln_lambda = log((double)prm->lambda); a.k = prm->k;
        a.accept = out->accept_prob ? out->accept_prob : w.accept;
        a.logq = out->logq ? out->logq : w.logq;
        a.logp = out->logp ? out->logp : w.logp;
        a.logratio = out->logratio ? out->logratio : w.logratio;
        a.zapprox = out->z_approx ? out->z_approx : w.zapprox;
        a.distill = (prm->flags & JP_FLAG_DISTILL_KL) ? 1 : 0;
        a.kl = out->distill_kl ? out->distill_kl : w.kl;
        a.lse_q = w.lse_q; a.lse_p = w.lse_p;
        a.mask = out->mask ? out->mask : w.mask;
        a.rowflag = w.rowflag;
        a.usize = out->union_size;
        a.topk_a = out->topk_actor; a.topk_p = out->topk_policy;
        const bool lp = (prm->flags & JP_FLAG_TOPK_LOGPROBS) != 0;
        a.topk_a_lq = lp ? out->topk_actor_logq : nullptr;
        a.topk_p_lp = lp ? out->topk_policy_logp : nullptr;
        a.V_total = V; a.state = (unsigned char *)base + pl.off_state; a.state_stride = (int64_t)pl.state_stride;

        jp::GemmArgs g{};
        g.A[0] = H_policy; g.Bt[0] = base + pl.off_wt_p; g.C[0] = (float *)(base + pl.off_lp); g.K[0] = (int)d_policy;
        g.A[1] = H_actor; g.Bt[1] = base + pl.off_wt_a; g.C[1] = (float *)(base + pl.off_lq); g.K[1] = (int)d_actor;
        g.M = (int)T; g.N = (int)pl.npad; g.nproblems = 2; g.ldc = pl.ldc;
        float *const c_policy = (float *)(base + pl.off_lp), *const c_actor = (float *)(base + pl.off_lq);
        int64_t group_base = 0, group_cols = 0, groups_done = 0;

        for (int64_t j = 0; j < pl.nchunks; ++j) {
            const int64_t v0 = j * pl.chunk;
            const int ncols = (int)((V - v0) < pl.chunk ? (V - v0) : pl.chunk);
            // the last chunk is multiplied only up to its own width rounded to the column tile
            const int nthis = (ncols + jp::LMHEAD_N_ALIGN - 1) / jp::LMHEAD_N_ALIGN * jp::LMHEAD_N_ALIGN;
            g.N = nthis;
            const int64_t slot = j % pl.group;                // where this chunk sits inside the group buffer
            g.C[0] = c_policy + slot * pl.chunk;
            g.C[1] = c_actor + slot * pl.chunk;
            if (slot == 0) { group_base = v0; group_cols = 0; }
            group_cols += ncols;
            if (!vmajor) {
                if (jp::launch_transpose_chunk(W_policy, V, (int)d_policy, v0, ncols, nthis, base + pl.off_wt_p, st) != hipSuccess) return JP_ERR_HIP;
                if (jp::launch_transpose_chunk(W_actor, V, (int)d_actor, v0, ncols, nthis, base + pl.off_wt_a, st) != hipSuccess) return JP_ERR_HIP;
            } else if (ncols == nthis) {
                // [V, d] weights: a chunk of whole column tiles is already the GEMM's second operand
                g.Bt[0] = (const char *)W_policy + (size_t)v0 * (size_t)d_policy * 2;
                g.Bt[1] = (const char *)W_actor + (size_t)v0 * (size_t)d_actor * 2;
                if (jp::launch_touch_rows(g.Bt[0], (int64_t)nthis * d_policy * 2, base + pl.off_wt_p, st) != hipSuccess) return JP_ERR_HIP;
                if (jp::launch_touch_rows(g.Bt[1], (int64_t)nthis * d_actor * 2, base + pl.off_wt_a, st) != hipSuccess) return JP_ERR_HIP;
            } else {
                if (jp::launch_copy_rows_chunk(W_policy, (int)d_policy, v0, ncols, nthis, base + pl.off_wt_p, st) != hipSuccess) return JP_ERR_HIP;
                if (jp::launch_copy_rows_chunk(W_actor, (int)d_actor, v0, ncols, nthis, base + pl.off_wt_a, st) != hipSuccess) return JP_ERR_HIP;
                g.Bt[0] = base + pl.off_wt_p;
                g.Bt[1] = base + pl.off_wt_a;
            }
            if (jp::launch_gemm_pair(g, st) != hipSuccess) return JP_ERR_HIP;
            const bool last = j + 1 == pl.nchunks;
            if (slot + 1 == pl.group || last) {               // the group is complete: one row-stage launch over it
                a.V = group_cols; a.id_base = group_base; a.carry_in = groups_done > 0; a.carry_out = !last;
                a.waves = (prm->flags & JP_FLAG_ONE_WAVE_PER_ROW) ? 1 : jp::waves_per_row(T, group_cols, 4);
                if (jp::launch_rows_carry(a, st) != hipSuccess) return JP_ERR_HIP;
                ++groups_done;
            }
        }
    }
    return finalize_impl(T, sampled_ids, uniforms, ref_logprob, prm, out, workspace, workspace_bytes, st,
                         uniforms != nullptr);
}

size_t jp_obrs_workspace_bytes(int64_t T, int64_t V, int32_t k, jp_dtype dt, uint32_t flags)
{
    (void)flags;
    if (T < 0 || T > 0x7fffffffLL || V <= 0 || k < 1 || (dt != JP_F32 && dt != JP_BF16)) return 0;
    return carve(nullptr, T).bytes;
}

jp_status jp_obrs_rows(const void *actor_logits, const void *policy_logits, int64_t T, int64_t V,
                       int64_t row_stride, jp_dtype dt, const int32_t *sampled_ids,
                       const float *uniforms, const jp_obrs_params *prm, const jp_obrs_outputs *out,
                       void *workspace, size_t workspace_bytes, void *stream)
{
    return rows_impl(actor_logits, policy_logits, T, V, row_stride, dt, sampled_ids, uniforms, prm, out,
                     workspace, workspace_bytes, (hipStream_t)stream, false);
}

jp_status jp_obrs_finalize(int64_t T, const int32_t *sampled_ids, const float *ref_logprob,
                           const jp_obrs_params *prm, const jp_obrs_outputs *out, void *workspace,
                           size_t workspace_bytes, void *stream)
{
    // Whether uniforms were supplied is not known here: the caller states it through
    // JP_FLAG_ALPHA_EXPECTED (set it when the row stage ran without uniforms).
    return finalize_impl(T, sampled_ids, nullptr, ref_logprob, prm, out, workspace, workspace_bytes,
                         (hipStream_t)stream, true);
}

jp_status jp_obrs_forward(const void *actor_logits, const void *policy_logits, int64_t T, int64_t V,
                          int64_t row_stride, jp_dtype dt, const int32_t *sampled_ids,
                          const float *uniforms, const float *ref_logprob, const jp_obrs_params *prm,
                          const jp_obrs_outputs *out, void *workspace, size_t workspace_bytes,
                          void *stream)
{
    jp_status s = rows_impl(actor_logits, policy_logits, T, V, row_stride, dt, sampled_ids, uniforms, prm,
                            out, workspace, workspace_bytes, (hipStream_t)stream, true);
    if (s != JP_OK) return s;
    return finalize_impl(T, sampled_ids, uniforms, ref_logprob, prm, out, workspace, workspace_bytes,
                         (hipStream_t)stream, uniforms != nullptr);
}

/* jp_obrs_forward on the library's static scratch instead of a caller's workspace. */
jp_status jp_obrs_forward_static(const void *actor_logits, const void *policy_logits, int64_t T, int64_t V,
                                 int64_t row_stride, jp_dtype dt, const int32_t *sampled_ids,
                                 const float *uniforms, const float *ref_logprob, const jp_obrs_params *prm,
                                 const jp_obrs_outputs *out, void *stream)
{
    if (T > JP_STATIC_MAX_T) return JP_ERR_TOO_LARGE;       // before anything touches the GPU
    if (T < 0) return JP_ERR_SHAPE;
    if (carve(nullptr, T).bytes > STATIC_SCRATCH_BYTES) return JP_ERR_TOO_LARGE;
    if (!prm || !out) return JP_ERR_NULL;
    // every argument error is reported before the scratch is looked up (which needs a GPU)
    jp_status s = check_shape(T, V, row_stride, dt);
    if (s == JP_OK) s = check_params(prm, V, true);
    if (s != JP_OK) return s;
    if (T > 0 && (!actor_logits || !policy_logits || !sampled_ids)) return JP_ERR_NULL;
    const size_t esz = dt == JP_BF16 ? 2 : 4;
    if (!aligned16(actor_logits) || !aligned16(policy_logits) || ((size_t)row_stride * esz) % 16 != 0) return JP_ERR_ALIGN;
    void *ws = nullptr;
    s = static_scratch(&ws);
    if (s != JP_OK) return s;
    return jp_obrs_forward(actor_logits, policy_logits, T, V, row_stride, dt, sampled_ids, uniforms, ref_logprob,
                           prm, out, ws, STATIC_SCRATCH_BYTES, stream);
}

/* Whole hot path with the actor side as the rollout phase stored it (ids + log-probabilities). */
jp_status jp_obrs_forward_stored(const void *policy_logits, int64_t T, int64_t V, int64_t row_stride,
                                 jp_dtype dt, const int32_t *actor_topk_ids, const float *actor_topk_logprob,
                                 const float *actor_logprob_x, const int32_t *sampled_ids,
                                 const float *uniforms, const float *ref_logprob, const jp_obrs_params *prm,
                                 jp_tail_rule tail_rule, const jp_obrs_outputs *out, void *workspace,
                                 size_t workspace_bytes, void *stream)
{
    if (!prm || !out) return JP_ERR_NULL;
    jp_status s = check_shape(T, V, row_stride, dt);
    if (s != JP_OK) return s;
    s = check_params(prm, V, true);
    if (s != JP_OK) return s;
    if (prm->flags & (JP_FLAG_EXACT_Z | JP_FLAG_DISTILL_KL)) return JP_ERR_UNSUPPORTED;   // need the actor row
    if (tail_rule != JP_TAIL_DROP && tail_rule != JP_TAIL_KTH && tail_rule != JP_TAIL_REST) return JP_ERR_PARAM;
    if (T > 0 && (!policy_logits || !sampled_ids || !actor_topk_ids || !actor_topk_logprob || !actor_logprob_x))
        return JP_ERR_NULL;
    const size_t esz = dt == JP_BF16 ? 2 : 4;
    if (!aligned16(policy_logits) || ((size_t)row_stride * esz) % 16 != 0) return JP_ERR_ALIGN;
    if (!workspace || workspace_bytes < jp_obrs_workspace_bytes(T, V, prm->k, dt, prm->flags)) return JP_ERR_WORKSPACE;
    if (((uintptr_t)workspace & (ALIGN - 1)) != 0) return JP_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    if (T > 0) {
        const Workspace w = carve(workspace, T);
        jp::RowArgs a{};
        a.actor = nullptr; a.policy = policy_logits; a.T = T; a.V = V; a.stride = row_stride;
        a.ids = sampled_ids; a.uni = uniforms; a.lambda = prm->lambda; a.ln_lambda = log((double)prm->lambda);
        a.k = prm->k;
        a.accept = out->accept_prob ? out->accept_prob : w.accept;
        a.logq = out->logq ? out->logq : w.logq;
        a.logp = out->logp ? out->logp : w.logp;
        a.logratio = out->logratio ? out->logratio : w.logratio;
        a.zapprox = out->z_approx ? out->z_approx : w.zapprox;
        a.kl = w.kl;
        a.lse_q = w.lse_q; a.lse_p = w.lse_p;
        a.mask = out->mask ? out->mask : w.mask;
        a.rowflag = w.rowflag;
        a.usize = out->union_size;
        a.topk_a = nullptr; a.topk_p = out->topk_policy;
        a.topk_a_lq = nullptr;
        a.topk_p_lp = (prm->flags & JP_FLAG_TOPK_LOGPROBS) ? out->topk_policy_logp : nullptr;
        a.stored_ids = actor_topk_ids; a.stored_logq = actor_topk_logprob; a.stored_logq_x = actor_logprob_x;
        a.tail_rule = (int)tail_rule;
        a.waves = (prm->flags & JP_FLAG_ONE_WAVE_PER_ROW) ? 1 : jp::waves_per_row(T, V, dt == JP_BF16 ? 2 : 4);
        if (jp::launch_rows_stored(a, (int)dt, st) != hipSuccess) return JP_ERR_HIP;
    }
    return finalize_impl(T, sampled_ids, uniforms, ref_logprob, prm, out, workspace, workspace_bytes, st,
                         uniforms != nullptr);
}

jp_status jp_obrs_token_logprob(const void *logits, int64_t T, int64_t V, int64_t row_stride, jp_dtype dt,
                                const int32_t *sampled_ids, float *out_logprob, void *stream)
{
    jp_status s = check_shape(T, V, row_stride, dt);
    if (s != JP_OK) return s;
    if (T > 0 && (!logits || !sampled_ids || !out_logprob)) return JP_ERR_NULL;
    const size_t esz = dt == JP_BF16 ? 2 : 4;
    if (!aligned16(logits) || ((size_t)row_stride * esz) % 16 != 0) return JP_ERR_ALIGN;
    jp::LogprobArgs a{logits, T, V, row_stride, sampled_ids, out_logprob};
    if (jp::launch_token_logprob(a, (int)dt, (hipStream_t)stream) != hipSuccess) return JP_ERR_HIP;
    return JP_OK;
}

size_t jp_obrs_forward3_workspace_bytes(int64_t T, int64_t V, int32_t k, jp_dtype dt, uint32_t flags)
{
    const size_t base = jp_obrs_workspace_bytes(T, V, k, dt, flags);
    return base ? base + round_up((size_t)T * 4) : 0;
}

jp_status jp_obrs_forward3(const void *actor_logits, const void *policy_new_logits, const void *policy_ref_logits,
                           int32_t target_is_ref, int64_t T, int64_t V, int64_t row_stride, jp_dtype dt,
                           const int32_t *sampled_ids, const float *uniforms, const jp_obrs_params *prm,
                           const jp_obrs_outputs *out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!prm || !out) return JP_ERR_NULL;
    if (T > 0 && !policy_ref_logits) return JP_ERR_NULL;
    if (target_is_ref)
        return jp_obrs_forward(actor_logits, policy_ref_logits, T, V, row_stride, dt, sampled_ids, uniforms,
                               nullptr, prm, out, workspace, workspace_bytes, stream);
    const size_t base = jp_obrs_workspace_bytes(T, V, prm->k, dt, prm->flags);
    if (base == 0) return JP_ERR_SHAPE;
    if (!workspace || workspace_bytes < base + round_up((size_t)(T > 0 ? T : 0) * 4)) return JP_ERR_WORKSPACE;
    float *ref_lp = (float *)((char *)workspace + base);
    // argument errors of the main call are reported before anything is launched
    if (T > 0 && (!actor_logits || !policy_new_logits || !sampled_ids)) return JP_ERR_NULL;
    jp_status s = check_shape(T, V, row_stride, dt);
    if (s == JP_OK) s = check_params(prm, V, true);
    if (s != JP_OK) return s;
    const size_t esz = dt == JP_BF16 ? 2 : 4;
    if (!aligned16(actor_logits) || !aligned16(policy_new_logits) || !aligned16(policy_ref_logits) ||
        ((size_t)row_stride * esz) % 16 != 0 || ((uintptr_t)workspace & (ALIGN - 1)) != 0)
        return JP_ERR_ALIGN;
    s = jp_obrs_token_logprob(policy_ref_logits, T, V, row_stride, dt, sampled_ids, ref_lp, stream);
    if (s != JP_OK) return s;
    return jp_obrs_forward(actor_logits, policy_new_logits, T, V, row_stride, dt, sampled_ids, uniforms,
                           ref_lp, prm, out, workspace, base, stream);
}

/* Per-row scaling factor for an acceptance budget (Theorem 2). */
jp_status jp_obrs_lambda_for_budget(const void *actor_logits, const void *policy_logits, int64_t T, int64_t V,
                                    int64_t row_stride, jp_dtype dt, const float *row_target, float target,
                                    float *out_lambda, const void *workspace, size_t workspace_bytes,
                                    void *stream)
{
    jp_status s = check_shape(T, V, row_stride, dt);
    if (s != JP_OK) return s;
    if (!row_target && (!(target > 0.f) || target > 1.f)) return JP_ERR_PARAM;
    if (T > 0 && (!actor_logits || !policy_logits || !out_lambda)) return JP_ERR_NULL;
    const size_t esz = dt == JP_BF16 ? 2 : 4;
    if (!aligned16(actor_logits) || !aligned16(policy_logits) || ((size_t)row_stride * esz) % 16 != 0) return JP_ERR_ALIGN;
    const Workspace w = carve(const_cast<void *>(workspace), T);
    if (!workspace || workspace_bytes < w.bytes) return JP_ERR_WORKSPACE;
    if (((uintptr_t)workspace & (ALIGN - 1)) != 0) return JP_ERR_ALIGN;
    if (T == 0) return JP_OK;
    jp::BudgetArgs b{};
    b.actor = actor_logits; b.policy = policy_logits; b.T = T; b.V = V; b.stride = row_stride;
    b.lse_q = w.lse_q; b.lse_p = w.lse_p; b.rowflag = w.rowflag;
    b.row_target = row_target; b.target = target; b.lambda_out = out_lambda;
    b.eps_rel = dt == JP_BF16 ? 1e-4f : 1e-6f;         // a tenth of the float tolerance of the other outputs
    if (jp::launch_budget(b, (int)dt, (hipStream_t)stream) != hipSuccess) return JP_ERR_HIP;
    return JP_OK;
}

size_t jp_obrs_budget_scratch_bytes(void) { return round_up(sizeof(jp::BudgetBatchState)); }

/* One scaling factor for the whole batch: mean_t Z_t(lambda) = target. */
jp_status jp_obrs_lambda_for_budget_batch(const void *actor_logits, const void *policy_logits, int64_t T,
                                          int64_t V, int64_t row_stride, jp_dtype dt, float target,
                                          float *out_lambda, const void *workspace, size_t workspace_bytes,
                                          void *scratch, size_t scratch_bytes, void *stream)
{
    jp_status s = check_shape(T, V, row_stride, dt);
    if (s != JP_OK) return s;
    if (!(target > 0.f) || target > 1.f) return JP_ERR_PARAM;
    if (!out_lambda || (T > 0 && (!actor_logits || !policy_logits))) return JP_ERR_NULL;
    const size_t esz = dt == JP_BF16 ? 2 : 4;
    if (!aligned16(actor_logits) || !aligned16(policy_logits) || ((size_t)row_stride * esz) % 16 != 0) return JP_ERR_ALIGN;
    const Workspace w = carve(const_cast<void *>(workspace), T);
    if (!workspace || workspace_bytes < w.bytes) return JP_ERR_WORKSPACE;
    if (!scratch || scratch_bytes < jp_obrs_budget_scratch_bytes()) return JP_ERR_WORKSPACE;
    if (((uintptr_t)workspace & (ALIGN - 1)) != 0 || ((uintptr_t)scratch & 15u) != 0) return JP_ERR_ALIGN;
    jp::BudgetArgs b{};
    b.actor = actor_logits; b.policy = policy_logits; b.T = T; b.V = V; b.stride = row_stride;
    b.lse_q = w.lse_q; b.lse_p = w.lse_p; b.rowflag = w.rowflag;
    b.row_target = nullptr; b.target = target; b.lambda_out = nullptr;
    b.eps_rel = dt == JP_BF16 ? 1e-4f : 1e-6f;
    if (jp::launch_budget_batch(b, (int)dt, (jp::BudgetBatchState *)scratch, out_lambda, (hipStream_t)stream) != hipSuccess)
        return JP_ERR_HIP;
    return JP_OK;
}

/* Gradient of the distillation term with respect to the actor logits (second streaming pass). */
jp_status jp_obrs_distill_grad(const void *actor_logits, const void *policy_logits, int64_t T, int64_t V,
                               int64_t row_stride, jp_dtype dt, const float *row_scale, float scale,
                               void *grad_actor, int64_t grad_row_stride, jp_dtype grad_dt,
                               const void *workspace, size_t workspace_bytes, void *stream)
{
    jp_status s = check_shape(T, V, row_stride, dt);
    if (s != JP_OK) return s;
    if (grad_dt != JP_F32 && grad_dt != JP_BF16) return JP_ERR_UNSUPPORTED;
    if (grad_row_stride < V) return JP_ERR_SHAPE;
    if (!isfinite(scale)) return JP_ERR_PARAM;
    if (T > 0 && (!actor_logits || !policy_logits || !grad_actor)) return JP_ERR_NULL;
    const size_t esz = dt == JP_BF16 ? 2 : 4, gsz = grad_dt == JP_BF16 ? 2 : 4;
    if (!aligned16(actor_logits) || !aligned16(policy_logits) || ((size_t)row_stride * esz) % 16 != 0) return JP_ERR_ALIGN;
    if (!aligned16(grad_actor) || ((size_t)grad_row_stride * gsz) % 16 != 0) return JP_ERR_ALIGN;
    const Workspace w = carve(const_cast<void *>(workspace), T);
    if (!workspace || workspace_bytes < w.bytes) return JP_ERR_WORKSPACE;
    if (((uintptr_t)workspace & (ALIGN - 1)) != 0) return JP_ERR_ALIGN;
    if (T == 0) return JP_OK;
    jp::GradArgs g{};
    g.actor = actor_logits; g.policy = policy_logits; g.T = T; g.V = V; g.stride = row_stride;
    g.lse_q = w.lse_q; g.lse_p = w.lse_p; g.rowflag = w.rowflag;
    g.row_scale = row_scale; g.scale = scale;
    g.grad = grad_actor; g.grad_stride = grad_row_stride;
    if (jp::launch_distill_grad(g, (int)dt, (int)grad_dt, (hipStream_t)stream) != hipSuccess) return JP_ERR_HIP;
    return JP_OK;
}

const char *jp_status_string(int32_t status)
{
    switch (status) {
    case JP_OK: return "ok";
    case JP_ERR_NULL: return "required pointer is NULL";
    case JP_ERR_SHAPE: return "invalid shape";
    case JP_ERR_PARAM: return "invalid parameter";
    case JP_ERR_ALIGN: return "pointer or row pitch not 16-byte aligned";
    case JP_ERR_WORKSPACE: return "workspace missing or too small";
    case JP_ERR_UNSUPPORTED: return "unsupported dtype, flag or k";
    case JP_ERR_HIP: return "HIP launch failed";
    case JP_ERR_TOO_LARGE: return "more token positions than the static scratch of the no-allocation entry point holds";
    }
    return "unknown status";
}

int jp_obrs_abi_version(void) { return 9; }

}  // extern "C"
