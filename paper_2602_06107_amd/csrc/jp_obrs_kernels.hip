// OBRS hot path of Jackpot for gfx950 (MI355X): the kernels around the row kernel.
//
// The optional second sweep that computes the normaliser of Eq. obrs_dist over the whole vocabulary,
// the log-probability of the sampled token under one more logit tensor, the scaling factor for an
// acceptance budget (Sec. 3.3, Theorem 2), the gradient of the distillation term of Sec. 4.2 (3),
// and the batch stage: the statistics of Sec. 4.4.2 and the weights of Alg. 1 step 3.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "jp_device_utils.h"
#include "jp_obrs_internal.h"

namespace jp {

// =================================================================================================
// Exact normaliser (diagnostic): Z_t = sum_v min(q_v, p_v/lambda) = sum_v 2^min(aq_v, ap_v) with
// aq = (lq - LSEq) log2e, ap = (lp - LSEp - ln lambda) log2e.  One wavefront per row.
// =================================================================================================
// W > 1: a row goes to W wavefronts of one workgroup, each with a contiguous run of the sweep
// iterations (small batches, where one wave per row leaves the chip idle); wave 0 adds the parts.
template <class ET, int W = 1>
__global__ __launch_bounds__(64 * W) void zexact_kernel(ZExactArgs A)
{
    constexpr int VEC = ET::VEC;
    const int lane = threadIdx.x & (WAVE - 1);
    const int wv = W > 1 ? __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)) : 0;
    const int64_t t = blockIdx.x;
    const uint8_t flag = A.rowflag[t];
    if (flag != ROW_OK) {
        if (threadIdx.x == 0) A.zexact[t] = (flag == ROW_PADDING) ? 0.f : __uint_as_float(0x7fc00000u);
        return;
    }
    const char *rowq = (const char *)A.actor + (size_t)t * (size_t)A.stride * ET::ESZ;
    const char *rowp = (const char *)A.policy + (size_t)t * (size_t)A.stride * ET::ESZ;
    const int64_t V = A.V;
    const uint32_t nfull = (uint32_t)(V / VEC);
    const int tail = (int)(V - (int64_t)nfull * VEC);
    const uint32_t nchunks = nfull + (tail ? 1u : 0u);
    const float Aq = (float)(A.lse_q[t] * LOG2E_D);
    const float Ap = (float)((A.lse_p[t] + log((double)A.lambda)) * LOG2E_D);
    // Two-level sum per lane: a chunk is summed by itself, chunk sums go to `s`, and every
    // BLOCK_CHUNKS chunks `s` is folded into `hi`.  No single accumulator then takes more than a
    // few dozen additions, which matters for rows of tied logits: thousands of EQUAL terms added to
    // one fp32 accumulator round the same way every time and drift by 1e-5 of the sum and more.
    // (fp32 logits are held to 1e-5 and get the two levels; bf16 logits, held to 1e-3, keep two
    // plain accumulators.)
    constexpr bool TWO_LEVEL = ET::ESZ == 4;
    float s = 0.f, s1 = 0.f, hi = 0.f;
    int until_fold = BLOCK_CHUNKS;
    auto account = [&](const float (&fq)[VEC], const float (&fp)[VEC]) {
        float a = 0.f, b = 0.f;
#pragma unroll
        for (int j = 0; j < VEC; j += 2) {
            a += __builtin_amdgcn_exp2f(fminf(__builtin_fmaf(fq[j], LOG2E_F, -Aq), __builtin_fmaf(fp[j], LOG2E_F, -Ap)));
            b += __builtin_amdgcn_exp2f(fminf(__builtin_fmaf(fq[j + 1], LOG2E_F, -Aq), __builtin_fmaf(fp[j + 1], LOG2E_F, -Ap)));
        }
        if constexpr (TWO_LEVEL) {
            s += a + b;
            if (--until_fold == 0) { hi += s; s = 0.f; until_fold = BLOCK_CHUNKS; }
        } else {
            s += a; s1 += b;
        }
    };
    const uint32_t nit = nfull / WAVE;                      // iterations in which every lane has a full chunk
    const uint32_t it_lo = W > 1 ? (uint32_t)((uint64_t)nit * (uint32_t)wv / W) : 0u;
    const uint32_t it_hi = W > 1 ? (uint32_t)((uint64_t)nit * (uint32_t)(wv + 1) / W) : nit;
    if (it_hi > it_lo) {
        constexpr int D = 3;                                // non-temporal loads in flight per tensor and lane
        const uint32_t last = it_hi - 1;
        u32x4 wq[D], wp[D];
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const uint32_t n = (it_lo + (uint32_t)d < last ? it_lo + (uint32_t)d : last) * WAVE + lane;
            wq[d] = stream_load(as_global_vec(rowq) + n);
            wp[d] = stream_load(as_global_vec(rowp) + n);
        }
        for (uint32_t it = it_lo; it < it_hi; it += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                const u32x4 cq = wq[d], cp = wp[d];
                const uint32_t n = (it + D + d < last ? it + D + d : last) * WAVE + lane;
                wq[d] = stream_load(as_global_vec(rowq) + n);
                wp[d] = stream_load(as_global_vec(rowp) + n);
                if (d == 0 || it + d < it_hi) {
                    float fq[VEC], fp[VEC];
                    ET::unpack(cq, fq);
                    ET::unpack(cp, fp);
                    account(fq, fp);
                }
            }
        }
    }
    if (W == 1 || wv == W - 1) {                            // the remainder belongs to the last wave
        const uint32_t c = nit * WAVE + lane;
        if (c < nchunks) {
            float fq[VEC], fp[VEC];
            load_chunk<ET>(rowq, c, nfull, tail, fq);
            load_chunk<ET>(rowp, c, nfull, tail, fp);
            account(fq, fp);
        }
    }
    double Z = wave_sum((double)hi + (double)s + (double)s1);
    if constexpr (W > 1) {
        __shared__ double part[W];
        if (lane == 0) part[wv] = Z;
        __syncthreads();
        if (wv > 0) return;
        Z = 0.0;
#pragma unroll
        for (int w = 0; w < W; ++w) Z += part[w];
    }
    if (lane == 0) A.zexact[t] = (float)Z;
}

// =================================================================================================
// log softmax(l_t)[x_t] for one logit tensor: how log p_ref(a_t) of Alg. 1 (Phase 2, step 1) is read
// off a third tensor.  One wavefront per row, one sweep: per-lane exponent reference (moved only
// when a chunk maximum exceeds it by the margin) and sum, combined across the wave at the end.
// =================================================================================================
// W > 1: rows split over W wavefronts as in zexact_kernel.
template <class ET, int W = 1>
__global__ __launch_bounds__(64 * W) void token_logprob_kernel(LogprobArgs A)
{
    constexpr int VEC = ET::VEC;
    const int lane = threadIdx.x & (WAVE - 1);
    const int wv = W > 1 ? __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)) : 0;
    const int64_t t = blockIdx.x;
    const int x = A.ids[t];
    const int64_t V = A.V;
    if (x < 0 || x >= V) {
        if (threadIdx.x == 0) A.out[t] = x < 0 ? 0.f : __uint_as_float(0x7fc00000u);
        return;
    }
    const char *row = (const char *)A.logits + (size_t)t * (size_t)A.stride * ET::ESZ;
    const gvec_ptr v = as_global_vec(row);
    const uint32_t nfull = (uint32_t)(V / VEC);
    const int tail = (int)(V - (int64_t)nfull * VEC);
    const uint32_t nchunks = nfull + (tail ? 1u : 0u);
    const uint32_t nit = nfull / WAVE;
    constexpr bool TWO_LEVEL = ET::ESZ == 4;                        // (two-level sum as in zexact_kernel)
    float M2 = M2_UNSET, mthr = -2.0e38f, s = 0.f, hi = 0.f;
    int until_fold = BLOCK_CHUNKS;
    auto consume = [&](const float (&f)[VEC], bool valid) {
        const float m = max_of<VEC>(f);
        if (valid && m > mthr) {                                    // rare: move this lane's reference
            const float newM2 = m * LOG2E_F;
            const float rescale = __builtin_amdgcn_exp2f(M2 - newM2);
            s *= rescale;
            if constexpr (TWO_LEVEL) hi *= rescale;
            M2 = newM2;
            mthr = m + RESCALE_MARGIN2 / LOG2E_F;
        }
        if (valid) s += sum_exp2<VEC>(f, M2);
        if constexpr (TWO_LEVEL) {
            if (--until_fold == 0) { hi += s; s = 0.f; until_fold = BLOCK_CHUNKS; }
        }
    };
    const uint32_t it_lo = W > 1 ? (uint32_t)((uint64_t)nit * (uint32_t)wv / W) : 0u;
    const uint32_t it_hi = W > 1 ? (uint32_t)((uint64_t)nit * (uint32_t)(wv + 1) / W) : nit;
    if (it_hi > it_lo) {
        constexpr int D = 4;
        const uint32_t last = it_hi - 1;
        u32x4 w[D];
#pragma unroll
        for (int d = 0; d < D; ++d) w[d] = stream_load(v + ((it_lo + (uint32_t)d < last ? it_lo + (uint32_t)d : last) * WAVE + lane));
        for (uint32_t it = it_lo; it < it_hi; it += D) {
            u32x4 c[D];
#pragma unroll
            for (int d = 0; d < D; ++d) c[d] = w[d];
#pragma unroll
            for (int d = 0; d < D; ++d) w[d] = stream_load(v + ((it + D + d < last ? it + D + d : last) * WAVE + lane));
#pragma unroll
            for (int d = 0; d < D; ++d) {
                if (d == 0 || it + d < it_hi) {
                    float f[VEC];
                    ET::unpack(c[d], f);
                    consume(f, true);
                }
            }
        }
    }
    if (W == 1 || wv == W - 1) {                            // the remainder belongs to the last wave
        const uint32_t c = nit * WAVE + lane;
        if (c < nchunks) {
            float f[VEC];
            load_chunk<ET>(row, c, nfull, tail, f);
            consume(f, true);
        }
    }
    // combine the 64 (reference, sum) pairs: common reference = the largest, sums rescaled to it
    float Mw = uniform_f(wave_max(M2));
    double S = wave_sum(M2 == M2_UNSET ? 0.0 : ((double)hi + (double)s) * (double)__builtin_amdgcn_exp2f(M2 - Mw));
    if constexpr (W > 1) {                                  // the same combination once more, over the waves
        __shared__ double part_s[W];
        __shared__ float part_m[W];
        if (lane == 0) { part_s[wv] = S; part_m[wv] = Mw; }
        __syncthreads();
        if (wv > 0) return;
        float Mall = part_m[0];
#pragma unroll
        for (int w = 1; w < W; ++w) Mall = fmaxf(Mall, part_m[w]);
        S = 0.0;
#pragma unroll
        for (int w = 0; w < W; ++w) S += part_s[w] * (double)__builtin_amdgcn_exp2f(part_m[w] - Mall);
        Mw = Mall;
    }
    const double lse = ((double)Mw + log2_of_sum(S)) * LN2_D;
    const double lp = (double)ET::load1(row, x) - lse;
    if (lane == 0) A.out[t] = isfinite(lse) ? (float)lp : __uint_as_float(0x7fc00000u);
}

// =================================================================================================
// Scaling factor for an acceptance budget (Sec. 3.3, Theorem 2): per row the lambda with
// Z(lambda) = sum_v min(q_v, p_v / lambda) = abar.  With d_v = log2(p_v / q_v),
//   Z(2^x) = sum_{d_v > x} q_v + 2^-x sum_{d_v <= x} p_v
// is non-increasing in x, so the crossing is bracketed by histogram sweeps of the row pair.
//   * The first sweep only has to say roughly where the crossing is: it puts the q-mass of every
//     token into 512 bins of width 1/16 over [-16, 16), the first and the last bin also taking
//     what lies beyond, out to +-64 (one exponential and one 32-bit integer LDS atomic per token:
//     2^-31 units, rounded, two copies per bin against same-address collisions) and prices the
//     p-mass of a bin as its q-mass times 2^(bin centre).  Inside the resolved part that is off by
//     at most a factor 2^(+-1/32) on every token; the bracket for the next sweep is the bin of the
//     crossing found that way with a bin on either side.  Narrow bins matter twice: lanes of one
//     instruction seldom meet in a bin, and few tokens fall into the bracket of the next sweep.
//   * Every later sweep is exact: the mass outside the bracket [lo, hi) goes to per-lane sums (one
//     exponential per token: p below the bracket, q above it), the tokens inside it to 256 fine bins
//     (float64 LDS atomics; the bins belong to this wave alone and the hardware takes the lanes of an
//     instruction in a fixed order, so the sums are reproducible).  If the crossing is not inside
//     after all (a degenerate row), the bracket moves to that side and widens; if it is, the sweep
//     ends with the closed form lambda = B / (abar - A) on the crossing bin, A the q-mass above it
//     and B the p-mass at or below it, which is exact up to the tokens inside that one bin: their
//     mass times the bin width.  Where that product is not negligible against the budget (a heavy
//     token next to the crossing), one more sweep splits the bin again.
// On the rollout shape two sweeps are enough (fine bins 0.0007 wide in log2 lambda).
// abar at the keepable mass (abar = 1) returns the smallest ratio, the largest lambda that still
// accepts everything.
// =================================================================================================
constexpr int BUDGET_COARSE = 512, BUDGET_FINE = 256, BUDGET_MAX_SWEEPS = 6;
constexpr float BUDGET_RANGE = 64.f;                       // the search covers ratios in [2^-64, 2^64)
constexpr float BUDGET_CRANGE = 16.f;                      // the coarse bins resolve [2^-16, 2^16): the first and
                                                           // the last one also take what lies beyond, out to the range
constexpr float BUDGET_COARSE_W = 2.f * BUDGET_CRANGE / (float)BUDGET_COARSE;
constexpr int BUDGET_CPL = BUDGET_COARSE / WAVE, BUDGET_FPL = BUDGET_FINE / WAVE;    // bins per lane
constexpr double BUDGET_FIX31 = 2147483648.0;              // 2^31

// Sweep of one row pair with `account(fq, fp)` called on every chunk (padding of the ragged last
// chunk arrives as -inf in both rows: probability 0 under both models).
// part / parts: the wave takes the part-th of `parts` contiguous runs of the sweep iterations (rows
// split over the waves of a workgroup); the remainder belongs to the last part.
template <class ET, class F>
__device__ __forceinline__ void budget_for_each_chunk(const char *rowq, const char *rowp, int64_t V, F account,
                                                      int part = 0, int parts = 1)
{
    constexpr int VEC = ET::VEC;
    const int lane = threadIdx.x & (WAVE - 1);
    const uint32_t nfull = (uint32_t)(V / VEC);
    const int tail = (int)(V - (int64_t)nfull * VEC);
    const uint32_t nchunks = nfull + (tail ? 1u : 0u);
    const uint32_t nit_all = nfull / WAVE;              // iterations in which every lane has a full chunk
    const uint32_t it_lo = (uint32_t)((uint64_t)nit_all * (uint32_t)part / (uint32_t)parts);
    const uint32_t nit = (uint32_t)((uint64_t)nit_all * (uint32_t)(part + 1) / (uint32_t)parts);   // end of this run
    if (nit > it_lo) {
        constexpr int D = 3;                            // loads in flight per tensor and lane
        const uint32_t last = nit - 1;
        u32x4 wq[D], wp[D];
#pragma unroll
        for (int d2 = 0; d2 < D; ++d2) {
            const uint32_t n = (it_lo + (uint32_t)d2 < last ? it_lo + (uint32_t)d2 : last) * WAVE + lane;
            wq[d2] = stream_load(as_global_vec(rowq) + n);
            wp[d2] = stream_load(as_global_vec(rowp) + n);
        }
        for (uint32_t it = it_lo; it < nit; it += D) {
#pragma unroll
            for (int d2 = 0; d2 < D; ++d2) {
                const u32x4 cq = wq[d2], cp = wp[d2];
                const uint32_t n = (it + D + d2 < last ? it + D + d2 : last) * WAVE + lane;
                wq[d2] = stream_load(as_global_vec(rowq) + n);
                wp[d2] = stream_load(as_global_vec(rowp) + n);
                if (d2 == 0 || it + d2 < nit) {
                    float fq[VEC], fp[VEC];
                    ET::unpack(cq, fq);
                    ET::unpack(cp, fp);
                    account(fq, fp);
                }
            }
        }
    }
    const uint32_t c = nit_all * WAVE + lane;
    if (part == parts - 1 && c < nchunks) {
        float fq[VEC], fp[VEC];
        load_chunk<ET>(rowq, c, nfull, tail, fq);
        load_chunk<ET>(rowp, c, nfull, tail, fp);
        account(fq, fp);
    }
}

// First sweep: q-mass of every token into the coarse bins `hist` ([1 + bin][2 copies], 2^-31 units).
// A ratio beyond the resolved part goes to the first or the last bin; one below the whole range (a
// token the target cannot emit has d = -inf) keeps none of its q-mass at any lambda of the range and
// goes to entry 0, which nobody reads.
template <class ET>
__device__ __forceinline__ void budget_coarse_sweep(const char *rowq, const char *rowp, int64_t V, float Aq, float Ap,
                                                    uint32_t *hist, int part = 0, int parts = 1)
{
    constexpr int VEC = ET::VEC;
    const int lane = threadIdx.x & (WAVE - 1);
    // (rows split over `parts` waves: they share the bins, whose integer sums do not depend on order)
    for (int e = threadIdx.x; e < 2 * (BUDGET_COARSE + 1); e += WAVE * parts) hist[e] = 0u;
    if (parts > 1) __syncthreads(); else lds_sync();
    const float dA = Ap - Aq;
    const float inv_w = 1.f / BUDGET_COARSE_W;
    const float off = BUDGET_CRANGE * inv_w + 1.f;
    const uint32_t copy = (uint32_t)lane & 1u;
    budget_for_each_chunk<ET>(rowq, rowp, V, [&](const float (&fq)[VEC], const float (&fp)[VEC]) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
            const float q = __builtin_amdgcn_exp2f(__builtin_fmaf(fq[j], LOG2E_F, -Aq));
            const float d = __builtin_fmaf(fp[j] - fq[j], LOG2E_F, -dA);          // log2(p / q); NaN when both are 0
            int b = (int)__builtin_fmaf(d, inv_w, off);                           // 1 + bin (saturates; NaN gives 0: q is 0 then)
            b = b < 1 ? (d >= -BUDGET_RANGE ? 1 : 0) : (b < BUDGET_COARSE ? b : BUDGET_COARSE);
            atomicAdd(&hist[((uint32_t)b << 1) | copy], (uint32_t)__builtin_fmaf(q, (float)BUDGET_FIX31, 0.5f));
        }
    }, part, parts);
    if (parts > 1) __syncthreads(); else lds_sync();
}

// The smallest finite log2 ratio of a row pair (one more sweep, only for a budget at the keepable
// mass, where every lambda up to the smallest ratio accepts everything).
template <class ET>
__device__ __forceinline__ float budget_min_ratio(const char *rowq, const char *rowp, int64_t V, float Aq, float Ap,
                                                  int part = 0, int parts = 1)
{
    constexpr int VEC = ET::VEC;
    const float dA = Ap - Aq;
    float dmin = __uint_as_float(0x7f800000u);
    budget_for_each_chunk<ET>(rowq, rowp, V, [&](const float (&fq)[VEC], const float (&fp)[VEC]) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
            const float d = __builtin_fmaf(fp[j] - fq[j], LOG2E_F, -dA);
            dmin = (d > -3.0e38f && d < 3.0e38f) ? fminf(dmin, d) : dmin;
        }
    }, part, parts);
    return -uniform_f(wave_max(-dmin));
}

// A later sweep for the bracket [lo, hi): the exact mass outside it (qa above, pb below, per-lane
// sums) and the q- and p-mass of the tokens inside it in the fine bins hq / hp (BUDGET_FINE + 1
// entries each: a product that rounds up to the bin count lands in the extra one, which is folded
// into the last bin).
template <class ET>
__device__ __forceinline__ void budget_fine_sweep(const char *rowq, const char *rowp, int64_t V, float Aq, float Ap,
                                                  float lo, float hi, double *hq, double *hp, double &qa, double &pb,
                                                  int part = 0, int parts = 1)
{
    // (rows split over waves: every wave has bins of its own, hq / hp, and returns its share of qa, pb)
    constexpr int VEC = ET::VEC;
    const int lane = threadIdx.x & (WAVE - 1);
    for (int e = lane; e < BUDGET_FINE + 1; e += WAVE) { hq[e] = 0.0; hp[e] = 0.0; }
    lds_sync();
    const float width = hi - lo;
    const float inv_w = (float)BUDGET_FINE / width;
    const float Apl = Ap + lo;
    const uint32_t width_bits = __float_as_uint(width);
    const float scale_below = __builtin_amdgcn_exp2f(lo);
    double not_below = 0.0, below_p = 0.0;
    budget_for_each_chunk<ET>(rowq, rowp, V, [&](const float (&fq)[VEC], const float (&fp)[VEC]) {
        float nbf = 0.f, pbf = 0.f;
        float dl[VEC], e[VEC];
        bool any = false;
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
            // below the bracket a token pays p / lambda at every lambda of it, from the bracket up it
            // keeps q: 2^min(aq, ap - lo) is q there and p 2^-lo below (NaN, both probabilities 0,
            // counts as not below: q = 0)
            const float aq = __builtin_fmaf(fq[j], LOG2E_F, -Aq), apl = __builtin_fmaf(fp[j], LOG2E_F, -Apl);
            dl[j] = apl - aq;                                                      // d - lo
            e[j] = __builtin_amdgcn_exp2f(fminf(aq, apl));
            const bool below = dl[j] < 0.f;
            pbf += below ? e[j] : 0.f;
            nbf += below ? 0.f : e[j];
            any |= __float_as_uint(dl[j]) < width_bits;                           // 0 <= d - lo < width
        }
        not_below += (double)nbf;
        below_p += (double)pbf;
        if (__ballot(any)) {
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                if (__float_as_uint(dl[j]) < width_bits) {
                    const int b = (int)(dl[j] * inv_w);                            // <= BUDGET_FINE
                    // (float64 bins: thousands of equal terms, a row of tied logits, added to one
                    // fp32 bin round the same way every time and drift by 1e-4 of the sum)
                    atomicAdd(&hq[b], (double)e[j]);
                    atomicAdd(&hp[b], (double)__builtin_amdgcn_exp2f(__builtin_fmaf(fp[j], LOG2E_F, -Ap)));
                }
            }
        }
    }, part, parts);
    lds_sync();
    if (lane == 0) { hq[BUDGET_FINE - 1] += hq[BUDGET_FINE]; hp[BUDGET_FINE - 1] += hp[BUDGET_FINE]; }
    lds_sync();
    double inq = 0.0;
    for (int e2 = lane; e2 < BUDGET_FINE; e2 += WAVE) inq += hq[e2];
    pb = below_p * (double)scale_below;
    qa = wave_sum(not_below) - wave_sum(inq);          // (wave total, on every lane)
    qa = qa > 0.0 ? qa : 0.0;
}

// Exclusive sums over the lanes of a wave through LDS: for lane l the sum of `q` over the lanes
// after it and of `p` over the lanes before it.  sq_ / sp_: 64 doubles each.
__device__ __forceinline__ void budget_lane_sums(double q, double p, double *sq_, double *sp_, double &q_after,
                                                 double &p_before, double &q_all, double &p_all)
{
    const int lane = threadIdx.x;
    lds_sync();
    sq_[lane] = q; sp_[lane] = p;
    lds_sync();
    q_after = 0.0; p_before = 0.0; q_all = 0.0; p_all = 0.0;
#pragma unroll 4
    for (int j = 0; j < WAVE; ++j) {
        const double qj = sq_[j], pj = sp_[j];
        q_after += j > lane ? qj : 0.0;
        p_before += j < lane ? pj : 0.0;
        q_all += qj;
        p_all += pj;
    }
    lds_sync();
}

// What a sweep found.  `goal` is the value Z must reach (abar, or abar times the number of rows when
// the masses are sums over a batch).
struct BudgetFound {
    int where;              // -1: crossing below lo, 0: inside (bin_lo .. bin_lo + bin_w), +1: above hi
    float bin_lo, bin_w;
    double lambda;          // closed form on the crossing bin (where == 0) or beyond the bracket (where == +1)
    double bin_q;           // q-mass of the tokens inside the crossing bin
};

// Lane l brings the masses of NB consecutive bins (bins l NB .. l NB + NB - 1 of width w from lo).
template <int NB>
__device__ __forceinline__ BudgetFound budget_scan(double goal, double A_above, double B_below, const double (&q)[NB],
                                                   const double (&p)[NB], float lo, float w, double *sq_, double *sp_)
{
    const int lane = threadIdx.x;
    double tq = 0.0, tp = 0.0;
#pragma unroll
    for (int j = 0; j < NB; ++j) { tq += q[j]; tp += p[j]; }
    double q_after, p_before, q_all, p_all;
    budget_lane_sums(tq, tp, sq_, sp_, q_after, p_before, q_all, p_all);
    // Z at the lower edge of every bin: the q-mass from this bin up, the p-mass of the bins below it
    double qsuf[NB], ppre[NB];
    int n_true = 0;
    {
        double qs = q_after + tq, pp = p_before;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            qsuf[j] = qs; ppre[j] = pp;
            const float edge = lo + w * (float)(lane * NB + j);
            const double z = A_above + qs + (B_below + pp) * (double)__builtin_amdgcn_exp2f(-edge);
            n_true += __popcll(__ballot(z >= goal));
            qs -= q[j];
            pp += p[j];
        }
    }
    BudgetFound r;
    const float hi = lo + w * (float)(WAVE * NB);
    const double z_hi = A_above + (B_below + p_all) * (double)__builtin_amdgcn_exp2f(-hi);
    r.bin_lo = lo; r.bin_w = w; r.bin_q = 0.0; r.lambda = 0.0;
    if (n_true == 0) { r.where = -1; return r; }
    if (z_hi >= goal) {
        r.where = 1;
        r.lambda = (B_below + p_all) / (goal - A_above);         // every ratio up to hi is below lambda
        return r;
    }
    const int g = n_true - 1;                                    // Z(edge g) >= goal > Z(edge g + 1)
    const int owner = g / NB, jj = g - owner * NB;
    double a_end = 0.0, b_end = 0.0, bq = 0.0;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        if (j == jj) { a_end = A_above + qsuf[j] - q[j]; b_end = B_below + ppre[j] + p[j]; bq = q[j]; }
    }
    a_end = lane_value_d(a_end, owner); b_end = lane_value_d(b_end, owner); bq = lane_value_d(bq, owner);
    r.where = 0;
    r.bin_lo = lo + w * (float)g;
    r.bin_q = bq;
    double lambda = b_end / (goal - a_end);
    const double l_lo = (double)__builtin_amdgcn_exp2f(r.bin_lo), l_hi = (double)__builtin_amdgcn_exp2f(r.bin_lo + w);
    r.lambda = lambda < l_lo ? l_lo : (lambda > l_hi ? l_hi : lambda);
    return r;
}

// After the first sweep: Z(lambda -> 0) is all the mass that can be kept at all.  A budget at (or
// within rounding of) it is met by every lambda up to the smallest ratio, which is the answer; Z is
// flat there, so a bracket search would be deciding on rounding noise: BUDGET_KEEP_ALL.  Otherwise
// the bracket for the exact sweeps: the coarse bin of the approximate crossing and one bin on
// either side (BUDGET_SEARCH).
enum { BUDGET_SEARCH = 0, BUDGET_DONE = 1, BUDGET_KEEP_ALL = 2 };
__device__ __forceinline__ int budget_after_coarse(double goal, const double (&q)[BUDGET_CPL], double *sq_, double *sp_,
                                                   float &lo, float &hi)
{
    const int lane = threadIdx.x;
    double p[BUDGET_CPL];
#pragma unroll
    for (int j = 0; j < BUDGET_CPL; ++j) {
        const float mid = -BUDGET_CRANGE + BUDGET_COARSE_W * ((float)(lane * BUDGET_CPL + j) + 0.5f);
        p[j] = q[j] * (double)__builtin_amdgcn_exp2f(mid);
    }
    double tq = 0.0;
#pragma unroll
    for (int j = 0; j < BUDGET_CPL; ++j) tq += q[j];
    const double zmax = wave_sum(tq);
    if (goal >= zmax * (1.0 - 1e-6)) return BUDGET_KEEP_ALL;
    const BudgetFound f = budget_scan<BUDGET_CPL>(goal, 0.0, 0.0, q, p, -BUDGET_CRANGE, BUDGET_COARSE_W, sq_, sp_);
    float centre = f.bin_lo;                                      // where == 0
    if (f.where < 0) centre = -BUDGET_CRANGE;
    if (f.where > 0) centre = BUDGET_CRANGE - BUDGET_COARSE_W;
    lo = centre - BUDGET_COARSE_W;
    hi = centre + 2.f * BUDGET_COARSE_W;
    if (lo < -BUDGET_CRANGE) lo = -BUDGET_RANGE;                  // the first and the last bin reach out to the range
    if (hi > BUDGET_CRANGE) hi = BUDGET_RANGE;
    return BUDGET_SEARCH;
}

// After an exact sweep of [lo, hi): BUDGET_DONE (lambda set), BUDGET_KEEP_ALL (the crossing lies
// below every ratio of the range), or BUDGET_SEARCH with the next bracket.
// eps: the error of Z that is negligible (absolute); last: no further sweep is allowed.
__device__ __forceinline__ int budget_after_fine(const BudgetFound &f, double eps, bool last, float &lo, float &hi,
                                                 double &lambda)
{
    const float width = hi - lo;
    if (f.where == 0) {
        // tokens inside the crossing bin are priced as if they lay below lambda: off by at most
        // their q-mass times (2^bin width - 1)
        const double err = f.bin_q * ((double)__builtin_amdgcn_exp2f(f.bin_w) - 1.0);
        lambda = f.lambda;
        if (err <= eps || f.bin_w < 1e-6f || last) return BUDGET_DONE;
        lo = f.bin_lo;
        hi = f.bin_lo + f.bin_w;
        return BUDGET_SEARCH;
    }
    if (f.where > 0) {
        lambda = f.lambda;
        if (hi >= BUDGET_RANGE || last) return BUDGET_DONE;       // beyond 2^64: every ratio is below lambda
        lo = hi;
        hi = fminf(hi + 8.f * width, BUDGET_RANGE);
        return BUDGET_SEARCH;
    }
    if (lo <= -BUDGET_RANGE) return BUDGET_KEEP_ALL;
    lambda = (double)__builtin_amdgcn_exp2f(lo);
    if (last) return BUDGET_DONE;
    hi = lo;
    lo = fmaxf(lo - 8.f * width, -BUDGET_RANGE);
    return BUDGET_SEARCH;
}

// W > 1: a row goes to W wavefronts of one workgroup (small batches, as in the row stage).  Every
// wave sweeps its run of the row; the integer bins of the first sweep are shared, the float64 bins
// of the exact sweeps are per wave and added up in wave order, and wave 0 alone runs the scans and
// tells the others through LDS how the search goes on.
template <class ET, int W = 1>
__global__ __launch_bounds__(64 * W, W == 1 ? 6 : 4) void budget_kernel(BudgetArgs A)
{
    // coarse bins (2 x 513 32-bit words); for W = 1 later the fine q / p bins (2 x 257 doubles)
    __shared__ __attribute__((aligned(8))) uint32_t hist[4 * (BUDGET_FINE + 1) > 2 * (BUDGET_COARSE + 1) ? 4 * (BUDGET_FINE + 1) : 2 * (BUDGET_COARSE + 1)];
    __shared__ double sq_[WAVE], sp_[WAVE];
    __shared__ double fine[W > 1 ? W : 1][W > 1 ? 2 * (BUDGET_FINE + 1) : 1];   // split rows: the fine bins of every wave
    __shared__ double s_out[W > 1 ? W : 1][2];                                  // ... and its mass outside the bracket
    __shared__ float s_min[W > 1 ? W : 1];
    __shared__ float s_lo, s_hi;
    __shared__ int s_state;
    const int lane = threadIdx.x & (WAVE - 1);
    const int wv = W > 1 ? __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)) : 0;
    double *const hq = W > 1 ? fine[wv] : (double *)hist, *const hp = hq + BUDGET_FINE + 1;
    const int64_t t = blockIdx.x;
    const float NaN = __uint_as_float(0x7fc00000u);
    const uint8_t flag = A.rowflag[t];
    const float abar_f = A.row_target ? A.row_target[t] : A.target;
    if (flag != ROW_OK || !(abar_f > 0.f) || abar_f > 1.f) {
        if (threadIdx.x == 0) A.lambda_out[t] = flag == ROW_PADDING ? 0.f : NaN;
        return;
    }
    const char *rowq = (const char *)A.actor + (size_t)t * (size_t)A.stride * ET::ESZ;
    const char *rowp = (const char *)A.policy + (size_t)t * (size_t)A.stride * ET::ESZ;
    const float Aq = (float)(A.lse_q[t] * LOG2E_D);
    const float Ap = (float)(A.lse_p[t] * LOG2E_D);
    const double goal = (double)abar_f;
    const double eps = goal * (double)A.eps_rel;

    budget_coarse_sweep<ET>(rowq, rowp, A.V, Aq, Ap, hist, wv, W);
    float lo = -BUDGET_RANGE, hi = BUDGET_RANGE;
    double lambda = 0.0;
    int state = BUDGET_SEARCH;
    if (wv == 0) {
        double cq[BUDGET_CPL];
#pragma unroll
        for (int j = 0; j < BUDGET_CPL; ++j) {
            const int b = 1 + lane * BUDGET_CPL + j;              // (entry 0 holds what no lambda keeps)
            cq[j] = ((double)hist[2 * b] + (double)hist[2 * b + 1]) / BUDGET_FIX31;
        }
        state = budget_after_coarse(goal, cq, sq_, sp_, lo, hi);
        if (W > 1 && lane == 0) { s_state = state; s_lo = lo; s_hi = hi; }
    }
    if constexpr (W > 1) {
        __syncthreads();
        state = s_state; lo = s_lo; hi = s_hi;
    }
    for (int sweep = 1; sweep < BUDGET_MAX_SWEEPS && state == BUDGET_SEARCH; ++sweep) {
        double qa, pb;
        budget_fine_sweep<ET>(rowq, rowp, A.V, Aq, Ap, lo, hi, hq, hp, qa, pb, wv, W);
        double A_above = qa, B_below = wave_sum(pb);
        if constexpr (W > 1) {
            if (lane == 0) { s_out[wv][0] = A_above; s_out[wv][1] = B_below; }
            __syncthreads();                                  // every wave's bins and outside masses are complete
        }
        if (wv == 0) {
            double fq[BUDGET_FPL], fp[BUDGET_FPL];
#pragma unroll
            for (int j = 0; j < BUDGET_FPL; ++j) { fq[j] = hq[lane * BUDGET_FPL + j]; fp[j] = hp[lane * BUDGET_FPL + j]; }
            if constexpr (W > 1) {
#pragma unroll
                for (int w = 1; w < W; ++w) {                 // in wave order: the same sums on every run
                    const double *oq = fine[w], *op = oq + BUDGET_FINE + 1;
#pragma unroll
                    for (int j = 0; j < BUDGET_FPL; ++j) { fq[j] += oq[lane * BUDGET_FPL + j]; fp[j] += op[lane * BUDGET_FPL + j]; }
                    A_above += s_out[w][0]; B_below += s_out[w][1];
                }
            }
            const BudgetFound f = budget_scan<BUDGET_FPL>(goal, A_above, B_below, fq, fp, lo, (hi - lo) / (float)BUDGET_FINE, sq_, sp_);
            state = budget_after_fine(f, eps, sweep == BUDGET_MAX_SWEEPS - 1, lo, hi, lambda);
            if (W > 1 && lane == 0) { s_state = state; s_lo = lo; s_hi = hi; }
        }
        if constexpr (W > 1) {
            __syncthreads();                                  // (also: nobody reads the bins any more)
            state = s_state; lo = s_lo; hi = s_hi;
        }
    }
    if (state == BUDGET_KEEP_ALL) {
        float dmin = budget_min_ratio<ET>(rowq, rowp, A.V, Aq, Ap, wv, W);
        if constexpr (W > 1) {
            if (lane == 0) s_min[wv] = dmin;
            __syncthreads();
#pragma unroll
            for (int w = 0; w < W; ++w) dmin = fminf(dmin, s_min[w]);
        }
        lambda = (double)__builtin_amdgcn_exp2f(dmin);
    }
    if (threadIdx.x == 0) A.lambda_out[t] = (float)lambda;
}

// The same search for one lambda of a whole batch, mean_t Z_t(lambda) = abar: the bins of all rows are
// summed in device memory (64-bit fixed point, so the sums are order-independent), a one-wave kernel
// between the sweeps finds the next bracket, and nothing goes through the host.
__global__ void budget_batch_init_kernel(BudgetBatchState *S)
{
    const int lane = threadIdx.x;
    for (int e = lane; e < BUDGET_COARSE; e += WAVE) S->coarse[e] = 0;
    for (int e = lane; e < BUDGET_FINE; e += WAVE) { S->fq[e] = 0; S->fp[e] = 0; }
    if (lane == 0) {
        S->lo = -BUDGET_RANGE; S->hi = BUDGET_RANGE; S->done = 0; S->lambda = 0.0;
        S->n_rows = 0; S->above = 0; S->below = 0; S->dmin_ord = 0x7fffffff;
    }
}

// float <-> int with the same order (for an atomic minimum over floats)
__device__ __forceinline__ int float_order_int(float f)
{
    const int i = __float_as_int(f);
    return i ^ ((i >> 31) & 0x7fffffff);
}

// (W > 1 in the three sweep kernels below: rows split over W waves as in budget_kernel; the sums in
// device memory are integers, so every wave adds its own share and nothing has to be merged.)
template <class ET, int W = 1>
__global__ __launch_bounds__(64 * W, W == 1 ? 6 : 4) void budget_batch_coarse_kernel(BudgetArgs A, BudgetBatchState *S)
{
    __shared__ uint32_t hist[2 * (BUDGET_COARSE + 1)];
    const int wv = W > 1 ? __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)) : 0;
    const int64_t t = blockIdx.x;
    if (A.rowflag[t] != ROW_OK) return;
    const char *rowq = (const char *)A.actor + (size_t)t * (size_t)A.stride * ET::ESZ;
    const char *rowp = (const char *)A.policy + (size_t)t * (size_t)A.stride * ET::ESZ;
    budget_coarse_sweep<ET>(rowq, rowp, A.V, (float)(A.lse_q[t] * LOG2E_D), (float)(A.lse_p[t] * LOG2E_D), hist, wv, W);
    for (int b = threadIdx.x; b < BUDGET_COARSE; b += WAVE * W) {
        const unsigned long long u = (unsigned long long)hist[2 * (b + 1)] + (unsigned long long)hist[2 * (b + 1) + 1];
        if (u) atomicAdd(&S->coarse[b], u);                   // 2^-31 units: integer sums, any order
    }
    if (threadIdx.x == 0) atomicAdd(&S->n_rows, 1ull);
}

__global__ __launch_bounds__(64) void budget_batch_after_coarse_kernel(BudgetBatchState *S, float target, float *out_lambda)
{
    __shared__ double sq_[WAVE], sp_[WAVE];
    const int lane = threadIdx.x;
    const unsigned long long n = S->n_rows;
    double cq[BUDGET_CPL];
#pragma unroll
    for (int j = 0; j < BUDGET_CPL; ++j) cq[j] = (double)S->coarse[lane * BUDGET_CPL + j] / BUDGET_FIX31;
    float lo = -BUDGET_RANGE, hi = BUDGET_RANGE;
    int state = BUDGET_DONE;
    if (n > 0) state = budget_after_coarse((double)target * (double)n, cq, sq_, sp_, lo, hi);
    if (lane == 0) {
        S->lo = lo; S->hi = hi;
        S->done = state;
        if (n == 0) {                                       // no valid row
            S->lambda = __longlong_as_double(0x7ff8000000000000LL);
            *out_lambda = __uint_as_float(0x7fc00000u);
        }
    }
}

// Only when the search ended with "every lambda up to the smallest ratio": that ratio, over all rows.
template <class ET, int W = 1>
__global__ __launch_bounds__(64 * W, W == 1 ? 6 : 4) void budget_batch_min_ratio_kernel(BudgetArgs A, BudgetBatchState *S)
{
    const int wv = W > 1 ? __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)) : 0;
    const int64_t t = blockIdx.x;
    if (S->done != BUDGET_KEEP_ALL || A.rowflag[t] != ROW_OK) return;
    const char *rowq = (const char *)A.actor + (size_t)t * (size_t)A.stride * ET::ESZ;
    const char *rowp = (const char *)A.policy + (size_t)t * (size_t)A.stride * ET::ESZ;
    const float dmin = budget_min_ratio<ET>(rowq, rowp, A.V, (float)(A.lse_q[t] * LOG2E_D), (float)(A.lse_p[t] * LOG2E_D), wv, W);
    if ((threadIdx.x & (WAVE - 1)) == 0) atomicMin(&S->dmin_ord, float_order_int(dmin));
}

__global__ void budget_batch_min_ratio_finish_kernel(BudgetBatchState *S, float *out_lambda)
{
    if (threadIdx.x != 0 || S->done != BUDGET_KEEP_ALL) return;
    const int o = S->dmin_ord;
    const float dmin = __int_as_float(o ^ ((o >> 31) & 0x7fffffff));
    S->lambda = (double)__builtin_amdgcn_exp2f(dmin);
    S->done = BUDGET_DONE;
    *out_lambda = (float)S->lambda;
}

template <class ET, int W = 1>
__global__ __launch_bounds__(64 * W, W == 1 ? 6 : 4) void budget_batch_fine_kernel(BudgetArgs A, BudgetBatchState *S)
{
    __shared__ double bins[W][2 * (BUDGET_FINE + 1)];        // every wave its own
    const int lane = threadIdx.x & (WAVE - 1);
    const int wv = W > 1 ? __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)) : 0;
    double *const hq = bins[wv], *const hp = hq + BUDGET_FINE + 1;
    const int64_t t = blockIdx.x;
    if (S->done != BUDGET_SEARCH || A.rowflag[t] != ROW_OK) return;
    const char *rowq = (const char *)A.actor + (size_t)t * (size_t)A.stride * ET::ESZ;
    const char *rowp = (const char *)A.policy + (size_t)t * (size_t)A.stride * ET::ESZ;
    double qa, pb;
    budget_fine_sweep<ET>(rowq, rowp, A.V, (float)(A.lse_q[t] * LOG2E_D), (float)(A.lse_p[t] * LOG2E_D), S->lo, S->hi, hq, hp, qa, pb, wv, W);
    const double A_above = qa, B_below = wave_sum(pb);
    for (int b = lane; b < BUDGET_FINE; b += WAVE) {
        const unsigned long long uq = (unsigned long long)(hq[b] * 4294967296.0), up = (unsigned long long)(hp[b] * 4294967296.0);
        if (uq) atomicAdd(&S->fq[b], uq);                    // 2^-32 units: integer sums, any order
        if (up) atomicAdd(&S->fp[b], up);
    }
    if (lane == 0) {
        atomicAdd(&S->above, (unsigned long long)(A_above * 4294967296.0));
        atomicAdd(&S->below, (unsigned long long)(B_below * 4294967296.0));
    }
}

__global__ __launch_bounds__(64) void budget_batch_after_fine_kernel(BudgetBatchState *S, float target, float eps_rel, int last,
                                                                     float *out_lambda)
{
    __shared__ double sq_[WAVE], sp_[WAVE];
    const int lane = threadIdx.x;
    if (S->done != BUDGET_SEARCH) return;
    const double unit = 1.0 / 4294967296.0;
    const double goal = (double)target * (double)S->n_rows;
    double fq[BUDGET_FPL], fp[BUDGET_FPL];
#pragma unroll
    for (int j = 0; j < BUDGET_FPL; ++j) {
        fq[j] = (double)S->fq[lane * BUDGET_FPL + j] * unit;
        fp[j] = (double)S->fp[lane * BUDGET_FPL + j] * unit;
    }
    float lo = S->lo, hi = S->hi;
    const BudgetFound f = budget_scan<BUDGET_FPL>(goal, (double)S->above * unit, (double)S->below * unit, fq, fp, lo,
                                                  (hi - lo) / (float)BUDGET_FINE, sq_, sp_);
    double lambda = 0.0;
    const int state = budget_after_fine(f, goal * (double)eps_rel, last != 0, lo, hi, lambda);
    lds_sync();
    for (int e = lane; e < BUDGET_FINE; e += WAVE) { S->fq[e] = 0; S->fp[e] = 0; }     // the next sweep starts from empty bins
    if (lane == 0) {
        S->above = 0; S->below = 0;
        S->lo = lo; S->hi = hi;
        S->done = state;
        if (state == BUDGET_DONE) { S->lambda = lambda; *out_lambda = (float)lambda; }
    }
}

// =================================================================================================
// Gradient of the distillation term KL(SG(p) || q) of Sec. 4.2 (3) with respect to the actor
// logits: g_t[v] = w_t (q_t(v) - p_t(v)), q = 2^(lq log2e - LSEq log2e), p likewise.  A second
// streaming pass: reads both logit rows once, writes one row.  A workgroup of 256 threads covers
// GRAD_CHUNKS 16-byte pieces per thread of one row.  One piece per thread measured fastest on the
// rollout shape (6.4 TB/s against 6.2 with two and 5.6 with four): with eight waves per SIMD
// resident, few requests per wave keep the accesses in flight within a narrow address window.
// =================================================================================================
constexpr int GRAD_THREADS = 256;
constexpr int GRAD_CHUNKS = 1;

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)     // round to nearest even
{
    const bf16x2_t r = __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t);
    return __builtin_bit_cast(uint32_t, r);
}
struct Bf16Out {
    static constexpr int ESZ = 2;
    static __device__ __forceinline__ void store1(char *row, int64_t i, float v)
    {
        ((uint16_t *)row)[i] = (uint16_t)pack_bf16x2(v, 0.f);
    }
    template <int VEC> static __device__ __forceinline__ void store(char *row, uint32_t c, const float (&g)[VEC])
    {
        uint32_t w[VEC / 2];
#pragma unroll
        for (int j = 0; j < VEC / 2; ++j) w[j] = pack_bf16x2(g[2 * j], g[2 * j + 1]);
        // written once, not read again by this pass: non-temporal stores
        if constexpr (VEC == 8) __builtin_nontemporal_store(u32x4{w[0], w[1], w[2], w[3]}, (u32x4 *)row + c);
        else __builtin_nontemporal_store(((uint64_t)w[1] << 32) | w[0], (uint64_t *)row + c);
    }
};
struct F32Out {
    static constexpr int ESZ = 4;
    static __device__ __forceinline__ void store1(char *row, int64_t i, float v) { ((float *)row)[i] = v; }
    template <int VEC> static __device__ __forceinline__ void store(char *row, uint32_t c, const float (&g)[VEC])
    {
#pragma unroll
        for (int j = 0; j < VEC / 4; ++j)
            __builtin_nontemporal_store(u32x4{__float_as_uint(g[4 * j]), __float_as_uint(g[4 * j + 1]),
                                              __float_as_uint(g[4 * j + 2]), __float_as_uint(g[4 * j + 3])},
                                        (u32x4 *)row + ((size_t)c * (VEC / 4) + j));
    }
};

// What one thread reads per request.  By default a 16-byte piece of each row.  For bf16 logits with
// an fp32 gradient an 8-byte piece (4 elements), two requests per thread: its result is 16 bytes, so
// every load and store instruction of a wave still covers one contiguous span (a 16-byte piece would
// make each lane write 32 bytes in two stores with a stride between lanes).
template <class ET> struct GradPiece {
    using Raw = u32x4;
    static constexpr int VEC = ET::VEC, CHUNKS = GRAD_CHUNKS;
    static __device__ __forceinline__ Raw load(const char *row, uint32_t c) { return stream_load(as_global_vec(row) + c); }
    static __device__ __forceinline__ void unpack(const Raw w, float (&f)[VEC]) { ET::unpack(w, f); }
};
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
struct Bf16HalfPiece {
    using Raw = u32x2;
    static constexpr int VEC = 4, CHUNKS = 2;
    static __device__ __forceinline__ Raw load(const char *row, uint32_t c)
    {
        return __builtin_nontemporal_load((const __attribute__((address_space(1))) u32x2 *)(uintptr_t)row + c);
    }
    static __device__ __forceinline__ void unpack(const Raw w, float (&f)[VEC])
    {
        f[0] = __uint_as_float(w.x << 16); f[1] = __uint_as_float(w.x & 0xffff0000u);
        f[2] = __uint_as_float(w.y << 16); f[3] = __uint_as_float(w.y & 0xffff0000u);
    }
};

template <class ET, class OT, class PC = GradPiece<ET>>
__global__ __launch_bounds__(GRAD_THREADS) void distill_grad_kernel(GradArgs A)
{
    constexpr int VEC = PC::VEC;
    constexpr int CHUNKS = PC::CHUNKS;
    // one-dimensional launch, segments of a row adjacent: consecutive workgroups stream consecutive memory
    const int64_t t = blockIdx.x / A.segs;
    const uint32_t seg = blockIdx.x - (uint32_t)t * A.segs;
    const int64_t V = A.V;
    const uint32_t nfull = (uint32_t)(V / VEC);
    const int tail = (int)(V - (int64_t)nfull * VEC);
    const char *rowq = (const char *)A.actor + (size_t)t * (size_t)A.stride * ET::ESZ;
    const char *rowp = (const char *)A.policy + (size_t)t * (size_t)A.stride * ET::ESZ;
    char *rowg = (char *)A.grad + (size_t)t * (size_t)A.grad_stride * OT::ESZ;
    // This workgroup covers chunks [seg_begin, seg_end) of the row in batches of CHUNKS pieces
    // per thread.  A batch is loaded, computed and stored with nothing carried to the next one:
    // short-lived workgroups with few registers, many of them resident, stream faster here than a
    // software pipeline inside a longer-lived one (the launcher gives at most one batch per
    // workgroup unless the grid would grow past its limit).  The loads go out before the row constants are read.
    const uint32_t seg_begin = seg * A.seg_chunks;
    const uint32_t seg_end = seg_begin + A.seg_chunks < nfull ? seg_begin + A.seg_chunks : nfull;
    typename PC::Raw rq[CHUNKS], rp[CHUNKS];
    auto request = [&](uint32_t base) {
#pragma unroll
        for (int u = 0; u < CHUNKS; ++u) {
            uint32_t c = base + u * GRAD_THREADS + threadIdx.x;
            c = c < seg_end ? c : seg_end - 1;           // clamp: a harmless repeat, never stored
            rq[u] = PC::load(rowq, c);
            rp[u] = PC::load(rowp, c);
        }
    };
    if (seg_begin < seg_end) request(seg_begin);
    const bool live = A.rowflag[t] == ROW_OK;
    const float w = live ? A.scale * (A.row_scale ? A.row_scale[t] : 1.f) : 0.f;
    const float Aq = live ? (float)(A.lse_q[t] * LOG2E_D) : 0.f;
    const float Ap = live ? (float)(A.lse_p[t] * LOG2E_D) : 0.f;
    auto grad_of = [&](float lq, float lp) {
        const float q = __builtin_amdgcn_exp2f(__builtin_fmaf(lq, LOG2E_F, -Aq));
        const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(lp, LOG2E_F, -Ap));
        return live ? w * (q - p) : 0.f;               // rows outside the loss get exact zeros
    };
    for (uint32_t base = seg_begin; base < seg_end; base += GRAD_THREADS * CHUNKS) {
        if (base != seg_begin) request(base);
#pragma unroll
        for (int u = 0; u < CHUNKS; ++u) {
            const uint32_t c = base + u * GRAD_THREADS + threadIdx.x;
            if (c < seg_end) {
                float fq[VEC], fp[VEC], g[VEC];
                PC::unpack(rq[u], fq);
                PC::unpack(rp[u], fp);
#pragma unroll
                for (int j = 0; j < VEC; ++j) g[j] = grad_of(fq[j], fp[j]);
                OT::template store<VEC>(rowg, c, g);
            }
        }
    }
    // the ragged end of the row, element by element
    if (seg == 0 && (int)threadIdx.x < tail) {
        const int64_t i = (int64_t)nfull * VEC + threadIdx.x;
        OT::store1(rowg, i, grad_of(ET::load1(rowq, i), ET::load1(rowp, i)));
    }
}

// =================================================================================================
// Batch stage (Sec. 4.4.2 and Alg. 1 step 3) in one launch.  Every workgroup sums the whole batch
// in the same fixed order (per-thread strided sums, wave butterflies, then the 16 wave partials in
// index order), so all workgroups hold bit-identical statistics, run to run as well; each then
// writes the weights of its own slice of tokens.  Workgroup 0 writes the stats struct.
//   alpha_hat = accepted / proposed;  kappa = alpha_hat / mean_t Z_approx,t
//   Z_t = kappa Z_approx,t;  w_t = Z_t max(lambda, p(x)/q(x));
//   rho_t = min(w_t, c1) * min(p_ref(x)/p(x), c2)
// =================================================================================================
constexpr int FINALIZE_THREADS = 1024;
constexpr int FINALIZE_WAVES = FINALIZE_THREADS / WAVE;


__global__ __launch_bounds__(FINALIZE_THREADS) void finalize_kernel(FinalizeArgs A)
{
    __shared__ double sh_z[FINALIZE_WAVES], sh_a[FINALIZE_WAVES], sh_ze[FINALIZE_WAVES], sh_kl[FINALIZE_WAVES];
    __shared__ long long sh_n[FINALIZE_WAVES], sh_acc[FINALIZE_WAVES];
    __shared__ unsigned sh_err[FINALIZE_WAVES];
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), wv = tid / WAVE;
    double z = 0.0, a = 0.0, ze = 0.0, kl = 0.0;
    long long n = 0, nacc = 0;
    unsigned err = 0;
    // Inputs of this thread's first token of the weight pass, fetched before the reduction so
    // their latency overlaps it.
    const int64_t t0 = (int64_t)blockIdx.x * FINALIZE_THREADS + tid;
    const bool has0 = t0 < A.T && (A.w || A.rho);
    const uint8_t f0 = has0 ? A.rowflag[t0] : (uint8_t)ROW_PADDING;
    const float z0 = has0 ? A.zapprox[t0] : 0.f;
    const float lr0 = has0 ? A.logratio[t0] : 0.f;
    const float ref0 = (has0 && A.ref_logprob) ? A.ref_logprob[t0] - A.logp[t0] : 0.f;
    // Loads of eight rows are issued together (no branch between them) to overlap their latency.
    constexpr int U = 8;
    for (int64_t base = tid; base < A.T; base += (int64_t)U * FINALIZE_THREADS) {
        uint8_t f[U], mk[U];
        float zv[U], av[U], zev[U], klv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t t = base + (int64_t)u * FINALIZE_THREADS;
            const bool in = t < A.T;
            f[u] = in ? A.rowflag[t] : (uint8_t)ROW_PADDING;
            mk[u] = (in && A.mask) ? A.mask[t] : (uint8_t)0;
            zv[u] = in ? A.zapprox[t] : 0.f;
            av[u] = in ? A.accept[t] : 0.f;
            zev[u] = (in && A.zexact) ? A.zexact[t] : 0.f;
            klv[u] = (in && A.kl) ? A.kl[t] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (f[u] == ROW_OK) {
                n += 1;
                nacc += (long long)mk[u];
                z += (double)zv[u];
                a += (double)av[u];
                ze += (double)zev[u];
                kl += (double)klv[u];
            } else if (f[u] == ROW_BAD_ID) {
                err |= JP_DATA_ERR_ID_RANGE;
            } else if (f[u] == ROW_NONFINITE) {
                err |= JP_DATA_ERR_NONFINITE;
            }
        }
    }
    z = wave_sum(z); a = wave_sum(a); ze = wave_sum(ze); kl = wave_sum(kl);
    n = wave_sum_i((int)n); nacc = wave_sum_i((int)nacc);      // per-thread counts are < 2^21
    err = wave_or(err);
    if (lane == 0) { sh_z[wv] = z; sh_a[wv] = a; sh_ze[wv] = ze; sh_kl[wv] = kl; sh_n[wv] = n; sh_acc[wv] = nacc; sh_err[wv] = err; }
    __syncthreads();
    z = a = ze = kl = 0.0; n = nacc = 0; err = 0;
#pragma unroll
    for (int i = 0; i < FINALIZE_WAVES; ++i) {
        z += sh_z[i]; a += sh_a[i]; ze += sh_ze[i]; kl += sh_kl[i]; n += sh_n[i]; nacc += sh_acc[i]; err |= sh_err[i];
    }
    const double nn = (double)n;
    const double mean_z = z / nn, mean_a = a / nn;
    const double alpha = A.alpha_expected ? mean_a : (double)nacc / nn;
    const double kappa = alpha / mean_z;
    if (blockIdx.x == 0 && tid == 0) {
        jp_obrs_stats st;
        st.n_valid = n;
        st.n_accept = nacc;
        st.alpha_hat = alpha;
        st.mean_z_approx = mean_z;
        st.kappa = kappa;
        st.mean_z_exact = A.zexact ? ze / nn : __longlong_as_double(0x7ff8000000000000LL);
        st.mean_accept = mean_a;
        st.error_flags = err | (n == 0 ? (unsigned)JP_DATA_ERR_EMPTY : 0u);
        st.reserved = 0;
        st.mean_distill_kl = A.kl ? kl / nn : __longlong_as_double(0x7ff8000000000000LL);
        *A.stats = st;
    }
    if (!A.w && !A.rho) return;
    const double lam = (double)A.lambda;
    auto weigh = [&](int64_t t, uint8_t f, float zap, float lr, float refdiff) {
        float w, rho;
        if (f == ROW_PADDING) {
            w = 0.f; rho = 0.f;
        } else if (f != ROW_OK) {
            w = rho = __uint_as_float(0x7fc00000u);
        } else {
            const double zt = kappa * (double)zap;
            const double ratio = (double)__builtin_amdgcn_exp2f(lr * LOG2E_F);      // p(x)/q(x)
            const double wd = zt * (lam > ratio ? lam : ratio);
            // F(w): truncation (Alg. 1 step 3), identity, or two-sided truncation (Sec. 2)
            double rd = wd < (double)A.c1 ? wd : (double)A.c1;
            if (A.f_mode == JP_F_IDENTITY) rd = wd;
            else if (A.f_mode == JP_F_BAND) rd = (wd >= (double)A.f_lo && wd <= (double)A.f_hi) ? wd : 0.0;
            if (A.ref_logprob) {
                const double rr = (double)__builtin_amdgcn_exp2f(refdiff * LOG2E_F); // p_ref(x)/p(x)
                rd *= rr < (double)A.c2 ? rr : (double)A.c2;
            }
            w = (float)wd; rho = (float)rd;
        }
        if (A.w) A.w[t] = w;
        if (A.rho) A.rho[t] = rho;
    };
    if (t0 < A.T) weigh(t0, f0, z0, lr0, ref0);
    const int64_t step = (int64_t)gridDim.x * FINALIZE_THREADS;
    for (int64_t t = t0 + step; t < A.T; t += step)
        weigh(t, A.rowflag[t], A.zapprox[t], A.logratio[t],
              A.ref_logprob ? A.ref_logprob[t] - A.logp[t] : 0.f);
}

// ---- launchers ------------------------------------------------------------------------------

// Small batches of long rows: four waves per row in the plain sweeps, by the rule of the row stage.
static bool split_rows(int64_t T, int64_t V, int dtype) { return waves_per_row(T, V, dtype == JP_BF16 ? 2 : 4) == 4; }

hipError_t launch_zexact(const ZExactArgs &a, int dtype, hipStream_t st)
{
    if (a.T <= 0) return hipSuccess;
    const dim3 grid((unsigned)a.T), block(WAVE);
    if (a.waves >= 4) {
        if (dtype == JP_BF16) hipLaunchKernelGGL((zexact_kernel<Bf16Elem, 4>), grid, dim3(4 * WAVE), 0, st, a);
        else hipLaunchKernelGGL((zexact_kernel<F32Elem, 4>), grid, dim3(4 * WAVE), 0, st, a);
        return hipGetLastError();
    }
    if (dtype == JP_BF16) hipLaunchKernelGGL((zexact_kernel<Bf16Elem>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((zexact_kernel<F32Elem>), grid, block, 0, st, a);
    return hipGetLastError();
}

hipError_t launch_finalize(const FinalizeArgs &a, hipStream_t st)
{
    int64_t blocks = (a.T + FINALIZE_THREADS - 1) / FINALIZE_THREADS;
    blocks = blocks < 1 ? 1 : (blocks > 64 ? 64 : blocks);
    hipLaunchKernelGGL(finalize_kernel, dim3((unsigned)blocks), dim3(FINALIZE_THREADS), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_token_logprob(const LogprobArgs &a, int dtype, hipStream_t st)
{
    if (a.T <= 0) return hipSuccess;
    const dim3 grid((unsigned)a.T), block(WAVE);
    if (split_rows(a.T, a.V, dtype)) {
        if (dtype == JP_BF16) hipLaunchKernelGGL((token_logprob_kernel<Bf16Elem, 4>), grid, dim3(4 * WAVE), 0, st, a);
        else hipLaunchKernelGGL((token_logprob_kernel<F32Elem, 4>), grid, dim3(4 * WAVE), 0, st, a);
        return hipGetLastError();
    }
    if (dtype == JP_BF16) hipLaunchKernelGGL((token_logprob_kernel<Bf16Elem>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((token_logprob_kernel<F32Elem>), grid, block, 0, st, a);
    return hipGetLastError();
}

hipError_t launch_budget(const BudgetArgs &a, int dtype, hipStream_t st)
{
    if (a.T <= 0) return hipSuccess;
    const dim3 grid((unsigned)a.T), block(WAVE);
    if (split_rows(a.T, a.V, dtype)) {
        if (dtype == JP_BF16) hipLaunchKernelGGL((budget_kernel<Bf16Elem, 4>), grid, dim3(4 * WAVE), 0, st, a);
        else hipLaunchKernelGGL((budget_kernel<F32Elem, 4>), grid, dim3(4 * WAVE), 0, st, a);
        return hipGetLastError();
    }
    if (dtype == JP_BF16) hipLaunchKernelGGL((budget_kernel<Bf16Elem>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((budget_kernel<F32Elem>), grid, block, 0, st, a);
    return hipGetLastError();
}

template <class ET, int W>
static void launch_budget_batch_w(const BudgetArgs &a, BudgetBatchState *S, float *out_lambda, hipStream_t st)
{
    const dim3 grid((unsigned)(a.T > 0 ? a.T : 1)), one(WAVE), block(WAVE * W);
    hipLaunchKernelGGL(budget_batch_init_kernel, dim3(1), one, 0, st, S);
    if (a.T > 0) hipLaunchKernelGGL((budget_batch_coarse_kernel<ET, W>), grid, block, 0, st, a, S);
    hipLaunchKernelGGL(budget_batch_after_coarse_kernel, dim3(1), one, 0, st, S, a.target, out_lambda);
    // the exact sweeps: as many launches as the search may need; once it has finished the rest return at once
    for (int sweep = 1; sweep < BUDGET_MAX_SWEEPS; ++sweep) {
        if (a.T > 0) hipLaunchKernelGGL((budget_batch_fine_kernel<ET, W>), grid, block, 0, st, a, S);
        hipLaunchKernelGGL(budget_batch_after_fine_kernel, dim3(1), one, 0, st, S, a.target, a.eps_rel,
                           sweep == BUDGET_MAX_SWEEPS - 1 ? 1 : 0, out_lambda);
    }
    if (a.T > 0) hipLaunchKernelGGL((budget_batch_min_ratio_kernel<ET, W>), grid, block, 0, st, a, S);
    hipLaunchKernelGGL(budget_batch_min_ratio_finish_kernel, dim3(1), one, 0, st, S, out_lambda);
}

hipError_t launch_budget_batch(const BudgetArgs &a, int dtype, BudgetBatchState *S, float *out_lambda, hipStream_t st)
{
    const bool split = split_rows(a.T, a.V, dtype);
    if (dtype == JP_BF16) {
        if (split) launch_budget_batch_w<Bf16Elem, 4>(a, S, out_lambda, st);
        else launch_budget_batch_w<Bf16Elem, 1>(a, S, out_lambda, st);
    } else {
        if (split) launch_budget_batch_w<F32Elem, 4>(a, S, out_lambda, st);
        else launch_budget_batch_w<F32Elem, 1>(a, S, out_lambda, st);
    }
    return hipGetLastError();
}

hipError_t launch_distill_grad(const GradArgs &a, int dtype, int grad_dtype, hipStream_t st)
{
    const bool half_piece = dtype == JP_BF16 && grad_dtype != JP_BF16;
    const int vec = dtype == JP_BF16 && !half_piece ? 8 : 4;
    const int64_t nfull = a.V / vec;
    const int64_t per_batch = (int64_t)GRAD_THREADS * (half_piece ? Bf16HalfPiece::CHUNKS : GRAD_CHUNKS);
    const int64_t batches = nfull > 0 ? (nfull + per_batch - 1) / per_batch : 1;
    // One batch per workgroup where the grid allows it; the row is cut into equal segments (a
    // multiple of 256 bytes each) so that the last workgroup of a row is as long as the others.
    int64_t segs = batches;
    while (segs * a.T > 0x7fffffffLL) segs = (segs + 1) / 2;  // grid.x limit: longer segments
    int64_t seg_chunks = nfull > 0 ? (nfull + segs - 1) / segs : 1;
    seg_chunks = (seg_chunks + 15) / 16 * 16;
    segs = nfull > 0 ? (nfull + seg_chunks - 1) / seg_chunks : 1;
    GradArgs g = a;
    g.seg_chunks = (uint32_t)seg_chunks;
    g.segs = (uint32_t)segs;
    const dim3 grid((unsigned)(a.T * segs));
    if (dtype == JP_BF16 && grad_dtype == JP_BF16)
        hipLaunchKernelGGL((distill_grad_kernel<Bf16Elem, Bf16Out>), grid, dim3(GRAD_THREADS), 0, st, g);
    else if (dtype == JP_BF16)
        hipLaunchKernelGGL((distill_grad_kernel<Bf16Elem, F32Out, Bf16HalfPiece>), grid, dim3(GRAD_THREADS), 0, st, g);
    else if (grad_dtype == JP_BF16)
        hipLaunchKernelGGL((distill_grad_kernel<F32Elem, Bf16Out>), grid, dim3(GRAD_THREADS), 0, st, g);
    else
        hipLaunchKernelGGL((distill_grad_kernel<F32Elem, F32Out>), grid, dim3(GRAD_THREADS), 0, st, g);
    return hipGetLastError();
}

}  // namespace jp
