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
template <class ET>
__global__ __launch_bounds__(64) void zexact_kernel(ZExactArgs A)
{
    constexpr int VEC = ET::VEC;
    const int lane = threadIdx.x;
    const int64_t t = blockIdx.x;
    const uint8_t flag = A.rowflag[t];
    if (flag != ROW_OK) {
        if (lane == 0) A.zexact[t] = (flag == ROW_PADDING) ? 0.f : __uint_as_float(0x7fc00000u);
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
    float s0 = 0.f, s1 = 0.f;
    auto account = [&](const float (&fq)[VEC], const float (&fp)[VEC]) {
#pragma unroll
        for (int j = 0; j < VEC; j += 2) {
            s0 += __builtin_amdgcn_exp2f(fminf(__builtin_fmaf(fq[j], LOG2E_F, -Aq), __builtin_fmaf(fp[j], LOG2E_F, -Ap)));
            s1 += __builtin_amdgcn_exp2f(fminf(__builtin_fmaf(fq[j + 1], LOG2E_F, -Aq), __builtin_fmaf(fp[j + 1], LOG2E_F, -Ap)));
        }
    };
    const uint32_t nit = nfull / WAVE;                      // iterations in which every lane has a full chunk
    if (nit > 0) {
        constexpr int D = 3;                                // non-temporal loads in flight per tensor and lane
        const uint32_t last = nit - 1;
        u32x4 wq[D], wp[D];
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const uint32_t n = ((uint32_t)d < last ? (uint32_t)d : last) * WAVE + lane;
            wq[d] = stream_load(as_global_vec(rowq) + n);
            wp[d] = stream_load(as_global_vec(rowp) + n);
        }
        for (uint32_t it = 0; it < nit; it += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                const u32x4 cq = wq[d], cp = wp[d];
                const uint32_t n = (it + D + d < last ? it + D + d : last) * WAVE + lane;
                wq[d] = stream_load(as_global_vec(rowq) + n);
                wp[d] = stream_load(as_global_vec(rowp) + n);
                if (d == 0 || it + d < nit) {
                    float fq[VEC], fp[VEC];
                    ET::unpack(cq, fq);
                    ET::unpack(cp, fp);
                    account(fq, fp);
                }
            }
        }
    }
    {
        const uint32_t c = nit * WAVE + lane;
        if (c < nchunks) {
            float fq[VEC], fp[VEC];
            load_chunk<ET>(rowq, c, nfull, tail, fq);
            load_chunk<ET>(rowp, c, nfull, tail, fp);
            account(fq, fp);
        }
    }
    const double Z = wave_sum((double)s0 + (double)s1);
    if (lane == 0) A.zexact[t] = (float)Z;
}

// =================================================================================================
// log softmax(l_t)[x_t] for one logit tensor: how log p_ref(a_t) of Alg. 1 (Phase 2, step 1) is read
// off a third tensor.  One wavefront per row, one sweep: per-lane exponent reference (moved only
// when a chunk maximum exceeds it by the margin) and sum, combined across the wave at the end.
// =================================================================================================
template <class ET>
__global__ __launch_bounds__(64) void token_logprob_kernel(LogprobArgs A)
{
    constexpr int VEC = ET::VEC;
    const int lane = threadIdx.x;
    const int64_t t = blockIdx.x;
    const int x = A.ids[t];
    const int64_t V = A.V;
    if (x < 0 || x >= V) {
        if (lane == 0) A.out[t] = x < 0 ? 0.f : __uint_as_float(0x7fc00000u);
        return;
    }
    const char *row = (const char *)A.logits + (size_t)t * (size_t)A.stride * ET::ESZ;
    const gvec_ptr v = as_global_vec(row);
    const uint32_t nfull = (uint32_t)(V / VEC);
    const int tail = (int)(V - (int64_t)nfull * VEC);
    const uint32_t nchunks = nfull + (tail ? 1u : 0u);
    const uint32_t nit = nfull / WAVE;
    float M2 = M2_UNSET, mthr = -2.0e38f, s = 0.f;
    auto consume = [&](const float (&f)[VEC], bool valid) {
        const float m = max_of<VEC>(f);
        if (valid && m > mthr) {                                    // rare: move this lane's reference
            const float newM2 = m * LOG2E_F;
            s *= __builtin_amdgcn_exp2f(M2 - newM2);
            M2 = newM2;
            mthr = m + RESCALE_MARGIN2 / LOG2E_F;
        }
        if (valid) s += sum_exp2<VEC>(f, M2);
    };
    if (nit > 0) {
        constexpr int D = 4;
        const uint32_t last = nit - 1;
        u32x4 w[D];
#pragma unroll
        for (int d = 0; d < D; ++d) w[d] = stream_load(v + (((uint32_t)d < last ? (uint32_t)d : last) * WAVE + lane));
        for (uint32_t it = 0; it < nit; it += D) {
            u32x4 c[D];
#pragma unroll
            for (int d = 0; d < D; ++d) c[d] = w[d];
#pragma unroll
            for (int d = 0; d < D; ++d) w[d] = stream_load(v + ((it + D + d < last ? it + D + d : last) * WAVE + lane));
#pragma unroll
            for (int d = 0; d < D; ++d) {
                if (d == 0 || it + d < nit) {
                    float f[VEC];
                    ET::unpack(c[d], f);
                    consume(f, true);
                }
            }
        }
    }
    {
        const uint32_t c = nit * WAVE + lane;
        if (c < nchunks) {
            float f[VEC];
            load_chunk<ET>(row, c, nfull, tail, f);
            consume(f, true);
        }
    }
    // combine the 64 (reference, sum) pairs: common reference = the largest, sums rescaled to it
    const float Mw = uniform_f(wave_max(M2));
    const double S = wave_sum(M2 == M2_UNSET ? 0.0 : (double)(s * __builtin_amdgcn_exp2f(M2 - Mw)));
    const double lse = ((double)Mw + log2_of_sum(S)) * LN2_D;
    const double lp = (double)ET::load1(row, x) - lse;
    if (lane == 0) A.out[t] = isfinite(lse) ? (float)lp : __uint_as_float(0x7fc00000u);
}

// =================================================================================================
// Scaling factor for an acceptance budget (Sec. 3.3, Theorem 2): per row the lambda with
// Z(lambda) = sum_v min(q_v, p_v / lambda) = abar.  With d_v = log2(p_v / q_v),
//   Z(2^x) = sum_{d_v > x} q_v + 2^-x sum_{d_v <= x} p_v
// is non-increasing in x, so the crossing is bracketed by histogram passes: a pass sweeps the row,
// adds q_v and p_v of the tokens inside the current bracket [lo, hi) to 64 bins in LDS (float64
// atomics; the bins belong to this wave alone and the hardware takes the lanes of an instruction in
// a fixed order, so the sums are reproducible; 8 copies per bin keep same-address collisions to
// eight lanes) and the mass outside it to two per-lane sums; the bin whose edges straddle abar is
// the next bracket.  After BUDGET_PASSES passes the bracket is 128 / 64^3 = 4.9e-4 wide in log2
// lambda and lambda = B / (abar - A) with A the q-mass above it and B the p-mass at or below it;
// that closed form is exact up to the few tokens whose ratio lies inside the last bracket (their
// mass times the bracket width, ~1e-8 of Z for a vocabulary of 1e5 tokens).
// abar = 1 returns the smallest ratio (the largest lambda that still accepts everything).
// =================================================================================================
constexpr int BUDGET_BINS = 64, BUDGET_COPIES = 8, BUDGET_PASSES = 3;
constexpr float BUDGET_RANGE = 64.f;                       // first bracket: ratios in [2^-64, 2^64)

// x in [0, 1] as an integer multiple of 2^-40, truncated: the 24-bit significand shifted into place.
// (Integer LDS atomics take same-address collisions faster than float64 ones; the first pass, where
// most tokens share a few bins, uses them.)
constexpr double BUDGET_FIX40 = 1099511627776.0;           // 2^40
__device__ __forceinline__ unsigned long long to_fixed40(float x)
{
    const uint32_t bits = __float_as_uint(x);
    const uint32_t m = (bits & 0x7fffffu) | 0x800000u;      // significand with its leading one
    uint32_t sh = 142u - (bits >> 23);                      // x = m 2^(e-150): (m 2^32) >> (142 - e) = x 2^40
    sh = sh < 63u ? sh : 63u;                               // below 2^-40 (and zero): nothing left
    return ((unsigned long long)m << 32) >> sh;
}

// One histogram sweep of a row pair for the bracket [lo, hi): q- and p-mass of the tokens inside it
// go to the LDS bins hq / hp, the mass outside it to the per-lane sums qa (above) and
// pb (below).  The first pass (FIRST) covers every ratio: it runs without branches, puts a ratio
// beyond the range into the nearest edge bin (the later passes sum the mass outside their bracket
// themselves, so this only has to find the bracket) and tracks the smallest log2 ratio.
template <class ET, bool FIRST>
__device__ __forceinline__ void budget_sweep(const char *rowq, const char *rowp, int64_t V, float Aq, float Ap,
                                             float lo, float hi, double *hq,
                                             double *hp, double &qa, double &pb, float &dmin)
{
    constexpr int VEC = ET::VEC;
    const int lane = threadIdx.x;
    const uint32_t nfull = (uint32_t)(V / VEC);
    const int tail = (int)(V - (int64_t)nfull * VEC);
    const uint32_t nchunks = nfull + (tail ? 1u : 0u);
    const int copy = lane & (BUDGET_COPIES - 1);
    for (int e = lane; e < BUDGET_BINS * BUDGET_COPIES; e += WAVE) { hq[e] = 0.0; hp[e] = 0.0; }   // all bits zero: also integer 0
    lds_sync();
    const float inv_w = (float)BUDGET_BINS / (hi - lo);
    qa = 0.0;
    pb = 0.0;
    auto account = [&](const float (&fq)[VEC], const float (&fp)[VEC]) {
        if constexpr (FIRST) {
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                const float aq = __builtin_fmaf(fq[j], LOG2E_F, -Aq), ap = __builtin_fmaf(fp[j], LOG2E_F, -Ap);
                const float d = ap - aq;
                // A ratio below the range keeps none of its q-mass at any lambda of the range, one
                // above it pays none of its p-mass; NaN (both probabilities 0) adds two zeros to bin 0.
                int b = (int)((d - lo) * inv_w);
                b = b < 0 ? 0 : (b < BUDGET_BINS - 1 ? b : BUDGET_BINS - 1);
                const float qv = d >= lo ? __builtin_amdgcn_exp2f(aq) : 0.f;
                const float pv = d < hi ? __builtin_amdgcn_exp2f(ap) : 0.f;
                atomicAdd((unsigned long long *)&hq[b * BUDGET_COPIES + copy], to_fixed40(qv));
                atomicAdd((unsigned long long *)&hp[b * BUDGET_COPIES + copy], to_fixed40(pv));
                // the smallest ratio among tokens that both models can emit (finite d)
                dmin = (d > -3.0e38f && d < 3.0e38f) ? fminf(dmin, d) : dmin;
            }
        } else {
            float pbf = 0.f, qaf = 0.f;                 // this chunk's mass below / above the bracket
            float dv[VEC], apv[VEC], one[VEC];
            bool any = false;
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                const float aq = __builtin_fmaf(fq[j], LOG2E_F, -Aq);
                apv[j] = __builtin_fmaf(fp[j], LOG2E_F, -Ap);
                dv[j] = apv[j] - aq;
                // a token outside the bracket needs only one of its two probabilities: p below it, q above
                const bool below = dv[j] < lo;
                one[j] = __builtin_amdgcn_exp2f(below ? apv[j] : aq);
                pbf += below ? one[j] : 0.f;            // at or below every lambda of the bracket
                qaf += dv[j] >= hi ? one[j] : 0.f;      // above every lambda of the bracket
                any |= dv[j] >= lo && dv[j] < hi;       // (both probabilities 0 give NaN: no mass)
            }
            pb += (double)pbf;
            qa += (double)qaf;
            // late passes: the bracket is narrow and most chunks of a wave hold nothing inside it
            if (__ballot(any)) {
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    if (dv[j] >= lo && dv[j] < hi) {
                        int b = (int)((dv[j] - lo) * inv_w);
                        b = b < BUDGET_BINS - 1 ? b : BUDGET_BINS - 1;
                        atomicAdd(&hq[b * BUDGET_COPIES + copy], (double)one[j]);
                        atomicAdd(&hp[b * BUDGET_COPIES + copy], (double)__builtin_amdgcn_exp2f(apv[j]));
                    }
                }
            }
        }
    };
    const uint32_t nit = nfull / WAVE;                  // iterations in which every lane has a full chunk
    if (nit > 0) {
        constexpr int D = 3;                            // loads in flight per tensor and lane
        const uint32_t last = nit - 1;
        u32x4 wq[D], wp[D];
#pragma unroll
        for (int d2 = 0; d2 < D; ++d2) {
            const uint32_t n = ((uint32_t)d2 < last ? (uint32_t)d2 : last) * WAVE + lane;
            wq[d2] = stream_load(as_global_vec(rowq) + n);
            wp[d2] = stream_load(as_global_vec(rowp) + n);
        }
        for (uint32_t it = 0; it < nit; it += D) {
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
    {
        const uint32_t c = nit * WAVE + lane;
        if (c < nchunks) {
            float fq[VEC], fp[VEC];
            load_chunk<ET>(rowq, c, nfull, tail, fq);
            load_chunk<ET>(rowp, c, nfull, tail, fp);
            account(fq, fp);
        }
    }
    lds_sync();
}

// Lane b's bin b summed over its copies: integers in 2^-40 units after the first pass, float64 after the others.
__device__ __forceinline__ void budget_bin_sums(const double *hq, const double *hp, bool first_pass, double &q, double &p)
{
    const int lane = threadIdx.x;
    if (first_pass) {
        unsigned long long uq = 0, up = 0;
#pragma unroll 4
        for (int c2 = 0; c2 < BUDGET_COPIES; ++c2) {
            uq += ((const unsigned long long *)hq)[lane * BUDGET_COPIES + c2];
            up += ((const unsigned long long *)hp)[lane * BUDGET_COPIES + c2];
        }
        q = (double)uq / BUDGET_FIX40;
        p = (double)up / BUDGET_FIX40;
    } else {
        q = 0.0; p = 0.0;
#pragma unroll 4
        for (int c2 = 0; c2 < BUDGET_COPIES; ++c2) { q += hq[lane * BUDGET_COPIES + c2]; p += hp[lane * BUDGET_COPIES + c2]; }
    }
}

// One step of the bracket search, run by a whole wave: lane b brings the q- and p-mass of bin b
// (Qb, Pbin); A_above / B_below are the masses outside the bracket, `goal` the value Z must reach
// (abar, or abar times the number of rows when the masses are sums over a batch); dmin the
// smallest log2 ratio seen.  Narrows [lo, hi) to the bin that straddles the goal, or finishes
// (returns true) with lambda.  sq_ / sp_: BUDGET_BINS doubles of LDS each.
__device__ __forceinline__ bool budget_step(double goal, double A_above, double B_below, double Qb, double Pbin,
                                            float &lo, float &hi, int pass, float dmin, double *sq_, double *sp_,
                                            double &lambda)
{
    const int lane = threadIdx.x;
    sq_[lane] = Qb; sp_[lane] = Pbin;
    lds_sync();
    // the q-mass of the bins from this lane's up, the p-mass of the bins below it
    double Qsuf = 0.0, Ppre = 0.0, Ptot = 0.0;
#pragma unroll 4
    for (int j = 0; j < BUDGET_BINS; ++j) {
        const double qj = sq_[j], pj = sp_[j];
        Qsuf += j >= lane ? qj : 0.0;
        Ppre += j < lane ? pj : 0.0;
        Ptot += pj;
    }
    lds_sync();
    const float w = (hi - lo) / (float)BUDGET_BINS;
    const float edge = lo + w * (float)lane;            // lower edge of this lane's bin
    const double Zedge = A_above + Qsuf + (B_below + Ppre) * (double)__builtin_amdgcn_exp2f(-edge);
    const double Zhi = A_above + (B_below + Ptot) * (double)__builtin_amdgcn_exp2f(-hi);
    const int n_true = __popcll(__ballot(Zedge >= goal));
    // Z(lambda -> 0) is all the mass that can be kept at all.  A budget at (or within rounding of)
    // it is met by every lambda up to the smallest ratio, which is the answer; Z is flat there,
    // so the bracket search would be deciding on rounding noise.
    const double Zmax = A_above + lane_value_d(Qsuf, 0);
    if (pass == 0 && (n_true == 0 || goal >= Zmax * (1.0 - 1e-6))) {
        lambda = (double)__builtin_amdgcn_exp2f(dmin);
        return true;
    }
    if (pass == 0 && Zhi >= goal) {
        lambda = (B_below + Ptot) / (goal - A_above);   // beyond 2^64: every ratio is below lambda
        return true;
    }
    int bstar = n_true > 0 ? n_true - 1 : 0;
    bstar = bstar < BUDGET_BINS - 1 ? bstar : BUDGET_BINS - 1;
    // masses as seen by lane bstar, made wave-uniform
    const double Qs = lane_value_d(Qsuf, bstar), Pp = lane_value_d(Ppre, bstar);
    const double Qself = lane_value_d(Qb, bstar), Pself = lane_value_d(Pbin, bstar);
    const float nlo = lo + w * (float)bstar;
    lo = nlo;
    hi = nlo + w;
    if (pass == BUDGET_PASSES - 1) {
        const double Aend = A_above + (Qs - Qself), Bend = B_below + Pp + Pself;
        lambda = Bend / (goal - Aend);
        const double l_lo = (double)__builtin_amdgcn_exp2f(nlo), l_hi = (double)__builtin_amdgcn_exp2f(nlo + w);
        lambda = lambda < l_lo ? l_lo : (lambda > l_hi ? l_hi : lambda);
        return true;
    }
    return false;
}

template <class ET>
__global__ __launch_bounds__(64, 4) void budget_kernel(BudgetArgs A)
{
    __shared__ double hq[BUDGET_BINS * BUDGET_COPIES], hp[BUDGET_BINS * BUDGET_COPIES];
    __shared__ double sq_[BUDGET_BINS], sp_[BUDGET_BINS];
    const int lane = threadIdx.x;
    const int64_t t = blockIdx.x;
    const float NaN = __uint_as_float(0x7fc00000u);
    const uint8_t flag = A.rowflag[t];
    const float abar_f = A.row_target ? A.row_target[t] : A.target;
    if (flag != ROW_OK || !(abar_f > 0.f) || abar_f > 1.f) {
        if (lane == 0) A.lambda_out[t] = flag == ROW_PADDING ? 0.f : NaN;
        return;
    }
    const char *rowq = (const char *)A.actor + (size_t)t * (size_t)A.stride * ET::ESZ;
    const char *rowp = (const char *)A.policy + (size_t)t * (size_t)A.stride * ET::ESZ;
    const float Aq = (float)(A.lse_q[t] * LOG2E_D);
    const float Ap = (float)(A.lse_p[t] * LOG2E_D);
    float lo = -BUDGET_RANGE, hi = BUDGET_RANGE;
    double lambda = 0.0;
    float dmin = __uint_as_float(0x7f800000u);
    for (int pass = 0; pass < BUDGET_PASSES; ++pass) {
        double qa, pb;
        if (pass == 0) budget_sweep<ET, true>(rowq, rowp, A.V, Aq, Ap, lo, hi, hq, hp, qa, pb, dmin);
        else budget_sweep<ET, false>(rowq, rowp, A.V, Aq, Ap, lo, hi, hq, hp, qa, pb, dmin);
        const double A_above = wave_sum(qa), B_below = wave_sum(pb);
        // lane b owns bin b
        double uq, up;
        budget_bin_sums(hq, hp, pass == 0, uq, up);
        const float dmin_w = pass == 0 ? -uniform_f(wave_max(-dmin)) : 0.f;
        if (budget_step((double)abar_f, A_above, B_below, uq, up, lo, hi,
                        pass, dmin_w, sq_, sp_, lambda))
            break;
    }
    if (lane == 0) A.lambda_out[t] = (float)lambda;
}

// The same search for one lambda of a whole batch, mean_t Z_t(lambda) = abar: the bins of all rows are
// summed in device memory (64-bit fixed point, 2^-32 units, so the sums are order-independent), a
// one-wave kernel narrows the bracket between the sweeps, and nothing goes through the host.
__global__ void budget_batch_init_kernel(BudgetBatchState *S)
{
    const int lane = threadIdx.x;
    S->bq[lane] = 0; S->bp[lane] = 0;
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

template <class ET>
__global__ __launch_bounds__(64, 4) void budget_batch_pass_kernel(BudgetArgs A, BudgetBatchState *S, int pass)
{
    __shared__ double hq[BUDGET_BINS * BUDGET_COPIES], hp[BUDGET_BINS * BUDGET_COPIES];
    const int lane = threadIdx.x;
    const int64_t t = blockIdx.x;
    if (S->done || A.rowflag[t] != ROW_OK) return;
    const char *rowq = (const char *)A.actor + (size_t)t * (size_t)A.stride * ET::ESZ;
    const char *rowp = (const char *)A.policy + (size_t)t * (size_t)A.stride * ET::ESZ;
    const float Aq = (float)(A.lse_q[t] * LOG2E_D);
    const float Ap = (float)(A.lse_p[t] * LOG2E_D);
    const float lo = S->lo, hi = S->hi;
    float dmin = __uint_as_float(0x7f800000u);
    double qa, pb;
    if (pass == 0) budget_sweep<ET, true>(rowq, rowp, A.V, Aq, Ap, lo, hi, hq, hp, qa, pb, dmin);
    else budget_sweep<ET, false>(rowq, rowp, A.V, Aq, Ap, lo, hi, hq, hp, qa, pb, dmin);
    const double A_above = wave_sum(qa), B_below = wave_sum(pb);
    double dq, dp;
    budget_bin_sums(hq, hp, pass == 0, dq, dp);
    const unsigned long long uq = (unsigned long long)(dq * 4294967296.0), up = (unsigned long long)(dp * 4294967296.0);
    if (uq) atomicAdd(&S->bq[lane], uq);                    // 2^-32 units: integer sums, any order
    if (up) atomicAdd(&S->bp[lane], up);
    if (pass == 0) dmin = -uniform_f(wave_max(-dmin));
    if (lane == 0) {
        atomicAdd(&S->above, (unsigned long long)(A_above * 4294967296.0));
        atomicAdd(&S->below, (unsigned long long)(B_below * 4294967296.0));
        if (pass == 0) {
            atomicAdd(&S->n_rows, 1ull);
            atomicMin(&S->dmin_ord, float_order_int(dmin));
        }
    }
}

__global__ __launch_bounds__(64) void budget_batch_scan_kernel(BudgetBatchState *S, float target, int pass, float *out_lambda)
{
    __shared__ double sq_[BUDGET_BINS], sp_[BUDGET_BINS];
    const int lane = threadIdx.x;
    if (S->done) return;
    const double unit = 1.0 / 4294967296.0;
    const unsigned long long n = S->n_rows;
    const double Qb = (double)S->bq[lane] * unit, Pbin = (double)S->bp[lane] * unit;
    const double A_above = (double)S->above * unit, B_below = (double)S->below * unit;
    float lo = S->lo, hi = S->hi;
    const int o = S->dmin_ord;
    const float dmin = __int_as_float(o ^ ((o >> 31) & 0x7fffffff));
    double lambda = 0.0;
    bool done;
    if (n == 0) {                                           // no valid row
        lambda = __longlong_as_double(0x7ff8000000000000LL);
        done = true;
    } else {
        done = budget_step((double)target * (double)n, A_above, B_below, Qb, Pbin, lo, hi, pass, dmin, sq_, sp_, lambda);
    }
    lds_sync();
    S->bq[lane] = 0; S->bp[lane] = 0;                       // the next sweep starts from empty bins
    if (lane == 0) {
        S->above = 0; S->below = 0;
        S->lo = lo; S->hi = hi;
        if (done) { S->done = 1; S->lambda = lambda; *out_lambda = (float)lambda; }
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

hipError_t launch_zexact(const ZExactArgs &a, int dtype, hipStream_t st)
{
    if (a.T <= 0) return hipSuccess;
    const dim3 grid((unsigned)a.T), block(WAVE);
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
    if (dtype == JP_BF16) hipLaunchKernelGGL((token_logprob_kernel<Bf16Elem>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((token_logprob_kernel<F32Elem>), grid, block, 0, st, a);
    return hipGetLastError();
}

hipError_t launch_budget(const BudgetArgs &a, int dtype, hipStream_t st)
{
    if (a.T <= 0) return hipSuccess;
    const dim3 grid((unsigned)a.T), block(WAVE);
    if (dtype == JP_BF16) hipLaunchKernelGGL((budget_kernel<Bf16Elem>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((budget_kernel<F32Elem>), grid, block, 0, st, a);
    return hipGetLastError();
}

hipError_t launch_budget_batch(const BudgetArgs &a, int dtype, BudgetBatchState *S, float *out_lambda, hipStream_t st)
{
    hipLaunchKernelGGL(budget_batch_init_kernel, dim3(1), dim3(WAVE), 0, st, S);
    for (int pass = 0; pass < BUDGET_PASSES; ++pass) {
        if (a.T > 0) {
            const dim3 grid((unsigned)a.T), block(WAVE);
            if (dtype == JP_BF16) hipLaunchKernelGGL((budget_batch_pass_kernel<Bf16Elem>), grid, block, 0, st, a, S, pass);
            else hipLaunchKernelGGL((budget_batch_pass_kernel<F32Elem>), grid, block, 0, st, a, S, pass);
        }
        hipLaunchKernelGGL(budget_batch_scan_kernel, dim3(1), dim3(WAVE), 0, st, S, a.target, pass, out_lambda);
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
