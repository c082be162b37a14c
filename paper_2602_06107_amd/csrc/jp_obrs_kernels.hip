// OBRS hot path of Jackpot for gfx950 (MI355X): device kernels.
//
// One 64-lane wavefront owns one token position.  It streams the actor and the policy logit
// rows once with 16-byte loads and keeps, per row:
//   * a running sum of 2^(l*log2(e) - M2) against a wave-uniform reference M2 (log-sum-exp),
//   * a bounded buffer of "chunk descriptors" (chunk maximum, chunk index) in LDS from which
//     the k chunks with the largest maxima survive (the k largest elements of a row always lie
//     inside the k chunks with the largest maxima),
// then expands the surviving chunks into elements, ranks them by (logit desc, id asc), forms the
// union of the two top-k lists and the normaliser estimate of Sec. 4.4.1, and the per-token
// acceptance probability of Eq. obrs_accept.  A second, optional sweep computes the normaliser
// of Eq. obrs_dist over the whole vocabulary; two small kernels do the batch statistics of
// Sec. 4.4.2 and the weights of Alg. 1 step 3.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "jp_obrs_internal.h"

namespace jp {

namespace {

constexpr int WAVE = 64;
constexpr float LOG2E_F = 1.4426950408889634f;
constexpr double LOG2E_D = 1.4426950408889634074;
constexpr double LN2_D = 0.69314718055994530942;
// The exponent reference moves only when a logit exceeds it by this many powers of two, so a
// row sum stays below 2^64 * V, far inside fp32 range.
constexpr float RESCALE_MARGIN2 = 64.0f;
constexpr float M2_UNSET = -3.0e38f;

__device__ __forceinline__ float neg_inf() { return __uint_as_float(0xff800000u); }

// 16 bytes of logits as a native vector (kept in four VGPRs), loaded through the global address
// space so the compiler emits global_load_dwordx4 and can keep several loads in flight.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint64_t u64x2 __attribute__((ext_vector_type(2)));
typedef const __attribute__((address_space(1))) u32x4 *gvec_ptr;
__device__ __forceinline__ gvec_ptr as_global_vec(const void *p) { return (gvec_ptr)(uintptr_t)p; }
// Streaming load: the logits are read once, so they are fetched with the non-temporal hint and
// do not displace each other in L2 (measured: 6.9 TB/s against 6.1 TB/s for plain loads).
__device__ __forceinline__ u32x4 stream_load(gvec_ptr p) { return __builtin_nontemporal_load(p); }

// Order-preserving map float -> uint32 (-0 is folded onto +0 so that equal values get equal keys).
__device__ __forceinline__ uint32_t ord32(float f)
{
    const uint32_t u = __float_as_uint(f + 0.0f);             // -0 + 0 = +0 (round to nearest)
    return u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);
}
__device__ __forceinline__ float unord32(uint32_t o)
{
    return __uint_as_float((o & 0x80000000u) ? (o ^ 0x80000000u) : ~o);
}

__device__ __forceinline__ int lane_prefix(uint64_t m)
{
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}
__device__ __forceinline__ int uniform_i(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ float uniform_f(float v)
{
    return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(v)));
}
__device__ __forceinline__ uint32_t uniform_u(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }
__device__ __forceinline__ uint64_t uniform_u64(uint64_t v)
{
    return ((uint64_t)uniform_u((uint32_t)(v >> 32)) << 32) | uniform_u((uint32_t)v);
}

// Wave-wide reductions on the VALU (data-parallel primitives, no LDS traffic): butterflies inside
// each quad (quad_perm), rotations by 4 and 8 inside each row of 16 lanes, then the four row
// results are read out and combined in a fixed order, so every lane gets the same bits.
template <int CTRL> __device__ __forceinline__ int dpp_mov(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, false);
}
constexpr int DPP_QUAD_XOR1 = 0xB1, DPP_QUAD_XOR2 = 0x4E, DPP_ROW_ROR4 = 0x124, DPP_ROW_ROR8 = 0x128;

template <int CTRL> __device__ __forceinline__ float dpp_f(float v) { return __int_as_float(dpp_mov<CTRL>(__float_as_int(v))); }
template <int CTRL> __device__ __forceinline__ double dpp_d(double v)
{
    return __hiloint2double(dpp_mov<CTRL>(__double2hiint(v)), dpp_mov<CTRL>(__double2loint(v)));
}
__device__ __forceinline__ double lane_value_d(double v, int l)
{
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), l), __builtin_amdgcn_readlane(__double2loint(v), l));
}

__device__ __forceinline__ float wave_max(float v)
{
    v = fmaxf(v, dpp_f<DPP_QUAD_XOR1>(v));
    v = fmaxf(v, dpp_f<DPP_QUAD_XOR2>(v));
    v = fmaxf(v, dpp_f<DPP_ROW_ROR4>(v));
    v = fmaxf(v, dpp_f<DPP_ROW_ROR8>(v));
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}
__device__ __forceinline__ double wave_sum(double v)
{
    v += dpp_d<DPP_QUAD_XOR1>(v);
    v += dpp_d<DPP_QUAD_XOR2>(v);
    v += dpp_d<DPP_ROW_ROR4>(v);
    v += dpp_d<DPP_ROW_ROR8>(v);
    return ((lane_value_d(v, 0) + lane_value_d(v, 16)) + lane_value_d(v, 32)) + lane_value_d(v, 48);
}
__device__ __forceinline__ int wave_sum_i(int v)
{
    v += dpp_mov<DPP_QUAD_XOR1>(v);
    v += dpp_mov<DPP_QUAD_XOR2>(v);
    v += dpp_mov<DPP_ROW_ROR4>(v);
    v += dpp_mov<DPP_ROW_ROR8>(v);
    return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) +
           __builtin_amdgcn_readlane(v, 32) + __builtin_amdgcn_readlane(v, 48);
}
__device__ __forceinline__ unsigned wave_or(unsigned v)
{
    const uint64_t any = __ballot(v != 0);
    unsigned r = 0;
#pragma unroll
    for (int b = 0; b < 3; ++b) r |= (__ballot((v >> b) & 1u) != 0) ? (1u << b) : 0u;   // three flag bits exist
    return any ? r : 0u;
}

// Single-wave workgroups: this orders LDS traffic between lanes (and stops the compiler from
// moving LDS accesses across it).
__device__ __forceinline__ void lds_sync() { __syncthreads(); }

// Value of lane (lane ^ L): data-parallel primitives inside a row of 16 lanes where one exists,
// the LDS crossbar (no memory access) otherwise.
template <int L> __device__ __forceinline__ uint32_t xor_lane(uint32_t v)
{
    static_assert(L == 1 || L == 2 || L == 4 || L == 8 || L == 16 || L == 32, "lane distance");
    if constexpr (L == 1) return (uint32_t)dpp_mov<DPP_QUAD_XOR1>((int)v);
    else if constexpr (L == 2) return (uint32_t)dpp_mov<DPP_QUAD_XOR2>((int)v);
    else if constexpr (L == 8) return (uint32_t)dpp_mov<DPP_ROW_ROR8>((int)v);
    else if constexpr (L == 32) return (uint32_t)__builtin_amdgcn_ds_bpermute((int)((threadIdx.x ^ 32u) << 2), (int)v);
    else return (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, 0x1F | (L << 10));   // bit mode: and 0x1f, or 0, xor L
}
template <int L> __device__ __forceinline__ uint64_t xor_lane(uint64_t v)
{
    return ((uint64_t)xor_lane<L>((uint32_t)(v >> 32)) << 32) | xor_lane<L>((uint32_t)v);
}

// Bitonic sorting network over the 64 * R keys of a wave, descending; key e of the sequence is
// register (e % R) of lane (e / R), so the exchanges at distance < R stay inside a lane.
template <class SK, int R, int K2, int J> __device__ __forceinline__ void bitonic_layer(SK (&v)[R], int lane)
{
    if constexpr (J < R) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if ((r & J) == 0) {
                const bool desc = (K2 < R) ? ((r & K2) == 0) : ((lane & (K2 / R)) == 0 || K2 == WAVE * R);
                const SK a = v[r], b = v[r | J];
                const bool g = a > b;
                const SK hi = g ? a : b, lo = g ? b : a;
                v[r] = desc ? hi : lo;
                v[r | J] = desc ? lo : hi;
            }
        }
    } else {
        constexpr int L = J / R;
        const bool lower = (lane & L) == 0;
        const bool desc = (lane & (K2 / R)) == 0 || K2 == WAVE * R;
        const bool keep_max = lower == desc;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const SK p = xor_lane<L>(v[r]);
            const bool g = v[r] > p;
            v[r] = (g == keep_max) ? v[r] : p;
        }
    }
    if constexpr (J > 1) bitonic_layer<SK, R, K2, J / 2>(v, lane);
}
template <class SK, int R, int K2> __device__ __forceinline__ void bitonic_merge_from(SK (&v)[R], int lane)
{
    bitonic_layer<SK, R, K2, K2 / 2>(v, lane);
    if constexpr (K2 < WAVE * R) bitonic_merge_from<SK, R, K2 * 2>(v, lane);
}
template <class SK, int R> __device__ __forceinline__ void bitonic_sort_desc(SK (&v)[R], int lane)
{
    bitonic_merge_from<SK, R, 2>(v, lane);
}

// ---- element types ------------------------------------------------------------------------

struct Bf16Elem {
    static constexpr int VEC = 8;           // elements per 16-byte load
    static constexpr int ESZ = 2;
    static __device__ __forceinline__ void unpack(const u32x4 w, float (&f)[VEC])
    {
        f[0] = __uint_as_float(w.x << 16); f[1] = __uint_as_float(w.x & 0xffff0000u);
        f[2] = __uint_as_float(w.y << 16); f[3] = __uint_as_float(w.y & 0xffff0000u);
        f[4] = __uint_as_float(w.z << 16); f[5] = __uint_as_float(w.z & 0xffff0000u);
        f[6] = __uint_as_float(w.w << 16); f[7] = __uint_as_float(w.w & 0xffff0000u);
    }
    static __device__ __forceinline__ float load1(const char *row, int64_t i)
    {
        return __uint_as_float((uint32_t)((const uint16_t *)row)[i] << 16);
    }
    // Candidate key for the final ranking: 16 value bits, then the complement of the candidate's
    // position in the buffer.  Candidates are buffered in ascending id order, so an unsigned
    // compare orders the keys by (value desc, id asc).
    using SortKey = uint32_t;
    static __device__ __forceinline__ SortKey make_sort(uint32_t ord, uint32_t pos) { return (ord & 0xffff0000u) | (0xffffu - pos); }
    static __device__ __forceinline__ uint32_t sort_ord(SortKey k) { return k & 0xffff0000u; }
    static __device__ __forceinline__ uint32_t sort_pos(SortKey k) { return 0xffffu - (k & 0xffffu); }
    static __device__ __forceinline__ float sort_value(SortKey k)
    {
        const uint32_t o = k & 0xffff0000u;
        return __uint_as_float((o & 0x80000000u) ? (o ^ 0x80000000u) : (~o & 0xffff0000u));
    }
};

struct F32Elem {
    static constexpr int VEC = 4;
    static constexpr int ESZ = 4;
    static __device__ __forceinline__ void unpack(const u32x4 w, float (&f)[VEC])
    {
        f[0] = __uint_as_float(w.x); f[1] = __uint_as_float(w.y);
        f[2] = __uint_as_float(w.z); f[3] = __uint_as_float(w.w);
    }
    static __device__ __forceinline__ float load1(const char *row, int64_t i) { return ((const float *)row)[i]; }
    using SortKey = uint64_t;               // 32 value bits, then the complement of the position
    static __device__ __forceinline__ SortKey make_sort(uint32_t ord, uint32_t pos) { return ((uint64_t)ord << 32) | (uint64_t)(0xffffffffu - pos); }
    static __device__ __forceinline__ uint32_t sort_ord(SortKey k) { return (uint32_t)(k >> 32); }
    static __device__ __forceinline__ uint32_t sort_pos(SortKey k) { return 0xffffffffu - (uint32_t)k; }
    static __device__ __forceinline__ float sort_value(SortKey k) { return unord32((uint32_t)(k >> 32)); }
};

// ---- chunk descriptors: (chunk maximum, chunk index) packed so that an unsigned compare orders
// them by (maximum desc, index asc).  Valid keys are never 0. --------------------------------

struct Key32 {                     // bf16 only: 16 value bits + 16 index bits
    using Key = uint32_t;
    static constexpr int KEYBITS = 32;
    static constexpr int VALBITS = 16;
    static __device__ __forceinline__ Key make(float cmax, uint32_t c) { return (ord32(cmax) & 0xffff0000u) | (0xffffu - c); }
    static __device__ __forceinline__ uint32_t ord(Key k) { return k & 0xffff0000u; }
    static __device__ __forceinline__ uint32_t chunk(Key k) { return 0xffffu - (k & 0xffffu); }
    static __device__ __forceinline__ float value(Key k)
    {
        uint32_t o = k & 0xffff0000u;
        return __uint_as_float((o & 0x80000000u) ? (o ^ 0x80000000u) : (~o & 0xffff0000u));
    }
};

struct Key64 {
    using Key = uint64_t;
    static constexpr int KEYBITS = 64;
    static constexpr int VALBITS = 32;
    static __device__ __forceinline__ Key make(float cmax, uint32_t c) { return ((uint64_t)ord32(cmax) << 32) | (uint64_t)(0xffffffffu - c); }
    static __device__ __forceinline__ uint32_t ord(Key k) { return (uint32_t)(k >> 32); }
    static __device__ __forceinline__ uint32_t chunk(Key k) { return 0xffffffffu - (uint32_t)k; }
    static __device__ __forceinline__ float value(Key k) { return unord32((uint32_t)(k >> 32)); }
};

template <class Key> __device__ __forceinline__ Key uniform_key(Key k);
template <> __device__ __forceinline__ uint32_t uniform_key<uint32_t>(uint32_t k) { return uniform_u(k); }
template <> __device__ __forceinline__ uint64_t uniform_key<uint64_t>(uint64_t k) { return uniform_u64(k); }

// Threshold the streaming loop compares chunk maxima against: the value part of `k`, or -inf
// while no threshold has been established.
template <class KT> __device__ __forceinline__ float threshold_value(typename KT::Key k)
{
    float v = KT::value(k);
    return (KT::ord(k) <= 0x007fffffu) ? neg_inf() : v;     // ord(-inf) = 0x007fffff
}

// ---- keep the k largest of cnt keys held in buf (LDS) -----------------------------------------
// Bitwise radix select over wave ballots.  After the value bits the loop may stop early: the
// prefix found so far is a lower bound of the k-th largest key with at least k keys above it,
// which is all the streaming filter needs.  exact=true runs every bit, leaving exactly
// min(cnt, k) keys.  Returns the new count; `prefix` receives the bound (0 if cnt < k).
template <class KT, int NS>
__device__ __forceinline__ int select_top_keys(typename KT::Key *buf, int cnt, int k, bool exact,
                                               int early_limit, typename KT::Key &prefix_out)
{
    using Key = typename KT::Key;
    const int lane = threadIdx.x;
    lds_sync();
    Key kk[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        int e = s * WAVE + lane;
        kk[s] = (e < cnt) ? buf[e] : (Key)0;
    }
    Key prefix = 0;
    int bit = KT::KEYBITS - 1;
    auto step = [&](int b) {
        Key cand = prefix | ((Key)1 << b);
        int n = 0;
#pragma unroll
        for (int s = 0; s < NS; ++s) n += __popcll(__ballot(kk[s] >= cand));
        if (n >= k) prefix = cand;
    };
    for (; bit >= KT::KEYBITS - KT::VALBITS; --bit) step(bit);
    int nge = 0;
#pragma unroll
    for (int s = 0; s < NS; ++s) nge += __popcll(__ballot(kk[s] >= prefix && kk[s] != 0));
    if (exact || nge > early_limit) {
        for (; bit >= 0; --bit) step(bit);
    }
    lds_sync();
    int n = 0;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        bool keep = kk[s] >= prefix && kk[s] != 0;
        uint64_t m = __ballot(keep);
        if (keep) buf[n + lane_prefix(m)] = kk[s];
        n += __popcll(m);
    }
    lds_sync();
    prefix_out = prefix;
    return n;
}

// Per-row, per-tensor streaming state.  Everything except `s` is wave-uniform.
template <class Key> struct Stream {
    float s;          // per-lane partial sum of 2^(l*log2e - M2)
    float M2;         // exponent reference (log2 domain)
    float mthr;       // logits above this force M2 to move
    float tauv;       // chunk maxima below this cannot enter the top-k
    Key tauk;         // exact form of the same bound (keys below it are not inserted)
    int cnt;          // descriptors currently buffered
    float d;          // policy stream only: per-lane sum of 2^(lp*log2e - M2) * (lp - lq)
};

template <class KT, int C, int NS>
__device__ __forceinline__ void offer_chunk(Stream<typename KT::Key> &st, typename KT::Key *buf,
                                            float cmax, uint32_t c, bool pass, int k)
{
    using Key = typename KT::Key;
    const Key key = KT::make(cmax, c);
    const bool ins = pass && key >= st.tauk;
    const uint64_t bm = __ballot(ins);
    if (bm) {
        if (ins) buf[st.cnt + lane_prefix(bm)] = key;
        st.cnt += __popcll(bm);
        if (st.cnt + WAVE > C) {
            Key pre;
            st.cnt = select_top_keys<KT, NS>(buf, st.cnt, k, false, C / 2, pre);
            pre = uniform_key<Key>(pre);
            st.tauk = pre > (Key)1 ? pre : (Key)1;
            st.tauv = uniform_f(threshold_value<KT>(st.tauk));
        }
    }
}

// A chunk maximum above st.mthr moves the exponent reference of the stream.
template <class Key>
__device__ __forceinline__ void raise_reference(Stream<Key> &st, float cmax, bool pass)
{
    const float wm = uniform_f(wave_max(pass ? cmax : neg_inf()));
    const float newM2 = wm * LOG2E_F;
    const float rescale = __builtin_amdgcn_exp2f(st.M2 - newM2);
    st.s *= rescale;
    st.d *= rescale;
    st.M2 = newM2;
    st.mthr = wm + RESCALE_MARGIN2 / LOG2E_F;
}

// log2 of a positive float sum: exponent plus hardware log2 of the mantissa in [1, 2), so the
// absolute error stays near 1e-7 whatever the magnitude.  0 -> -inf, inf/NaN propagate.
__device__ __forceinline__ double log2_of_sum(double S)
{
    const float f = (float)S;
    if (!(f > 0.f) || !(f < __uint_as_float(0x7f800000u))) return (double)__builtin_amdgcn_logf(f);
    const int e = __builtin_amdgcn_frexp_expf(f);            // f = m * 2^e, m in [0.5, 1)
    const float m2 = __builtin_amdgcn_frexp_mantf(f) * 2.0f;
    return (double)(e - 1) + (double)__builtin_amdgcn_logf(m2);
}

// Policy-row sum that also accumulates e_v (lp_v - lq_v), the numerator of the distillation
// term KL(p || q) = sum_v p_v (lp_v - lq_v) - (LSE_p - LSE_q) (Sec. 4.2 (3), Eq. distill_loss).
// lp_v = -inf gives e_v = 0; the difference is floored so that 0 * (-inf) cannot appear.
template <int VEC>
__device__ __forceinline__ float sum_exp2_kl(const float (&fp)[VEC], const float (&fq)[VEC], float M2, float &dacc)
{
    float a = 0.f, b = 0.f, da = 0.f, db = 0.f;
#pragma unroll
    for (int j = 0; j < VEC; j += 2) {
        const float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(fp[j], LOG2E_F, -M2));
        const float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(fp[j + 1], LOG2E_F, -M2));
        a += e0;
        b += e1;
        da = __builtin_fmaf(e0, fmaxf(fp[j] - fq[j], -1.0e30f), da);
        db = __builtin_fmaf(e1, fmaxf(fp[j + 1] - fq[j + 1], -1.0e30f), db);
    }
    dacc += da + db;
    return a + b;
}

template <int VEC> __device__ __forceinline__ float max_of(const float (&f)[VEC])
{
    float m = f[0];
#pragma unroll
    for (int j = 1; j < VEC; ++j) m = fmaxf(m, f[j]);
    return m;
}

template <int VEC> __device__ __forceinline__ float sum_exp2(const float (&f)[VEC], float M2)
{
    float a = 0.f, b = 0.f;
#pragma unroll
    for (int j = 0; j < VEC; j += 2) {
        a += __builtin_amdgcn_exp2f(__builtin_fmaf(f[j], LOG2E_F, -M2));
        b += __builtin_amdgcn_exp2f(__builtin_fmaf(f[j + 1], LOG2E_F, -M2));
    }
    return a + b;
}

// Load chunk c of a row: a plain 16-byte load for full chunks, element loads (padded with -inf)
// for the ragged tail chunk.
template <class ET>
__device__ __forceinline__ void load_chunk(const char *row, uint32_t c, uint32_t nfull, int tail,
                                           float (&f)[ET::VEC])
{
    if (c < nfull) {
        ET::unpack(as_global_vec(row)[c], f);
    } else {
#pragma unroll
        for (int j = 0; j < ET::VEC; ++j)
            f[j] = (j < tail) ? ET::load1(row, (int64_t)c * ET::VEC + j) : neg_inf();
    }
}

}  // namespace

// =================================================================================================
// Row kernel: S1-S5 of the hot path for one token position per wavefront.
// =================================================================================================
//
// CARRY = true is the vocabulary-chunked form used when the logits are produced chunk by chunk
// (fused lm_head): the row covers ids [id_base, id_base + V) of a vocabulary of V_total tokens,
// the running row state (exponent reference and sum of both rows, sampled-token logits, the two
// top-k lists so far with both logits of every entry) is read from / written to a per-row record,
// and only the launch of the last chunk runs the union / normaliser / acceptance step.
template <class ET, class KT, int KC, bool CARRY, bool DISTILL, bool STORED = false>
__global__ __launch_bounds__(64, (KC <= 64 ? (sizeof(typename KT::Key) > 4 ? 7 : 8) : (sizeof(typename KT::Key) > 4 ? 1 : (KC <= 128 ? 6 : 4)))) void row_kernel(RowArgs A)
{
    using Key = typename KT::Key;
    constexpr int VEC = ET::VEC;
    constexpr int C = (KC >= 256 ? 3 : 4) * KC;   // descriptor buffer capacity per tensor
    constexpr int NS = C / WAVE;
    constexpr int E = 2 * KC;             // element candidate capacity = keys of the sorting network
    constexpr int R = E / WAVE;
    using SK = typename ET::SortKey;

    // One LDS pool, used twice: during the sweep it holds the two descriptor buffers; once the
    // surviving descriptors sit in registers it holds the element candidates of the expansion.
    constexpr int DS = 2 * KC / WAVE;                               // descriptor registers per lane
    constexpr int DESC_BYTES = 2 * C * (int)sizeof(Key);
    constexpr int CAND_BYTES = E * ((int)sizeof(SK) + 8);
    constexpr int UNION_BYTES = (3 * KC + 2 * KC + (STORED ? 2 * KC : 0)) * 4;   // list 1, hash table, first-occurrence table
    constexpr int POOL_BYTES0 = DESC_BYTES > CAND_BYTES ? DESC_BYTES : CAND_BYTES;
    constexpr int POOL_BYTES = ((POOL_BYTES0 > UNION_BYTES ? POOL_BYTES0 : UNION_BYTES) + 15) / 16 * 16;
    __shared__ __attribute__((aligned(16))) unsigned char pool[POOL_BYTES];
    Key *const s_desc0 = (Key *)pool;
    Key *const s_desc1 = s_desc0 + C;
    SK *const s_key = (SK *)pool;                                   // candidate sort keys
    uint32_t *const s_cid = (uint32_t *)(pool + E * sizeof(SK));    // candidate token ids
    uint32_t *const s_oth = s_cid + E;                              // the other tensor's logit
    // The two ranked lists (ids, own logits, the other tensor's logits).  List 1 is only written
    // when the candidates of tensor 1 are no longer needed and takes their place in the pool.
    __shared__ uint32_t list0[3 * KC];
    uint32_t *const l_id[2] = {list0, (uint32_t *)pool};
    float *const l_a[2] = {(float *)(list0 + KC), (float *)pool + KC};
    float *const l_b[2] = {(float *)(list0 + 2 * KC), (float *)pool + 2 * KC};

    const int lane = threadIdx.x;
    const int64_t t = blockIdx.x;
    const int k = A.k;
    const int64_t V = A.V;
    const float NaN = __uint_as_float(0x7fc00000u);

    const int x = A.ids[t];
    const int64_t V_total = CARRY ? A.V_total : V;
    const int64_t id_base = CARRY ? A.id_base : 0;
    const bool carry_in = CARRY && A.carry_in, carry_out = CARRY && A.carry_out;
    unsigned char *const state = CARRY ? A.state + (size_t)t * (size_t)A.state_stride : nullptr;
    CarryHeader *const hdr = (CarryHeader *)state;
    uint32_t *const st_id0 = (uint32_t *)(state + sizeof(CarryHeader));     // [2][3][KC] words
    if (x < 0 || x >= V_total) {          // padding row, or a sampled id outside the vocabulary
        if (carry_out) return;            // reported by the launch of the last chunk
        const bool pad = x < 0;
        const float fill = pad ? 0.f : NaN;
        if (lane == 0) {
            A.rowflag[t] = pad ? ROW_PADDING : ROW_BAD_ID;
            A.accept[t] = fill; A.logq[t] = fill; A.logp[t] = fill; A.logratio[t] = fill;
            A.zapprox[t] = fill; A.lse_q[t] = fill; A.lse_p[t] = fill;
            if (A.mask) A.mask[t] = 0;
            if (A.usize) A.usize[t] = 0;
            if (DISTILL) A.kl[t] = fill;
        }
        for (int r = lane; r < k; r += WAVE) {
            if (A.topk_a) A.topk_a[t * k + r] = -1;
            if (A.topk_p) A.topk_p[t * k + r] = -1;
            if (A.topk_a_lq) A.topk_a_lq[t * k + r] = fill;
            if (A.topk_p_lp) A.topk_p_lp[t * k + r] = fill;
        }
        return;
    }

    const char *rowq = (const char *)A.actor + (size_t)t * (size_t)A.stride * ET::ESZ;
    const char *rowp = (const char *)A.policy + (size_t)t * (size_t)A.stride * ET::ESZ;
    const gvec_ptr vq = as_global_vec(rowq);
    const gvec_ptr vp = as_global_vec(rowp);
    const uint32_t nfull = (uint32_t)(V / VEC);
    const int tail = (int)(V - (int64_t)nfull * VEC);
    const uint32_t nchunks = nfull + (tail ? 1u : 0u);
    const uint32_t nit = nfull / WAVE;

    Stream<Key> sq{0.f, M2_UNSET, -2.0e38f, neg_inf(), (Key)1, 0};
    Stream<Key> sp{0.f, M2_UNSET, -2.0e38f, neg_inf(), (Key)1, 0};
    int nl_in[2] = {0, 0};                // entries of the carried top-k lists
    float xq_in = 0.f, xp_in = 0.f;
    int have_x = 0;
    if (carry_in) {
        // Resume the scan: the carried sums go to lane 0, and a full carried list bounds what can
        // still enter the top-k (its k-th value), exactly as if the sweep had never stopped.
        sq.M2 = hdr->M2[0]; sp.M2 = hdr->M2[1];
        if (lane == 0) { sq.s = (float)hdr->S[0]; sp.s = (float)hdr->S[1]; sp.d = (float)hdr->D; }
        if (sq.M2 != M2_UNSET) sq.mthr = (sq.M2 + RESCALE_MARGIN2) / LOG2E_F;
        if (sp.M2 != M2_UNSET) sp.mthr = (sp.M2 + RESCALE_MARGIN2) / LOG2E_F;
        nl_in[0] = hdr->nl[0]; nl_in[1] = hdr->nl[1];
        xq_in = hdr->x_logit[0]; xp_in = hdr->x_logit[1]; have_x = hdr->have_x;
        if (nl_in[0] >= k) {
            const float vk = __uint_as_float(st_id0[(0 * 3 + 1) * KC + (k - 1)]);
            const Key b = KT::make(vk, 0xffffffffu);
            sq.tauk = b > (Key)1 ? b : (Key)1;
            sq.tauv = threshold_value<KT>(sq.tauk);
        }
        if (nl_in[1] >= k) {
            const float vk = __uint_as_float(st_id0[(1 * 3 + 1) * KC + (k - 1)]);
            const Key b = KT::make(vk, 0xffffffffu);
            sp.tauk = b > (Key)1 ? b : (Key)1;
            sp.tauv = threshold_value<KT>(sp.tauk);
        }
    }

    auto consume = [&](const float (&fq)[VEC], const float (&fp)[VEC], uint32_t c, bool valid) {
        const float mq = STORED ? 0.f : max_of<VEC>(fq), mp = max_of<VEC>(fp);
        const bool pq = !STORED && valid && (mq >= sq.tauv);
        const bool pp = valid && (mp >= sp.tauv);
        const uint64_t bq = STORED ? 0 : __ballot(pq), bp = __ballot(pp);
        if (bq | bp) {
            if (bq) offer_chunk<KT, C, NS>(sq, s_desc0, mq, c, pq, k);
            if (bp) offer_chunk<KT, C, NS>(sp, s_desc1, mp, c, pp, k);
            // a value above the margin of an exponent reference is also above the top-k bound
            const bool rq = pq && mq > sq.mthr, rp = pp && mp > sp.mthr;
            if (__ballot(rq || rp)) {
                if (__ballot(rq)) raise_reference(sq, mq, pq);
                if (__ballot(rp)) raise_reference(sp, mp, pp);
            }
        }
        if constexpr (!STORED) sq.s += sum_exp2<VEC>(fq, sq.M2);
        if constexpr (DISTILL) sp.s += sum_exp2_kl<VEC>(fp, fq, sp.M2, sp.d);
        else sp.s += sum_exp2<VEC>(fp, sp.M2);
    };

    // ---- streaming sweep: iterations in which every lane owns a full 16-byte chunk ----------
    if (nit > 0) {
        // Two 16-byte loads per tensor stay in flight per lane: the loads for iterations it+2 and
        // it+3 are issued before iterations it and it+1 are consumed (indices clamp at the end).
        const uint32_t last = nit - 1;
        const uint32_t second = (last < 1u ? last : 1u) * WAVE + lane;
        u32x4 wq0 = stream_load(vq + lane), wp0 = stream_load(vp + lane);
        u32x4 wq1 = stream_load(vq + second), wp1 = stream_load(vp + second);
        for (uint32_t it = 0; it < nit; it += 2) {
            const u32x4 cq0 = wq0, cp0 = wp0, cq1 = wq1, cp1 = wp1;
            const uint32_t n0 = (it + 2 < last ? it + 2 : last) * WAVE + lane;
            const uint32_t n1 = (it + 3 < last ? it + 3 : last) * WAVE + lane;
            wq0 = stream_load(vq + n0); wp0 = stream_load(vp + n0);
            wq1 = stream_load(vq + n1); wp1 = stream_load(vp + n1);
            float fq[VEC], fp[VEC];
            ET::unpack(cq0, fq);
            ET::unpack(cp0, fp);
            consume(fq, fp, it * WAVE + lane, true);
            if (it + 1 < nit) {
                ET::unpack(cq1, fq);
                ET::unpack(cp1, fp);
                consume(fq, fp, (it + 1) * WAVE + lane, true);
            }
        }
    }
    // ---- remainder: fewer than 64 chunks, the last of which may be ragged ------------------------
    {
        const uint32_t c = nit * WAVE + lane;
        if (nit * WAVE < nchunks) {
            float fq[VEC], fp[VEC];
            const bool valid = c < nchunks;
            if (valid) {
                if constexpr (!STORED) load_chunk<ET>(rowq, c, nfull, tail, fq);
                load_chunk<ET>(rowp, c, nfull, tail, fp);
            } else {
#pragma unroll
                for (int j = 0; j < VEC; ++j) { fq[j] = neg_inf(); fp[j] = neg_inf(); }
            }
            consume(fq, fp, c, valid);
        }
    }

    // ---- log-sum-exp of both rows (log2 domain until the last step) -----------------------------
    const double Sq = wave_sum((double)sq.s), Sp = wave_sum((double)sp.s);
    const double Dp = DISTILL ? wave_sum((double)sp.d) : 0.0;
    // stored form: the actor side arrives as log-probabilities, i.e. logits whose log-sum-exp is 0
    const double lse_q = STORED ? 0.0 : ((double)sq.M2 + log2_of_sum(Sq)) * LN2_D;
    const double lse_p = ((double)sp.M2 + log2_of_sum(Sp)) * LN2_D;
    const double ln_lambda = A.ln_lambda;

    // logits of the sampled token (from this chunk if it holds x, else the carried ones)
    const bool x_here = (int64_t)x >= id_base && (int64_t)x < id_base + V;
    const float xq = STORED ? A.stored_logq_x[t] : (x_here ? ET::load1(rowq, (int64_t)x - id_base) : xq_in);
    const float xp = x_here ? ET::load1(rowp, (int64_t)x - id_base) : xp_in;
    const double lq_x = (double)xq, lp_x = (double)xp;
    const double logq_x = lq_x - lse_q, logp_x = lp_x - lse_p;
    const double logratio = logp_x - logq_x;
    // a = min(1, p(x) / (lambda q(x))), taken in the log2 domain
    double acc = (double)__builtin_amdgcn_exp2f((float)((logratio - ln_lambda) * LOG2E_D));
    acc = acc < 1.0 ? acc : 1.0;
    const bool finite_row = isfinite(lse_q) && isfinite(lse_p) && isfinite(logratio);

    // ---- top-k of both rows: k best chunks -> their elements -> rank by (value desc, id asc) ----
    Key kth[2];
    int nc[2];
    // The value bits of the k-th largest chunk maximum are enough: every chunk at or above that
    // value is expanded and the element ranking below is exact.  Only a large plateau of equal
    // maxima makes the select run to the last bit (leaving exactly k chunks).
    nc[0] = STORED ? 0 : uniform_i(select_top_keys<KT, NS>(s_desc0, sq.cnt, k, false, 2 * KC, kth[0]));
    nc[1] = uniform_i(select_top_keys<KT, NS>(s_desc1, sp.cnt, k, false, 2 * KC, kth[1]));
    Key dk[2][DS];                                                  // at most 2*KC survive per tensor
#pragma unroll
    for (int sl = 0; sl < DS; ++sl) {
        const int e = sl * WAVE + lane;
        dk[0][sl] = (!STORED && e < nc[0]) ? s_desc0[e] : (Key)0;
        dk[1][sl] = e < nc[1] ? s_desc1[e] : (Key)0;
    }
    lds_sync();                                                     // the pool now belongs to the candidates

    int nl[2];
    auto expand = [&](auto tensor_c) {
        constexpr int i = decltype(tensor_c)::value;
        const char *rowA = i == 0 ? rowq : rowp;     // the tensor ranked here
        const char *rowB = i == 0 ? rowp : rowq;     // the other one
        // A candidate needs ord >= thr_ord (the k-th largest chunk maximum) and, once k candidates
        // have been ranked, ord > above_ord (their k-th value: all of them have smaller ids).
        uint32_t thr_ord = (nc[i] >= k) ? KT::ord(uniform_key<Key>(kth[i])) : 0u;
        uint32_t above_ord = 0u;
        bool have_above = false;
        int nS = 0;
        if (CARRY && nl_in[i] > 0) {
            // The carried list seeds the candidates (all its ids are below this chunk's); when it
            // is full its k-th value is a second lower bound of the final k-th value.
            const uint32_t *cid = st_id0 + (i * 3 + 0) * KC, *ca = cid + KC, *cb = ca + KC;
            for (int r = lane; r < nl_in[i]; r += WAVE) {
                s_key[r] = ET::make_sort(ord32(__uint_as_float(ca[r])), (uint32_t)r);
                s_cid[r] = cid[r];
                s_oth[r] = cb[r];
            }
            nS = nl_in[i];
            if (nl_in[i] >= k) {
                const uint32_t ok = ord32(__uint_as_float(ca[k - 1]));
                thr_ord = ok > thr_ord ? ok : thr_ord;
            }
        }

        // The other tensor's logit of a candidate is fetched once the candidate set is known
        // (entries [filled, nS) still lack it); the loads of one pass are independent.
        int filled = nS;
        auto fill_other = [&]() {
            lds_sync();
            for (int e = filled + lane; e < nS; e += WAVE)
                s_oth[e] = STORED ? 0u : __float_as_uint(ET::load1(rowB, (int64_t)s_cid[e] - id_base));
            filled = nS;
        };
        // Sort the nS buffered candidates.  Candidates are buffered in ascending id order among
        // equal values, and the key carries the buffer position, so the descending sort is the
        // (value desc, id asc) order.  Lane l ends up with ranks l R .. l R + R - 1 and the id and
        // other-tensor logit that go with them.
        SK v[R];
        uint32_t gid[R], goth[R];
        auto sort_candidates = [&]() {
            lds_sync();
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int e = lane * R + r;
                v[r] = e < nS ? s_key[e] : (SK)0;
            }
            bitonic_sort_desc<SK, R>(v, lane);
            const int keep = nS < k ? nS : k;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                uint32_t pos = ET::sort_pos(v[r]);
                pos = pos < (uint32_t)(E - 1) ? pos : (uint32_t)(E - 1);
                const bool live = lane * R + r < keep;
                gid[r] = live ? s_cid[pos] : 0u;
                goth[r] = live ? s_oth[pos] : 0u;
            }
            lds_sync();                                   // everything needed from the buffer is in registers
            return keep;
        };
        // Make room: keep only the k best so far, in rank order (which keeps equal values in id order).
        auto compact = [&]() {
            fill_other();
            const int keep = sort_candidates();
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int q = lane * R + r;
                if (q < keep) {
                    s_key[q] = ET::make_sort(ord32(ET::sort_value(v[r])), (uint32_t)q);
                    s_cid[q] = gid[r];
                    s_oth[q] = goth[r];
                }
            }
            nS = keep;
            filled = keep;
            lds_sync();
            if (keep >= k) {
                const SK kk = s_key[k - 1];
                above_ord = uniform_u(ord32(ET::sort_value(kk)));
                have_above = true;
            }
        };

        // The surviving chunks of this tensor are requested up to four per lane at a time, before
        // the first of them is looked at.
        constexpr int PF = DS > 4 ? 4 : DS;
        u32x4 raw[PF];
#pragma unroll
        for (int sl = 0; sl < DS; ++sl) {
            if (sl * WAVE >= nc[i]) break;
            if (sl % PF == 0) {
#pragma unroll
                for (int u = 0; u < PF; ++u) {
                    const bool full = (sl + u) * WAVE + lane < nc[i] && KT::chunk(dk[i][sl + u]) < nfull;
                    raw[u] = full ? as_global_vec(rowA)[KT::chunk(dk[i][sl + u])] : u32x4{0u, 0u, 0u, 0u};
                }
            }
            const bool has = sl * WAVE + lane < nc[i];
            const uint32_t c = has ? KT::chunk(dk[i][sl]) : 0u;
            float fa[VEC];
            if (has && c < nfull) {
                ET::unpack(raw[sl % PF], fa);
            } else if (has) {
                load_chunk<ET>(rowA, c, nfull, tail, fa);            // the ragged last chunk
            } else {
#pragma unroll
                for (int j = 0; j < VEC; ++j) fa[j] = neg_inf();
            }
            // bit j: element j of this lane's chunk is a candidate
            auto candidates = [&](bool mine) {
                uint32_t m = 0;
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    const uint32_t o = ord32(fa[j]);
                    const bool ok = mine && (int64_t)c * VEC + j < V && o >= thr_ord && (!have_above || o > above_ord);
                    m |= ok ? (1u << j) : 0u;
                }
                return m;
            };
            // Descriptors are in ascending chunk order, so appending lane by lane, element by
            // element keeps the buffer in ascending id order.
            auto append = [&](uint32_t m) {
                const int cnt = __popc(m);
                int pre = 0, tot = 0;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const uint64_t bm = __ballot((cnt >> b) & 1);
                    pre += lane_prefix(bm) << b;
                    tot += __popcll(bm) << b;
                }
                uint32_t pos = (uint32_t)(nS + pre);
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    if ((m >> j) & 1u) {
                        s_key[pos] = ET::make_sort(ord32(fa[j]), pos);
                        s_cid[pos] = (uint32_t)(id_base + (int64_t)c * VEC + j);
                        ++pos;
                    }
                }
                nS += tot;
            };
            const uint32_t m_all = candidates(has);
            if (nS + wave_sum_i(__popc(m_all)) <= E) {
                append(m_all);
            } else {
                // Too many for the buffer at once: eight lanes (at most 64 candidates) at a time,
                // ranking and keeping the k best whenever the next group might not fit.
                for (int g = 0; g < WAVE / 8; ++g) {
                    if (nS + WAVE > E) compact();
                    append(candidates(has && (lane >> 3) == g));
                }
            }
        }
        fill_other();
        nl[i] = sort_candidates();
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int q = lane * R + r;
            if (q < nl[i]) {
                l_id[i][q] = gid[r];
                l_a[i][q] = ET::sort_value(v[r]);
                l_b[i][q] = __uint_as_float(goth[r]);
            }
        }
        lds_sync();
    };
    if constexpr (STORED) nl[0] = 0;
    else expand(std::integral_constant<int, 0>{});
    expand(std::integral_constant<int, 1>{});

    // Chunked stored form: the target logit of a stored id is picked up by the launch whose chunk
    // holds it and kept in the row record (in list 0's id slots, which this form never uses).
    float *const st_slp = (float *)st_id0;
    if constexpr (CARRY && STORED) {
        for (int r = lane; r < k; r += WAVE) {
            const int64_t id = (int64_t)A.stored_ids[t * k + r];
            if (id >= id_base && id < id_base + V) st_slp[r] = ET::load1(rowp, id - id_base);
        }
    }

    if (carry_out) {                      // hand the row state to the launch of the next chunk
        if (lane == 0) {
            hdr->M2[0] = sq.M2; hdr->M2[1] = sp.M2;
            hdr->S[0] = Sq; hdr->S[1] = Sp; hdr->D = Dp;
            hdr->nl[0] = nl[0]; hdr->nl[1] = nl[1];
            hdr->x_logit[0] = xq; hdr->x_logit[1] = xp;
            hdr->have_x = (have_x || x_here) ? 1 : 0;
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            uint32_t *cid = st_id0 + (i * 3 + 0) * KC, *ca = cid + KC, *cb = ca + KC;
            for (int r = lane; r < nl[i]; r += WAVE) {
                cid[r] = l_id[i][r];
                ca[r] = __float_as_uint(l_a[i][r]);
                cb[r] = __float_as_uint(l_b[i][r]);
            }
        }
        return;
    }

    // ---- V_k = union of the two lists; Z_approx = sum over V_k of min(q, p/lambda) -------------
    // In the log domain min(q, p/lambda) = exp(min(lq - LSEq, lp - LSEp - ln lambda)).
    double zsum = 0.0;
    int ucount = 0;
    // Membership of the policy list's ids in the actor list through a small open-addressing hash
    // table (load factor <= 1/2) in the LDS pool, behind list 1.
    constexpr int HT = 2 * KC;
    uint32_t *const tab = (uint32_t *)pool + 3 * KC;
    auto table_insert = [&](uint32_t id) {                  // returns the slot that holds id
        uint32_t slot = (id * 2654435761u) >> 7 & (HT - 1);
        for (int tries = 0; tries < HT; ++tries) {
            const uint32_t old = atomicCAS(&tab[slot], 0xffffffffu, id);
            if (old == 0xffffffffu || old == id) break;
            slot = (slot + 1) & (HT - 1);
        }
        return slot;
    };
    double tail_dq = 0.0;                 // stored form: log q assumed for a token outside the stored list
    if constexpr (STORED) {
        // The actor list as the rollout phase stored it (Alg. 1, Phase 1): ids and log-probabilities.
        // A slot with an id outside [0, V) is unused; of a repeated id the first occurrence counts
        // (decided by an atomic minimum over positions, so the outcome does not depend on timing).
        uint32_t *const first = tab + HT;
        constexpr int SR = KC / WAVE;
        uint32_t sid[SR], sslot[SR];
        float slq[SR];
        lds_sync();
        for (int e = lane; e < 2 * HT; e += WAVE) tab[e] = 0xffffffffu;     // table and first[]
        lds_sync();
#pragma unroll
        for (int s2 = 0; s2 < SR; ++s2) {
            const int r = s2 * WAVE + lane;
            const int32_t raw_id = r < k ? A.stored_ids[t * k + r] : -1;
            const bool ok = raw_id >= 0 && (int64_t)raw_id < V_total;
            sid[s2] = ok ? (uint32_t)raw_id : 0xffffffffu;
            slq[s2] = ok ? A.stored_logq[t * k + r] : 0.f;
            sslot[s2] = 0;
            if (ok) {
                sslot[s2] = table_insert(sid[s2]);
                atomicMin(&first[sslot[s2]], (uint32_t)r);
            }
        }
        lds_sync();
        float kth = __uint_as_float(0x7f800000u);           // smallest stored log-probability
        double mass = 0.0;
        int n = 0;
#pragma unroll
        for (int s2 = 0; s2 < SR; ++s2) {
            const int r = s2 * WAVE + lane;
            const bool keep = sid[s2] != 0xffffffffu && first[sslot[s2]] == (uint32_t)r;
            if (keep) {
                const double dq = (double)slq[s2];
                // (the lane that wrote record entry r above is the lane that reads it here)
                const float lp_s = CARRY ? st_slp[r] : ET::load1(rowp, (int64_t)sid[s2]);
                const double dp = (double)lp_s - lse_p - ln_lambda;
                zsum += (double)__builtin_amdgcn_exp2f((float)((dq < dp ? dq : dp) * LOG2E_D));
                mass += (double)__builtin_amdgcn_exp2f((float)(dq * LOG2E_D));
                kth = fminf(kth, slq[s2]);
                ucount += 1;
            }
        }
        n = wave_sum_i(ucount);
        kth = -uniform_f(wave_max(-kth));
        mass = wave_sum(mass);
        if (n == 0) kth = 0.f;                              // nothing stored: the bound is log 1
        const double neg_inf_d = -__builtin_inf();
        if (A.tail_rule == 0 || (int64_t)n == V_total) {
            tail_dq = neg_inf_d;
        } else if (A.tail_rule == 1) {
            tail_dq = (double)kth;
        } else {
            const double rest = mass < 1.0 ? 1.0 - mass : 0.0;
            const double share = rest / (double)(V_total - n);
            tail_dq = share > 0.0 ? (double)(__builtin_amdgcn_logf((float)share)) * LN2_D : neg_inf_d;
            tail_dq = tail_dq < (double)kth ? tail_dq : (double)kth;
        }
    } else {
        for (int r = lane; r < nl[0]; r += WAVE) {
            const double dq = (double)l_a[0][r] - lse_q;
            const double dp = (double)l_b[0][r] - lse_p - ln_lambda;
            zsum += (double)__builtin_amdgcn_exp2f((float)((dq < dp ? dq : dp) * LOG2E_D));
            ucount += 1;
            if (A.topk_a) A.topk_a[t * k + r] = (int32_t)l_id[0][r];
            if (A.topk_a_lq) A.topk_a_lq[t * k + r] = finite_row ? (float)dq : NaN;
        }
        lds_sync();
        for (int e = lane; e < HT; e += WAVE) tab[e] = 0xffffffffu;
        lds_sync();
        for (int r = lane; r < nl[0]; r += WAVE) table_insert(l_id[0][r]);
    }
    lds_sync();
    for (int r = lane; r < nl[1]; r += WAVE) {
        const uint32_t id = l_id[1][r];
        bool dup = false;
        uint32_t slot = (id * 2654435761u) >> 7 & (HT - 1);
        for (int tries = 0; tries < HT; ++tries) {
            const uint32_t v = tab[slot];
            if (v == id) { dup = true; break; }
            if (v == 0xffffffffu) break;
            slot = (slot + 1) & (HT - 1);
        }
        const double dp0 = (double)l_a[1][r] - lse_p;
        const double dq = STORED ? tail_dq : (double)l_b[1][r] - lse_q;
        const double dp = dp0 - ln_lambda;
        if (!dup) {
            zsum += (double)__builtin_amdgcn_exp2f((float)((dq < dp ? dq : dp) * LOG2E_D));
            ucount += 1;
        }
        if (A.topk_p) A.topk_p[t * k + r] = (int32_t)id;
        if (A.topk_p_lp) A.topk_p_lp[t * k + r] = finite_row ? (float)dp0 : NaN;
    }
    const double z_approx = wave_sum(zsum);
    const int usize = wave_sum_i(ucount);

    if (lane == 0) {
        A.rowflag[t] = finite_row ? ROW_OK : ROW_NONFINITE;
        A.lse_q[t] = lse_q;
        A.lse_p[t] = lse_p;
        A.logq[t] = finite_row ? (float)logq_x : NaN;
        A.logp[t] = finite_row ? (float)logp_x : NaN;
        A.logratio[t] = finite_row ? (float)logratio : NaN;
        A.accept[t] = finite_row ? (float)acc : NaN;
        A.zapprox[t] = finite_row ? (float)z_approx : NaN;
        if (A.mask) A.mask[t] = (finite_row && A.uni && (double)A.uni[t] < acc) ? 1 : 0;
        if (A.usize) A.usize[t] = usize;
        // KL(p || q) = sum_v p_v (lp_v - lq_v) - (LSE_p - LSE_q)
        if (DISTILL) A.kl[t] = finite_row ? (float)(Dp / Sp - (lse_p - lse_q)) : NaN;
    }
}

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

template <class ET, class KT>
static hipError_t launch_rows_k(const RowArgs &a, hipStream_t st)
{
    const dim3 grid((unsigned)a.T), block(WAVE);
    if (a.distill) {
        if (a.k <= 64) hipLaunchKernelGGL((row_kernel<ET, KT, 64, false, true>), grid, block, 0, st, a);
        else if (a.k <= 128) hipLaunchKernelGGL((row_kernel<ET, KT, 128, false, true>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((row_kernel<ET, KT, 256, false, true>), grid, block, 0, st, a);
    } else {
        if (a.k <= 64) hipLaunchKernelGGL((row_kernel<ET, KT, 64, false, false>), grid, block, 0, st, a);
        else if (a.k <= 128) hipLaunchKernelGGL((row_kernel<ET, KT, 128, false, false>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((row_kernel<ET, KT, 256, false, false>), grid, block, 0, st, a);
    }
    return hipGetLastError();
}

hipError_t launch_rows_carry(const RowArgs &a, hipStream_t st)
{
    if (a.T <= 0) return hipSuccess;
    const dim3 grid((unsigned)a.T), block(WAVE);
    if (a.distill) {
        if (a.k <= 64) hipLaunchKernelGGL((row_kernel<F32Elem, Key64, 64, true, true>), grid, block, 0, st, a);
        else if (a.k <= 128) hipLaunchKernelGGL((row_kernel<F32Elem, Key64, 128, true, true>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((row_kernel<F32Elem, Key64, 256, true, true>), grid, block, 0, st, a);
    } else {
        if (a.k <= 64) hipLaunchKernelGGL((row_kernel<F32Elem, Key64, 64, true, false>), grid, block, 0, st, a);
        else if (a.k <= 128) hipLaunchKernelGGL((row_kernel<F32Elem, Key64, 128, true, false>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((row_kernel<F32Elem, Key64, 256, true, false>), grid, block, 0, st, a);
    }
    return hipGetLastError();
}

hipError_t launch_rows_carry_stored(const RowArgs &a, hipStream_t st)
{
    if (a.T <= 0) return hipSuccess;
    const dim3 grid((unsigned)a.T), block(WAVE);
    if (a.k <= 64) hipLaunchKernelGGL((row_kernel<F32Elem, Key64, 64, true, false, true>), grid, block, 0, st, a);
    else if (a.k <= 128) hipLaunchKernelGGL((row_kernel<F32Elem, Key64, 128, true, false, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((row_kernel<F32Elem, Key64, 256, true, false, true>), grid, block, 0, st, a);
    return hipGetLastError();
}

hipError_t launch_rows(const RowArgs &a, int dtype, hipStream_t st)
{
    if (a.T <= 0) return hipSuccess;
    if (dtype == JP_BF16) {
        const int64_t nchunks = (a.V + Bf16Elem::VEC - 1) / Bf16Elem::VEC;
        if (nchunks <= 65535) return launch_rows_k<Bf16Elem, Key32>(a, st);
        return launch_rows_k<Bf16Elem, Key64>(a, st);
    }
    return launch_rows_k<F32Elem, Key64>(a, st);
}

template <class ET, class KT>
static hipError_t launch_rows_stored_k(const RowArgs &a, hipStream_t st)
{
    const dim3 grid((unsigned)a.T), block(WAVE);
    if (a.k <= 64) hipLaunchKernelGGL((row_kernel<ET, KT, 64, false, false, true>), grid, block, 0, st, a);
    else if (a.k <= 128) hipLaunchKernelGGL((row_kernel<ET, KT, 128, false, false, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((row_kernel<ET, KT, 256, false, false, true>), grid, block, 0, st, a);
    return hipGetLastError();
}

hipError_t launch_rows_stored(const RowArgs &a, int dtype, hipStream_t st)
{
    if (a.T <= 0) return hipSuccess;
    if (dtype == JP_BF16) {
        const int64_t nchunks = (a.V + Bf16Elem::VEC - 1) / Bf16Elem::VEC;
        if (nchunks <= 65535) return launch_rows_stored_k<Bf16Elem, Key32>(a, st);
        return launch_rows_stored_k<Bf16Elem, Key64>(a, st);
    }
    return launch_rows_stored_k<F32Elem, Key64>(a, st);
}

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
