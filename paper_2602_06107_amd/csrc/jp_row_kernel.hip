// OBRS hot path of Jackpot for gfx950 (MI355X): the row kernel.
//
// One 64-lane wavefront owns one token position.  It streams the actor and the policy logit
// rows once with 16-byte loads and keeps, per row:
//   * a running sum of 2^(l*log2(e) - M2) against a wave-uniform reference M2 (log-sum-exp),
//   * a bounded buffer of "chunk descriptors" (chunk maximum, chunk index) in LDS from which
//     the k chunks with the largest maxima survive (the k largest elements of a row always lie
//     inside the k chunks with the largest maxima),
// then expands the surviving chunks into elements, ranks them by (logit desc, id asc), forms the
// union of the two top-k lists and the normaliser estimate of Sec. 4.4.1, and the per-token
// acceptance probability of Eq. obrs_accept.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "jp_device_utils.h"
#include "jp_obrs_internal.h"

namespace jp {

namespace {

// Candidate key for the final ranking: the logit's order-preserving bits, then the complement of
// the candidate's position in the buffer.  Candidates are buffered in ascending id order, so an
// unsigned compare orders the keys by (value desc, id asc).
template <class ET> struct SortOf;
template <> struct SortOf<Bf16Elem> {
    using SortKey = uint32_t;               // 16 value bits + 16 position bits
    static __device__ __forceinline__ SortKey make_sort(uint32_t ord, uint32_t pos) { return (ord & 0xffff0000u) | (0xffffu - pos); }
    static __device__ __forceinline__ uint32_t sort_pos(SortKey k) { return 0xffffu - (k & 0xffffu); }
    static __device__ __forceinline__ float sort_value(SortKey k)
    {
        const uint32_t o = k & 0xffff0000u;
        return __uint_as_float((o & 0x80000000u) ? (o ^ 0x80000000u) : (~o & 0xffff0000u));
    }
};
template <> struct SortOf<F32Elem> {
    using SortKey = uint64_t;               // 32 value bits, then the complement of the position
    static __device__ __forceinline__ SortKey make_sort(uint32_t ord, uint32_t pos) { return ((uint64_t)ord << 32) | (uint64_t)(0xffffffffu - pos); }
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
    const int lane = threadIdx.x & (WAVE - 1);
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
    float hi, dhi;    // fp32 logits only: what `s` / `d` held at the last fold of the two-level sum
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
template <bool TWO_LEVEL, class Key>
__device__ __forceinline__ void raise_reference(Stream<Key> &st, float cmax, bool pass)
{
    const float wm = uniform_f(wave_max(pass ? cmax : neg_inf()));
    const float newM2 = wm * LOG2E_F;
    const float rescale = __builtin_amdgcn_exp2f(st.M2 - newM2);
    st.s *= rescale;
    st.d *= rescale;
    if constexpr (TWO_LEVEL) { st.hi *= rescale; st.dhi *= rescale; }
    st.M2 = newM2;
    st.mthr = wm + RESCALE_MARGIN2 / LOG2E_F;
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
//
// W > 1 gives a row to W wavefronts of one workgroup (for batches too small to fill the chip with
// one wave per row, where a single wave's instruction stream, not the memory system, sets the
// time of a row): wave w sweeps the w-th of W contiguous runs of chunks with descriptor buffers of
// its own and keeps its best C / W descriptors per tensor; then the sums of all waves go to wave 0
// and the surviving descriptors are put together in wave order (which is chunk order, so ties
// still resolve towards the smaller id).  With two tensors wave 0 ranks the actor's top-k while
// wave 1 ranks the policy's in a candidate pool of its own and hands the list over through LDS;
// wave 0 alone runs the union and the outputs exactly as for W = 1.  In the stored-actor form
// wave 0 does all of it.  In the chunked forms the carried sums enter through wave 0, every wave
// starts from the carried thresholds, and wave 0 writes the record.
template <class ET, class KT, int KC, bool CARRY, bool DISTILL, bool STORED = false, int W = 1>
__global__ __launch_bounds__(64 * W, (KC <= 64 ? (sizeof(typename KT::Key) > 4 ? 7 : 8) : (sizeof(typename KT::Key) > 4 ? 1 : (KC <= 128 ? 6 : 4)))) void row_kernel(RowArgs A)
{
    using Key = typename KT::Key;
    constexpr int VEC = ET::VEC;
    constexpr int C = (KC >= 256 ? 3 : 4) * KC;   // descriptor buffer capacity per tensor
    constexpr int NS = C / WAVE;
    constexpr int E = 2 * KC;             // element candidate capacity = keys of the sorting network
    constexpr int R = E / WAVE;
    using SO = SortOf<ET>;
    using SK = typename SO::SortKey;
    const int lane = threadIdx.x & (WAVE - 1);
    const int wv = W > 1 ? __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)) : 0;
    // Split rows with two tensors: after the sweep wave 0 ranks the actor's top-k while wave 1 ranks
    // the policy's, each with a candidate pool of its own.
    constexpr bool PAR = W > 1 && !STORED;

    // One LDS pool, used twice: during the sweep it holds the two descriptor buffers; once the
    // surviving descriptors sit in registers it holds the element candidates of the expansion.
    constexpr int DS = 2 * KC / WAVE;                               // descriptor registers per lane
    constexpr int DESC_BYTES = 2 * C * (int)sizeof(Key);
    constexpr int CAND_BYTES = E * ((int)sizeof(SK) + 8);
    constexpr int UNION_BYTES = (3 * KC + 2 * KC + (STORED ? 2 * KC : 0)) * 4;   // list 1, hash table, first-occurrence table
    constexpr int POOL_BYTES0 = DESC_BYTES > CAND_BYTES ? DESC_BYTES : CAND_BYTES;
    constexpr int POOL_BYTES = ((POOL_BYTES0 > UNION_BYTES ? POOL_BYTES0 : UNION_BYTES) + 15) / 16 * 16;
    __shared__ __attribute__((aligned(16))) unsigned char pool[POOL_BYTES];
    // split rows: descriptor buffers of waves 1 .. W-1, and what every wave hands to wave 0
    static_assert(W == 1 || W * KC <= C, "C / W descriptors per wave must hold the k best");
    __shared__ __attribute__((aligned(16))) Key s_more[W > 1 ? (W - 1) * 2 * C : 1];
    static_assert(!PAR || CAND_BYTES <= DESC_BYTES, "wave 1 reuses its descriptor buffers as its candidate pool");
    __shared__ double s_part[W > 1 ? W : 1][3];                     // sums of actor / policy, distillation sum
    __shared__ float s_pref[W > 1 ? W : 1][2];                      // their exponent references
    __shared__ int s_pcnt[W > 1 ? W : 1][2];                        // descriptors kept
    Key *const s_desc0 = (W > 1 && wv > 0) ? s_more + (size_t)(wv - 1) * 2 * C : (Key *)pool;
    Key *const s_desc1 = s_desc0 + C;
    unsigned char *const cpool = (PAR && wv == 1) ? (unsigned char *)s_more : pool;   // this wave's candidate pool
    SK *const s_key = (SK *)cpool;                                  // candidate sort keys
    uint32_t *const s_cid = (uint32_t *)(cpool + E * sizeof(SK));   // candidate token ids
    uint32_t *const s_oth = s_cid + E;                              // the other tensor's logit
    // The two ranked lists (ids, own logits, the other tensor's logits).  List 1 is only written
    // when the candidates of tensor 1 are no longer needed and takes their place in the pool (of
    // the wave that ranked it: wave 0 copies it from wave 1's pool before the union).
    __shared__ uint32_t list0[3 * KC];
    uint32_t *const l_id[2] = {list0, (uint32_t *)cpool};
    float *const l_a[2] = {(float *)(list0 + KC), (float *)cpool + KC};
    float *const l_b[2] = {(float *)(list0 + 2 * KC), (float *)cpool + 2 * KC};

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
        if (W > 1 && wv > 0) return;
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

    Stream<Key> sq{0.f, M2_UNSET, -2.0e38f, neg_inf(), (Key)1, 0, 0.f, 0.f, 0.f};
    Stream<Key> sp{0.f, M2_UNSET, -2.0e38f, neg_inf(), (Key)1, 0, 0.f, 0.f, 0.f};
    // fp32 logits are held to 1e-5: the lane sums are then kept in two levels (chunk sums go to `s`,
    // `s` is folded into `hi` every BLOCK_CHUNKS chunks), because thousands of EQUAL terms (a row of
    // tied logits) added to one fp32 accumulator round the same way every time and drift by 1e-5
    // of the sum.  bf16 logits are held to 1e-3 and keep the single accumulator (and its register).
    constexpr bool TWO_LEVEL = ET::ESZ == 4;
    int nl_in[2] = {0, 0};                // entries of the carried top-k lists
    float xq_in = 0.f, xp_in = 0.f;
    int have_x = 0;
    if (carry_in) {
        // Resume the scan: the carried sums go to lane 0, and a full carried list bounds what can
        // still enter the top-k (its k-th value), exactly as if the sweep had never stopped.
        sq.M2 = hdr->M2[0]; sp.M2 = hdr->M2[1];
        if (lane == 0 && wv == 0) { sq.s = (float)hdr->S[0]; sp.s = (float)hdr->S[1]; sp.d = (float)hdr->D; }
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
                if (__ballot(rq)) raise_reference<TWO_LEVEL>(sq, mq, pq);
                if (__ballot(rp)) raise_reference<TWO_LEVEL>(sp, mp, pp);
            }
        }
        if constexpr (!STORED) sq.s += sum_exp2<VEC>(fq, sq.M2);
        if constexpr (DISTILL) sp.s += sum_exp2_kl<VEC>(fp, fq, sp.M2, sp.d);
        else sp.s += sum_exp2<VEC>(fp, sp.M2);
    };

    // ---- streaming sweep: iterations in which every lane owns a full 16-byte chunk ----------
    // (iterations [it_lo, it_hi) belong to this wave: all of them when a wave has the whole row)
    const uint32_t it_lo = W > 1 ? (uint32_t)((uint64_t)nit * (uint32_t)wv / W) : 0u;
    const uint32_t it_hi = W > 1 ? (uint32_t)((uint64_t)nit * (uint32_t)(wv + 1) / W) : nit;
    if (it_hi > it_lo) {
        // Two 16-byte loads per tensor stay in flight per lane: the loads for iterations it+2 and
        // it+3 are issued before iterations it and it+1 are consumed (indices clamp at the end).
        const uint32_t last = it_hi - 1;
        const uint32_t second = (it_lo + 1u < last ? it_lo + 1u : last) * WAVE + lane;
        u32x4 wq0 = stream_load(vq + it_lo * WAVE + lane), wp0 = stream_load(vp + it_lo * WAVE + lane);
        u32x4 wq1 = stream_load(vq + second), wp1 = stream_load(vp + second);
        for (uint32_t it = it_lo; it < it_hi; it += 2) {
            const u32x4 cq0 = wq0, cp0 = wp0, cq1 = wq1, cp1 = wp1;
            const uint32_t n0 = (it + 2 < last ? it + 2 : last) * WAVE + lane;
            const uint32_t n1 = (it + 3 < last ? it + 3 : last) * WAVE + lane;
            wq0 = stream_load(vq + n0); wp0 = stream_load(vp + n0);
            wq1 = stream_load(vq + n1); wp1 = stream_load(vp + n1);
            float fq[VEC], fp[VEC];
            ET::unpack(cq0, fq);
            ET::unpack(cp0, fp);
            consume(fq, fp, it * WAVE + lane, true);
            if (it + 1 < it_hi) {
                ET::unpack(cq1, fq);
                ET::unpack(cp1, fp);
                consume(fq, fp, (it + 1) * WAVE + lane, true);
            }
            if constexpr (TWO_LEVEL) {
                if (((it - it_lo) / 2) % (BLOCK_CHUNKS / 2) == BLOCK_CHUNKS / 2 - 1) {
                    sq.hi += sq.s; sq.s = 0.f;
                    sp.hi += sp.s; sp.s = 0.f;
                    if constexpr (DISTILL) { sp.dhi += sp.d; sp.d = 0.f; }
                }
            }
        }
    }
    // ---- remainder: fewer than 64 chunks, the last of which may be ragged (the last wave's) -----
    if (W == 1 || wv == W - 1) {
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

    double Sq = wave_sum((double)sq.hi + (double)sq.s), Sp = wave_sum((double)sp.hi + (double)sp.s);
    double Dp = DISTILL ? wave_sum((double)sp.dhi + (double)sp.d) : 0.0;
    if constexpr (W > 1) {
        // ---- split rows: every wave hands its sums to wave 0 and its best descriptors to the wave
        // that ranks the tensor (wave 0; wave 1 for the policy when both tensors are swept) ----------
        constexpr int LIM = C / W;                // >= KC >= k: the k best chunks of a run survive
        Key unused;
        const int n0 = uniform_i(select_top_keys<KT, NS>(s_desc0, sq.cnt, k, false, LIM, unused));
        const int n1 = uniform_i(select_top_keys<KT, NS>(s_desc1, sp.cnt, k, false, LIM, unused));
        if (lane == 0) {
            s_part[wv][0] = Sq; s_part[wv][1] = Sp; s_part[wv][2] = Dp;
            s_pref[wv][0] = sq.M2; s_pref[wv][1] = sp.M2;
            s_pcnt[wv][0] = n0; s_pcnt[wv][1] = n1;
        }
        __syncthreads();
        if (!PAR && wv > 0) return;
        // The lists of the waves are concatenated in wave (= chunk) order behind wave 0's own, which
        // already sit at the front of the pool's two buffers.
        Key *const m0 = (Key *)pool, *const m1 = m0 + C;
        if (wv == 0) {
            int c0 = n0;
            float Mq = sq.M2, Mp = sp.M2;
#pragma unroll
            for (int w = 1; w < W; ++w) {
                const Key *src0 = s_more + (size_t)(w - 1) * 2 * C;
                const int a0 = s_pcnt[w][0];
                for (int e = lane; e < a0; e += WAVE) m0[c0 + e] = src0[e];
                c0 += a0;
                Mq = fmaxf(Mq, s_pref[w][0]); Mp = fmaxf(Mp, s_pref[w][1]);
            }
            sq.cnt = c0;
            // sums on the common (largest) exponent reference, as the lanes of one wave have them
            Sq = 0.0; Sp = 0.0; Dp = 0.0;
#pragma unroll
            for (int w = 0; w < W; ++w) {
                const double fq2 = (double)__builtin_amdgcn_exp2f(s_pref[w][0] - Mq);
                const double fp2 = (double)__builtin_amdgcn_exp2f(s_pref[w][1] - Mp);
                Sq += s_part[w][0] * fq2; Sp += s_part[w][1] * fp2; Dp += s_part[w][2] * fp2;
            }
            sq.M2 = Mq; sp.M2 = Mp;
        }
        if (wv == (PAR ? 1 : 0)) {
            int c1 = s_pcnt[0][1];
#pragma unroll
            for (int w = 1; w < W; ++w) {
                const Key *src1 = s_more + (size_t)(w - 1) * 2 * C + C;
                const int a1 = s_pcnt[w][1];
                for (int e = lane; e < a1; e += WAVE) m1[c1 + e] = src1[e];
                c1 += a1;
            }
            sp.cnt = c1;
        }
        lds_sync();
    }

    // ---- log-sum-exp of both rows (log2 domain until the last step) -----------------------------
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
    const bool on0 = !PAR || wv == 0, on1 = !PAR || wv == 1;        // which tensor this wave ranks
    Key *const d0 = (Key *)pool, *const d1 = d0 + C;                // the (merged) descriptor lists
    nc[0] = 0; nc[1] = 0;
    kth[0] = 0; kth[1] = 0;
    if (!STORED && on0) nc[0] = uniform_i(select_top_keys<KT, NS>(d0, sq.cnt, k, false, 2 * KC, kth[0]));
    if (on1) nc[1] = uniform_i(select_top_keys<KT, NS>(d1, sp.cnt, k, false, 2 * KC, kth[1]));
    Key dk[2][DS];                                                  // at most 2*KC survive per tensor
#pragma unroll
    for (int sl = 0; sl < DS; ++sl) {
        const int e = sl * WAVE + lane;
        dk[0][sl] = (!STORED && e < nc[0]) ? d0[e] : (Key)0;
        dk[1][sl] = e < nc[1] ? d1[e] : (Key)0;
    }
    // the pools now belong to the candidates (split rows: wave 1's own buffers, which wave 0 has
    // finished reading, and the pool, whose policy descriptors wave 1 holds in registers)
    if constexpr (PAR) __syncthreads();
    else lds_sync();

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
                s_key[r] = SO::make_sort(ord32(__uint_as_float(ca[r])), (uint32_t)r);
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
        uint32_t gid[R], goth[R], nopay[R] = {};
        auto sort_candidates = [&]() {
            lds_sync();
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int e = lane * R + r;
                v[r] = e < nS ? s_key[e] : (SK)0;
            }
            bitonic_sort_desc<SK, R, false>(v, nopay, lane);
            const int keep = nS < k ? nS : k;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                uint32_t pos = SO::sort_pos(v[r]);
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
                    s_key[q] = SO::make_sort(ord32(SO::sort_value(v[r])), (uint32_t)q);
                    s_cid[q] = gid[r];
                    s_oth[q] = goth[r];
                }
            }
            nS = keep;
            filled = keep;
            lds_sync();
            if (keep >= k) {
                const SK kk = s_key[k - 1];
                above_ord = uniform_u(ord32(SO::sort_value(kk)));
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
                        s_key[pos] = SO::make_sort(ord32(fa[j]), pos);
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
                l_a[i][q] = SO::sort_value(v[r]);
                l_b[i][q] = __uint_as_float(goth[r]);
            }
        }
        lds_sync();
    };
    nl[0] = 0; nl[1] = 0;
    if constexpr (!STORED) {
        if (on0) expand(std::integral_constant<int, 0>{});
    }
    if (on1) expand(std::integral_constant<int, 1>{});
    if constexpr (PAR) {
        if (wv == 1 && lane == 0) s_pcnt[1][1] = nl[1];
        __syncthreads();
        if (wv > 0) return;
        nl[1] = s_pcnt[1][1];
        const uint32_t *const theirs = (const uint32_t *)s_more;    // list 1 as wave 1 left it
        for (int r = lane; r < nl[1]; r += WAVE) {
            l_id[1][r] = theirs[r];
            l_a[1][r] = __uint_as_float(theirs[KC + r]);
            l_b[1][r] = __uint_as_float(theirs[2 * KC + r]);
        }
        lds_sync();
    }

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

// ---- launchers ------------------------------------------------------------------------------

// SPLIT: also instantiate the forms that give a row to two or four waves (a.waves).
template <class ET, class KT, bool SPLIT, bool DISTILL>
static hipError_t launch_rows_kd(const RowArgs &a, hipStream_t st)
{
    const dim3 grid((unsigned)a.T), block(WAVE);
    if constexpr (SPLIT) {
        // four waves need room for 4 k descriptors in wave 0's buffer: not at k > 128
        const int w = a.waves >= 4 && a.k <= 128 ? 4 : (a.waves >= 2 ? 2 : 1);
        if (w == 4) {
            const dim3 b4(4 * WAVE);
            if (a.k <= 64) hipLaunchKernelGGL((row_kernel<ET, KT, 64, false, DISTILL, false, 4>), grid, b4, 0, st, a);
            else hipLaunchKernelGGL((row_kernel<ET, KT, 128, false, DISTILL, false, 4>), grid, b4, 0, st, a);
            return hipGetLastError();
        }
        if (w == 2) {
            const dim3 b2(2 * WAVE);
            if (a.k <= 64) hipLaunchKernelGGL((row_kernel<ET, KT, 64, false, DISTILL, false, 2>), grid, b2, 0, st, a);
            else if (a.k <= 128) hipLaunchKernelGGL((row_kernel<ET, KT, 128, false, DISTILL, false, 2>), grid, b2, 0, st, a);
            else hipLaunchKernelGGL((row_kernel<ET, KT, 256, false, DISTILL, false, 2>), grid, b2, 0, st, a);
            return hipGetLastError();
        }
    }
    if (a.k <= 64) hipLaunchKernelGGL((row_kernel<ET, KT, 64, false, DISTILL>), grid, block, 0, st, a);
    else if (a.k <= 128) hipLaunchKernelGGL((row_kernel<ET, KT, 128, false, DISTILL>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((row_kernel<ET, KT, 256, false, DISTILL>), grid, block, 0, st, a);
    return hipGetLastError();
}

template <class ET, class KT, bool SPLIT>
static hipError_t launch_rows_k(const RowArgs &a, hipStream_t st)
{
    return a.distill ? launch_rows_kd<ET, KT, SPLIT, true>(a, st) : launch_rows_kd<ET, KT, SPLIT, false>(a, st);
}

// The vocabulary-chunked forms (fp32 logit chunks, 64-bit keys): the same split by a.waves.
template <bool DISTILL, bool STORED>
static hipError_t launch_rows_carry_ds(const RowArgs &a, hipStream_t st)
{
    const dim3 grid((unsigned)a.T), block(WAVE);
    const int w = a.waves >= 4 && a.k <= 128 ? 4 : (a.waves >= 2 ? 2 : 1);
    if (w == 4) {
        const dim3 b4(4 * WAVE);
        if (a.k <= 64) hipLaunchKernelGGL((row_kernel<F32Elem, Key64, 64, true, DISTILL, STORED, 4>), grid, b4, 0, st, a);
        else hipLaunchKernelGGL((row_kernel<F32Elem, Key64, 128, true, DISTILL, STORED, 4>), grid, b4, 0, st, a);
        return hipGetLastError();
    }
    if (w == 2) {
        const dim3 b2(2 * WAVE);
        if (a.k <= 64) hipLaunchKernelGGL((row_kernel<F32Elem, Key64, 64, true, DISTILL, STORED, 2>), grid, b2, 0, st, a);
        else if (a.k <= 128) hipLaunchKernelGGL((row_kernel<F32Elem, Key64, 128, true, DISTILL, STORED, 2>), grid, b2, 0, st, a);
        else hipLaunchKernelGGL((row_kernel<F32Elem, Key64, 256, true, DISTILL, STORED, 2>), grid, b2, 0, st, a);
        return hipGetLastError();
    }
    if (a.k <= 64) hipLaunchKernelGGL((row_kernel<F32Elem, Key64, 64, true, DISTILL, STORED>), grid, block, 0, st, a);
    else if (a.k <= 128) hipLaunchKernelGGL((row_kernel<F32Elem, Key64, 128, true, DISTILL, STORED>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((row_kernel<F32Elem, Key64, 256, true, DISTILL, STORED>), grid, block, 0, st, a);
    return hipGetLastError();
}

hipError_t launch_rows_carry(const RowArgs &a, hipStream_t st)
{
    if (a.T <= 0) return hipSuccess;
    return a.distill ? launch_rows_carry_ds<true, false>(a, st) : launch_rows_carry_ds<false, false>(a, st);
}

hipError_t launch_rows_carry_stored(const RowArgs &a, hipStream_t st)
{
    if (a.T <= 0) return hipSuccess;
    return launch_rows_carry_ds<false, true>(a, st);
}

hipError_t launch_rows(const RowArgs &a, int dtype, hipStream_t st)
{
    if (a.T <= 0) return hipSuccess;
    if (dtype == JP_BF16) {
        const int64_t nchunks = (a.V + Bf16Elem::VEC - 1) / Bf16Elem::VEC;
        if (nchunks <= 65535) return launch_rows_k<Bf16Elem, Key32, true>(a, st);
        return launch_rows_k<Bf16Elem, Key64, false>(a, st);
    }
    return launch_rows_k<F32Elem, Key64, true>(a, st);
}

template <class ET, class KT, bool SPLIT>
static hipError_t launch_rows_stored_k(const RowArgs &a, hipStream_t st)
{
    const dim3 grid((unsigned)a.T), block(WAVE);
    if constexpr (SPLIT) {
        const int w = a.waves >= 4 && a.k <= 128 ? 4 : (a.waves >= 2 ? 2 : 1);
        if (w == 4) {
            const dim3 b4(4 * WAVE);
            if (a.k <= 64) hipLaunchKernelGGL((row_kernel<ET, KT, 64, false, false, true, 4>), grid, b4, 0, st, a);
            else hipLaunchKernelGGL((row_kernel<ET, KT, 128, false, false, true, 4>), grid, b4, 0, st, a);
            return hipGetLastError();
        }
        if (w == 2) {
            const dim3 b2(2 * WAVE);
            if (a.k <= 64) hipLaunchKernelGGL((row_kernel<ET, KT, 64, false, false, true, 2>), grid, b2, 0, st, a);
            else if (a.k <= 128) hipLaunchKernelGGL((row_kernel<ET, KT, 128, false, false, true, 2>), grid, b2, 0, st, a);
            else hipLaunchKernelGGL((row_kernel<ET, KT, 256, false, false, true, 2>), grid, b2, 0, st, a);
            return hipGetLastError();
        }
    }
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
        if (nchunks <= 65535) return launch_rows_stored_k<Bf16Elem, Key32, true>(a, st);
        return launch_rows_stored_k<Bf16Elem, Key64, false>(a, st);
    }
    return launch_rows_stored_k<F32Elem, Key64, true>(a, st);
}

}  // namespace jp
