// Device-side helpers shared by the kernels of the OBRS hot path (gfx950, 64-lane wavefronts):
// streaming loads, order-preserving float keys, wave-wide reductions on the VALU, a bitonic sorting
// network over the registers of a wave, and the two element types (bf16 / fp32 logits).
#ifndef JP_DEVICE_UTILS_H
#define JP_DEVICE_UTILS_H

#include <hip/hip_runtime.h>
#include <stdint.h>

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
constexpr int BLOCK_CHUNKS = 48;                       // chunk sums per lane between two folds of a two-level sum

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

// Lanes of the wave for which `pred` holds, as a mask in scalar registers (the compare that made
// `pred` writes the mask directly; the generic __ballot goes through a vector register).
__device__ __forceinline__ uint64_t ballot64(bool pred) { return __builtin_amdgcn_ballot_w64(pred); }

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
// bitwise AND / OR of a 32-bit value over the wave (every lane gets the result)
__device__ __forceinline__ uint32_t wave_and(uint32_t v)
{
    v &= (uint32_t)dpp_mov<DPP_QUAD_XOR1>((int)v);
    v &= (uint32_t)dpp_mov<DPP_QUAD_XOR2>((int)v);
    v &= (uint32_t)dpp_mov<DPP_ROW_ROR4>((int)v);
    v &= (uint32_t)dpp_mov<DPP_ROW_ROR8>((int)v);
    return (uint32_t)(__builtin_amdgcn_readlane((int)v, 0) & __builtin_amdgcn_readlane((int)v, 16) &
                      __builtin_amdgcn_readlane((int)v, 32) & __builtin_amdgcn_readlane((int)v, 48));
}
__device__ __forceinline__ uint32_t wave_or32(uint32_t v)
{
    v |= (uint32_t)dpp_mov<DPP_QUAD_XOR1>((int)v);
    v |= (uint32_t)dpp_mov<DPP_QUAD_XOR2>((int)v);
    v |= (uint32_t)dpp_mov<DPP_ROW_ROR4>((int)v);
    v |= (uint32_t)dpp_mov<DPP_ROW_ROR8>((int)v);
    return (uint32_t)(__builtin_amdgcn_readlane((int)v, 0) | __builtin_amdgcn_readlane((int)v, 16) |
                      __builtin_amdgcn_readlane((int)v, 32) | __builtin_amdgcn_readlane((int)v, 48));
}
__device__ __forceinline__ unsigned wave_or(unsigned v)
{
    const uint64_t any = __ballot(v != 0);
    unsigned r = 0;
#pragma unroll
    for (int b = 0; b < 3; ++b) r |= (__ballot((v >> b) & 1u) != 0) ? (1u << b) : 0u;   // three flag bits exist
    return any ? r : 0u;
}

// Single-wave workgroups: the LDS unit executes the LDS instructions of one wave in program
// order, so a value written by one lane is seen by a later read of another lane without any
// wait.  What is needed is only that the compiler keeps that program order (it cannot see the
// cross-lane dependence): a wavefront-scope fence and a scheduling barrier, neither of which
// emits an instruction.  Unlike __syncthreads() this does not wait for the global loads in
// flight, so a select or a drain in the middle of the sweep does not stall the stream.
__device__ __forceinline__ void lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

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
// register (e % R) of lane (e / R), so the exchanges at distance < R stay inside a lane.  With
// PAY a 32-bit payload travels with every key.
template <class SK, int R, int K2, int J, bool PAY>
__device__ __forceinline__ void bitonic_layer(SK (&v)[R], uint32_t (&pay)[R], int lane)
{
    if constexpr (J < R) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if ((r & J) == 0) {
                const bool desc = (K2 < R) ? ((r & K2) == 0) : ((lane & (K2 / R)) == 0 || K2 == WAVE * R);
                const SK a = v[r], b = v[r | J];
                const bool g = a > b;
                const bool swap = g != desc;              // descending wants the larger key first
                v[r] = swap ? b : a;
                v[r | J] = swap ? a : b;
                if constexpr (PAY) {
                    const uint32_t pa = pay[r], pb = pay[r | J];
                    pay[r] = swap ? pb : pa;
                    pay[r | J] = swap ? pa : pb;
                }
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
            const bool mine = (v[r] > p) == keep_max;
            v[r] = mine ? v[r] : p;
            if constexpr (PAY) {
                const uint32_t pp = xor_lane<L>(pay[r]);
                pay[r] = mine ? pay[r] : pp;
            }
        }
    }
    if constexpr (J > 1) bitonic_layer<SK, R, K2, J / 2, PAY>(v, pay, lane);
}
template <class SK, int R, int K2, bool PAY>
__device__ __forceinline__ void bitonic_merge_from(SK (&v)[R], uint32_t (&pay)[R], int lane)
{
    bitonic_layer<SK, R, K2, K2 / 2, PAY>(v, pay, lane);
    if constexpr (K2 < WAVE * R) bitonic_merge_from<SK, R, K2 * 2, PAY>(v, pay, lane);
}
// Keys must be distinct where the payload matters (equal keys may exchange payloads).
template <class SK, int R, bool PAY>
__device__ __forceinline__ void bitonic_sort_desc(SK (&v)[R], uint32_t (&pay)[R], int lane)
{
    bitonic_merge_from<SK, R, 2, PAY>(v, pay, lane);
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
};

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

}  // namespace jp
#endif
