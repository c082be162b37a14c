// Fused lm_head path for gfx950: logits of one vocabulary chunk are produced on the matrix cores
// (bf16 x bf16 -> fp32, v_mfma_f32_32x32x16_bf16) straight from the hidden states and the vocabulary
// projection, and handed to the row kernel chunk by chunk, so the [T, V] logit tensors never
// exist.  Two kernels live here:
//   * transpose_chunk_kernel: W[d, V] (vocabulary contiguous) -> Wt[n, d] for the columns of one
//     chunk, so that both GEMM operands are contiguous along the contraction dimension (16-byte
//     pieces on both sides, through an LDS tile);
//   * gemm_tn_kernel: C[M, N] = A[M, K] * Bt[N, K]^T with 256x256x64 workgroup tiles, XOR-swizzled
//     LDS tiles filled straight from global memory round a five-slot ring, 2x2 waves of 128x128
//     (4x4 MFMA blocks each).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <type_traits>

#include "jp_obrs_internal.h"

namespace jp {

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef const __attribute__((address_space(1))) u32x4 *gvec_ptr;

typedef const __attribute__((address_space(1))) void *gvoid_ptr;
typedef __attribute__((address_space(3))) void *lvoid_ptr;

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int GEMM_THREADS = 256;
constexpr int TILE_BYTES = BM * BK * 2;            // 32 KB per operand tile
constexpr int ROW_BYTES = BK * 2;                  // 128 B: eight 16-byte pieces per tile row
constexpr int NU = 5;                              // LDS ring: five operand-tile slots, the whole 160 KB
// s_waitcnt immediates (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8).
constexpr int WAIT_VM0 = 0x0F70;                   // vmcnt(0)
constexpr int WAIT_VM8_LGKM0 = 0x0078;             // vmcnt(8) lgkmcnt(0)
constexpr int WAIT_VM24 = 0x4F78;                  // vmcnt(24)

// Piece p (0..7) of tile row r is stored at piece p ^ ((r >> 1) & 7).  The LDS serves 256 bytes
// (64 banks) per cycle, i.e. 16 lanes of a 16-byte access: consecutive rows alternate between the
// two 128-byte halves of the bank space, and rows of equal parity get distinct pieces, so the 16
// rows a fragment read touches per cycle are conflict-free (measured with SQ_LDS_BANK_CONFLICT).
__device__ __forceinline__ int tile_offset(int row, int piece) { return row * ROW_BYTES + ((piece ^ ((row >> 1) & 7)) << 4); }

}  // namespace

// -------------------------------------------------------------------------------------------------
// Wt[n, kk] = W[kk, v0 + n] for n < ncols (zero for ncols <= n < npad), kk < d.
// A workgroup moves a tile of 64 k-rows x 128 vocabulary columns: it reads 16-byte pieces along
// the vocabulary (the contiguous direction of W), scatters their eight elements into an LDS tile
// held column-major, and writes 16-byte pieces along k (the contiguous direction of Wt).  Pieces
// that are not 16-byte aligned in W (v0 or ldw not a multiple of 8), or that cross the end of
// the chunk, are read element by element.  d is a multiple of 64 (checked by the caller).
// -------------------------------------------------------------------------------------------------
constexpr int TR_K = 64, TR_N = 128, TR_PITCH = TR_K + 2;     // LDS pitch in elements: an odd number of 32-bit words,
                                                              // so the eight rows a piece scatters to fall into different banks
__global__ __launch_bounds__(256) void transpose_chunk_kernel(const uint16_t *__restrict__ W, int64_t ldw,
                                                              int d, int64_t v0, int ncols, int npad,
                                                              uint16_t *__restrict__ Wt)
{
    __shared__ __attribute__((aligned(4))) uint16_t tile[TR_N][TR_PITCH];
    const int n0 = blockIdx.x * TR_N, k0 = blockIdx.y * TR_K;
    const int tid = threadIdx.x;
    const bool aligned = ((v0 | ldw) & 7) == 0 && ((uintptr_t)W & 15) == 0;
    {
        const int piece = tid & 15, krow = tid >> 4;          // 16 pieces of 8 columns per k-row, 16 k-rows per pass
#pragma unroll
        for (int pass = 0; pass < TR_K / 16; ++pass) {
            const int kk = pass * 16 + krow, n = n0 + piece * 8;
            uint16_t e[8];
            const uint16_t *src = W + (int64_t)(k0 + kk) * ldw + v0 + n;
            if (aligned && n + 8 <= ncols) {
                const u32x4 v = *(const u32x4 *)src;
#pragma unroll
                for (int j = 0; j < 4; ++j) { e[2 * j] = (uint16_t)(v[j] & 0xffffu); e[2 * j + 1] = (uint16_t)(v[j] >> 16); }
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) e[j] = n + j < ncols ? src[j] : (uint16_t)0;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) tile[piece * 8 + j][kk] = e[j];
        }
    }
    __syncthreads();
    {
        const int piece = tid & 7, nrow = tid >> 3;           // 8 pieces of 8 k per column, 32 columns per pass
#pragma unroll
        for (int pass = 0; pass < TR_N / 32; ++pass) {
            const int nl = pass * 32 + nrow, n = n0 + nl;
            const uint32_t *row = (const uint32_t *)&tile[nl][piece * 8];      // (4-byte aligned: the pitch is 33 words)
            const u32x4 v = {row[0], row[1], row[2], row[3]};
            if (n < npad) *(u32x4 *)(Wt + (int64_t)n * d + k0 + piece * 8) = v;
        }
    }
}

// -------------------------------------------------------------------------------------------------
// C[m, n] = sum_k A[m, k] * Bt[n, k]; A: [M, K] bf16, Bt: [N, K] bf16, C: [M, ldc] fp32.
// K is a multiple of 64 and N a multiple of 256 (the caller pads Bt with zero rows); M is free.
// blockIdx.z selects one of two independent problems (policy / actor head) sharing M, N, ldc.
//
// Operand tiles go from global memory straight into LDS (global_load_lds_dwordx4: no staging
// registers, no ds_write).  A wave instruction of that kind writes 64 x 16 bytes to consecutive
// LDS addresses, which is 8 tile rows of 128 bytes (whole cache lines on the global side); the
// swizzle is applied on the global side (which 16-byte piece of its row a lane fetches), so the
// LDS image is the same as if it had been written piece by piece.  The operand tiles of
// successive k-tiles, A(0) B(0) A(1) B(1) ..., go round a ring of five 32 KB slots.
// -------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(GEMM_THREADS, 1) void gemm_tn_kernel(GemmArgs G)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];   // ring of NU operand-tile slots
    const int z = blockIdx.z;
    const unsigned char *A = (const unsigned char *)G.A[z];
    const unsigned char *B = (const unsigned char *)G.Bt[z];
    float *C = G.C[z];
    const int K = G.K[z];
    const int M = G.M;

    // XCD-aware tile order: the hardware deals consecutive workgroups round-robin to the 8 XCDs;
    // give every XCD a contiguous run of tiles, walked 8 row-tiles at a time so that the 32
    // workgroups an XCD runs together share 8 A row-tiles and 4 B column-tiles in its L2.
    const int tiles_m = (M + BM - 1) / BM, tiles_n = G.N / BN;
    const int ntiles = tiles_m * tiles_n;
    int id = blockIdx.x;
    {
        const int per = (ntiles + 7) / 8;
        const int cand = (id % 8) * per + id / 8;
        // only a remap when every XCD gets a full share; otherwise keep the launch order
        id = (ntiles % 8 == 0) ? cand : id;
    }
    constexpr int GM = 8;
    const int group = id / (GM * tiles_n);
    const int gm = (tiles_m - group * GM) < GM ? (tiles_m - group * GM) : GM;
    const int in_group = id - group * GM * tiles_n;
    const int tile_m = group * GM + in_group % gm;
    const int tile_n = in_group / gm;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;                 // 2 x 2 waves, 128 x 128 each
    const int li = lane & 31, lg = lane >> 5;                // MFMA row/col index, k-group

    // Loads: per operand tile a wave fetches tile rows [64 wave + 8 i, +8), i < 8.  Lane l lands at
    // LDS piece (l & 7) of row (l >> 3) of that group, so it fetches logical piece
    // (l & 7) ^ swizzle(row), and swizzle(row) = (row >> 1) & 7 = 4 (i & 1) + ((l >> 4) & 3).
    const int64_t ldk = (int64_t)K * 2;                      // bytes per row of A / Bt
    const unsigned char *abase = A + (int64_t)tile_m * BM * ldk;     // wave-uniform tile origins
    const unsigned char *bbase = B + (int64_t)tile_n * BN * ldk;
    uint32_t oa[8], ob[8];                                   // byte offsets of this lane's pieces
    {
        const int last = M - 1 - tile_m * BM;                // rows past M repeat the last row (never stored)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int piece = (lane & 7) ^ (4 * (i & 1) + ((lane >> 4) & 3));
            const int r = wave * 64 + i * 8 + (lane >> 3);
            const int ra = r < last ? r : last;
            oa[i] = (uint32_t)ra * (uint32_t)ldk + piece * 16;
            ob[i] = (uint32_t)r * (uint32_t)ldk + piece * 16;
        }
    }
    const int nk = K / BK;
    // quarter q (0..3) of the loads of operand tile `which` (0 = A, 1 = B) of k-tile kt into ring slot `slot`
    auto issue_quarter = [&](int which, int kt, int slot, int q) __attribute__((always_inline)) {
        const int kc = kt < nk ? kt : nk - 1;                // past the end: a harmless repeat into a free slot
        unsigned char *dst = lds + slot * TILE_BYTES + wave * 8192;
#pragma unroll
        for (int i = 2 * q; i < 2 * q + 2; ++i) {
            const unsigned char *src = which ? bbase + ob[i] : abase + oa[i];
            __builtin_amdgcn_global_load_lds((gvoid_ptr)(uintptr_t)(src + kc * ROW_BYTES), (lvoid_ptr)(dst + i * 1024), 16, 0, 0);
        }
    };
    auto issue_tile = [&](int which, int kt, int slot) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < 4; ++q) issue_quarter(which, kt, slot, q);
    };

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    uint32_t fa_off[4], fb_off[4];                           // fragment addresses of the four k-steps
#pragma unroll
    for (int s2 = 0; s2 < 4; ++s2) {
        fa_off[s2] = (uint32_t)tile_offset(wm * 128 + li, 2 * s2 + lg);
        fb_off[s2] = (uint32_t)tile_offset(wn * 128 + li, 2 * s2 + lg);
    }
    bf16x8 fa[2][4], fb[2][4];
    auto lfrag = [&](int slot_a, int slot_b, int s2) __attribute__((always_inline)) {
        const unsigned char *ta = lds + slot_a * TILE_BYTES, *tb = lds + slot_b * TILE_BYTES;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            fa[s2 & 1][i] = *(const bf16x8 *)(ta + fa_off[s2] + i * 32 * ROW_BYTES);
            fb[s2 & 1][i] = *(const bf16x8 *)(tb + fb_off[s2] + i * 32 * ROW_BYTES);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    auto mfma_row = [&](int s2, int i) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[s2 & 1][i], fb[s2 & 1][j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    };
    auto ring_next = [](int slot, int by) { slot += by; return slot >= NU ? slot - NU : slot; };

    // Ring schedule.  While k-tile kt is multiplied out of slots sa (A) and sb (B), the slots
    // after them hold A(kt+1), B(kt+1) and A(kt+2), landed or in flight.  Late in tile kt, once
    // its last fragments are in registers, every wave waits for its own share of tile kt+1 (all
    // but the newest 8 loads, which are A(kt+2)); the barrier makes every wave's share visible
    // and proves that nobody reads the slots of tile kt any more, which then take B(kt+2) and
    // A(kt+3).  Fragment reads are issued a whole k-step before they are used, and the loads are
    // dealt out four at a time between MFMA rows.
    int sa = 0, sb = 1;
    issue_tile(0, 0, 0);
    issue_tile(1, 0, 1);
    issue_tile(0, 1, 2);
    issue_tile(1, 1, 3);
    issue_tile(0, 2, 4);
    __builtin_amdgcn_s_waitcnt(WAIT_VM24);
    __syncthreads();
    lfrag(sa, sb, 0);
    for (int kt = 0; kt < nk; ++kt) {
        const int sa1 = ring_next(sa, 2), sb1 = ring_next(sb, 2);
        mfma_row(0, 0);
        lfrag(sa, sb, 1);
        mfma_row(0, 1);
        mfma_row(0, 2);
        mfma_row(0, 3);
        mfma_row(1, 0);
        lfrag(sa, sb, 2);
        mfma_row(1, 1);
        mfma_row(1, 2);
        mfma_row(1, 3);
        mfma_row(2, 0);
        lfrag(sa, sb, 3);
        mfma_row(2, 1);
        mfma_row(2, 2);
        __builtin_amdgcn_s_waitcnt(WAIT_VM8_LGKM0);
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
        mfma_row(2, 3);
        lfrag(sa1, sb1, 0);                                  // past the end: reads a stale slot, unused
        mfma_row(3, 0);
        issue_quarter(1, kt + 2, sa, 0);                     // B(kt+2) takes A(kt)'s slot,
        issue_quarter(1, kt + 2, sa, 1);
        __builtin_amdgcn_sched_barrier(0);
        mfma_row(3, 1);
        issue_quarter(1, kt + 2, sa, 2);
        issue_quarter(1, kt + 2, sa, 3);
        __builtin_amdgcn_sched_barrier(0);
        mfma_row(3, 2);
        issue_quarter(0, kt + 3, sb, 0);                     // A(kt+3) takes B(kt)'s slot
        issue_quarter(0, kt + 3, sb, 1);
        __builtin_amdgcn_sched_barrier(0);
        mfma_row(3, 3);
        issue_quarter(0, kt + 3, sb, 2);
        issue_quarter(0, kt + 3, sb, 3);
        __builtin_amdgcn_sched_barrier(0);
        sa = sa1;
        sb = sb1;
    }
    __builtin_amdgcn_s_waitcnt(WAIT_VM0);                    // no load may still be writing LDS at exit

    // D layout of the 32x32 MFMA: lane holds column (lane & 31); register r is row
    // 8 (r / 4) + 4 (lane >> 5) + (r & 3).
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = tile_m * BM + wm * 128 + i * 32 + 8 * (r >> 2) + 4 * lg + (r & 3);
            if (row < M) {
                float *crow = C + (int64_t)row * G.ldc + tile_n * BN + wn * 128 + li;
#pragma unroll
                for (int j = 0; j < 4; ++j) __builtin_nontemporal_store(acc[i][j][r], crow + j * 32);
            }
        }
    }
}

// Wt[n, :] = W[v0 + n, :] for n < ncols, zero rows up to npad: the vocabulary-major weight layout needs
// no transpose, only this padded copy for the last, partial chunk.  d is a multiple of 64.
__global__ __launch_bounds__(256) void copy_rows_chunk_kernel(const u32x4 *__restrict__ W, int d16, int64_t v0,
                                                              int ncols, int npad, u32x4 *__restrict__ Wt)
{
    const int64_t total = (int64_t)npad * d16;               // 16-byte pieces
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t n = i / d16;
        Wt[i] = n < ncols ? W[(v0 + n) * d16 + (i - n * d16)] : u32x4{0u, 0u, 0u, 0u};
    }
}

// Reads `n16` 16-byte pieces and keeps nothing: [V, d] weights are multiplied in place, and a chunk
// that the GEMM meets cold in HBM costs it 6 % (its k-loop waits on operand latency), while a chunk
// that has just been read sits in the 256 MB Infinity Cache.  The transposed layout gets the same
// effect for free from its transpose.  (The store can practically never happen; it keeps the loads.)
__global__ __launch_bounds__(256) void touch_rows_kernel(const u32x4 *__restrict__ W, int64_t n16, uint32_t *sink)
{
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (int64_t)gridDim.x * blockDim.x) {
        const u32x4 v = W[i];
        acc ^= v;
    }
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u && (acc[0] & acc[1]) == 0x7f4a7c15u) *sink = acc[2];
}

hipError_t launch_touch_rows(const void *W, int64_t bytes, void *sink, hipStream_t st)
{
    const int64_t n16 = bytes / 16;
    if (n16 <= 0) return hipSuccess;
    // a chunk that cannot stay in the Infinity Cache beside its logits (the wide chunks of small
    // batches) would only be read twice
    if (bytes > ((int64_t)96 << 20)) return hipSuccess;
    const unsigned blocks = (unsigned)((n16 + 255) / 256 < 2048 ? (n16 + 255) / 256 : 2048);
    hipLaunchKernelGGL(touch_rows_kernel, dim3(blocks), dim3(256), 0, st, (const u32x4 *)W, n16, (uint32_t *)sink);
    return hipGetLastError();
}

hipError_t launch_copy_rows_chunk(const void *W, int d, int64_t v0, int ncols, int npad, void *Wt, hipStream_t st)
{
    const int d16 = d / 8;
    const int64_t total = (int64_t)npad * d16;
    const unsigned blocks = (unsigned)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
    hipLaunchKernelGGL(copy_rows_chunk_kernel, dim3(blocks), dim3(256), 0, st, (const u32x4 *)W, d16, v0, ncols, npad,
                       (u32x4 *)Wt);
    return hipGetLastError();
}

hipError_t launch_transpose_chunk(const void *W, int64_t ldw, int d, int64_t v0, int ncols, int npad,
                                  void *Wt, hipStream_t st)
{
    const dim3 grid((unsigned)((npad + TR_N - 1) / TR_N), (unsigned)(d / TR_K));
    hipLaunchKernelGGL(transpose_chunk_kernel, grid, dim3(256), 0, st, (const uint16_t *)W, ldw, d, v0, ncols,
                       npad, (uint16_t *)Wt);
    return hipGetLastError();
}

hipError_t launch_gemm_pair(const GemmArgs &g, hipStream_t st)
{
    const int lds_bytes = NU * TILE_BYTES;      // 160 KB ring
    // More than 64 KB of dynamic LDS has to be allowed once per device; later launches (also ones
    // recorded into a graph) then make no call besides the launch itself.  The flag is only ever set,
    // through an atomic, after the attribute call has succeeded; two threads racing on a device's
    // first call both make that (idempotent) call.
    static std::atomic<bool> allowed[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64 || !allowed[dev].load(std::memory_order_acquire)) {
        e = hipFuncSetAttribute((const void *)gemm_tn_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        if (dev >= 0 && dev < 64) allowed[dev].store(true, std::memory_order_release);
    }
    const int tiles = ((g.M + BM - 1) / BM) * (g.N / BN);
    hipLaunchKernelGGL(gemm_tn_kernel, dim3((unsigned)tiles, 1, (unsigned)g.nproblems), dim3(GEMM_THREADS), lds_bytes, st, g);
    return hipGetLastError();
}

}  // namespace jp
