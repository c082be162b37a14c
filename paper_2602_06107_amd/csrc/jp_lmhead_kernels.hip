// Fused lm_head path for gfx950: logits of one vocabulary chunk are produced on the matrix cores
// (bf16 x bf16 -> fp32, v_mfma_f32_32x32x16_bf16) straight from the hidden states and the vocabulary
// projection, and handed to the row kernel chunk by chunk, so the [T, V] logit tensors never
// exist.  Two kernels live here:
//   * transpose_chunk_kernel: W[d, V] (vocabulary contiguous) -> Wt[n, d] for the columns of one
//     chunk, so that both GEMM operands are contiguous along the contraction dimension;
//   * gemm_tn_kernel: C[M, N] = A[M, K] * Bt[N, K]^T with 256x256x64 workgroup tiles, XOR-swizzled
//     LDS tiles, register-staged double buffering, 2x2 waves of 128x128 (4x4 MFMA blocks each).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "jp_obrs_internal.h"

namespace jp {

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef const __attribute__((address_space(1))) u32x4 *gvec_ptr;

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int GEMM_THREADS = 256;
constexpr int TILE_BYTES = BM * BK * 2;            // 32 KB per operand tile
constexpr int ROW_BYTES = BK * 2;                  // 128 B: eight 16-byte pieces per tile row

// Piece p (0..7) of tile row r is stored at piece p ^ ((r >> 1) & 7).  The LDS serves 256 bytes
// (64 banks) per cycle, i.e. 16 lanes of a 16-byte access: consecutive rows alternate between the
// two 128-byte halves of the bank space, and rows of equal parity get distinct pieces, so the 16
// rows a fragment read touches per cycle are conflict-free (measured with SQ_LDS_BANK_CONFLICT).
__device__ __forceinline__ int tile_offset(int row, int piece) { return row * ROW_BYTES + ((piece ^ ((row >> 1) & 7)) << 4); }

}  // namespace

// -------------------------------------------------------------------------------------------------
// Wt[n, kk] = W[kk, v0 + n] for n < ncols (zero for ncols <= n < npad), kk < d.
// -------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void transpose_chunk_kernel(const uint16_t *__restrict__ W, int64_t ldw,
                                                              int d, int64_t v0, int ncols, int npad,
                                                              uint16_t *__restrict__ Wt)
{
    __shared__ uint16_t tile[64][66];
    const int n0 = blockIdx.x * 64, k0 = blockIdx.y * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int kk = i * 4 + ty, n = n0 + tx;
        uint16_t v = 0;
        if (k0 + kk < d && n < ncols) v = W[(int64_t)(k0 + kk) * ldw + v0 + n];
        tile[kk][tx] = v;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int n = n0 + i * 4 + ty, kk = k0 + tx;
        if (n < npad && kk < d) Wt[(int64_t)n * d + kk] = tile[tx][i * 4 + ty];
    }
}

// -------------------------------------------------------------------------------------------------
// C[m, n] = sum_k A[m, k] * Bt[n, k]; A: [M, K] bf16, Bt: [N, K] bf16, C: [M, ldc] fp32.
// K is a multiple of 64 and N a multiple of 256 (the caller pads Bt with zero rows); M is free.
// blockIdx.z selects one of two independent problems (policy / actor head) sharing M, N, ldc.
// -------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(GEMM_THREADS, 1) void gemm_tn_kernel(GemmArgs G)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];   // 2 stages x (A tile, B tile)
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

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;                 // 2 x 2 waves, 128 x 128 each
    const int li = lane & 31, lg = lane >> 5;                // MFMA row/col index, k-group

    // staging: thread owns piece (tid & 7) of rows (tid >> 3) + 32 i, i < 8, of both tiles
    const int sp = tid & 7, sr = tid >> 3;
    const int64_t ldk = (int64_t)K * 2;                      // bytes per row of A / Bt
    const unsigned char *abase = A + (int64_t)tile_m * BM * ldk;     // wave-uniform tile origins
    const unsigned char *bbase = B + (int64_t)tile_n * BN * ldk;
    uint32_t oa[8], ob[8];                                   // byte offsets inside the tile's rows
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        int ra = sr + 32 * i;
        const int last = M - 1 - tile_m * BM;                // rows past M repeat the last row (never stored)
        ra = ra < last ? ra : last;
        oa[i] = (uint32_t)ra * (uint32_t)ldk + sp * 16;
        ob[i] = (uint32_t)(sr + 32 * i) * (uint32_t)ldk + sp * 16;
    }

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // Global -> register -> LDS staging with the memory instructions spread between the MFMAs:
    // during k-tile kt the 16 ds_writes that put tile kt+1 (already in registers) into the other
    // LDS stage ride behind the first 32 MFMAs, and the 16 global loads of tile kt+2 ride behind
    // the last 32, so neither the vector-memory nor the LDS queue ever stalls the matrix pipe and
    // every load has about one and a half k-tiles (~1.3 us) to arrive.
    u32x4 stg[16];                                           // pieces 0-7: A rows, 8-15: Bt rows
    const int nk = K / BK;
    const uint32_t st_off = (uint32_t)tile_offset(sr, sp);   // rows 32 apart share their swizzle
    auto gload_piece = [&](int kt, int p) __attribute__((always_inline)) {
        const int kc = kt < nk ? kt : nk - 1;                // past the end: a harmless repeat
        stg[p] = p < 8 ? *(gvec_ptr)(uintptr_t)(abase + oa[p] + kc * ROW_BYTES)
                       : *(gvec_ptr)(uintptr_t)(bbase + ob[p - 8] + kc * ROW_BYTES);
    };
    auto lstore_piece = [&](int stage, int p) __attribute__((always_inline)) {
        unsigned char *t = lds + stage * 2 * TILE_BYTES + st_off + (p < 8 ? 0 : TILE_BYTES) + (p & 7) * 32 * ROW_BYTES;
        *(u32x4 *)t = stg[p];
    };
    uint32_t fa_off[BK / 16], fb_off[BK / 16];               // fragment addresses of the 4 k-steps
#pragma unroll
    for (int s2 = 0; s2 < BK / 16; ++s2) {
        fa_off[s2] = (uint32_t)tile_offset(wm * 128 + li, 2 * s2 + lg);
        fb_off[s2] = (uint32_t)(TILE_BYTES + tile_offset(wn * 128 + li, 2 * s2 + lg));
    }

#pragma unroll
    for (int p = 0; p < 16; ++p) gload_piece(0, p);
#pragma unroll
    for (int p = 0; p < 16; ++p) lstore_piece(0, p);
#pragma unroll
    for (int p = 0; p < 16; ++p) gload_piece(1, p);
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int stage = kt & 1;
        const unsigned char *ts = lds + stage * 2 * TILE_BYTES;
        bf16x8 fa[2][4], fb[2][4];
        auto lfrag = [&](int s2, int b2) __attribute__((always_inline)) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                fa[b2][i] = *(const bf16x8 *)(ts + fa_off[s2] + i * 32 * ROW_BYTES);
                fb[b2][i] = *(const bf16x8 *)(ts + fb_off[s2] + i * 32 * ROW_BYTES);
            }
        };
        lfrag(0, 0);
#pragma unroll
        for (int s2 = 0; s2 < BK / 16; ++s2) {
            if (s2 + 1 < BK / 16) lfrag(s2 + 1, (s2 + 1) & 1);   // fragments one k-step ahead
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[s2 & 1][i], fb[s2 & 1][j], acc[i][j], 0, 0, 0);
                const int r = s2 * 4 + i;                    // 16 MFMA rows per k-tile
                if (r < 8) {
                    lstore_piece(stage ^ 1, 2 * r);
                    lstore_piece(stage ^ 1, 2 * r + 1);
                } else {
                    gload_piece(kt + 2, 2 * (r - 8));
                    gload_piece(kt + 2, 2 * (r - 8) + 1);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __syncthreads();
    }

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
                for (int j = 0; j < 4; ++j) crow[j * 32] = acc[i][j][r];
            }
        }
    }
}

hipError_t launch_transpose_chunk(const void *W, int64_t ldw, int d, int64_t v0, int ncols, int npad,
                                  void *Wt, hipStream_t st)
{
    const dim3 grid((unsigned)((npad + 63) / 64), (unsigned)((d + 63) / 64));
    hipLaunchKernelGGL(transpose_chunk_kernel, grid, dim3(256), 0, st, (const uint16_t *)W, ldw, d, v0, ncols,
                       npad, (uint16_t *)Wt);
    return hipGetLastError();
}

hipError_t launch_gemm_pair(const GemmArgs &g, hipStream_t st)
{
    const int lds_bytes = 4 * TILE_BYTES;      // 128 KB: two stages of an A tile and a B tile
    hipError_t e = hipFuncSetAttribute((const void *)gemm_tn_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return e;
    const int tiles = ((g.M + BM - 1) / BM) * (g.N / BN);
    hipLaunchKernelGGL(gemm_tn_kernel, dim3((unsigned)tiles, 1, (unsigned)g.nproblems), dim3(GEMM_THREADS), lds_bytes, st, g);
    return hipGetLastError();
}

}  // namespace jp
