// bf16 GEMM on the gfx950 matrix cores:  C[M,N] = A[M,K] * W[N,K]^T, fp32
// accumulation.  Both operands are contiguous along K, so global loads, LDS
// tiles and MFMA fragments all move 16-byte chunks of 8 K-elements.
//
// A workgroup owns a BM x BN tile of C and walks K in steps of 64 with two LDS
// stages: while the matrix cores consume stage s, the next K-slab is already
// in flight from HBM into registers and is written to stage s^1 afterwards.
// Wave (wm, wn) owns a (BM/WM) x (BN/WN) sub-tile made of 32x32 MFMA tiles.
//
// Epilogues: plain bf16 store; residual add (bf16 residual in, fp32 out -- or
// fp32 residual in, bf16 out: the residual stream between the two halves of a
// layer stays in fp32, so it is rounded to bf16 once per layer); SiLU(gate)*up,
// where gate and up columns alternate in blocks of 32 so that both sit in the
// same lane.
#include "common.h"
#include "mfma.h"

namespace mvla {

constexpr int BK = 64;

// Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2.
// Every XCD gets one contiguous range of the tile sequence, and the sequence
// itself runs through groups of GROUP_M row-tiles column by column, so the ~32
// tiles an XCD has in flight form a GROUP_M x (32/GROUP_M) patch that re-uses
// both its activation rows and its weight panel out of that L2.
constexpr int GROUP_M = 8;
__device__ __forceinline__ bool tile_coords(int tiles_m, int tiles_n, int* tm, int* tn) {
    const int total = tiles_m * tiles_n;
    const int per_xcd = (total + 7) >> 3;
    const int lin = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (lin >= total) return false;
    const int group_tiles = GROUP_M * tiles_n;
    const int g = lin / group_tiles, r = lin % group_tiles;
    const int gm = min(GROUP_M, tiles_m - g * GROUP_M);  // rows in this (maybe last) group
    *tm = g * GROUP_M + r % gm;
    *tn = r / gm;
    return true;
}

template <int BM, int BN, int WM, int WN, int EPI>
__global__ __launch_bounds__(WM * WN * 64) void gemm_kernel(
    const bf16_t* __restrict__ A, int lda, const bf16_t* __restrict__ W, int M, int N, int K,
    void* __restrict__ Cv, int ldc, const void* __restrict__ Rv, int ldr, int tiles_m,
    int tiles_n) {
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM, TN = BN / WN;  // wave tile
    constexpr int FM = TM / 32, FN = TN / 32;  // MFMA tiles per wave
    constexpr int A_CH = BM * 8 / NT, B_CH = BN * 8 / NT;
    static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile/thread mismatch");
    static_assert(EPI != EPI_SILU_MUL || FN % 2 == 0, "gate/up pairs must share a wave");

    extern __shared__ uint4 lds[];
    uint4* As = lds;                 // [2][BM*8]
    uint4* Bs = lds + 2 * BM * 8;    // [2][BN*8]

    int tile_m, tile_n;
    if (!tile_coords(tiles_m, tiles_n, &tile_m, &tile_n)) return;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    // global source of every 16-byte chunk this thread stages
    const uint4* a_src[A_CH];
    const uint4* b_src[B_CH];
    int a_dst[A_CH], b_dst[B_CH];
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
        const int cid = tid + i * NT, row = cid >> 3, ch = cid & 7;
        const int gr = min(m0 + row, M - 1);
        a_src[i] = reinterpret_cast<const uint4*>(A + (size_t)gr * lda) + ch;
        a_dst[i] = lds_slot(row, ch);
    }
#pragma unroll
    for (int i = 0; i < B_CH; ++i) {
        const int cid = tid + i * NT, row = cid >> 3, ch = cid & 7;
        const int gr = min(n0 + row, N - 1);
        b_src[i] = reinterpret_cast<const uint4*>(W + (size_t)gr * K) + ch;
        b_dst[i] = lds_slot(row, ch);
    }

    f32x16_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    uint4 a_reg[A_CH], b_reg[B_CH];
    const int k_tiles = K / BK;
#pragma unroll
    for (int i = 0; i < A_CH; ++i) a_reg[i] = a_src[i][0];
#pragma unroll
    for (int i = 0; i < B_CH; ++i) b_reg[i] = b_src[i][0];
#pragma unroll
    for (int i = 0; i < A_CH; ++i) As[a_dst[i]] = a_reg[i];
#pragma unroll
    for (int i = 0; i < B_CH; ++i) Bs[b_dst[i]] = b_reg[i];
    __syncthreads();

    const int frag_row = lane & 31, frag_g = lane >> 5;
    for (int kt = 0; kt < k_tiles; ++kt) {
        const int cur = kt & 1;
        // next K-slab goes into flight before the matrix cores start on this one (the last
        // iteration re-fetches its own slab: harmless, keeps the loop free of branches)
        const int nk = min(kt + 1, k_tiles - 1) * 8;
#pragma unroll
        for (int i = 0; i < A_CH; ++i) a_reg[i] = a_src[i][nk];
#pragma unroll
        for (int i = 0; i < B_CH; ++i) b_reg[i] = b_src[i][nk];
        const uint4* Ac = As + cur * BM * 8;
        const uint4* Bc = Bs + cur * BN * 8;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            uint4 af[FM], bfr[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i)
                af[i] = Ac[lds_slot(wm * TM + i * 32 + frag_row, ks * 2 + frag_g)];
#pragma unroll
            for (int j = 0; j < FN; ++j)
                bfr[j] = Bc[lds_slot(wn * TN + j * 32 + frag_row, ks * 2 + frag_g)];
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j) acc[i][j] = mfma32(af[i], bfr[j], acc[i][j]);
        }
        uint4* An = As + (cur ^ 1) * BM * 8;
        uint4* Bn = Bs + (cur ^ 1) * BN * 8;
#pragma unroll
        for (int i = 0; i < A_CH; ++i) An[a_dst[i]] = a_reg[i];
#pragma unroll
        for (int i = 0; i < B_CH; ++i) Bn[b_dst[i]] = b_reg[i];
        __syncthreads();
    }

    // ---- epilogue: lane holds column (lane%32) and rows mfma32_row(v, lane) of each tile ----
    const int col_in_tile = lane & 31;
    bf16_t* C = static_cast<bf16_t*>(Cv);
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        const int row_base = m0 + wm * TM + i * 32;
        if (EPI == EPI_SILU_MUL) {
#pragma unroll
            for (int j = 0; j < FN; j += 2) {
                const int ncol = n0 + wn * TN + j * 32;  // gate block start (multiple of 64)
                const int ocol = (ncol >> 1) + col_in_tile;
                if (ncol + 32 + col_in_tile < N) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int row = row_base + mfma32_row(v, lane);
                        if (row < M) {
                            const float g = acc[i][j][v], u = acc[i][j + 1][v];
                            const float s = g / (1.f + __expf(-g));
                            C[(size_t)row * ldc + ocol] = f32_to_bf16(s * u);
                        }
                    }
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const int col = n0 + wn * TN + j * 32 + col_in_tile;
                if (col < N) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int row = row_base + mfma32_row(v, lane);
                        if (row < M) {
                            float val = acc[i][j][v];
                            if (EPI == EPI_RES_BF16_TO_F32) {
                                val += bf16_to_f32(
                                    static_cast<const bf16_t*>(Rv)[(size_t)row * ldr + col]);
                                static_cast<float*>(Cv)[(size_t)row * ldc + col] = val;
                            } else {
                                if (EPI == EPI_RES_F32_TO_BF16)
                                    val += static_cast<const float*>(Rv)[(size_t)row * ldr + col];
                                C[(size_t)row * ldc + col] = f32_to_bf16(val);
                            }
                        }
                    }
                }
            }
        }
    }
}

template <int BM, int BN, int WM, int WN>
static int launch_cfg(const bf16_t* A, int lda, const bf16_t* W, int M, int N, int K, void* C,
                      int ldc, const void* R, int ldr, int epi, hipStream_t st) {
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int total = tiles_m * tiles_n;
    const int grid = ((total + 7) / 8) * 8;
    const size_t lds = (size_t)2 * (BM + BN) * 8 * sizeof(uint4);
    dim3 block(WM * WN * 64);
#define MVLA_GEMM_LAUNCH(E)                                                                   \
    do {                                                                                      \
        auto kern = gemm_kernel<BM, BN, WM, WN, E>;                                           \
        if (lds > 64 * 1024) {                                                                \
            MVLA_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),           \
                                               hipFuncAttributeMaxDynamicSharedMemorySize,    \
                                               (int)lds));                                    \
        }                                                                                     \
        hipLaunchKernelGGL(kern, dim3(grid), block, lds, st, A, lda, W, M, N, K, C, ldc, R,   \
                           ldr, tiles_m, tiles_n);                                            \
    } while (0)
    if (epi == EPI_STORE) MVLA_GEMM_LAUNCH(EPI_STORE);
    else if (epi == EPI_RES_BF16_TO_F32) MVLA_GEMM_LAUNCH(EPI_RES_BF16_TO_F32);
    else if (epi == EPI_RES_F32_TO_BF16) MVLA_GEMM_LAUNCH(EPI_RES_F32_TO_BF16);
    else MVLA_GEMM_LAUNCH(EPI_SILU_MUL);
#undef MVLA_GEMM_LAUNCH
    MVLA_HIP_CHECK(hipGetLastError());
    return MVLA_OK;
}

int launch_gemm(const bf16_t* A, int lda, const bf16_t* W, int M, int N, int K, void* C, int ldc,
                const void* R, int ldr, int epilogue, hipStream_t st) {
    if (M <= 0 || N <= 0) return MVLA_OK;
    if (K % BK != 0 || lda % 8 != 0) return MVLA_EUNSUPPORTED;
    if (epilogue == EPI_SILU_MUL && N % 64 != 0) return MVLA_EUNSUPPORTED;
    // Large problems: 256x128 tiles (4 waves of 128x64).  Small M: 128x128 tiles.
    if (M >= 1024)
        return launch_cfg<256, 128, 2, 2>(A, lda, W, M, N, K, C, ldc, R, ldr, epilogue, st);
    return launch_cfg<128, 128, 2, 2>(A, lda, W, M, N, K, C, ldc, R, ldr, epilogue, st);
}

}  // namespace mvla
