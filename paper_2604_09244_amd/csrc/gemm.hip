// bf16 GEMM on the gfx950 matrix cores:  C[M,N] = A[M,K] * W[N,K]^T, fp32
// accumulation.  Both operands are contiguous along K, so HBM reads, LDS tiles
// and MFMA fragments all move 16-byte chunks of 8 K-elements.
//
// Data path.  K-slabs of the A and W tiles go from global memory straight into
// LDS (global_load_lds, 16 bytes per lane, no register staging) into a ring of
// NS stages, so the next slab(s) are in flight while the matrix cores work on
// the current one.  The LDS image is XOR-swizzled; because a direct load
// always lands its 64 lanes on 1 KiB of consecutive LDS, the swizzle is applied
// on the global side: lane l fetches the chunk that belongs at its slot.
// MFMA fragments are double-buffered in registers: the ds_reads of k-step s+1
// (and, across the stage barrier, of the next slab) are issued before the MFMAs
// of step s.
//
// Work split.  A workgroup owns a BM x BN tile; its waves own (BM/WM) x (BN/WN)
// sub-tiles of 32x32 MFMA blocks (wave rows overlap by a block where the 32-row
// blocks do not divide).  Tiles that fill whole rounds of the chip
// are computed start to finish by one workgroup.  The tiles of the last,
// partial round are cut along K into equal ranges of k-iterations handed out
// contiguously to the otherwise idle CUs; the pieces of a tile meet in an fp32
// partial buffer and whichever piece arrives last (integer arrival counter)
// adds them up in fixed piece order and runs the epilogue, so results do not
// depend on timing.
//
// Epilogues: the q/k/v projection (q and k columns rotated by the row's position
// on the fp32 accumulators and stored as bf16, v columns stored transposed for
// the attention kernel); residual add (bf16 residual in, fp32 out -- or
// fp32 residual in, bf16 out: the residual stream between the two halves of a
// layer stays in fp32, so it is rounded to bf16 once per layer); SiLU(gate)*up,
// where gate and up columns alternate in blocks of 32 (one 64-column group holds a
// gate block and its up block).  Every epilogue lays the accumulator tile down in
// LDS as fp32 rows first, so residual reads and result stores are 16 bytes per
// lane on whole cache lines; K-split tiles take the same route after the pieces
// are summed.
#include "common.h"
#include "mfma.h"

namespace mvla {

// direct global -> LDS copy of 16 bytes per lane: the wave's 64 lanes land on 1 KiB starting
// at the wave-uniform LDS byte address lds_addr.  Not tracked by the compiler's wait-count
// insertion; every consumer is ordered behind wait_vm<>() and a workgroup barrier.
__device__ __forceinline__ void dma16(const void* g, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr),
                 "v"(g)
                 : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_vm() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Partial sums cross between CUs (and XCDs, each with its own L2) through agent-coherent
// accesses, which go to the shared level of the memory system one access at a time; nothing
// here needs a whole-cache write-back or invalidate.
typedef float f32q_t __attribute__((ext_vector_type(4)));
// The wait states after the store keep the next VALU write away from the data registers
// (a store of more than 64 bits reads them late; the compiler cannot see that inside asm).
__device__ __forceinline__ void st16_coherent(float* p, f32q_t v) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 2" ::"v"(p), "v"(v) : "memory");
}
// Issues the load; the value may be used only after settle() has been applied to it.
__device__ __forceinline__ f32q_t ld16_coherent(const float* p) {
    f32q_t v;
    asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v) : "v"(p) : "memory");
    return v;
}
// Output (and residual) of the epilogues as a bounds-checked buffer: a lane whose byte offset lies
// at or beyond the record count is dropped (stores) or reads zeros (loads) by the hardware.  A
// lane that has nothing to write gets the offset OOB_OFFSET instead of a branch around its store:
// the stream of memory instructions is then the same for every lane, and the compiler's count of
// outstanding ones -- which places the waits for the residual reads -- is exact (a store that may
// or may not have been issued makes it wait for the stores before as well: loads and stores
// return in issue order).
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
constexpr int OOB_OFFSET = 0x7FFF0000;
__device__ __forceinline__ __amdgpu_buffer_rsrc_t buffer_of(const void* base, int bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes > 0 ? bytes : 0, 0x00020000);
}
__device__ __forceinline__ void settle(f32q_t& a, f32q_t& b, f32q_t& c, f32q_t& d) {
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d)::"memory");
}

constexpr int GROUP_M = 8;
constexpr int SK_MIN_ITERS = 8;    // smallest K-range worth its own workgroup (in slabs)
constexpr int SK_MAX_PIECES = 64;  // most pieces one tile is ever cut into

// An LDS row holds one K-slab of a tile row: CPR = BK/8 chunks of 16 bytes.  Chunk c of row r
// lives at slot r*CPR + (c ^ swz(r)) with swz(r) = (r >> 1) & 7 for 128-byte rows and
// (r >> 2) & 3 for 64-byte rows: both conflict-free for the 32-row x 16-byte fragment reads
// (measured: SQ_LDS_BANK_CONFLICT = 0).
template <int CPR>
__device__ __forceinline__ int swz(int row) {
    return CPR == 8 ? (row >> 1) & 7 : (row >> 2) & 3;
}

struct GemmPlan {
    int tiles_m, tiles_n, k_tiles;
    int dp_tiles;     // tiles computed whole by one workgroup
    int dp_grid;      // dp_tiles rounded up to a multiple of 8 (workgroup ids 0 .. dp_grid-1)
    int sk_tiles;     // tiles of the last partial round, split along K
    int sk_blocks;    // workgroups sharing the sk_tiles * k_tiles iterations
};

// Workgroup ids are dealt round-robin to the 8 XCDs (each has its own L2).  Give every XCD a
// contiguous range of the sequence, and run the sequence through groups of GROUP_M row-tiles
// column by column, so the tiles an XCD has in flight share activation rows and weight panels.
__device__ __forceinline__ int xcd_chunked(int id, int total) {
    return (id & 7) * ((total + 7) >> 3) + (id >> 3);  // may be >= total for padded ids
}
__device__ __forceinline__ void tile_of(int lin, int tiles_m, int tiles_n, int* tm, int* tn) {
    const int group_tiles = GROUP_M * tiles_n;
    const int g = lin / group_tiles, r = lin % group_tiles;
    const int gm = min(GROUP_M, tiles_m - g * GROUP_M);
    *tm = g * GROUP_M + r % gm;
    *tn = r / gm;
}

// Epilogue staging: the output tile goes through LDS as fp32 rows of BN + 4 floats (the 4 keep
// 16-byte accesses of 32 consecutive rows on different banks), RP rows per pass.  The whole tile
// in one pass if the LDS a workgroup may use holds it, else one wave row per pass.
template <int BM, int BN, int WM, int NS>
struct EpiGeom {
    static constexpr int LDT = BN + 4;
    static constexpr int CAP = (NS == 2 && BM == 128 && BN == 128) ? 76 * 1024 : 156 * 1024;
    static constexpr int TM = (BM / 32 + WM - 1) / WM * 32;   // rows of a wave row
    static constexpr int PASSES = BM * LDT * 4 <= CAP ? 1 : WM;
    static constexpr int RP = PASSES == 1 ? BM : TM;
    static constexpr int BYTES = RP * LDT * 4;
    static_assert(BYTES <= CAP, "epilogue tile does not fit the LDS");
    static_assert(TM * WM == BM || PASSES == WM, "overlapping wave rows go one per pass");
};

template <int BM, int BN, int BK, int WM, int WN, int NS, int EPI>
__global__ __launch_bounds__(WM * WN * 64) void gemm_kernel(
    const bf16_t* __restrict__ A, int lda, const bf16_t* __restrict__ W, int M, int N, int K,
    void* __restrict__ Cv, int ldc, const void* __restrict__ Rv, int ldr, GemmPlan plan,
    float* __restrict__ partial, uint32_t* __restrict__ counters, RopeEpilogue rope) {
    constexpr int NT = WM * WN * 64;
    constexpr int CPR = BK / 8;             // 16-byte chunks per LDS row
    constexpr int KS = BK / 16;             // MFMA k-steps per slab
    // A wave owns FM x FN accumulator blocks of 32x32.  When the tile's 32-row blocks do not
    // divide among the WM wave rows (288 rows on two wave rows), every wave row still takes
    // FM = ceil blocks and the last one starts early: the rows both cover are computed twice
    // (identical values) so that the main loop stays free of branches.
    constexpr int FM = (BM / 32 + WM - 1) / WM, TM = FM * 32, TN = BN / WN, FN = TN / 32;
    static_assert(BM % 32 == 0 && BN % (32 * WN) == 0 && TM <= BM, "");
    constexpr int STAGE = (BM + BN) * CPR;  // 16-byte slots per stage
    constexpr int A_SLOTS = BM * CPR, B_SLOTS = BN * CPR;   // 16-byte slots of the A and W tiles
    constexpr int A_LD = A_SLOTS / NT, B_LD = B_SLOTS / NT;
    constexpr int P = A_LD + B_LD;          // direct loads per thread per slab
    static_assert(A_SLOTS % NT == 0 && B_SLOTS % NT == 0, "tile/thread mismatch");
    static_assert(KS % 2 == 0 && NS >= 2, "");

    extern __shared__ uint4 lds[];
    __shared__ int sh_last;
    __shared__ int sh_slot[SK_MAX_PIECES];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int wrow0 = min(wm * TM, BM - TM);   // first tile row of this wave's blocks
    const int fr = lane & 31, fg = lane >> 5;
    const int k_tiles = plan.k_tiles;

    // ---- which part of which tile is ours --------------------------------------------------
    int n_seg_work;   // 1 for a whole tile, up to 2 for a K-range that straddles two tiles
    int it_begin = 0, it_end = 0, sk_id = 0;
    const bool is_dp = (int)blockIdx.x < plan.dp_grid;
    if (is_dp) {
        n_seg_work = xcd_chunked(blockIdx.x, plan.dp_tiles) < plan.dp_tiles ? 1 : 0;
    } else {
        // K-split workgroups in XCD-contiguous order too: the pieces of a tile, and the tiles that
        // share a weight panel, then run on one XCD at the same time and share its L2
        const int id = blockIdx.x - plan.dp_grid, x = id & 7;   // dp_grid is a multiple of 8
        sk_id = x * (plan.sk_blocks >> 3) + min(x, plan.sk_blocks & 7) + (id >> 3);
        const long total = (long)plan.sk_tiles * k_tiles;
        it_begin = (int)(total * sk_id / plan.sk_blocks);
        it_end = (int)(total * (sk_id + 1) / plan.sk_blocks);
        n_seg_work = (it_begin / k_tiles == (it_end - 1) / k_tiles) ? 1 : 2;
    }

    for (int seg = 0; seg < n_seg_work; ++seg) {
        int lin, k0, k1, sk_tile = -1, first_blk = 0, last_blk = 0;
        if (is_dp) {
            lin = xcd_chunked(blockIdx.x, plan.dp_tiles);
            k0 = 0;
            k1 = k_tiles;
        } else {
            const int it0 = seg == 0 ? it_begin : (it_begin / k_tiles + 1) * k_tiles;
            sk_tile = it0 / k_tiles;
            const int it1 = min(it_end, (sk_tile + 1) * k_tiles);
            k0 = it0 - sk_tile * k_tiles;
            k1 = it1 - sk_tile * k_tiles;
            lin = plan.dp_tiles + sk_tile;
            // workgroups whose ranges touch this tile: the one holding its first and its last slab
            const long total = (long)plan.sk_tiles * k_tiles;
            first_blk = (int)((((long)sk_tile * k_tiles + 1) * plan.sk_blocks - 1) / total);
            last_blk = (int)((((long)(sk_tile + 1) * k_tiles) * plan.sk_blocks - 1) / total);
        }
        int tile_m, tile_n;
        tile_of(lin, plan.tiles_m, plan.tiles_n, &tile_m, &tile_n);
        const int m0 = tile_m * BM, n0 = tile_n * BN;

        // ---- direct-load mapping: op i covers slot i*NT + tid of the A (or W) tile ----------
        const bf16_t* a_src[A_LD];
        const bf16_t* b_src[B_LD];
        uint32_t a_lds[A_LD], b_lds[B_LD];
        const uint32_t lds_base = (uint32_t)(uintptr_t)lds;
#pragma unroll
        for (int i = 0; i < A_LD; ++i) {
            const int sl = i * NT + tid, row = sl / CPR, ch = (sl % CPR) ^ swz<CPR>(row);
            a_src[i] = A + (size_t)min(m0 + row, M - 1) * lda + ch * 8;
            a_lds[i] = __builtin_amdgcn_readfirstlane(
                lds_base + (uint32_t)(i * NT + wave * 64) * 16u);
        }
#pragma unroll
        for (int i = 0; i < B_LD; ++i) {
            const int sl = i * NT + tid, row = sl / CPR, ch = (sl % CPR) ^ swz<CPR>(row);
            b_src[i] = W + (size_t)min(n0 + row, N - 1) * K + ch * 8;
            b_lds[i] = __builtin_amdgcn_readfirstlane(
                lds_base + (uint32_t)(A_SLOTS + i * NT + wave * 64) * 16u);
        }
        int a_row[FM], b_row[FN];
#pragma unroll
        for (int i = 0; i < FM; ++i) a_row[i] = wrow0 + i * 32 + fr;
#pragma unroll
        for (int j = 0; j < FN; ++j) b_row[j] = wn * TN + j * 32 + fr;

        f32x16_t acc[FM][FN];
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

#define MVLA_ISSUE(KT, STG)                                                                    \
    {                                                                                          \
        const int koff = min((KT), k1 - 1) * BK;                                               \
        const uint32_t soff = (uint32_t)(STG) * STAGE * 16u;                                   \
        _Pragma("unroll") for (int i = 0; i < A_LD; ++i) dma16(a_src[i] + koff, a_lds[i] + soff); \
        _Pragma("unroll") for (int i = 0; i < B_LD; ++i) dma16(b_src[i] + koff, b_lds[i] + soff); \
    }
#define MVLA_READ_FRAGS(AF, BF, STG, S)                                                        \
    {                                                                                          \
        const uint4* As_ = lds + (STG) * STAGE;                                                \
        const uint4* Bs_ = As_ + BM * CPR;                                                     \
        _Pragma("unroll") for (int i = 0; i < FM; ++i) AF[i] =                                 \
            As_[a_row[i] * CPR + (((S) * 2 + fg) ^ swz<CPR>(a_row[i]))];                            \
        _Pragma("unroll") for (int j = 0; j < FN; ++j) BF[j] =                                 \
            Bs_[b_row[j] * CPR + (((S) * 2 + fg) ^ swz<CPR>(b_row[j]))];                            \
    }
#define MVLA_MFMA(AF, BF)                                                                      \
    {                                                                                          \
        _Pragma("unroll") for (int i = 0; i < FM; ++i) _Pragma("unroll") for (int j = 0; j < FN; ++j) \
            acc[i][j] = mfma32(BF[j], AF[i], acc[i][j]);                                       \
    }

// Scheduling of one k-step: the fragment reads of the next step are dealt out between this
// step's MFMAs (MPR MFMAs, then one read, ...) instead of going out in one burst.
#define MVLA_SPREAD_READS                                                                      \
    {                                                                                          \
        constexpr int MPR = (FM * FN) / (FM + FN) > 0 ? (FM * FN) / (FM + FN) : 1;             \
        _Pragma("unroll") for (int r = 0; r < FM + FN; ++r) {                                  \
            __builtin_amdgcn_sched_group_barrier(0x008, MPR, 0);                               \
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                 \
        }                                                                                      \
        __builtin_amdgcn_sched_group_barrier(0x008, FM * FN, 0);                               \
        __builtin_amdgcn_sched_barrier(0);                                                     \
    }
// the MFMAs of one k-step with the direct loads of slab KT dealt out between them, one per MFMA
// (a wave that is alone on its SIMD would otherwise issue nothing to the matrix core while it
// sets up the loads)
#define MVLA_MFMA_ISSUE(AF, BF, KT, STG)                                                       \
    {                                                                                          \
        const int koff = min((KT), k1 - 1) * BK;                                               \
        const uint32_t soff = (uint32_t)(STG) * STAGE * 16u;                                   \
        int n_ = 0;                                                                            \
        _Pragma("unroll") for (int i = 0; i < FM; ++i) _Pragma("unroll") for (int j = 0; j < FN; ++j) { \
            acc[i][j] = mfma32(BF[j], AF[i], acc[i][j]);                                       \
            if (n_ < A_LD) dma16(a_src[n_ < A_LD ? n_ : 0] + koff, a_lds[n_ < A_LD ? n_ : 0] + soff); \
            else if (n_ < P) dma16(b_src[n_ < P ? n_ - A_LD : 0] + koff, b_lds[n_ < P ? n_ - A_LD : 0] + soff); \
            __builtin_amdgcn_sched_barrier(0);                                                 \
            ++n_;                                                                              \
        }                                                                                      \
        _Pragma("unroll") for (int r = FM * FN; r < P; ++r) {                                  \
            if (r < A_LD) dma16(a_src[r < A_LD ? r : 0] + koff, a_lds[r < A_LD ? r : 0] + soff);     \
            else dma16(b_src[r - A_LD] + koff, b_lds[r - A_LD] + soff);                        \
        }                                                                                      \
    }

        // every thread of the workgroup has left the previous segment's LDS reads behind
        __syncthreads();
        // ... and nothing the compiler keeps count of (a previous segment's epilogue loads and
        // stores) is outstanding any more: a wait it placed for those inside the main loop would
        // also wait for the loop's direct loads, which it does not see
        __builtin_amdgcn_s_waitcnt(0);
        // ---- prologue: NS-1 slabs in flight, then one more behind the first barrier ---------
#pragma unroll
        for (int s = 0; s < NS - 1; ++s) MVLA_ISSUE(k0 + s, s)
        uint4 af0[FM], bf0[FN], af1[FM], bf1[FN];
        wait_vm<(NS - 2) * P>();
        __syncthreads();
        if constexpr (NS >= 3 && KS == 4 && P >= 4) {   // (the loop's first three k-steps issue the rest)
            const int koff = min(k0 + NS - 1, k1 - 1) * BK;
            const uint32_t soff = (uint32_t)(NS - 1) * STAGE * 16u;
#pragma unroll
            for (int r = 0; r < P / 4; ++r) {
                if (r < A_LD) dma16(a_src[r < A_LD ? r : 0] + koff, a_lds[r < A_LD ? r : 0] + soff);
                else dma16(b_src[r < P ? r - A_LD : 0] + koff, b_lds[r < P ? r - A_LD : 0] + soff);
            }
        } else {
            MVLA_ISSUE(k0 + NS - 1, NS - 1)
        }
        MVLA_READ_FRAGS(af0, bf0, 0, 0)
        int stage = 0;
        // Four-wave shapes (registers to spare).  The load unit of a CU takes one 64-lane direct
        // load per 16 clocks, so the 64 loads of a 256x256x64 slab need 1024 clocks of it -- two
        // k-steps.  Issued all in the last k-step (as the other shapes do), they kept the waves
        // standing at load issue instead of feeding the matrix core: 1100 - 1800 clocks for that
        // k-step instead of 512 (cycle counters in a working copy).  Here a slab's fragments are
        // read two k-steps ahead -- those of k-steps 2 and 3 during k-step 0, those of the next
        // slab's k-steps 0 and 1 during k-step 3, one LDS read after each MFMA -- so the stage is
        // free after k-step 0 and the loads of slab kt+2 go out a third each over k-steps 1, 2
        // and 3, with the wait for slab kt+1 before the last.
        constexpr bool DEEP = WM * WN == 4 && NS == 2 && KS == 4 && P >= 3;
        // Shapes with three stages always have a free one: the loads of a slab go out a quarter
        // per k-step (the last k-step of one iteration and the first three of the next) instead
        // of all in one, for the same reason.
        constexpr bool SPREAD4 = NS >= 3 && KS == 4 && P >= 4;
        constexpr int NR = 2 * (FM + FN);   // fragment reads of two k-steps
// read number R of the fragments of k-steps SA (first FM + FN reads, into AFA/BFA) and
// SB (the rest, into AFB/BFB) of stage STG
#define MVLA_READ_ONE(AFA, BFA, AFB, BFB, STG, SA, SB, R)                                      \
    {                                                                                          \
        const uint4* As_ = lds + (STG) * STAGE;                                                \
        const uint4* Bs_ = As_ + BM * CPR;                                                     \
        const int set_ = (R) / (FM + FN), idx_ = (R) % (FM + FN);                              \
        const int ks_ = set_ == 0 ? (SA) : (SB);                                               \
        if (idx_ < FM) {                                                                       \
            const int ii_ = idx_ < FM ? idx_ : 0;                                              \
            const uint4 v_ = As_[a_row[ii_] * CPR + ((ks_ * 2 + fg) ^ swz<CPR>(a_row[ii_]))];  \
            if (set_ == 0) AFA[ii_] = v_; else AFB[ii_] = v_;                                  \
        } else {                                                                               \
            const int jj_ = idx_ >= FM ? idx_ - FM : 0;                                        \
            const uint4 v_ = Bs_[b_row[jj_] * CPR + ((ks_ * 2 + fg) ^ swz<CPR>(b_row[jj_]))];  \
            if (set_ == 0) BFA[jj_] = v_; else BFB[jj_] = v_;                                  \
        }                                                                                      \
    }
// the MFMAs of one k-step; after MFMA n comes fragment read n (of NRD) of (RSTG; SA, SB), and
// the direct loads [L0, L1) of slab KT into stage STG are dealt out evenly
#define MVLA_STEP(AF, BF, NRD, AFA, BFA, AFB, BFB, RSTG, SA, SB, KT, STG, L0, L1)            \
    {                                                                                          \
        const int koff = min((KT), k1 - 1) * BK;                                               \
        const uint32_t soff = (uint32_t)(STG) * STAGE * 16u;                                   \
        constexpr int NL_ = (L1) - (L0);                                                       \
        constexpr int EVERY_ = NL_ > 0 && (FM * FN) / (NL_ > 0 ? NL_ : 1) > 0 ? (FM * FN) / (NL_ > 0 ? NL_ : 1) : 1; \
        int n_ = 0, l_ = (L0);                                                                 \
        _Pragma("unroll") for (int i = 0; i < FM; ++i) _Pragma("unroll") for (int j = 0; j < FN; ++j) { \
            acc[i][j] = mfma32(BF[j], AF[i], acc[i][j]);                                       \
            if (n_ < (NRD)) MVLA_READ_ONE(AFA, BFA, AFB, BFB, RSTG, SA, SB, n_)                \
            if (n_ % EVERY_ == EVERY_ - 1 && l_ < (L1)) {                                      \
                if (l_ < A_LD) dma16(a_src[l_ < A_LD ? l_ : 0] + koff, a_lds[l_ < A_LD ? l_ : 0] + soff); \
                else dma16(b_src[l_ < P ? l_ - A_LD : 0] + koff, b_lds[l_ < P ? l_ - A_LD : 0] + soff);   \
                ++l_;                                                                          \
            }                                                                                  \
            __builtin_amdgcn_sched_barrier(0);                                                 \
            ++n_;                                                                              \
        }                                                                                      \
        _Pragma("unroll") for (int r = FM * FN; r < (NRD); ++r)                                \
            MVLA_READ_ONE(AFA, BFA, AFB, BFB, RSTG, SA, SB, r)                                 \
        _Pragma("unroll") for (int r = 0; r < P; ++r)                                          \
            if (r >= l_ && r < (L1)) {                                                         \
                if (r < A_LD) dma16(a_src[r < A_LD ? r : 0] + koff, a_lds[r < A_LD ? r : 0] + soff); \
                else dma16(b_src[r - A_LD] + koff, b_lds[r - A_LD] + soff);                    \
            }                                                                                  \
    }
        if constexpr (DEEP) {
            uint4 af2[FM], bf2[FN], af3[FM], bf3[FN];
            constexpr int L1_ = P / 3, L2_ = 2 * P / 3;
            MVLA_READ_FRAGS(af1, bf1, 0, 1)
            for (int kt = k0; kt < k1; ++kt) {
                const int nstage = stage ^ 1;
                // k-step 0, reading the fragments of k-steps 2 and 3: after it this slab is in registers
                MVLA_STEP(af0, bf0, NR, af2, bf2, af3, bf3, stage, 2, 3, kt + 2, stage, 0, 0)
                __syncthreads();   // ... for every wave: the stage is free for slab kt+2
                MVLA_STEP(af1, bf1, 0, af2, bf2, af3, bf3, stage, 2, 3, kt + 2, stage, 0, L1_)
                MVLA_STEP(af2, bf2, 0, af2, bf2, af3, bf3, stage, 2, 3, kt + 2, stage, L1_, L2_)
                // slab kt+1 has landed for every wave (the two thirds of slab kt+2 may be in flight)
                wait_vm<L2_>();
                __syncthreads();
                // k-step 3, reading the fragments of k-steps 0 and 1 of the next slab
                MVLA_STEP(af3, bf3, NR, af0, bf0, af1, bf1, nstage, 0, 1, kt + 2, stage, L2_, P)
                stage = nstage;
            }
        } else if constexpr (SPREAD4) {
            constexpr int Q1 = P / 4, Q2 = P / 2, Q3 = 3 * P / 4;
            for (int kt = k0; kt < k1; ++kt) {
                const int nstage = stage + 1 == NS ? 0 : stage + 1;
                const int pstage = stage == 0 ? NS - 1 : stage - 1;   // freed one iteration ago
                MVLA_STEP(af0, bf0, FM + FN, af1, bf1, af1, bf1, stage, 1, 1, kt + NS - 1, pstage, Q1, Q2)
                MVLA_STEP(af1, bf1, FM + FN, af0, bf0, af0, bf0, stage, 2, 2, kt + NS - 1, pstage, Q2, Q3)
                MVLA_STEP(af0, bf0, FM + FN, af1, bf1, af1, bf1, stage, 3, 3, kt + NS - 1, pstage, Q3, P)
                // slab kt+1 has landed for every wave; slab kt's stage is free for slab kt+NS
                wait_vm<(NS - 2) * P>();
                __syncthreads();
                MVLA_STEP(af1, bf1, FM + FN, af0, bf0, af0, bf0, nstage, 0, 0, kt + NS, stage, 0, Q1)
                stage = nstage;
            }
        } else
        for (int kt = k0; kt < k1; ++kt) {
            const int nstage = stage + 1 == NS ? 0 : stage + 1;
#pragma unroll
            for (int s = 0; s < KS - 2; s += 2) {
                MVLA_READ_FRAGS(af1, bf1, stage, s + 1)
                MVLA_MFMA(af0, bf0)
                MVLA_SPREAD_READS
                MVLA_READ_FRAGS(af0, bf0, stage, s + 2)
                MVLA_MFMA(af1, bf1)
                MVLA_SPREAD_READS
            }
            MVLA_READ_FRAGS(af1, bf1, stage, KS - 1)
            MVLA_MFMA(af0, bf0)
            MVLA_SPREAD_READS
            // slab kt+1 has landed for every wave; slab kt's stage is free for slab kt+NS
            wait_vm<(NS - 2) * P>();
            __syncthreads();
            MVLA_READ_FRAGS(af0, bf0, nstage, 0)
            __builtin_amdgcn_sched_barrier(0);
            MVLA_MFMA_ISSUE(af1, bf1, kt + NS, stage)
            stage = nstage;
        }
        wait_vm<0>();
#undef MVLA_ISSUE
#undef MVLA_READ_FRAGS
#undef MVLA_MFMA
#undef MVLA_MFMA_ISSUE
#undef MVLA_SPREAD_READS
#undef MVLA_READ_ONE
#undef MVLA_STEP

        // ---- K-split tiles: park the partial sums; the last piece to arrive finishes --------
        // (the four-wave 128x128-per-wave shape keeps its register budget for the main loop:
        // whole tiles only, the host never plans a K-split for it)
        constexpr bool HAS_SK = !(WM * WN == 4 && FM * FN >= 15);
        const int n_pieces = (!HAS_SK || is_dp) ? 1 : last_blk - first_blk + 1;
        if (HAS_SK && n_pieces > 1) {
            // slot 0 of a workgroup holds the piece of the tile its range starts in, slot 1 the next
            const int my_slot = 2 * sk_id + (seg == 0 ? 0 : 1);
            float* mine = partial + (size_t)my_slot * (BM * BN);
            // 16 bytes per lane: register quad c of block (i,j) goes to float offset
            // (((i*FN + j)*4 + c)*NT + tid)*4 of the slot
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        f32q_t q = {acc[i][j][4 * c], acc[i][j][4 * c + 1], acc[i][j][4 * c + 2],
                                    acc[i][j][4 * c + 3]};
                        st16_coherent(&mine[(((i * FN + j) * 4 + c) * NT + tid) * 4], q);
                    }
            wait_vm<0>();     // this thread's partial sums have reached the coherent level
            __syncthreads();  // ... and so have everyone else's in the workgroup
            if (tid == 0) {
                const uint32_t prev = __hip_atomic_fetch_add(&counters[sk_tile], 1u, __ATOMIC_RELAXED,
                                                             __HIP_MEMORY_SCOPE_AGENT);
                sh_last = (prev == (uint32_t)(n_pieces - 1));
                if (sh_last)
                    __hip_atomic_store(&counters[sk_tile], 0u, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
            }
            if (tid < n_pieces) {
                // piece of workgroup b: its slot 0 if b's range starts inside this tile, else 1
                const long total = (long)plan.sk_tiles * k_tiles;
                const int b = first_blk + tid;
                const int b_start_tile = (int)(total * b / plan.sk_blocks) / k_tiles;
                sh_slot[tid] = 2 * b + (b_start_tile == sk_tile ? 0 : 1);
            }
            __syncthreads();
            if (!sh_last) continue;
            // Sum the pieces in piece order (so the order of additions never depends on who came
            // last), several 16-byte loads in flight at a time; then the common epilogue below.
            // With few accumulator registers the own piece is taken from a register copy instead
            // of being read back, and two pieces are fetched per round trip.
            constexpr int NQ = FM * FN * 4;                       // quads per thread per piece
            // (not for the shape that runs two workgroups per CU: the copy would cost it that)
            constexpr bool KEEP_OWN = NQ <= 16 && !(NS == 2 && BM == 128 && BN == 128);
            constexpr int CH_MAX = (NQ <= 16) ? 16 : 8;           // quads in flight
            constexpr int CH = (CH_MAX >= 16 && NQ % 16 == 0) ? 16
                               : (CH_MAX >= 12 && NQ % 12 == 0) ? 12
                               : (NQ % 8 == 0) ? 8 : 4;
            static_assert(NQ % CH == 0 && CH % 4 == 0, "");
            constexpr int PPR = (KEEP_OWN && 2 * NQ <= 16) ? 2 : 1;   // pieces per round trip
            f32x16_t own[KEEP_OWN ? FM : 1][KEEP_OWN ? FN : 1];
            const int my_piece = KEEP_OWN ? sk_id - first_blk : -1;
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    if (KEEP_OWN) own[i][j] = acc[i][j];
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
                }
#pragma unroll 1
            for (int pc = 0; pc < n_pieces; pc += PPR) {
                if (PPR == 2) {
                    // both pieces of the pair in flight together (own piece: no load)
                    f32q_t t[2][NQ];
                    const int p1 = min(pc + 1, n_pieces - 1);
                    const float* s0 = partial + (size_t)sh_slot[pc] * (BM * BN) + tid * 4;
                    const float* s1 = partial + (size_t)sh_slot[p1] * (BM * BN) + tid * 4;
                    if (pc != my_piece)
#pragma unroll
                        for (int q = 0; q < NQ; ++q) t[0][q] = ld16_coherent(&s0[(size_t)q * NT * 4]);
                    if (pc + 1 < n_pieces && pc + 1 != my_piece)
#pragma unroll
                        for (int q = 0; q < NQ; ++q) t[1][q] = ld16_coherent(&s1[(size_t)q * NT * 4]);
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int q = 0; q < NQ; q += 4) settle(t[h][q], t[h][q + 1], t[h][q + 2], t[h][q + 3]);
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        if (pc + h >= n_pieces) break;
                        const bool mine = (pc + h == my_piece);
#pragma unroll
                        for (int q = 0; q < NQ; ++q) {
                            const int blk = q / 4, c = q % 4;
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                acc[blk / FN][blk % FN][4 * c + e] +=
                                    mine ? own[KEEP_OWN ? blk / FN : 0][KEEP_OWN ? blk % FN : 0][4 * c + e]
                                         : t[h][q][e];
                        }
                    }
                } else {
                    const bool mine = (pc == my_piece);
                    const float* src = partial + (size_t)sh_slot[pc] * (BM * BN) + tid * 4;
#pragma unroll
                    for (int q0 = 0; q0 < NQ; q0 += CH) {
                        f32q_t t[CH];
                        if (!mine) {
#pragma unroll
                            for (int q = 0; q < CH; ++q)
                                t[q] = ld16_coherent(&src[(size_t)(q0 + q) * NT * 4]);
                        }
#pragma unroll
                        for (int q = 0; q < CH; q += 4) settle(t[q], t[q + 1], t[q + 2], t[q + 3]);
#pragma unroll
                        for (int q = 0; q < CH; ++q) {
                            const int blk = (q0 + q) / 4, c = (q0 + q) % 4;
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                acc[blk / FN][blk % FN][4 * c + e] +=
                                    mine ? own[KEEP_OWN ? blk / FN : 0][KEEP_OWN ? blk % FN : 0][4 * c + e]
                                         : t[q][e];
                        }
                    }
                }
            }
        }

        // ---- epilogue through LDS: the MFMAs are issued with the weight fragment as the first
        // operand, so a lane of an accumulator block holds one tile row and its registers four
        // consecutive columns at a time: the tile is laid down as fp32 rows with 16-byte stores,
        // then every thread takes 8 consecutive columns of a row (4 where an fp32 matrix is read or
        // written), so the residual is read and the result written with one access per lane on
        // whole consecutive cache lines.  A pass covers as many tile rows as the LDS holds (a whole
        // number of wave rows); only the waves owning them write.
        using EG = EpiGeom<BM, BN, WM, NS>;
        constexpr int LDT = EG::LDT, PASSES = EG::PASSES, RP = EG::RP;
        constexpr int OUT_COLS = EPI == EPI_SILU_MUL ? BN / 2 : BN;   // output columns per tile
        static_assert(RP % 16 == 0, "row groups of 8 come in pairs");
        constexpr int ITEMS = RP * OUT_COLS / 8;                      // 8-column items per pass
        float* tile = reinterpret_cast<float*>(lds);
        // (the epilogue's per-thread indices are computed here, not before the main loop, where
        // the compiler would otherwise put them and keep them in registers the loop needs)
        int etid = tid;
        asm volatile("" : "+v"(etid));
        const int out_n0 = EPI == EPI_SILU_MUL ? n0 / 2 : n0;
        const int out_N = EPI == EPI_SILU_MUL ? N / 2 : N;
#pragma unroll 1
        for (int pass = 0; pass < PASSES; ++pass) {
            // first tile row of the pass (with overlapping wave rows the last pass starts early)
            const int prow0 = PASSES == 1 ? 0 : min(pass * TM, BM - TM);
            // q/k rotation: the position ids of this thread's items of the pass, fetched while
            // the tile is laid down (items: 8 columns of a half head, BN/16 per row)
            constexpr int PER_ROW = BN / 16;
            constexpr int QB = (FM * FN >= 8 && WM * WN >= 8) ? 2 : 4;   // items whose table rows fly together
            constexpr int NB = (RP * PER_ROW + QB * NT - 1) / (QB * NT);
            constexpr bool PREFETCH = EPI == EPI_QKV_ROPE && QB == 4;   // (registers to spare)
            int pos_pre[PREFETCH ? NB * QB : 1];
            if (PREFETCH && n0 < 2 * rope.D) {
#pragma unroll
                for (int q = 0; q < NB * QB; ++q) {
                    const int row = m0 + prow0 + min((etid + q * NT) / PER_ROW, RP - 1);
                    pos_pre[q] = rope.pos[min(row, M - 1)];
                }
            }
            // This pass's part of the output as a bounds-checked buffer (rows of the pass that
            // exist, the tile's columns that exist); offsets are relative to its first element.
            constexpr int ES = EPI == EPI_RES_BF16_TO_F32 ? 4 : 2;           // bytes per output element
            const int rows_here = min(RP, M - m0 - prow0);                    // (may be <= 0)
            const int cols_here = min(OUT_COLS, out_N - out_n0);
            const int r_lo = PASSES > 1 ? max(pass * TM - prow0, 0) : 0;      // rows below: the pass before wrote them
            const __amdgpu_buffer_rsrc_t c_buf = buffer_of(
                static_cast<char*>(Cv) + ((size_t)(m0 + prow0) * ldc + out_n0) * ES,
                rows_here > 0 ? ((rows_here - 1) * ldc + cols_here) * ES : 0);
            // Residual epilogues: an item is 4 columns of a row (16 bytes of fp32: a wave's load
            // or store covers consecutive whole cache lines; with 8-column items a lane's two
            // 16-byte fp32 accesses lay 32 bytes apart and a store burst of that form takes 1.4-1.8
            // times as long).  Items go in batches of RU whose residual reads are in flight
            // together, the first batch requested before the tile is laid down; reads and stores
            // are unconditional buffer accesses (behind a per-item branch the compiler made each
            // read wait for the one before it -- a memory round trip per item -- and behind
            // conditional stores for the stores before it).
            constexpr bool RES = EPI == EPI_RES_BF16_TO_F32 || EPI == EPI_RES_F32_TO_BF16;
            // (register room: the four-wave 256x256 shape has its accumulators in the second
            // register file and takes 16 items per batch; the others 16 registers' worth; shapes
            // with no registers to spare request after the lay-down)
            constexpr bool BIG = WM * WN == 4 && BM == 256 && BN == 256;
            constexpr bool TIGHT = (WM * WN == 8 && BM == 256 && BN == 256) || BM == 288 ||
                                   (WM * WN == 4 && BM == 128);
            constexpr int IPR = OUT_COLS / 4;                                 // items per tile row
            constexpr int RPT = (RP * IPR + NT - 1) / NT;                     // items per thread and pass
            constexpr int RREG = EPI == EPI_RES_BF16_TO_F32 ? 2 : 4;          // registers per item
            constexpr int RES_ES = EPI == EPI_RES_BF16_TO_F32 ? 2 : 4;        // bytes per residual element
            constexpr int RU_MAX = BIG ? 16 : 16 / RREG;
            constexpr int RU = RPT < RU_MAX ? RPT : RU_MAX, RNB = (RPT + RU - 1) / RU;
            // item k of this thread: row r of the pass and first column c4 of the tile.  Where the
            // threads of the workgroup cover whole rows, the column is the same for every item
            // and the row advances by a constant: no divisions, offsets by one addition.
            constexpr bool WHOLE_ROWS = NT % IPR == 0;
            constexpr int RSTEP = WHOLE_ROWS ? NT / IPR : 0;
            int ftid = etid;   // (thread index as the items' second half sees it: set after the lay-down)
            auto item_rc = [&](int t, int k, int& r, int& c4) __attribute__((always_inline)) {
                if (WHOLE_ROWS) {
                    r = t / IPR + k * RSTEP;
                    c4 = (t % IPR) * 4;
                } else {
                    const int it = t + k * NT;
                    r = it / IPR;
                    c4 = (it % IPR) * 4;
                }
            };
            const __amdgpu_buffer_rsrc_t r_buf = buffer_of(
                RES ? static_cast<const char*>(Rv) + ((size_t)(m0 + prow0) * ldr + out_n0) * RES_ES : nullptr,
                RES && rows_here > 0 ? ((rows_here - 1) * ldr + cols_here) * RES_ES : 0);
            u32x2_t rh_[RES ? RU : 1];    // bf16 residual (4 values)
            u32x4_t rf_[RES ? RU : 1];    // fp32 residual
            auto res_request = [&](int b) __attribute__((always_inline)) {
#pragma unroll
                for (int u = 0; u < RU; ++u) {
                    int r, c4;
                    item_rc(etid, b * RU + u, r, c4);
                    const int off = (min(r, RP - 1) * ldr + c4) * RES_ES;   // (beyond the records: zeros)
                    if (EPI == EPI_RES_BF16_TO_F32)
                        rh_[u] = __builtin_amdgcn_raw_buffer_load_b64(r_buf, off, 0, 0);
                    else
                        rf_[u] = __builtin_amdgcn_raw_buffer_load_b128(r_buf, off, 0, 0);
                }
            };
            auto res_finish = [&](int b) __attribute__((always_inline)) {
#pragma unroll
                for (int u = 0; u < RU; ++u) {
                    int r, c4;
                    item_rc(ftid, b * RU + u, r, c4);
                    const bool ok = r >= r_lo && r < rows_here && c4 < cols_here;
                    const int off = ok ? (r * ldc + c4) * ES : OOB_OFFSET;
                    const float4 t = *reinterpret_cast<const float4*>(tile + min(r, RP - 1) * LDT + c4);
                    if (EPI == EPI_RES_BF16_TO_F32) {
                        const u32x2_t h = rh_[u];
                        const u32x4_t o = {__float_as_uint(t.x + __uint_as_float(h.x << 16)),
                                           __float_as_uint(t.y + __uint_as_float(h.x & 0xFFFF0000u)),
                                           __float_as_uint(t.z + __uint_as_float(h.y << 16)),
                                           __float_as_uint(t.w + __uint_as_float(h.y & 0xFFFF0000u))};
                        __builtin_amdgcn_raw_buffer_store_b128(o, c_buf, off, 0, 0);
                    } else {
                        const u32x4_t q = rf_[u];
                        const u32x2_t o = {pack_bf16x2(t.x + __uint_as_float(q.x), t.y + __uint_as_float(q.y)),
                                           pack_bf16x2(t.z + __uint_as_float(q.z), t.w + __uint_as_float(q.w))};
                        __builtin_amdgcn_raw_buffer_store_b64(o, c_buf, off, 0, 0);
                    }
                    // (items stay in order: with nothing conditional left the scheduler would
                    // otherwise read the tile rows of all items first and run out of registers)
                    if (u % 4 == 3) __builtin_amdgcn_sched_barrier(0);
                }
            };
            if constexpr (RES && !TIGHT) res_request(0);
            __syncthreads();   // previous readers of the LDS (fragments or the last pass) are done
            if (PASSES == 1 || wm == pass) {
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const int r = wrow0 - prow0 + i * 32 + fr;
                            const int c = wn * TN + j * 32 + 8 * q + 4 * fg;
                            *reinterpret_cast<float4*>(tile + r * LDT + c) =
                                make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1],
                                            acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
                        }
            }
            __syncthreads();
            // (what the items need beyond their residual is computed from here on, not before
            // the lay-down, where it would be held in registers across it)
            asm volatile("" : "+v"(ftid));
            if (EPI == EPI_QKV_ROPE) {
                const int DH = rope.dh, HALF = DH >> 1, CPH = HALF >> 3;   // 16-byte chunks per half head
                if (n0 < 2 * rope.D) {
                    // q or k columns: every item is 8 columns of the first half of a head and
                    // their partners dh/2 further on (tiles hold whole heads: BN % dh == 0; a row
                    // has BN/16 items whatever dh is).  Items are taken a few at a time so that the
                    // table rows of a batch are in flight together.
#pragma unroll
                    for (int jb = 0; jb < NB; ++jb) {
                        const int it0 = etid + jb * QB * NT;
                        int r[QB], col[QB], c8[QB], p[QB];
                        bool ok[QB];
#pragma unroll
                        for (int u = 0; u < QB; ++u) {
                            const int it = it0 + u * NT;
                            r[u] = min(it / PER_ROW, RP - 1);
                            const int rest = it % PER_ROW;
                            c8[u] = (rest % CPH) * 8;
                            col[u] = (rest / CPH) * DH + c8[u];   // column in the tile
                            const int row = m0 + prow0 + r[u];
                            ok[u] = it < RP * PER_ROW && r[u] >= r_lo && r[u] < rows_here && col[u] < cols_here;
                            p[u] = PREFETCH ? pos_pre[PREFETCH ? jb * QB + u : 0] : rope.pos[min(row, M - 1)];
                        }
                        float4 cs[QB][2], sn[QB][2];
#pragma unroll
                        for (int u = 0; u < QB; ++u) {
                            const size_t toff = (size_t)min(max(p[u], 0), rope.rope_len - 1) * HALF + c8[u];
                            cs[u][0] = *reinterpret_cast<const float4*>(rope.rc + toff);
                            cs[u][1] = *reinterpret_cast<const float4*>(rope.rc + toff + 4);
                            sn[u][0] = *reinterpret_cast<const float4*>(rope.rs + toff);
                            sn[u][1] = *reinterpret_cast<const float4*>(rope.rs + toff + 4);
                        }
#pragma unroll
                        for (int u = 0; u < QB; ++u) {
                            const float* ta = tile + r[u] * LDT + col[u];
                            const float4 a0 = *reinterpret_cast<const float4*>(ta);
                            const float4 a1 = *reinterpret_cast<const float4*>(ta + 4);
                            const float4 b0 = *reinterpret_cast<const float4*>(ta + HALF);
                            const float4 b1 = *reinterpret_cast<const float4*>(ta + HALF + 4);
                            const float a[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
                            const float b[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
                            const float c[8] = {cs[u][0].x, cs[u][0].y, cs[u][0].z, cs[u][0].w,
                                                cs[u][1].x, cs[u][1].y, cs[u][1].z, cs[u][1].w};
                            const float sv[8] = {sn[u][0].x, sn[u][0].y, sn[u][0].z, sn[u][0].w,
                                                 sn[u][1].x, sn[u][1].y, sn[u][1].z, sn[u][1].w};
                            uint32_t wa[4], wb[4];
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                wa[e] = pack_bf16x2(a[2 * e] * c[2 * e] - b[2 * e] * sv[2 * e],
                                                    a[2 * e + 1] * c[2 * e + 1] - b[2 * e + 1] * sv[2 * e + 1]);
                                wb[e] = pack_bf16x2(b[2 * e] * c[2 * e] + a[2 * e] * sv[2 * e],
                                                    b[2 * e + 1] * c[2 * e + 1] + a[2 * e + 1] * sv[2 * e + 1]);
                            }
                            const int off = ok[u] ? (r[u] * ldc + col[u]) * 2 : OOB_OFFSET;
                            const u32x4_t oa = {wa[0], wa[1], wa[2], wa[3]}, ob = {wb[0], wb[1], wb[2], wb[3]};
                            __builtin_amdgcn_raw_buffer_store_b128(oa, c_buf, off, 0, 0);
                            __builtin_amdgcn_raw_buffer_store_b128(ob, c_buf, off + HALF * 2, 0, 0);
                            __builtin_amdgcn_sched_barrier(0);   // (one item's tile reads at a time: registers)
                        }
                    }
                } else {
                    // v columns, transposed into vt[b, h, d, s]: an item is one column and one
                    // group of 8 tokens aligned in s (one 16-byte store).  The rows of the pass are
                    // walked sample by sample (a uniform loop: one division per sample, none per
                    // item); within a sample's rows the groups are [8j, 8j+8) of its tokens, the
                    // groups cut by the ends of the rows are stored token by token by the two
                    // passes (or tiles) that hold their rows, and whoever stores a sample's last
                    // token clears the padding behind it.  A half-wave runs over 32 columns, the
                    // two halves over alternate groups: LDS reads without bank conflicts.
                    const int H = rope.D / DH, S = rope.S, S_pad = rope.S_pad;
                    const int g_base = m0 + prow0;                                  // global row of LDS row 0
                    const int g_lo = m0 + (PASSES > 1 ? max(prow0, pass * TM) : 0);  // rows this pass owns
                    const int g_hi = min(g_base + RP, M);
                    constexpr int NW = NT / 64, NCH = BN / 32;     // waves; 32-column chunks of the tile
                    constexpr int WPC = NW > NCH ? NW / NCH : 1;   // waves sharing a chunk (over groups)
                    const int vlane = ftid & 63, vwave = ftid >> 6;
                    const int g_first = (vlane >> 5) + 2 * (NW > NCH ? vwave / NCH : 0);
                    constexpr int G_STEP = 2 * WPC;
                    for (int g_a = g_lo; g_a < g_hi;) {
                        const int bs = g_a / S, g_s = bs * S, g_e = min(g_hi, g_s + S);
                        const int s_a = g_a - g_s, s_e = g_e - g_s;   // tokens [s_a, s_e) of sample bs are ours
                        const int r_off = g_s - g_base;               // LDS row of token s: s + r_off
                        const int j_hi = (s_e + 7) >> 3;
#pragma unroll 1
                        for (int ch = NW > NCH ? vwave % NCH : vwave; ch < NCH && (NW <= NCH || vwave < WPC * NCH);
                             ch += NW) {
                            const int d = ch * 32 + (vlane & 31);
                            const int vcol = n0 - 2 * rope.D + d, hd = vcol / DH, dd = vcol - hd * DH;
                            bf16_t* dst = rope.vt + ((size_t)(bs * H + hd) * DH + dd) * S_pad;
                            const float* src = tile + r_off * LDT + d;     // (+ s * LDT: token s)
                            if (n0 + d >= N) continue;
#pragma unroll 1
                            for (int j = (s_a >> 3) + g_first; j < j_hi; j += G_STEP) {
                                const int s_al = j * 8;
                                const int lo = max(s_a, s_al), hi = min(s_e, s_al + 8);
                                if (lo == s_al && hi == s_al + 8) {          // a whole group of ours
                                    const float* q = src + s_al * LDT;
                                    *reinterpret_cast<uint4*>(dst + s_al) =
                                        make_uint4(pack_bf16x2(q[0], q[LDT]), pack_bf16x2(q[2 * LDT], q[3 * LDT]),
                                                   pack_bf16x2(q[4 * LDT], q[5 * LDT]),
                                                   pack_bf16x2(q[6 * LDT], q[7 * LDT]));
                                    if (hi == S)
                                        for (int z = s_al + 8; z < S_pad; z += 8)
                                            *reinterpret_cast<uint4*>(dst + z) = make_uint4(0, 0, 0, 0);
                                } else if (lo == s_al && hi == S) {          // the sample's short last group, all ours
                                    float v[8];
#pragma unroll
                                    for (int i = 0; i < 8; ++i)
                                        v[i] = s_al + i < hi ? src[min(s_al + i, hi - 1) * LDT] : 0.f;
                                    *reinterpret_cast<uint4*>(dst + s_al) =
                                        make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]),
                                                   pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
                                    for (int z = s_al + 8; z < S_pad; z += 8)
                                        *reinterpret_cast<uint4*>(dst + z) = make_uint4(0, 0, 0, 0);
                                } else {                                     // cut by the ends of our rows
#pragma unroll 1
                                    for (int t = lo; t < hi; ++t) {
                                        dst[t] = (bf16_t)(pack_bf16x2(src[t * LDT], 0.f) & 0xFFFFu);
                                        if (t == S - 1)
                                            for (int z = S; z < S_pad; ++z) dst[z] = 0;
                                    }
                                }
                            }
                        }
                        g_a = g_e;
                    }
                }
                continue;
            }
            if constexpr (RES) {
                if constexpr (TIGHT) res_request(0);
#pragma unroll 1
                for (int b = 0; b < RNB; ++b) {
                    res_finish(b);
                    if (b + 1 < RNB) res_request(b + 1);
                }
                continue;
            }
            // SiLU(gate) * up: 8 output columns per item (16 bytes of bf16), two items at a time
            constexpr int U = 2;
#pragma unroll 1
            for (int it0 = etid; it0 < ITEMS; it0 += U * NT) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int it = it0 + u * NT;
                    const int r = min(it / (OUT_COLS / 8), RP - 1), c8 = it % (OUT_COLS / 8);
                    const bool ok = it < ITEMS && r >= r_lo && r < rows_here && c8 * 8 < cols_here;
                    // gate block [64q, 64q+32) and up block [64q+32, 64q+64) of the tile
                    const int oc = c8 * 8;                      // output column within the tile
                    const float* g = tile + r * LDT + (oc >> 5) * 64 + (oc & 31);
                    const float4 g0 = *reinterpret_cast<const float4*>(g);
                    const float4 g1 = *reinterpret_cast<const float4*>(g + 4);
                    const float4 u0 = *reinterpret_cast<const float4*>(g + 32);
                    const float4 u1 = *reinterpret_cast<const float4*>(g + 36);
                    const float gv[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
                    const float uv[8] = {u0.x, u0.y, u0.z, u0.w, u1.x, u1.y, u1.z, u1.w};
                    // SiLU(g) u = g u / (1 + e^-g); the hardware reciprocal (1 ulp) is far inside
                    // what the bf16 result keeps
                    float x[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        x[e] = gv[e] * uv[e] * __builtin_amdgcn_rcpf(1.f + __expf(-gv[e]));
                    const u32x4_t o = {pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3]),
                                       pack_bf16x2(x[4], x[5]), pack_bf16x2(x[6], x[7])};
                    __builtin_amdgcn_raw_buffer_store_b128(o, c_buf, ok ? (r * ldc + oc) * 2 : OOB_OFFSET, 0, 0);
                }
            }
        }
    }
}

// ---- host side ------------------------------------------------------------------------------
// Compute units of the current device: sets how many workgroups are resident at once (the round
// size of the tile plan) and the size of the K-split partial buffer.  Asked once; 256 (MI355X)
// when there is no device to ask.
int device_cu_count() {
    static int cached = 0;
    if (cached > 0) return cached;
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) {
        (void)hipGetLastError();
        return 256;
    }
    cached = n;
    return n;
}

// Split of the tile set into whole-tile workgroups and K-split workgroups for `slots`
// concurrently resident workgroups.
static GemmPlan make_plan(int M, int N, int K, int BM, int BN, int BK, int slots, int sk_pct) {
    GemmPlan p;
    p.tiles_m = (M + BM - 1) / BM;
    p.tiles_n = (N + BN - 1) / BN;
    p.k_tiles = K / BK;
    const int tiles = p.tiles_m * p.tiles_n;
    const int rem = tiles % slots;
    // a last round that is at least sk_pct % full is not worth cutting up
    if (rem == 0 || rem * 100 >= slots * sk_pct) {
        p.dp_tiles = tiles;
        p.dp_grid = (tiles + 7) / 8 * 8;
        p.sk_tiles = 0;
        p.sk_blocks = 0;
        return p;
    }
    p.dp_tiles = tiles - rem;
    p.dp_grid = (p.dp_tiles + 7) / 8 * 8;
    p.sk_tiles = rem;
    const long iters = (long)rem * p.k_tiles;
    long blocks = slots;
    if (iters / blocks < SK_MIN_ITERS) blocks = iters / SK_MIN_ITERS;
    if (blocks > (long)rem * (SK_MAX_PIECES / 2 - 1)) blocks = (long)rem * (SK_MAX_PIECES / 2 - 1);
    if (blocks < rem) blocks = rem;  // a workgroup never spans more than two tiles
    p.sk_blocks = (int)blocks;
    return p;
}

// Which part of the tile plan a launch covers: all of it, or -- when two kernels of the same tile
// size share one plan -- the whole tiles only, or the K-split tiles of the last round only.
enum PlanPart { PLAN_ALL = 0, PLAN_WHOLE_TILES = 1, PLAN_SPLIT_TILES = 2 };

// The plan for a tile shape, with the K-split dropped when the workspace has no room for it.
static GemmPlan plan_for(int M, int N, int K, int BM, int BN, int BK, int slots, int sk_pct,
                         size_t partial_bytes, int n_counters) {
    GemmPlan plan = make_plan(M, N, K, BM, BN, BK, slots, sk_pct);
    if (plan.sk_blocks > 0) {
        const size_t need = (size_t)2 * plan.sk_blocks * BM * BN * sizeof(float);
        if (need > partial_bytes || plan.sk_tiles > n_counters) {  // no room: whole tiles only
            plan.dp_tiles += plan.sk_tiles;
            plan.dp_grid = (plan.dp_tiles + 7) / 8 * 8;
            plan.sk_tiles = plan.sk_blocks = 0;
        }
    }
    return plan;
}

template <int BM, int BN, int BK, int WM, int WN, int NS>
static int launch_cfg(const bf16_t* A, int lda, const bf16_t* W, int M, int N, int K, void* C,
                      int ldc, const void* R, int ldr, int epi, int slots_per_cu, int sk_pct,
                      float* partial, size_t partial_bytes, uint32_t* counters, int n_counters,
                      const RopeEpilogue& rope, hipStream_t st, PlanPart part = PLAN_ALL) {
    constexpr bool has_sk = !(WM * WN == 4 && ((BM / 32 + WM - 1) / WM) * (BN / WN / 32) >= 15);
    GemmPlan plan = plan_for(M, N, K, BM, BN, BK, device_cu_count() * slots_per_cu,
                             (has_sk || part != PLAN_ALL) ? sk_pct : 0, partial_bytes, n_counters);
    if (part == PLAN_WHOLE_TILES) {
        plan.sk_tiles = plan.sk_blocks = 0;         // (their tiles are left to the other launch)
    } else if (part == PLAN_SPLIT_TILES) {
        if (plan.sk_blocks == 0) return MVLA_OK;
        plan.dp_grid = 0;                           // workgroup ids start at the K-split workgroups
    }
    if (!has_sk && plan.sk_blocks > 0) return MVLA_EINVAL;
    const int grid = plan.dp_grid + plan.sk_blocks;
    if (grid == 0) return MVLA_OK;
    const size_t stage_bytes = (size_t)NS * (BM + BN) * (BK / 8) * sizeof(uint4);
    const size_t epi_bytes = EpiGeom<BM, BN, WM, NS>::BYTES;
    const size_t lds = stage_bytes > epi_bytes ? stage_bytes : epi_bytes;
    dim3 block(WM * WN * 64);
    // the dynamic-LDS limit of a kernel is raised once per device (the size is a constant of the
    // instantiation), not on every launch
#define MVLA_GEMM_LAUNCH(E)                                                                   \
    do {                                                                                      \
        auto kern = gemm_kernel<BM, BN, BK, WM, WN, NS, E>;                                       \
        static bool lds_set[kMaxDevices] = {};                                                \
        int dev = 0;                                                                          \
        MVLA_HIP_CHECK(hipGetDevice(&dev));                                                   \
        if (dev < 0 || dev >= kMaxDevices || !lds_set[dev]) {                                 \
            MVLA_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),           \
                                               hipFuncAttributeMaxDynamicSharedMemorySize,    \
                                               (int)lds));                                    \
            if (dev >= 0 && dev < kMaxDevices) lds_set[dev] = true;                           \
        }                                                                                     \
        hipLaunchKernelGGL(kern, dim3(grid), block, lds, st, A, lda, W, M, N, K, C, ldc, R,   \
                           ldr, plan, partial, counters, rope);                               \
    } while (0)
    if (epi == EPI_QKV_ROPE) MVLA_GEMM_LAUNCH(EPI_QKV_ROPE);
    else if (epi == EPI_RES_BF16_TO_F32) MVLA_GEMM_LAUNCH(EPI_RES_BF16_TO_F32);
    else if (epi == EPI_RES_F32_TO_BF16) MVLA_GEMM_LAUNCH(EPI_RES_F32_TO_BF16);
    else MVLA_GEMM_LAUNCH(EPI_SILU_MUL);
#undef MVLA_GEMM_LAUNCH
    MVLA_HIP_CHECK(hipGetLastError());
    return MVLA_OK;
}

size_t gemm_partial_bytes() {
    // two partial tiles per K-split workgroup; 256x256 tiles on 256 slots == 128x128 on 512
    return (size_t)2 * device_cu_count() * 256 * 256 * sizeof(float);
}

// Tile configurations and the time one round of them takes at K = 4096 on this chip (measured
// once, microseconds; only their ratios matter for the choice below).
struct TileCfg {
    int BM, BN, slots_per_cu;
    float round_us;
    bool can_split;   // has the K-split path
};
constexpr int kNumCfgs = 7;
static const TileCfg kCfgs[kNumCfgs] = {
    {256, 256, 1, 105.f, true},   // K-slab 64, eight waves of 128x64, two stages
    {256, 128, 1, 62.f, true},    // K-slab 64, eight waves of 64x64, three stages
    {128, 128, 2, 67.f, true},    // K-slab 64, four waves of 64x64, two stages, two workgroups per CU
    {128, 128, 1, 35.f, true},    // K-slab 64, eight waves of 32x64, three stages
    {256, 256, 1, 98.f, true},    // K-slab 64, four waves of 128x128 (accumulators fill the second
                                  // register file, a third less LDS traffic per MFMA); a K-split last
                                  // round runs on the eight-wave kernel of the same tile size
    {192, 128, 1, 50.f, true},    // K-slab 64, eight waves of 96x32, three stages (row counts just over
                                  // 2x256 with few column tiles: three row tiles, K-split over all CUs)
    {288, 192, 1, 92.f, false},   // K-slab 64, four waves of 160x96 (the two wave rows overlap by one
                                  // 32-row block), accumulators in the second register file, whole
                                  // tiles only
};
constexpr int kSplitPct = 50;        // cut the last round along K only when it is under half full
constexpr float kSplitOverhead = 0.3f;  // cost of the partial-sum exchange, in rounds

// Estimated rounds of work for a tile configuration: whole rounds, plus the last partial
// round either as a full round or, when K-split, as its fill fraction plus the exchange cost.
static float estimate_us(const TileCfg& c, int M, int N, int K) {
    const long tiles = (long)((M + c.BM - 1) / c.BM) * ((N + c.BN - 1) / c.BN);
    const int slots = device_cu_count() * c.slots_per_cu;
    const long full = tiles / slots, rem = tiles % slots;
    float rounds = (float)full;
    if (rem)
        rounds += (c.can_split && rem * 100 < (long)slots * kSplitPct)
                      ? (float)rem / slots + kSplitOverhead : 1.f;
    return rounds * c.round_us * (float)K / 4096.f;
}

int gemm_num_configs() { return kNumCfgs; }

// The rotating q/k/v epilogue works on tiles that hold whole heads and lie inside one of the
// q, k, v column sections.
static bool cfg_runs(const TileCfg& c, int epilogue, const RopeEpilogue* rope) {
    return epilogue != EPI_QKV_ROPE || (c.BN % rope->dh == 0 && rope->D % c.BN == 0);
}

bool gemm_config_runs(int cfg, int epilogue, const RopeEpilogue* rope) {
    return cfg >= 0 && cfg < kNumCfgs && (epilogue != EPI_QKV_ROPE || rope) &&
           cfg_runs(kCfgs[cfg], epilogue, rope);
}

// force_cfg >= 0 picks that tile configuration and force_split_pct the K-split threshold
// (0 = never, 101 = whenever the last round is not full); force_cfg < 0, or a configuration
// that cannot run this epilogue, leaves the choice to the cost model.
int launch_gemm(const bf16_t* A, int lda, const bf16_t* W, int M, int N, int K, void* C, int ldc,
                const void* R, int ldr, int epilogue, float* partial, size_t partial_bytes,
                uint32_t* counters, int n_counters, int force_cfg, int force_split_pct,
                const RopeEpilogue* rope, hipStream_t st) {
    if (M <= 0 || N <= 0) return MVLA_OK;
    if (K < 64 || K % 64 != 0 || lda % 8 != 0) return MVLA_EUNSUPPORTED;
    if (epilogue == EPI_SILU_MUL && N % 64 != 0) return MVLA_EUNSUPPORTED;
    if (N % 8 != 0 || ldc % 8 != 0 || (R && ldr % 8 != 0)) return MVLA_EUNSUPPORTED;
    if (ldc > (1 << 20) || ldr > (1 << 20)) return MVLA_EUNSUPPORTED;   // (32-bit byte offsets inside a tile)
    if (epilogue == EPI_QKV_ROPE) {
        if (!rope || !rope->pos || !rope->rc || !rope->rs || rope->S <= 0 || rope->rope_len <= 0)
            return MVLA_EINVAL;
        if ((rope->dh != 64 && rope->dh != 128) || rope->D % rope->dh != 0) return MVLA_EUNSUPPORTED;
        // N = 3D: q, k, v; N = 2D: q and k; N = D: one of q, k alone (W points at its rows)
        if (N != 3 * rope->D && N != 2 * rope->D && N != rope->D) return MVLA_EINVAL;
        if ((N == 3 * rope->D) != (rope->vt != nullptr)) return MVLA_EINVAL;
        if (M % rope->S != 0 || rope->S_pad < rope->S || rope->S_pad % 8 != 0) return MVLA_EINVAL;
    }
    int best = -1, split_pct = kSplitPct;
    if (force_cfg >= 0 && force_cfg < kNumCfgs && cfg_runs(kCfgs[force_cfg], epilogue, rope)) {
        best = force_cfg;
        split_pct = force_split_pct;
    } else {
        float best_us = 0.f;
        for (int i = 0; i < kNumCfgs; ++i) {
            if (!cfg_runs(kCfgs[i], epilogue, rope)) continue;
            const float t = estimate_us(kCfgs[i], M, N, K);
            if (best < 0 || t < best_us) {
                best_us = t;
                best = i;
            }
        }
        if (best < 0) return MVLA_EUNSUPPORTED;
    }
    const RopeEpilogue rope_args = rope ? *rope : RopeEpilogue{};
#define MVLA_ARGS A, lda, W, M, N, K, C, ldc, R, ldr, epilogue, kCfgs[best].slots_per_cu, split_pct, \
                  partial, partial_bytes, counters, n_counters, rope_args, st
    switch (best) {
        case 0: return launch_cfg<256, 256, 64, 2, 4, 2>(MVLA_ARGS);
        case 1: return launch_cfg<256, 128, 64, 4, 2, 3>(MVLA_ARGS);
        case 2: return launch_cfg<128, 128, 64, 2, 2, 2>(MVLA_ARGS);
        case 3: return launch_cfg<128, 128, 64, 4, 2, 3>(MVLA_ARGS);
        case 4: {
            // four waves of 128x128 have no registers for the K-split exchange: when the last round
            // is to be cut, its tiles go to the eight-wave kernel of the same tile size in a second
            // launch (same plan, same tile numbering)
            const GemmPlan pl = plan_for(M, N, K, 256, 256, 64, device_cu_count(), split_pct,
                                         partial_bytes, n_counters);
            if (pl.sk_blocks == 0) return launch_cfg<256, 256, 64, 2, 2, 2>(MVLA_ARGS);
            const int rc = launch_cfg<256, 256, 64, 2, 2, 2>(MVLA_ARGS, PLAN_WHOLE_TILES);
            if (rc) return rc;
            return launch_cfg<256, 256, 64, 2, 4, 2>(MVLA_ARGS, PLAN_SPLIT_TILES);
        }
        case 5: return launch_cfg<192, 128, 64, 2, 4, 3>(MVLA_ARGS);
        default: return launch_cfg<288, 192, 64, 2, 2, 2>(MVLA_ARGS);
    }
#undef MVLA_ARGS
}

}  // namespace mvla
