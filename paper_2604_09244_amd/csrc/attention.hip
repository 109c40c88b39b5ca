// Causal flash attention on the gfx950 matrix cores.
//
// Both products are computed transposed so that a lane owns one query:
//   S^T = K * Q^T   (MFMA rows = keys, columns = queries)
//   O^T = V^T * P^T (MFMA rows = head-dim, columns = queries)
// The S^T accumulator layout (lane = query column, registers = key rows) is
// exactly the B-operand layout P^T needs, up to a fixed permutation of the 16
// keys of a step which the V^T fragments follow, so probabilities go from one
// product to the next without leaving registers.  Softmax statistics are
// per-lane scalars; the two lanes that share a query exchange one value per
// tile.  K tiles [64 keys x dh] and V^T tiles [dh x 64 keys] travel from global
// memory straight into a ring of LDS stages (global_load_lds, 16 bytes per
// lane; the XOR swizzle is applied on the global side because a direct load
// always lands a wave on 1 KiB of consecutive LDS), so the next tiles are in
// flight while the current one is consumed.  V^T is produced by the rotary
// kernel, which makes both tiles contiguous along the contraction axis of
// their product.
#include "common.h"
#include "mfma.h"

namespace mvla {

constexpr int ATT_THREADS = 256;
constexpr int ATT_QT = 128;  // queries per workgroup (32 per wave)
constexpr int ATT_KT = 64;   // keys per tile

// untracked direct global -> LDS copy (see gemm.hip): order consumers behind att_wait_vm + barrier
// (address = wave-uniform base + per-lane unsigned 32-bit byte offset)
__device__ __forceinline__ void att_dma16(const void* base, uint32_t off, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr),
                 "v"(off), "s"(base)
                 : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void att_wait_vm() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// K rows are dh/8 chunks long (16 or 8), V^T rows 8 chunks; conflict-free XOR patterns
template <int CPR>
__device__ __forceinline__ int att_swz(int row) {
    return CPR == 16 ? (row & 15) : ((row >> 1) & 7);
}

template <int DH, int NS>
__global__ __launch_bounds__(ATT_THREADS, 2) void attention_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, int ld, const bf16_t* __restrict__ vt,
    int S_pad, int S, int H, float scale_log2e, bf16_t* __restrict__ out, int ldo) {
    constexpr int CPR = DH / 8;           // 16-byte chunks per K row
    constexpr int STEPS = DH / 16;        // MFMA k-steps over the head dim
    constexpr int DB = DH / 32;           // 32-row blocks of O^T
    constexpr int K_SLOTS = ATT_KT * CPR, V_SLOTS = DH * 8, STAGE = K_SLOTS + V_SLOTS;
    constexpr int K_LD = K_SLOTS / ATT_THREADS, V_LD = V_SLOTS / ATT_THREADS;
    constexpr int P = K_LD + V_LD;        // direct loads per thread per tile

    extern __shared__ uint4 lds[];

    // Workgroups are dispatched in blockIdx order, x fastest.  Heads run along x and query tiles
    // along y, heavier (later) tiles first: a sample's tiles then start in order of decreasing
    // work across all its heads (the light ones fill the end instead of a heavy tile of the last
    // head starting late), and because the head count is a multiple of the 8 XCDs that workgroup
    // ids are dealt to, every tile of a head runs on the same XCD and finds its K/V in that L2.
    const int qtile = gridDim.y - 1 - blockIdx.y, h = blockIdx.x, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fr = lane & 31, fg = lane >> 5;
    const int q0 = qtile * ATT_QT;
    const int qw0 = q0 + wave * 32;           // first query of this wave
    const int my_q = qw0 + fr;                // this lane's query (sequence row)

    // B operand of S^T: this lane's query row
    uint4 qf[STEPS];
    {
        const bf16_t* src = q + ((size_t)b * S + min(my_q, S - 1)) * ld + h * DH + fg * 8;
#pragma unroll
        for (int st = 0; st < STEPS; ++st) qf[st] = *reinterpret_cast<const uint4*>(src + st * 16);
        // The fragments are pinned here, before any direct load is in flight: otherwise the
        // compiler's waits for these loads sit inside the key loop, where they would also wait
        // for the (untracked) direct loads of the next tile.
#pragma unroll
        for (int st = 0; st < STEPS; ++st)
            asm volatile("" : "+v"(qf[st].x), "+v"(qf[st].y), "+v"(qf[st].z), "+v"(qf[st].w));
    }

    const int last_row = min(q0 + ATT_QT, S) - 1;
    const int n_kt = last_row / ATT_KT + 1;   // key tiles this workgroup needs (causal)

    // direct-load mapping: op i of this thread covers slot i*256 + tid of the K (or V^T) tile
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds;
    // (bases are wave-uniform, the per-lane parts 32-bit byte offsets within one sample's keys
    // or one head's V^T: fewer address registers than one pointer per op)
    const bf16_t* k_base = k + (size_t)b * S * ld + h * DH;
    const bf16_t* v_base = vt + (size_t)(b * H + h) * DH * S_pad;
    int k_row[K_LD];
    uint32_t k_off[K_LD], k_lds[K_LD];
#pragma unroll
    for (int i = 0; i < K_LD; ++i) {
        const int sl = i * ATT_THREADS + tid, row = sl / CPR, ch = (sl % CPR) ^ att_swz<CPR>(row);
        k_row[i] = row;
        k_off[i] = (uint32_t)ch * 16u;
        k_lds[i] = __builtin_amdgcn_readfirstlane(lds_base + (uint32_t)(i * ATT_THREADS + wave * 64) * 16u);
    }
    uint32_t v_off[V_LD], v_lds[V_LD];
#pragma unroll
    for (int i = 0; i < V_LD; ++i) {
        const int sl = i * ATT_THREADS + tid, row = sl >> 3, ch = (sl & 7) ^ att_swz<8>(row);
        v_off[i] = ((uint32_t)row * (uint32_t)S_pad + (uint32_t)ch * 8u) * 2u;
        v_lds[i] = __builtin_amdgcn_readfirstlane(
            lds_base + (uint32_t)(K_SLOTS + i * ATT_THREADS + wave * 64) * 16u);
    }
#define ATT_ISSUE(KT, STG)                                                                  \
    {                                                                                       \
        const int kt_ = min((KT), n_kt - 1);                                                \
        const uint32_t soff = (uint32_t)(STG) * STAGE * 16u;                                \
        _Pragma("unroll") for (int i = 0; i < K_LD; ++i) {                                  \
            const int key = min(kt_ * ATT_KT + k_row[i], S - 1);                            \
            att_dma16(k_base, k_off[i] + (uint32_t)key * (uint32_t)ld * 2u, k_lds[i] + soff); \
        }                                                                                   \
        _Pragma("unroll") for (int i = 0; i < V_LD; ++i)                                    \
            att_dma16(v_base + kt_ * ATT_KT, v_off[i], v_lds[i] + soff);                    \
    }

    f32x16_t o_acc[DB];
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int v = 0; v < 16; ++v) o_acc[d][v] = 0.f;
    float run_m = -INFINITY, run_l = 0.f;   // run_l: this lane's share of the row sum

#pragma unroll
    for (int s = 0; s < NS - 1; ++s) ATT_ISSUE(s, s)

    int stage = 0;
    for (int kt = 0; kt < n_kt; ++kt) {
        // tile kt has landed for every wave; the stage of tile kt-1 is free for tile kt+NS-1
        att_wait_vm<(NS - 2) * P>();
        __syncthreads();
        {
            int nstage = stage + NS - 1;
            if (nstage >= NS) nstage -= NS;
            ATT_ISSUE(kt + NS - 1, nstage)
        }
        const int key0 = kt * ATT_KT;
        // a wave whose queries all precede this tile has nothing to add
        if (key0 <= qw0 + 31 && qw0 < S) {
            const uint4* Kc = lds + stage * STAGE;
            const uint2* Vc = reinterpret_cast<const uint2*>(Kc + K_SLOTS);
            // ---- S^T for the two 32-key halves of the tile
            // (the two independent accumulator chains alternate, so the matrix core does not
            // wait on its own results)
            f32x16_t s_acc[2];
            uint4 kf[2][STEPS];
#pragma unroll
            for (int st = 0; st < STEPS; ++st)
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const int row = t * 32 + fr;
                    kf[t][st] = Kc[row * CPR + ((st * 2 + fg) ^ att_swz<CPR>(row))];
                }
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) s_acc[t][v] = 0.f;
#pragma unroll
            for (int st = 0; st < STEPS; ++st)
#pragma unroll
                for (int t = 0; t < 2; ++t) s_acc[t] = mfma32(kf[t][st], qf[st], s_acc[t]);
            // V^T fragments of the first two head-dim blocks: in flight during the softmax arithmetic
            uint4 vfrag[2][4];
#pragma unroll
            for (int d = 0; d < 2; ++d) {
                const int row = min(d, DB - 1) * 32 + fr;
                const int sw = att_swz<8>(row);
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const uint2 lo = Vc[(row * 8 + ((ks * 2) ^ sw)) * 2 + fg];
                    const uint2 hi = Vc[(row * 8 + ((ks * 2 + 1) ^ sw)) * 2 + fg];
                    vfrag[d][ks] = make_uint4(lo.x, lo.y, hi.x, hi.y);
                }
            }
            // ---- (mask,) row max on the raw logits; only tiles that reach the diagonal or the end
            // of the sequence need the mask (wave-uniform test).  The softmax scale is positive, so
            // the max commutes with it, and scale and subtraction fuse into one FMA per logit (the
            // kernel is bound by vector-ALU issue, not by the matrix core).
            float tile_m = -INFINITY;
            if (key0 + ATT_KT - 1 <= qw0 && key0 + ATT_KT <= S) {
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int v = 0; v < 16; ++v) tile_m = fmaxf(tile_m, s_acc[t][v]);
            } else {
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int key = key0 + t * 32 + mfma32_row(v, lane);
                        const float x = (key <= my_q && key < S) ? s_acc[t][v] : -INFINITY;
                        s_acc[t][v] = x;
                        tile_m = fmaxf(tile_m, x);
                    }
            }
            tile_m = fmaxf(tile_m, __shfl_xor(tile_m, 32));
            const float new_m = fmaxf(run_m, tile_m);   // (raw logits) finite from the first tile on (key 0)
            const float neg_m = -new_m * scale_log2e;
            float psum = 0.f;
            uint4 pf[4];  // P^T B-operand fragments: one per 16-key step
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
                    float e[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        e[i] = __builtin_amdgcn_exp2f(fmaf(s_acc[t][hh * 8 + i], scale_log2e, neg_m));
                        psum += e[i];
                    }
                    pf[t * 2 + hh] = make_uint4(pack_bf16x2(e[0], e[1]), pack_bf16x2(e[2], e[3]),
                                                pack_bf16x2(e[4], e[5]), pack_bf16x2(e[6], e[7]));
                }
            // the running max rarely moves after the first tiles: rescale only when it did for
            // some query of the wave (a factor of exactly 1 otherwise)
            if (__any(new_m != run_m)) {
                const float corr = __builtin_amdgcn_exp2f((run_m - new_m) * scale_log2e);
                run_l *= corr;
#pragma unroll
                for (int d = 0; d < DB; ++d)
#pragma unroll
                    for (int v = 0; v < 16; ++v) o_acc[d][v] *= corr;
                run_m = new_m;
            }
            run_l += psum;
            // ---- O^T += V^T * P^T ; the A fragment takes keys {4g..4g+3, 8+4g..8+4g+3} of each
            // 16-key step, matching the key order of the P^T registers.  The fragments of a pair
            // of head-dim blocks are read ahead of their MFMAs (the first pair before the softmax
            // arithmetic above, see vfrag), so the matrix core does not wait on LDS latency.
#pragma unroll
            for (int dp = 0; dp < DB; dp += 2) {
                uint4 vnext[2][4];
                if (dp + 2 < DB) {
#pragma unroll
                    for (int d = 0; d < 2; ++d) {
                        const int row = (dp + 2 + d) * 32 + fr;
                        const int sw = att_swz<8>(row);
#pragma unroll
                        for (int ks = 0; ks < 4; ++ks) {
                            const uint2 lo = Vc[(row * 8 + ((ks * 2) ^ sw)) * 2 + fg];
                            const uint2 hi = Vc[(row * 8 + ((ks * 2 + 1) ^ sw)) * 2 + fg];
                            vnext[d][ks] = make_uint4(lo.x, lo.y, hi.x, hi.y);
                        }
                    }
                }
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                    for (int d = 0; d < 2; ++d)
                        if (dp + d < DB) o_acc[dp + d] = mfma32(vfrag[d][ks], pf[ks], o_acc[dp + d]);
#pragma unroll
                for (int d = 0; d < 2; ++d)
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks) vfrag[d][ks] = vnext[d][ks];
            }
        }
        stage = stage + 1 == NS ? 0 : stage + 1;
    }
    att_wait_vm<0>();
#undef ATT_ISSUE

    // ---- normalise and store: lane holds query my_q, rows = head-dim
    const float tot = run_l + __shfl_xor(run_l, 32);
    if (my_q < S) {
        const float inv = 1.0f / tot;
        bf16_t* orow = out + ((size_t)b * S + my_q) * ldo + h * DH;
#pragma unroll
        for (int d = 0; d < DB; ++d)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const int col = d * 32 + 8 * v4 + 4 * fg;
                uint2 w;
                w.x = pack_bf16x2(o_acc[d][v4 * 4 + 0] * inv, o_acc[d][v4 * 4 + 1] * inv);
                w.y = pack_bf16x2(o_acc[d][v4 * 4 + 2] * inv, o_acc[d][v4 * 4 + 3] * inv);
                *reinterpret_cast<uint2*>(orow + col) = w;
            }
    }
}

template <int DH, int NS>
static int launch_att(const bf16_t* q, const bf16_t* k, int ldqkv, const bf16_t* vt, int S_pad,
                      int B, int S, int H, bf16_t* out, int ldo, hipStream_t st) {
    dim3 grid(H, (S + ATT_QT - 1) / ATT_QT, B);
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)DH);
    const size_t lds = (size_t)NS * (ATT_KT * (DH / 8) + DH * 8) * sizeof(uint4);
    auto kern = attention_kernel<DH, NS>;
    static bool lds_set[kMaxDevices] = {};   // the dynamic-LDS limit is raised once per device
    int dev = 0;
    MVLA_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices || !lds_set[dev]) {
        MVLA_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        if (dev >= 0 && dev < kMaxDevices) lds_set[dev] = true;
    }
    hipLaunchKernelGGL(kern, grid, dim3(ATT_THREADS), lds, st, q, k, ldqkv, vt, S_pad, S, H,
                       scale_log2e, out, ldo);
    MVLA_HIP_CHECK(hipGetLastError());
    return MVLA_OK;
}

int launch_attention(const bf16_t* q, const bf16_t* k, int ldqkv, const bf16_t* vt, int S_pad,
                     int B, int S, int H, int dh, bf16_t* out, int ldo, hipStream_t st) {
    if (B <= 0 || S <= 0) return MVLA_OK;
    if (S_pad % ATT_KT != 0 || S_pad < S) return MVLA_EINVAL;
    // per-lane byte offsets inside one sample's keys / one head's V^T are 32-bit (kept below 2^31)
    if ((size_t)S * ldqkv * 2 >= ((size_t)1 << 31) || (size_t)dh * S_pad * 2 >= ((size_t)1 << 31))
        return MVLA_EUNSUPPORTED;
    // two stages of 32 KiB each: two workgroups per CU, whose waves overlap softmax and MFMA
    if (dh == 128) return launch_att<128, 2>(q, k, ldqkv, vt, S_pad, B, S, H, out, ldo, st);
    if (dh == 64) return launch_att<64, 2>(q, k, ldqkv, vt, S_pad, B, S, H, out, ldo, st);
    return MVLA_EUNSUPPORTED;
}

}  // namespace mvla
