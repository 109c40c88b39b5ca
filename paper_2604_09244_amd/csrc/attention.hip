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
// tile.  K tiles [64 keys x dh] and V^T tiles [dh x 64 keys] are staged in LDS
// (two stages, next tile in flight while the current one is consumed); V^T is
// produced by the rotary kernel, so both tiles are contiguous along the
// contraction axis of their product.
#include "common.h"
#include "mfma.h"

namespace mvla {

constexpr int ATT_THREADS = 256;
constexpr int ATT_QT = 128;  // queries per workgroup (32 per wave)
constexpr int ATT_KT = 64;   // keys per tile

template <int DH>
__global__ __launch_bounds__(ATT_THREADS) void attention_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, int ld, const bf16_t* __restrict__ vt,
    int S_pad, int S, int H, float scale_log2e, bf16_t* __restrict__ out, int ldo) {
    constexpr int CPR = DH / 8;           // 16-byte chunks per K row
    constexpr int STEPS = DH / 16;        // MFMA k-steps over the head dim
    constexpr int DB = DH / 32;           // 32-row blocks of O^T
    constexpr int K_CH = ATT_KT * CPR / ATT_THREADS;  // chunks per thread per K tile
    constexpr int V_CH = DH * 8 / ATT_THREADS;        // chunks per thread per V^T tile

    extern __shared__ uint4 lds[];
    uint4* Ks = lds;                          // [2][64 * CPR]
    uint4* Vs = lds + 2 * ATT_KT * CPR;       // [2][DH * 8]

    // heavier (later) query tiles first
    const int qtile = gridDim.x - 1 - blockIdx.x, h = blockIdx.y, b = blockIdx.z;
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
    }

    const int last_row = min(q0 + ATT_QT, S) - 1;
    const int n_kt = last_row / ATT_KT + 1;   // key tiles this workgroup needs (causal)

    // staging sources
    const bf16_t* k_src[K_CH];
    int k_dst[K_CH], k_row[K_CH];
#pragma unroll
    for (int i = 0; i < K_CH; ++i) {
        const int cid = tid + i * ATT_THREADS, row = cid / CPR, ch = cid % CPR;
        k_row[i] = row;
        k_src[i] = k + (size_t)b * S * ld + h * DH + ch * 8;
        k_dst[i] = row * CPR + (ch ^ (row & 7));
    }
    const bf16_t* v_src[V_CH];
    int v_dst[V_CH];
#pragma unroll
    for (int i = 0; i < V_CH; ++i) {
        const int cid = tid + i * ATT_THREADS, row = cid >> 3, ch = cid & 7;
        v_src[i] = vt + ((size_t)(b * H + h) * DH + row) * S_pad + ch * 8;
        v_dst[i] = lds_slot(row, ch);
    }
    uint4 k_reg[K_CH], v_reg[V_CH];
#define ATT_FETCH(KT)                                                                      \
    {                                                                                      \
        _Pragma("unroll") for (int i = 0; i < K_CH; ++i) {                                 \
            const int key = min((KT) * ATT_KT + k_row[i], S - 1);                          \
            k_reg[i] = *reinterpret_cast<const uint4*>(k_src[i] + (size_t)key * ld);       \
        }                                                                                  \
        _Pragma("unroll") for (int i = 0; i < V_CH; ++i) v_reg[i] =                        \
            *reinterpret_cast<const uint4*>(v_src[i] + (KT) * ATT_KT);                     \
    }
#define ATT_STASH(STAGE)                                                                   \
    {                                                                                      \
        uint4* Kd = Ks + (STAGE) * ATT_KT * CPR;                                           \
        uint4* Vd = Vs + (STAGE) * DH * 8;                                                 \
        _Pragma("unroll") for (int i = 0; i < K_CH; ++i) Kd[k_dst[i]] = k_reg[i];          \
        _Pragma("unroll") for (int i = 0; i < V_CH; ++i) Vd[v_dst[i]] = v_reg[i];          \
    }

    f32x16_t o_acc[DB];
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int v = 0; v < 16; ++v) o_acc[d][v] = 0.f;
    float run_m = -INFINITY, run_l = 0.f;   // run_l: this lane's share of the row sum

    ATT_FETCH(0)
    ATT_STASH(0)
    __syncthreads();

    for (int kt = 0; kt < n_kt; ++kt) {
        const int cur = kt & 1;
        const int nkt = min(kt + 1, n_kt - 1);  // unconditional: the last tile re-fetches itself
        ATT_FETCH(nkt)
        const int key0 = kt * ATT_KT;
        // a wave whose queries all precede this tile has nothing to add
        if (key0 <= qw0 + 31 && qw0 < S) {
            const uint4* Kc = Ks + cur * ATT_KT * CPR;
            const uint2* Vc = reinterpret_cast<const uint2*>(Vs + cur * DH * 8);
            // ---- S^T for the two 32-key halves of the tile
            f32x16_t s_acc[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
#pragma unroll
                for (int v = 0; v < 16; ++v) s_acc[t][v] = 0.f;
                const int row = t * 32 + fr;
#pragma unroll
                for (int st = 0; st < STEPS; ++st) {
                    const uint4 kf = Kc[row * CPR + ((st * 2 + fg) ^ (row & 7))];
                    s_acc[t] = mfma32(kf, qf[st], s_acc[t]);
                }
            }
            // ---- scale, mask, row max
            float tile_m = -INFINITY;
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = key0 + t * 32 + mfma32_row(v, lane);
                    const float x = (key <= my_q && key < S) ? s_acc[t][v] * scale_log2e : -INFINITY;
                    s_acc[t][v] = x;
                    tile_m = fmaxf(tile_m, x);
                }
            tile_m = fmaxf(tile_m, __shfl_xor(tile_m, 32));
            const float new_m = fmaxf(run_m, tile_m);   // finite from the first tile on (key 0)
            const float corr = __builtin_amdgcn_exp2f(run_m - new_m);
            run_m = new_m;
            float psum = 0.f;
            uint4 pf[4];  // P^T B-operand fragments: one per 16-key step
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
                    float e[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        e[i] = __builtin_amdgcn_exp2f(s_acc[t][hh * 8 + i] - new_m);
                        psum += e[i];
                    }
                    pf[t * 2 + hh] = make_uint4(pack_bf16x2(e[0], e[1]), pack_bf16x2(e[2], e[3]),
                                                pack_bf16x2(e[4], e[5]), pack_bf16x2(e[6], e[7]));
                }
            run_l = run_l * corr + psum;
#pragma unroll
            for (int d = 0; d < DB; ++d)
#pragma unroll
                for (int v = 0; v < 16; ++v) o_acc[d][v] *= corr;
            // ---- O^T += V^T * P^T ; the A fragment takes keys {4g..4g+3, 8+4g..8+4g+3} of each
            // 16-key step, matching the key order of the P^T registers
#pragma unroll
            for (int d = 0; d < DB; ++d) {
                const int row = d * 32 + fr;
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const uint2 lo = Vc[lds_slot(row, ks * 2) * 2 + fg];
                    const uint2 hi = Vc[lds_slot(row, ks * 2 + 1) * 2 + fg];
                    o_acc[d] = mfma32(make_uint4(lo.x, lo.y, hi.x, hi.y), pf[ks], o_acc[d]);
                }
            }
        }
        ATT_STASH(cur ^ 1)
        __syncthreads();
    }

#undef ATT_FETCH
#undef ATT_STASH
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

int launch_attention(const bf16_t* q, const bf16_t* k, int ldqkv, const bf16_t* vt, int S_pad,
                     int B, int S, int H, int dh, bf16_t* out, int ldo, hipStream_t st) {
    if (B <= 0 || S <= 0) return MVLA_OK;
    if (S_pad % ATT_KT != 0 || S_pad < S) return MVLA_EINVAL;
    dim3 grid((S + ATT_QT - 1) / ATT_QT, H, B);
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)dh);
    if (dh == 128) {
        const size_t lds = (size_t)2 * (ATT_KT * 16 + 128 * 8) * sizeof(uint4);
        MVLA_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(attention_kernel<128>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(attention_kernel<128>, grid, dim3(ATT_THREADS), lds, st, q, k, ldqkv, vt,
                           S_pad, S, H, scale_log2e, out, ldo);
    } else if (dh == 64) {
        const size_t lds = (size_t)2 * (ATT_KT * 8 + 64 * 8) * sizeof(uint4);
        hipLaunchKernelGGL(attention_kernel<64>, grid, dim3(ATT_THREADS), lds, st, q, k, ldqkv, vt,
                           S_pad, S, H, scale_log2e, out, ldo);
    } else {
        return MVLA_EUNSUPPORTED;
    }
    MVLA_HIP_CHECK(hipGetLastError());
    return MVLA_OK;
}

}  // namespace mvla
