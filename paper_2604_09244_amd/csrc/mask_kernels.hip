// Mask generation of the tri-stage framework for gfx950 (paper Sec. 4.1-4.4,
// Algorithm 1): per-patch L1 feature share (Eq. 1), and one workgroup per
// sample that clusters the patches' attention scores (1-D k-means, K = 3),
// applies the semantic rules with their two baselines, fuses with the
// dual-threshold candidates and writes the two retention masks (Eq. 10);
// then a scan that turns the masks into ascending token indices.
// Every reduction has a fixed shape, so results are reproducible bit for bit.
#include "common.h"

namespace mvla {

// ---------------------------------------------------------------------------
// Eq. 1: for patch p, l2 = |f_2D|_1 (row p), l3 = |f_3D|_1 (row n_patch + p);
// outputs l2/(l2+l3) and l3/(l2+l3), 0 when the denominator is 0.
// One workgroup per (patch, sample): waves 0-1 read the 2D row, waves 2-3 the
// 3D row, 16 bytes (8 bf16) per lane per access.
// ---------------------------------------------------------------------------
constexpr int FS_THREADS = 256;

__device__ inline float abs_sum8(uint4 v) {
    // bf16 -> fp32 is a 16-bit shift; |x| clears the sign bit
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        s += __uint_as_float((w[i] << 16) & 0x7fffffffu);
        s += __uint_as_float(w[i] & 0x7fff0000u);
    }
    return s;
}

__global__ __launch_bounds__(FS_THREADS) void feature_share_kernel(
    const uint4* __restrict__ feat, int S, int row_vec /* D*2/16 */, int n_patch,
    float* __restrict__ m2d, float* __restrict__ m3d) {
    __shared__ float part[FS_THREADS / 64];
    const int p = blockIdx.x, b = blockIdx.y;
    const int half = threadIdx.x >> 7, t = threadIdx.x & 127;
    const uint4* row = feat + ((size_t)b * S + (half ? n_patch + p : p)) * row_vec;
    float s = 0.f;
    for (int c = t; c < row_vec; c += FS_THREADS / 2) s += abs_sum8(row[c]);
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        const float l2 = part[0] + part[1], l3 = part[2] + part[3];
        const float den = l2 + l3;
        m2d[(size_t)b * n_patch + p] = den > 0.f ? l2 / den : 0.f;
        m3d[(size_t)b * n_patch + p] = den > 0.f ? l3 / den : 0.f;
    }
}

int launch_feature_share(const bf16_t* feat, int B, int S, int D, int n_patch, float* m2d,
                         float* m3d, hipStream_t st) {
    hipLaunchKernelGGL(feature_share_kernel, dim3(n_patch, B), dim3(FS_THREADS), 0, st,
                       reinterpret_cast<const uint4*>(feat), S, D / 8, n_patch, m2d, m3d);
    MVLA_HIP_CHECK(hipGetLastError());
    return MVLA_OK;
}

// ---------------------------------------------------------------------------
// Candidate sets and masks, one workgroup per sample.
// ---------------------------------------------------------------------------
constexpr int CM_THREADS = 256;
constexpr int CM_WAVES = CM_THREADS / 64;

struct CmShared {
    double d[3][CM_WAVES];
    int n[3][CM_WAVES];
    float f[2][CM_WAVES];
};

// sums three doubles and three counts over the workgroup, same order every time
__device__ inline void block_sum3(double s[3], int n[3], CmShared& sh) {
#pragma unroll
    for (int j = 0; j < 3; ++j)
        for (int o = 32; o > 0; o >>= 1) {
            s[j] += __shfl_xor(s[j], o);
            n[j] += __shfl_xor(n[j], o);
        }
    __syncthreads();
    if ((threadIdx.x & 63) == 0)
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            sh.d[j][threadIdx.x >> 6] = s[j];
            sh.n[j][threadIdx.x >> 6] = n[j];
        }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        double a = 0.0;
        int c = 0;
        for (int w = 0; w < CM_WAVES; ++w) {
            a += sh.d[j][w];
            c += sh.n[j][w];
        }
        s[j] = a;
        n[j] = c;
    }
}

enum : uint32_t { C_2D = 1u, C_3D = 2u };

__global__ __launch_bounds__(CM_THREADS) void candidate_kernel(
    const float* __restrict__ x_hat /* [4,B,P] */, const float* __restrict__ sal /* [B,2P] */,
    const float* __restrict__ u /* [B,P] */, int B, int P, int n_text, mvla_mask_rules rules,
    uint8_t* __restrict__ mask2d, uint8_t* __restrict__ mask3d, uint8_t* __restrict__ sem,
    int32_t* __restrict__ kept_len) {
    extern __shared__ float dyn[];
    float* score = dyn;                                         // [P]
    uint8_t* label = reinterpret_cast<uint8_t*>(dyn + P);       // [P]
    __shared__ CmShared sh;
    const int b = blockIdx.x, tid = threadIdx.x;
    const float* sal_b = sal + (size_t)b * 2 * P;

    // patch score: the 2D token's salience plus the 3D token's (summand of Eq. 3), in fp32
    float lo = INFINITY, hi = -INFINITY;
    for (int p = tid; p < P; p += CM_THREADS) {
        const float v = sal_b[p] + sal_b[P + p];
        score[p] = v;
        label[p] = 255;
        lo = fminf(lo, v);
        hi = fmaxf(hi, v);
    }
    for (int o = 32; o > 0; o >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, o));
        hi = fmaxf(hi, __shfl_xor(hi, o));
    }
    if ((tid & 63) == 0) {
        sh.f[0][tid >> 6] = lo;
        sh.f[1][tid >> 6] = hi;
    }
    __syncthreads();
    for (int w = 0; w < CM_WAVES; ++w) {
        lo = fminf(lo, sh.f[0][w]);
        hi = fmaxf(hi, sh.f[1][w]);
    }

    // Lloyd iterations (Sec. 4.2): centres start at min, mid-range, max; nearest centre, the
    // lower-numbered one on equal distance; a centre without points stays; stop when an
    // assignment repeats the previous one or after kmeans_max_iter assignments.
    double c0 = (double)lo, c2 = (double)hi, c1 = 0.5 * (c0 + c2);
    for (int it = 0; it < rules.kmeans_max_iter; ++it) {
        double s[3] = {0.0, 0.0, 0.0};
        int n[3] = {0, 0, 0};
        int changed = 0;
        for (int p = tid; p < P; p += CM_THREADS) {
            const double x = (double)score[p];
            const double d0 = fabs(x - c0), d1 = fabs(x - c1), d2 = fabs(x - c2);
            int l = 0;
            double best = d0;
            if (d1 < best) {
                best = d1;
                l = 1;
            }
            if (d2 < best) l = 2;
            changed |= (l != (int)label[p]);
            label[p] = (uint8_t)l;
            s[l] += x;
            n[l] += 1;
        }
        if (!__syncthreads_or(changed)) break;
        block_sum3(s, n, sh);
        if (n[0] > 0) c0 = s[0] / (double)n[0];
        if (n[1] > 0) c1 = s[1] / (double)n[1];
        if (n[2] > 0) c2 = s[2] / (double)n[2];
    }
    __syncthreads();

    // baselines: means of the two semantic indicators over the sample's patches (Eqs. 5, 6)
    const float* m3_s1 = x_hat + ((size_t)1 * B + b) * P;
    const float* m2_s2 = x_hat + ((size_t)2 * B + b) * P;
    const float* m3_s2 = x_hat + ((size_t)3 * B + b) * P;
    double mu[3] = {0.0, 0.0, 0.0};
    int unused[3] = {0, 0, 0};
    for (int p = tid; p < P; p += CM_THREADS) {
        mu[0] += (double)m2_s2[p];
        mu[1] += (double)m3_s2[p];
    }
    block_sum3(mu, unused, sh);
    const double mu2 = mu[0] / (double)P, mu3 = mu[1] / (double)P;

    int kept = 0;
    for (int p = tid; p < P; p += CM_THREADS) {
        // data-preprocessing stage (Sec. 4.1): dual threshold on the 3D feature share
        const float share3 = m3_s1[p];
        const uint32_t cand1 = share3 < rules.tau_2d ? C_2D : (share3 > rules.tau_3d ? C_3D : C_2D | C_3D);
        // semantic stage (Sec. 4.2): lowest centre = background, middle = robot, highest = object
        const int l = label[p];
        const float a2 = m2_s2[p], a3 = m3_s2[p];
        uint32_t cand2;
        if (l == 0)
            cand2 = u[(size_t)b * P + p] < rules.bg_drop ? 0u : (C_2D | C_3D);
        else if (l == 1)
            cand2 = (double)a3 > mu3 ? (C_2D | C_3D) : ((double)a2 > mu2 ? C_2D : 0u);
        else
            cand2 = (a2 > rules.obj_2d_min && a3 < rules.obj_3d_max) ? C_2D : (C_2D | C_3D);
        // fusion (Sec. 4.4): intersection, falling back to the semantic proposal when empty;
        // patches without a semantic proposal are dropped
        uint32_t fin = cand2 & cand1;
        if (fin == 0u) fin = cand2;
        mask2d[(size_t)b * P + p] = (uint8_t)(fin & C_2D ? 1 : 0);
        mask3d[(size_t)b * P + p] = (uint8_t)(fin & C_3D ? 1 : 0);
        if (sem) sem[(size_t)b * P + p] = (uint8_t)l;
        kept += (int)(fin & 1u) + (int)(fin >> 1);
    }
    double z[3] = {0.0, 0.0, 0.0};
    int cnt[3] = {kept, 0, 0};
    block_sum3(z, cnt, sh);
    if (tid == 0) kept_len[b] = cnt[0] + n_text;
}

int launch_candidate_masks(const float* x_hat, const float* sal, const float* u, int B, int P,
                           int n_text, const mvla_mask_rules& rules, uint8_t* mask2d,
                           uint8_t* mask3d, uint8_t* sem, int32_t* kept_len, hipStream_t st) {
    const size_t lds = (size_t)P * 4 + (((size_t)P + 3) & ~(size_t)3);
    hipLaunchKernelGGL(candidate_kernel, dim3(B), dim3(CM_THREADS), lds, st, x_hat, sal, u, B, P,
                       n_text, rules, mask2d, mask3d, sem, kept_len);
    MVLA_HIP_CHECK(hipGetLastError());
    return MVLA_OK;
}

// ---------------------------------------------------------------------------
// Masks -> ascending token indices (Eq. 10): kept 2D tokens, kept 3D tokens
// (offset by the patch count), all language tokens; the rest of the row up to
// S_pad repeats the last language token's index.  One workgroup per sample;
// a thread owns a contiguous run of the 2P flags, a block prefix sum places it.
// ---------------------------------------------------------------------------
constexpr int MI_THREADS = 256;

__global__ __launch_bounds__(MI_THREADS) void mask_index_kernel(
    const uint8_t* __restrict__ mask2d, const uint8_t* __restrict__ mask3d, int P, int n_text,
    int S_pad, int32_t* __restrict__ kept_idx) {
    __shared__ uint32_t wsum[MI_THREADS / 64];
    const int b = blockIdx.x, tid = threadIdx.x;
    const int n = 2 * P, per = (n + MI_THREADS - 1) / MI_THREADS;
    const int i0 = min(tid * per, n), i1 = min(i0 + per, n);
    const uint8_t* m2 = mask2d + (size_t)b * P;
    const uint8_t* m3 = mask3d + (size_t)b * P;
    uint32_t cnt = 0;
    for (int i = i0; i < i1; ++i) cnt += (i < P ? m2[i] : m3[i - P]) ? 1u : 0u;
    // inclusive scan over the threads
    uint32_t v = cnt;
    const int lane = tid & 63, wave = tid >> 6;
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = __shfl_up(v, o);
        if (lane >= o) v += t;
    }
    if (lane == 63) wsum[wave] = v;
    __syncthreads();
    uint32_t before = 0, total = 0;
    for (int w = 0; w < MI_THREADS / 64; ++w) {
        if (w < wave) before += wsum[w];
        total += wsum[w];
    }
    int32_t* out = kept_idx + (size_t)b * S_pad;
    int o = (int)(before + v - cnt);
    for (int i = i0; i < i1; ++i)
        if ((i < P ? m2[i] : m3[i - P]) && o < S_pad) out[o++] = i;
    const int len = (int)total + n_text;
    for (int j = (int)total + tid; j < S_pad; j += MI_THREADS)
        out[j] = j < len ? n + (j - (int)total) : n + n_text - 1;
}

int launch_mask_indices(const uint8_t* mask2d, const uint8_t* mask3d, int B, int P, int n_text,
                        int S_pad, int32_t* kept_idx, hipStream_t st) {
    hipLaunchKernelGGL(mask_index_kernel, dim3(B), dim3(MI_THREADS), 0, st, mask2d, mask3d, P,
                       n_text, S_pad, kept_idx);
    MVLA_HIP_CHECK(hipGetLastError());
    return MVLA_OK;
}

}  // namespace mvla
