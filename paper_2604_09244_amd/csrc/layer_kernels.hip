// Element-wise and small kernels of the decoder layer on gfx950: RMSNorm,
// rotary table, rotary embedding + V transpose, and the language-query scoring
// probabilities (paper Sec. 3.2: the attention rows that salience is read from).
#include "common.h"
#include "mfma.h"

namespace mvla {

// ---------------------------------------------------------------------------
// RMSNorm: out = x * gain / sqrt(mean(x^2) + eps), one wave per row, fp32 maths.
// ---------------------------------------------------------------------------
constexpr int NORM_THREADS = 256;

__global__ __launch_bounds__(NORM_THREADS) void rmsnorm_kernel(const uint4* __restrict__ x,
                                                               const uint4* __restrict__ gain,
                                                               int M, int row_vec, float inv_d,
                                                               float eps, uint4* __restrict__ out) {
    const int row = blockIdx.x * (NORM_THREADS / 64) + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (row >= M) return;
    const uint4* xr = x + (size_t)row * row_vec;
    float ss = 0.f;
    for (int c = lane; c < row_vec; c += 64) {
        const uint4 v = xr[c];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float lo = __uint_as_float(w[i] << 16), hi = __uint_as_float(w[i] & 0xFFFF0000u);
            ss += lo * lo + hi * hi;
        }
    }
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    const float scale = 1.0f / sqrtf(ss * inv_d + eps);
    uint4* orow = out + (size_t)row * row_vec;
    for (int c = lane; c < row_vec; c += 64) {
        const uint4 v = xr[c], g = gain[c];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w}, gw[4] = {g.x, g.y, g.z, g.w};
        uint32_t r[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float lo = __uint_as_float(w[i] << 16) * scale * __uint_as_float(gw[i] << 16);
            const float hi = __uint_as_float(w[i] & 0xFFFF0000u) * scale *
                             __uint_as_float(gw[i] & 0xFFFF0000u);
            r[i] = pack_bf16x2(lo, hi);
        }
        orow[c] = make_uint4(r[0], r[1], r[2], r[3]);
    }
}

int launch_rmsnorm(const bf16_t* x, const bf16_t* gain, int M, int D, float eps, bf16_t* out,
                   hipStream_t st) {
    if (M <= 0) return MVLA_OK;
    const int rows_per_block = NORM_THREADS / 64;
    hipLaunchKernelGGL(rmsnorm_kernel, dim3((M + rows_per_block - 1) / rows_per_block),
                       dim3(NORM_THREADS), 0, st, reinterpret_cast<const uint4*>(x),
                       reinterpret_cast<const uint4*>(gain), M, D / 8, 1.0f / (float)D, eps,
                       reinterpret_cast<uint4*>(out));
    MVLA_HIP_CHECK(hipGetLastError());
    return MVLA_OK;
}

// Same, reading the fp32 residual stream (eight floats per 16-byte output chunk).
__global__ __launch_bounds__(NORM_THREADS) void rmsnorm_f32_kernel(const float4* __restrict__ x,
                                                                   const uint4* __restrict__ gain,
                                                                   int M, int row_vec, float inv_d,
                                                                   float eps,
                                                                   uint4* __restrict__ out) {
    const int row = blockIdx.x * (NORM_THREADS / 64) + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (row >= M) return;
    const float4* xr = x + (size_t)row * row_vec * 2;
    float ss = 0.f;
    for (int c = lane; c < row_vec * 2; c += 64) {
        const float4 v = xr[c];
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    const float scale = 1.0f / sqrtf(ss * inv_d + eps);
    uint4* orow = out + (size_t)row * row_vec;
    for (int c = lane; c < row_vec; c += 64) {
        const float4 a = xr[2 * c], b = xr[2 * c + 1];
        const uint4 g = gain[c];
        const float xs[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        const uint32_t gw[4] = {g.x, g.y, g.z, g.w};
        uint32_t r[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            r[i] = pack_bf16x2(xs[2 * i] * scale * __uint_as_float(gw[i] << 16),
                               xs[2 * i + 1] * scale * __uint_as_float(gw[i] & 0xFFFF0000u));
        orow[c] = make_uint4(r[0], r[1], r[2], r[3]);
    }
}

int launch_rmsnorm_f32(const float* x, const bf16_t* gain, int M, int D, float eps, bf16_t* out,
                       hipStream_t st) {
    if (M <= 0) return MVLA_OK;
    const int rows_per_block = NORM_THREADS / 64;
    hipLaunchKernelGGL(rmsnorm_f32_kernel, dim3((M + rows_per_block - 1) / rows_per_block),
                       dim3(NORM_THREADS), 0, st, reinterpret_cast<const float4*>(x),
                       reinterpret_cast<const uint4*>(gain), M, D / 8, 1.0f / (float)D, eps,
                       reinterpret_cast<uint4*>(out));
    MVLA_HIP_CHECK(hipGetLastError());
    return MVLA_OK;
}

// ---------------------------------------------------------------------------
// Rotary table in fp64: angle = pos * base^(-2i/dh).
// ---------------------------------------------------------------------------
__global__ void rope_table_kernel(double base, int rope_len, int half, float* __restrict__ c,
                                  float* __restrict__ s) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= rope_len * half) return;
    const int pos = idx / half, i = idx % half;
    const double inv_freq = pow(base, -(double)i / (double)half);
    const double ang = (double)pos * inv_freq;
    c[idx] = (float)cos(ang);
    s[idx] = (float)sin(ang);
}

int launch_rope_table(double base, int rope_len, int dh, float* c, float* s, hipStream_t st) {
    const int n = rope_len * (dh / 2);
    if (n <= 0) return MVLA_OK;
    hipLaunchKernelGGL(rope_table_kernel, dim3((n + 255) / 256), dim3(256), 0, st, base, rope_len,
                       dh / 2, c, s);
    MVLA_HIP_CHECK(hipGetLastError());
    return MVLA_OK;
}

// ---------------------------------------------------------------------------
// Rotary embedding of q and k in place (rotate-half pairing: element i with
// i + dh/2) and transposition of v into vt[b, h, d, s] (row length S_pad,
// zero beyond S), which makes the keys the contiguous axis of the P*V operand.
// One workgroup handles 64 tokens of one head.
// ---------------------------------------------------------------------------
constexpr int ROPE_THREADS = 256;
constexpr int ROPE_TOK = 64;

template <int DH>
__global__ __launch_bounds__(ROPE_THREADS) void rope_split_kernel(
    bf16_t* __restrict__ qkv, const int32_t* __restrict__ pos, const float* __restrict__ rc,
    const float* __restrict__ rs, int rope_len, int S, int H, int S_pad, int n_sections,
    bf16_t* __restrict__ vt) {
    constexpr int HALF = DH / 2;
    constexpr int CH = HALF / 8;  // 16-byte chunks per half row
    const int s0 = blockIdx.x * ROPE_TOK, h = blockIdx.y, b = blockIdx.z;
    const int D = H * DH, ld = n_sections * D;
    const int tid = threadIdx.x;

    // q (section 0) and k (section 1)
    for (int item = tid; item < 2 * ROPE_TOK * CH; item += ROPE_THREADS) {
        const int sec = item / (ROPE_TOK * CH);
        const int rem = item % (ROPE_TOK * CH);
        const int t = rem / CH, c = rem % CH;
        const int s = s0 + t;
        if (s >= S) continue;
        const size_t m = (size_t)b * S + s;
        int p = pos[m];
        p = min(max(p, 0), rope_len - 1);
        bf16_t* base = qkv + m * ld + sec * D + h * DH;
        uint4 va = *reinterpret_cast<uint4*>(base + c * 8);
        uint4 vb = *reinterpret_cast<uint4*>(base + HALF + c * 8);
        const float4 c0 = *reinterpret_cast<const float4*>(rc + (size_t)p * HALF + c * 8);
        const float4 c1 = *reinterpret_cast<const float4*>(rc + (size_t)p * HALF + c * 8 + 4);
        const float4 s0v = *reinterpret_cast<const float4*>(rs + (size_t)p * HALF + c * 8);
        const float4 s1v = *reinterpret_cast<const float4*>(rs + (size_t)p * HALF + c * 8 + 4);
        const float cs[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
        const float sn[8] = {s0v.x, s0v.y, s0v.z, s0v.w, s1v.x, s1v.y, s1v.z, s1v.w};
        uint32_t aw[4] = {va.x, va.y, va.z, va.w}, bw[4] = {vb.x, vb.y, vb.z, vb.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float a0 = __uint_as_float(aw[i] << 16), a1 = __uint_as_float(aw[i] & 0xFFFF0000u);
            const float b0 = __uint_as_float(bw[i] << 16), b1 = __uint_as_float(bw[i] & 0xFFFF0000u);
            const float ra0 = a0 * cs[2 * i] - b0 * sn[2 * i];
            const float rb0 = b0 * cs[2 * i] + a0 * sn[2 * i];
            const float ra1 = a1 * cs[2 * i + 1] - b1 * sn[2 * i + 1];
            const float rb1 = b1 * cs[2 * i + 1] + a1 * sn[2 * i + 1];
            aw[i] = pack_bf16x2(ra0, ra1);
            bw[i] = pack_bf16x2(rb0, rb1);
        }
        *reinterpret_cast<uint4*>(base + c * 8) = make_uint4(aw[0], aw[1], aw[2], aw[3]);
        *reinterpret_cast<uint4*>(base + HALF + c * 8) = make_uint4(bw[0], bw[1], bw[2], bw[3]);
    }
    if (n_sections < 3) return;

    // v (section 2): [64 tokens x DH] -> LDS -> vt[d][s0 .. s0+63]
    __shared__ bf16_t tile[ROPE_TOK][DH + 2];  // +2: odd word stride, conflict-free column reads
    for (int item = tid; item < ROPE_TOK * (DH / 8); item += ROPE_THREADS) {
        const int t = item / (DH / 8), c = item % (DH / 8);
        const int s = s0 + t;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (s < S) v = *reinterpret_cast<const uint4*>(qkv + ((size_t)b * S + s) * ld + 2 * D +
                                                       h * DH + c * 8);
        uint32_t* dst = reinterpret_cast<uint32_t*>(&tile[t][c * 8]);
        dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
    }
    __syncthreads();
    bf16_t* vrow = vt + ((size_t)(b * H + h) * DH) * S_pad + s0;
    for (int item = tid; item < DH * (ROPE_TOK / 8); item += ROPE_THREADS) {
        const int d = item / (ROPE_TOK / 8), c = item % (ROPE_TOK / 8);
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            w[i] = (uint32_t)tile[c * 8 + 2 * i][d] | ((uint32_t)tile[c * 8 + 2 * i + 1][d] << 16);
        *reinterpret_cast<uint4*>(vrow + (size_t)d * S_pad + c * 8) =
            make_uint4(w[0], w[1], w[2], w[3]);
    }
}

int launch_rope_split(bf16_t* qkv, const int32_t* pos, const float* rc, const float* rs,
                      int rope_len, int B, int S, int H, int dh, int S_pad, bf16_t* vt,
                      hipStream_t st) {
    if (B <= 0 || S <= 0) return MVLA_OK;
    const int n_sections = vt ? 3 : 2;
    dim3 grid((S + ROPE_TOK - 1) / ROPE_TOK, H, B);
    if (dh == 128)
        hipLaunchKernelGGL(rope_split_kernel<128>, grid, dim3(ROPE_THREADS), 0, st, qkv, pos, rc,
                           rs, rope_len, S, H, S_pad, n_sections, vt);
    else if (dh == 64)
        hipLaunchKernelGGL(rope_split_kernel<64>, grid, dim3(ROPE_THREADS), 0, st, qkv, pos, rc,
                           rs, rope_len, S, H, S_pad, n_sections, vt);
    else
        return MVLA_EUNSUPPORTED;
    MVLA_HIP_CHECK(hipGetLastError());
    return MVLA_OK;
}

// ---------------------------------------------------------------------------
// Scoring probabilities of the last nq rows (the language-token queries):
//   P[b,h,i,:] = softmax_j( q_i . k_j / sqrt(dh) + key_bias[b,j] ),  j <= row(i).
// One workgroup per (32-query tile, head, sample).  Logits are MFMA tiles with
// queries on the rows and keys on the columns, so a register holds 32
// consecutive keys of one query across lanes and stores are coalesced.  Pass 1
// keeps a running max / sum per query; pass 2 recomputes the logits and writes
// normalised probabilities (nothing is staged in memory in between).
// ---------------------------------------------------------------------------
constexpr int SC_THREADS = 256;

template <int DH>
__global__ __launch_bounds__(SC_THREADS) void score_probs_kernel(
    const bf16_t* __restrict__ q, int ldq, const bf16_t* __restrict__ k, int ldk,
    const float* __restrict__ key_bias, int S, int H, int nq, float scale,
    float* __restrict__ probs) {
    constexpr int STEPS = DH / 16;
    const int qt = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fr = lane & 31, fg = lane >> 5;
    const int row0 = S - nq;            // sequence row of scoring query 0
    const int qi0 = qt * 32;            // first query of this tile

    // A operand: this lane's query row, all of dh
    uint4 qf[STEPS];
    {
        const int qi = min(qi0 + fr, nq - 1);
        const bf16_t* src = q + ((size_t)b * S + row0 + qi) * ldq + h * DH + fg * 8;
#pragma unroll
        for (int st = 0; st < STEPS; ++st) qf[st] = *reinterpret_cast<const uint4*>(src + st * 16);
    }
    const int n_kb = (S + 31) / 32;
    const bf16_t* kbase = k + (size_t)b * S * ldk + h * DH + fg * 8;
    const float* bias = key_bias ? key_bias + (size_t)b * S : nullptr;

    float run_m[16], run_l[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) { run_m[v] = -INFINITY; run_l[v] = 0.f; }

    __shared__ float sh_m[SC_THREADS / 64][32], sh_l[SC_THREADS / 64][32];

    for (int pass = 0; pass < 2; ++pass) {
        for (int kb = wave; kb < n_kb; kb += SC_THREADS / 64) {
            const int key = kb * 32 + fr;  // this lane's key column
            const int kr = min(key, S - 1);
            f32x16_t acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.f;
            const bf16_t* ksrc = kbase + (size_t)kr * ldk;
#pragma unroll
            for (int st = 0; st < STEPS; ++st) {
                const uint4 kf = *reinterpret_cast<const uint4*>(ksrc + st * 16);
                acc = mfma32(qf[st], kf, acc);
            }
            const float kbias = (bias && key < S) ? bias[key] : 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int qi = qi0 + mfma32_row(v, lane);
                const bool valid = key < S && key <= row0 + qi;
                const float logit = valid ? acc[v] * scale + kbias : -INFINITY;
                if (pass == 0) {
                    // per-lane running (max, sum) over this lane's key column
                    const float nm = fmaxf(run_m[v], logit);
                    if (nm != -INFINITY) {
                        run_l[v] = run_l[v] * __expf(run_m[v] - nm) + __expf(logit - nm);
                        run_m[v] = nm;
                    }
                } else if (qi < nq && key < S) {
                    const float p = valid ? __expf(logit - run_m[v]) * run_l[v] : 0.f;
                    probs[(((size_t)b * H + h) * nq + qi) * S + key] = p;
                }
            }
        }
        if (pass == 0) {
            // combine (max, sum) over the 32 lanes that share a query row, then over the
            // four waves; afterwards run_m = global max, run_l = 1 / global sum
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                for (int o = 16; o > 0; o >>= 1) {
                    const float om = __shfl_xor(run_m[v], o), ol = __shfl_xor(run_l[v], o);
                    const float nm = fmaxf(run_m[v], om);
                    if (nm != -INFINITY)
                        run_l[v] = run_l[v] * __expf(run_m[v] - nm) + ol * __expf(om - nm);
                    run_m[v] = nm;
                }
            }
            if (fr == 0) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    sh_m[wave][mfma32_row(v, lane)] = run_m[v];
                    sh_l[wave][mfma32_row(v, lane)] = run_l[v];
                }
            }
            __syncthreads();
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = mfma32_row(v, lane);
                float gm = -INFINITY;
                for (int w = 0; w < SC_THREADS / 64; ++w) gm = fmaxf(gm, sh_m[w][r]);
                float gl = 0.f;
                for (int w = 0; w < SC_THREADS / 64; ++w)
                    gl += (sh_m[w][r] == -INFINITY) ? 0.f : sh_l[w][r] * __expf(sh_m[w][r] - gm);
                run_m[v] = gm;
                run_l[v] = 1.0f / gl;
            }
        }
    }
}

int launch_score_probs(const bf16_t* q, int q_row_stride, const bf16_t* k, int k_row_stride,
                       const float* key_bias, int B, int S, int H, int dh, int nq, float* probs,
                       hipStream_t st) {
    if (B <= 0 || nq <= 0) return MVLA_OK;
    dim3 grid((nq + 31) / 32, H, B);
    const float scale = 1.0f / sqrtf((float)dh);
    if (dh == 128)
        hipLaunchKernelGGL(score_probs_kernel<128>, grid, dim3(SC_THREADS), 0, st, q, q_row_stride,
                           k, k_row_stride, key_bias, S, H, nq, scale, probs);
    else if (dh == 64)
        hipLaunchKernelGGL(score_probs_kernel<64>, grid, dim3(SC_THREADS), 0, st, q, q_row_stride,
                           k, k_row_stride, key_bias, S, H, nq, scale, probs);
    else
        return MVLA_EUNSUPPORTED;
    MVLA_HIP_CHECK(hipGetLastError());
    return MVLA_OK;
}

}  // namespace mvla
