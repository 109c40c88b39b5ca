// Element-wise and small kernels of the decoder layer on gfx950: RMSNorm,
// rotary table (the rotation itself and the V transpose happen in the q/k/v
// projection's epilogue, gemm.hip), and the language-query scoring
// probabilities (paper Sec. 3.2: the attention rows that salience is read from).
#include "common.h"
#include "mfma.h"

namespace mvla {

// ---------------------------------------------------------------------------
// RMSNorm: out = x * gain / sqrt(mean(x^2) + eps), fp32 maths, bf16 out.  One
// workgroup per row; a thread keeps its 16-byte chunks in registers between the
// sum of squares and the scaling, so the row is read once.
// ---------------------------------------------------------------------------
constexpr int NORM_THREADS = 256;
constexpr int NORM_MAX_CHUNKS = 4;  // per thread: D <= 256 * 4 * 8 = 8192

__device__ __forceinline__ float block_sum(float v, float* sh) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < NORM_THREADS / 64; ++w) t += sh[w];
    return t;
}

// IN_F32: the row is fp32 (the mid-layer residual stream), else bf16.
// tail > 0: the last `tail` rows of every sample of S rows are written a second time, packed
// into out_tail [B*tail, D], and their position ids are copied to pos_out [B*tail] (the scoring
// pass projects queries for those rows only).
template <bool IN_F32>
__global__ __launch_bounds__(NORM_THREADS) void rmsnorm_kernel(const void* __restrict__ xv,
                                                               const uint4* __restrict__ gain,
                                                               int row_vec /* D/8 */, float inv_d,
                                                               float eps, uint4* __restrict__ out,
                                                               int S, int tail,
                                                               uint4* __restrict__ out_tail,
                                                               const int32_t* __restrict__ pos,
                                                               int32_t* __restrict__ pos_out) {
    __shared__ float sh[NORM_THREADS / 64];
    const int row = blockIdx.x, tid = threadIdx.x;
    int trow = -1;                       // row of the packed tail matrix, if this is a tail row
    if (tail > 0) {
        const int b = row / S, s_ = row - b * S;
        if (s_ >= S - tail) trow = b * tail + s_ - (S - tail);
    }
    if (trow >= 0 && tid == 0) pos_out[trow] = pos[row];
    float vals[NORM_MAX_CHUNKS][8];
    float ss = 0.f;
#pragma unroll
    for (int k = 0; k < NORM_MAX_CHUNKS; ++k) {
        const int c = tid + k * NORM_THREADS;
        if (c < row_vec) {
            if (IN_F32) {
                const float4* xr = static_cast<const float4*>(xv) + (size_t)row * row_vec * 2;
                const float4 a = xr[2 * c], b = xr[2 * c + 1];
                vals[k][0] = a.x; vals[k][1] = a.y; vals[k][2] = a.z; vals[k][3] = a.w;
                vals[k][4] = b.x; vals[k][5] = b.y; vals[k][6] = b.z; vals[k][7] = b.w;
            } else {
                const uint4 v = (static_cast<const uint4*>(xv) + (size_t)row * row_vec)[c];
                const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    vals[k][2 * i] = __uint_as_float(w[i] << 16);
                    vals[k][2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
                }
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) ss += vals[k][i] * vals[k][i];
        }
    }
    ss = block_sum(ss, sh);
    const float scale = 1.0f / sqrtf(ss * inv_d + eps);
    uint4* optr = out + (size_t)row * row_vec;
    uint4* tptr = out_tail + (size_t)(trow >= 0 ? trow : 0) * row_vec;
#pragma unroll
    for (int k = 0; k < NORM_MAX_CHUNKS; ++k) {
        const int c = tid + k * NORM_THREADS;
        if (c < row_vec) {
            const uint4 g = gain[c];
            const uint32_t gw[4] = {g.x, g.y, g.z, g.w};
            uint32_t r[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                r[i] = pack_bf16x2(vals[k][2 * i] * scale * __uint_as_float(gw[i] << 16),
                                   vals[k][2 * i + 1] * scale * __uint_as_float(gw[i] & 0xFFFF0000u));
            optr[c] = make_uint4(r[0], r[1], r[2], r[3]);
            if (trow >= 0) tptr[c] = make_uint4(r[0], r[1], r[2], r[3]);
        }
    }
}

static int launch_rmsnorm_any(const void* x, bool f32, const bf16_t* gain, int M, int D, float eps,
                              bf16_t* out, hipStream_t st) {
    if (M <= 0) return MVLA_OK;
    if (D % 8 != 0 || D / 8 > NORM_THREADS * NORM_MAX_CHUNKS) return MVLA_EUNSUPPORTED;
    if (f32)
        hipLaunchKernelGGL(rmsnorm_kernel<true>, dim3(M), dim3(NORM_THREADS), 0, st, x,
                           reinterpret_cast<const uint4*>(gain), D / 8, 1.0f / (float)D, eps,
                           reinterpret_cast<uint4*>(out), 0, 0, nullptr, nullptr, nullptr);
    else
        hipLaunchKernelGGL(rmsnorm_kernel<false>, dim3(M), dim3(NORM_THREADS), 0, st, x,
                           reinterpret_cast<const uint4*>(gain), D / 8, 1.0f / (float)D, eps,
                           reinterpret_cast<uint4*>(out), 0, 0, nullptr, nullptr, nullptr);
    MVLA_HIP_CHECK(hipGetLastError());
    return MVLA_OK;
}

int launch_rmsnorm(const bf16_t* x, const bf16_t* gain, int M, int D, float eps, bf16_t* out,
                   hipStream_t st) {
    return launch_rmsnorm_any(x, false, gain, M, D, eps, out, st);
}
int launch_rmsnorm_f32(const float* x, const bf16_t* gain, int M, int D, float eps, bf16_t* out,
                       hipStream_t st) {
    return launch_rmsnorm_any(x, true, gain, M, D, eps, out, st);
}

int launch_rmsnorm_tail(const bf16_t* x, const int32_t* pos, const bf16_t* gain, int B, int S,
                        int tail, int D, float eps, bf16_t* out, bf16_t* out_tail, int32_t* pos_out,
                        hipStream_t st) {
    if (B <= 0 || S <= 0) return MVLA_OK;
    if (D % 8 != 0 || D / 8 > NORM_THREADS * NORM_MAX_CHUNKS) return MVLA_EUNSUPPORTED;
    if (tail <= 0 || tail > S || !pos || !pos_out || !out_tail) return MVLA_EINVAL;
    hipLaunchKernelGGL(rmsnorm_kernel<false>, dim3(B * S), dim3(NORM_THREADS), 0, st, x,
                       reinterpret_cast<const uint4*>(gain), D / 8, 1.0f / (float)D, eps,
                       reinterpret_cast<uint4*>(out), S, tail, reinterpret_cast<uint4*>(out_tail), pos,
                       pos_out);
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
// Scoring probabilities of the last nq rows (the language-token queries):
//   P[b,h,i,:] = softmax_j( q_i . k_j / sqrt(dh) + key_bias[b,j] ),  j <= row(i).
// One workgroup per (32-query tile, head, sample).  Logits are MFMA tiles with
// queries on the rows and keys on the columns, so a register holds 32
// consecutive keys of one query across lanes and stores are coalesced.  Pass 1
// keeps a running max / sum per query; pass 2 recomputes the logits and writes
// normalised probabilities (nothing is staged in memory in between).
// ---------------------------------------------------------------------------
constexpr int SC_THREADS = 256;

// COLSUM: instead of the probabilities, write for every key column j < n_out the sum of the
// probabilities over the tile's (up to 32) queries: out[b, h, tile, j].  The salience
// reduction then runs over H * tiles short rows and the [B,H,nq,S] tensor never exists.
template <int DH, bool COLSUM>
__global__ __launch_bounds__(SC_THREADS) void score_probs_kernel(
    const bf16_t* __restrict__ q, int ldq, int q_rows /* per sample */, const bf16_t* __restrict__ k,
    int ldk, const float* __restrict__ key_bias, int S, int H, int nq, float scale,
    float* __restrict__ probs, int n_out) {
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
        // q holds either all S rows of a sample or only its nq scoring rows
        const bf16_t* src = q + ((size_t)b * q_rows + (q_rows - nq) + qi) * ldq + h * DH + fg * 8;
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
        // the key fragments of the wave's next block are requested before this block's products
        // (rows past the end are clamped: loaded, never used)
        uint4 kf[STEPS], kn[STEPS];
        {
            const bf16_t* ksrc = kbase + (size_t)min(wave * 32 + fr, S - 1) * ldk;
#pragma unroll
            for (int st = 0; st < STEPS; ++st) kn[st] = *reinterpret_cast<const uint4*>(ksrc + st * 16);
        }
        for (int kb = wave; kb < n_kb; kb += SC_THREADS / 64) {
            const int key = kb * 32 + fr;  // this lane's key column
#pragma unroll
            for (int st = 0; st < STEPS; ++st) kf[st] = kn[st];
            {
                const bf16_t* nsrc = kbase + (size_t)min(key + (SC_THREADS / 64) * 32, S - 1) * ldk;
#pragma unroll
                for (int st = 0; st < STEPS; ++st)
                    kn[st] = *reinterpret_cast<const uint4*>(nsrc + st * 16);
            }
            f32x16_t acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
            for (int st = 0; st < STEPS; ++st) acc = mfma32(qf[st], kf[st], acc);
            const float kbias = (bias && key < S) ? bias[key] : 0.f;
            float csum = 0.f;
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
                    if (COLSUM) csum += p;
                    else probs[(((size_t)b * H + h) * nq + qi) * S + key] = p;
                }
            }
            if (COLSUM && pass == 1) {
                csum += __shfl_xor(csum, 32);      // the other 16 query rows of the tile
                if (fg == 0 && key < n_out)
                    probs[(((size_t)b * H + h) * gridDim.x + qt) * n_out + key] = csum;
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

// Single-pass variant for S <= 8 waves * KBW key blocks * 32 keys: every wave keeps the logits
// of its KBW key blocks in registers, so Q*K^T is computed once.
constexpr int SCR_THREADS = 512;
constexpr int SCR_WAVES = SCR_THREADS / 64;

template <int DH, int KBW, bool COLSUM>
__global__ __launch_bounds__(SCR_THREADS) void score_probs_reg_kernel(
    const bf16_t* __restrict__ q, int ldq, int q_rows /* per sample */, const bf16_t* __restrict__ k,
    int ldk, const float* __restrict__ key_bias, int S, int H, int nq, float scale,
    float* __restrict__ probs, int n_out) {
    constexpr int STEPS = DH / 16;
    const int qt = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fr = lane & 31, fg = lane >> 5;
    const int row0 = S - nq, qi0 = qt * 32;
    uint4 qf[STEPS];
    {
        const int qi = min(qi0 + fr, nq - 1);
        // q holds either all S rows of a sample or only its nq scoring rows
        const bf16_t* src = q + ((size_t)b * q_rows + (q_rows - nq) + qi) * ldq + h * DH + fg * 8;
#pragma unroll
        for (int st = 0; st < STEPS; ++st) qf[st] = *reinterpret_cast<const uint4*>(src + st * 16);
    }
    const int n_kb = (S + 31) / 32;
    const bf16_t* kbase = k + (size_t)b * S * ldk + h * DH + fg * 8;
    const float* bias = key_bias ? key_bias + (size_t)b * S : nullptr;

    f32x16_t lg[KBW];
    // key fragments of block i+1 are requested before the products of block i are issued
    // (rows past the end are clamped: loaded, never used)
    uint4 kf[2][STEPS];
    {
        const bf16_t* ksrc = kbase + (size_t)min(wave * 32 + fr, S - 1) * ldk;
#pragma unroll
        for (int st = 0; st < STEPS; ++st) kf[0][st] = *reinterpret_cast<const uint4*>(ksrc + st * 16);
    }
#pragma unroll
    for (int i = 0; i < KBW; ++i) {
        const int kb = wave + SCR_WAVES * i;
        const int key = kb * 32 + fr;
#pragma unroll
        for (int v = 0; v < 16; ++v) lg[i][v] = 0.f;
        if (i + 1 < KBW) {
            const bf16_t* nsrc = kbase + (size_t)min(key + SCR_WAVES * 32, S - 1) * ldk;
#pragma unroll
            for (int st = 0; st < STEPS; ++st)
                kf[(i + 1) & 1][st] = *reinterpret_cast<const uint4*>(nsrc + st * 16);
        }
        if (kb < n_kb) {   // wave-uniform
#pragma unroll
            for (int st = 0; st < STEPS; ++st) lg[i] = mfma32(qf[st], kf[i & 1][st], lg[i]);
        }
    }
    float run_m[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) run_m[v] = -INFINITY;
#pragma unroll
    for (int i = 0; i < KBW; ++i) {
        const int kb = wave + SCR_WAVES * i;
        const int key = kb * 32 + fr;
        const float kbias = (bias && key < S) ? bias[key] : 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int qi = qi0 + mfma32_row(v, lane);
            const bool valid = kb < n_kb && key < S && key <= row0 + qi;
            lg[i][v] = valid ? lg[i][v] * scale + kbias : -INFINITY;
            run_m[v] = fmaxf(run_m[v], lg[i][v]);
        }
    }
    __shared__ float sh_m[SCR_WAVES][32], sh_l[SCR_WAVES][32];
    // row maxima: over the 32 lanes of a half-wave, then over the waves
#pragma unroll
    for (int v = 0; v < 16; ++v)
        for (int o = 16; o > 0; o >>= 1) run_m[v] = fmaxf(run_m[v], __shfl_xor(run_m[v], o));
    if (fr == 0) {
#pragma unroll
        for (int v = 0; v < 16; ++v) sh_m[wave][mfma32_row(v, lane)] = run_m[v];
    }
    __syncthreads();
    float run_l[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int r = mfma32_row(v, lane);
        float gm = sh_m[0][r];
#pragma unroll
        for (int w = 1; w < SCR_WAVES; ++w) gm = fmaxf(gm, sh_m[w][r]);
        run_m[v] = gm;     // finite: key 0 is visible to every query
        run_l[v] = 0.f;
    }
#pragma unroll
    for (int i = 0; i < KBW; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            lg[i][v] = __expf(lg[i][v] - run_m[v]);   // exp(-inf) = 0 for masked entries
            run_l[v] += lg[i][v];
        }
#pragma unroll
    for (int v = 0; v < 16; ++v)
        for (int o = 16; o > 0; o >>= 1) run_l[v] += __shfl_xor(run_l[v], o);
    if (fr == 0) {
#pragma unroll
        for (int v = 0; v < 16; ++v) sh_l[wave][mfma32_row(v, lane)] = run_l[v];
    }
    __syncthreads();
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int r = mfma32_row(v, lane);
        float gl = 0.f;
#pragma unroll
        for (int w = 0; w < SCR_WAVES; ++w) gl += sh_l[w][r];
        run_l[v] = 1.0f / gl;
    }
#pragma unroll
    for (int i = 0; i < KBW; ++i) {
        const int kb = wave + SCR_WAVES * i;
        const int key = kb * 32 + fr;
        if (COLSUM) {
            float csum = 0.f;   // masked entries hold exp(-inf) = 0
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (qi0 + mfma32_row(v, lane) < nq) csum += lg[i][v] * run_l[v];
            csum += __shfl_xor(csum, 32);
            if (fg == 0 && kb < n_kb && key < n_out)
                probs[(((size_t)b * H + h) * gridDim.x + qt) * n_out + key] = csum;
        } else if (kb < n_kb && key < S) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int qi = qi0 + mfma32_row(v, lane);
                if (qi < nq) probs[(((size_t)b * H + h) * nq + qi) * S + key] = lg[i][v] * run_l[v];
            }
        }
    }
}

template <int DH, bool COLSUM>
static bool launch_score_reg(const bf16_t* q, int ldq, int q_rows, const bf16_t* k, int ldk,
                             const float* key_bias, int B, int S, int H, int nq, float scale,
                             float* out, int n_out, hipStream_t st) {
    dim3 grid((nq + 31) / 32, H, B);
    const int need = ((S + 31) / 32 + SCR_WAVES - 1) / SCR_WAVES;  // key blocks per wave
#define MVLA_SCR(KBW)                                                                       \
    hipLaunchKernelGGL((score_probs_reg_kernel<DH, KBW, COLSUM>), grid, dim3(SCR_THREADS), 0, st, \
                       q, ldq, q_rows, k, ldk, key_bias, S, H, nq, scale, out, n_out)
    if (need <= 3) MVLA_SCR(3);
    else if (need <= 6) MVLA_SCR(6);
    else if (need <= 8) MVLA_SCR(8);
    else return false;
#undef MVLA_SCR
    return true;
}

template <int DH, bool COLSUM>
static void launch_score_dh(const bf16_t* q, int ldq, int q_rows, const bf16_t* k, int ldk,
                            const float* key_bias, int B, int S, int H, int nq, float scale,
                            float* out, int n_out, hipStream_t st) {
    // register-resident single pass when the row fits, else two passes
    if (launch_score_reg<DH, COLSUM>(q, ldq, q_rows, k, ldk, key_bias, B, S, H, nq, scale, out, n_out,
                                     st))
        return;
    dim3 grid((nq + 31) / 32, H, B);
    hipLaunchKernelGGL((score_probs_kernel<DH, COLSUM>), grid, dim3(SC_THREADS), 0, st, q, ldq, q_rows,
                       k, ldk, key_bias, S, H, nq, scale, out, n_out);
}

// colsum_n == 0: out = probabilities [B,H,nq,S]; colsum_n > 0: out = per-tile column sums
// [B, H, ceil(nq/32), colsum_n] over the first colsum_n key columns.
int launch_score_probs(const bf16_t* q, int q_row_stride, bool q_tail_only, const bf16_t* k,
                       int k_row_stride, const float* key_bias, int B, int S, int H, int dh, int nq,
                       float* out, int colsum_n, hipStream_t st) {
    if (B <= 0 || nq <= 0) return MVLA_OK;
    const float scale = 1.0f / sqrtf((float)dh);
    const int q_rows = q_tail_only ? nq : S;
#define MVLA_SC(DH_, CS_)                                                                       \
    launch_score_dh<DH_, CS_>(q, q_row_stride, q_rows, k, k_row_stride, key_bias, B, S, H, nq, scale, \
                              out, colsum_n, st)
    if (dh == 128) {
        if (colsum_n > 0) MVLA_SC(128, true); else MVLA_SC(128, false);
    } else if (dh == 64) {
        if (colsum_n > 0) MVLA_SC(64, true); else MVLA_SC(64, false);
    } else {
        return MVLA_EUNSUPPORTED;
    }
#undef MVLA_SC
    MVLA_HIP_CHECK(hipGetLastError());
    return MVLA_OK;
}

}  // namespace mvla
