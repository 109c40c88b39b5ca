// Pruning-step kernels for gfx950: attention-column salience, modality budget,
// per-modality top-k selection, gather-compaction.  All are bandwidth- or
// latency-bound; none uses floating-point atomics, so every result is
// reproducible bit for bit.
#include "common.h"

namespace mvla {

// ---------------------------------------------------------------------------
// Salience (paper Sec. 3.2, Eq. 3): column sums of the language-query
// attention rows over the visual columns, divided by the number of rows.
//
// A wave is laid out as 4 row-groups x 16 lanes; a lane owns VEC consecutive
// columns, so one row-group reads 16*VEC consecutive floats of one row
// (coalesced 16-byte loads when VEC == 4).  Row-groups are folded with two
// wavefront shuffles, the block's four waves through LDS, and the blocks that
// share a column chunk through a partial buffer summed in fixed order by
// whichever of them arrives last (integer arrival counter, no float atomics).
// ---------------------------------------------------------------------------
// forward declarations of the per-sample steps that the fused kernel runs after the salience
struct FusedPrune {
    int n2, n3, n_text, k_total, min2, min3;
    int32_t* k2k3;
    int32_t* kept_idx;
    uint32_t* sample_counters;  // one arrival counter per sample (kept at zero between calls)
};
template <bool COHERENT>
__device__ __forceinline__ void finish_sample(const float* sal_b, const FusedPrune& f, int b,
                                              uint32_t* keys);

constexpr int SAL_THREADS = 256;
constexpr int SEL_THREADS = 256;    // selection (also the tail of the fused kernel)
constexpr int SEL_MAX_N = 16384;    // largest segment the selection stages in LDS
constexpr int SEL_SMALL_N = 64;     // up to here a direct rank count beats the threshold search (measured)
constexpr int SAL_LPR = 16;                        // lanes per row-group
constexpr int SAL_GROUPS = SAL_THREADS / SAL_LPR;  // 16 row-groups per block

// FUSED: the workgroup that completes the last column chunk of a sample goes on to split the
// budget and select that sample's tokens (same arithmetic as budget_kernel / select_kernel).
template <int VEC, bool FUSED>
__global__ __launch_bounds__(SAL_THREADS) void salience_kernel(
    const float* __restrict__ attn, int R, int S, int n_vis, int rows_per_split, int n_split,
    float inv_rows, float* __restrict__ sal, float* __restrict__ partial,
    uint32_t* __restrict__ counters, FusedPrune fused) {
    extern __shared__ uint32_t dyn_lds[];  // selection keys (fused variant only)
    constexpr int CW = SAL_LPR * VEC;  // columns per chunk
    const int chunk = blockIdx.x, split = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x;
    const int lane16 = tid % SAL_LPR;
    const int group = tid / SAL_LPR;
    const int col0 = chunk * CW + lane16 * VEC;
    const int r_begin = split * rows_per_split;
    const int r_end = min(R, r_begin + rows_per_split);
    const float* base = attn + (size_t)b * R * S;

    float acc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0.f;

    if (VEC == 4) {
        if (col0 + 3 < n_vis) {
            int r = r_begin + group;
            // four, then two independent loads in flight per lane
            for (; r + 3 * SAL_GROUPS < r_end; r += 4 * SAL_GROUPS) {
                const float4 a = *reinterpret_cast<const float4*>(base + (size_t)r * S + col0);
                const float4 c =
                    *reinterpret_cast<const float4*>(base + (size_t)(r + SAL_GROUPS) * S + col0);
                const float4 d =
                    *reinterpret_cast<const float4*>(base + (size_t)(r + 2 * SAL_GROUPS) * S + col0);
                const float4 e =
                    *reinterpret_cast<const float4*>(base + (size_t)(r + 3 * SAL_GROUPS) * S + col0);
                acc[0] += a.x; acc[1] += a.y; acc[2] += a.z; acc[3] += a.w;
                acc[0] += c.x; acc[1] += c.y; acc[2] += c.z; acc[3] += c.w;
                acc[0] += d.x; acc[1] += d.y; acc[2] += d.z; acc[3] += d.w;
                acc[0] += e.x; acc[1] += e.y; acc[2] += e.z; acc[3] += e.w;
            }
            for (; r + SAL_GROUPS < r_end; r += 2 * SAL_GROUPS) {
                const float4 a = *reinterpret_cast<const float4*>(base + (size_t)r * S + col0);
                const float4 c =
                    *reinterpret_cast<const float4*>(base + (size_t)(r + SAL_GROUPS) * S + col0);
                acc[0] += a.x; acc[1] += a.y; acc[2] += a.z; acc[3] += a.w;
                acc[0] += c.x; acc[1] += c.y; acc[2] += c.z; acc[3] += c.w;
            }
            for (; r < r_end; r += SAL_GROUPS) {
                const float4 a = *reinterpret_cast<const float4*>(base + (size_t)r * S + col0);
                acc[0] += a.x; acc[1] += a.y; acc[2] += a.z; acc[3] += a.w;
            }
        } else {
            for (int r = r_begin + group; r < r_end; r += SAL_GROUPS)
#pragma unroll
                for (int v = 0; v < VEC; ++v)
                    if (col0 + v < n_vis) acc[v] += base[(size_t)r * S + col0 + v];
        }
    } else {
        for (int r = r_begin + group; r < r_end; r += SAL_GROUPS)
#pragma unroll
            for (int v = 0; v < VEC; ++v)
                if (col0 + v < n_vis) acc[v] += base[(size_t)r * S + col0 + v];
    }

    // fold the wave's 4 row-groups (lanes l, l^16, l^32, l^48 own the same columns)
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
        acc[v] += __shfl_xor(acc[v], 16);
        acc[v] += __shfl_xor(acc[v], 32);
    }
    __shared__ float red[SAL_THREADS / 64][CW];
    __shared__ int is_last;
    const int wave = tid / 64, lane = tid % 64;
    if (lane < SAL_LPR) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) red[wave][lane * VEC + v] = acc[v];
    }
    __syncthreads();
    float tot = 0.f;
    const int c = chunk * CW + tid;
    if (tid < CW) {
#pragma unroll
        for (int w = 0; w < SAL_THREADS / 64; ++w) tot += red[w][tid];
    }
    // store of a finished salience value: plain, or agent-coherent when another workgroup
    // (maybe on another XCD) will read it in this same launch
    auto put = [&](float v) {
        if (FUSED)
            __hip_atomic_store(&sal[(size_t)b * n_vis + c], v, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        else
            sal[(size_t)b * n_vis + c] = v;
    };
    if (n_split == 1) {
        if (tid < CW && c < n_vis) put(tot * inv_rows);
        if (!FUSED) return;
    } else {
        // several blocks share this column chunk: publish, last arrival finishes
        float* pslot = partial + ((size_t)(b * gridDim.x + chunk) * n_split) * CW;
        // partial sums cross CUs/XCDs through agent-coherent accesses (no cache-wide flushes)
        if (tid < CW)
            __hip_atomic_store(&pslot[(size_t)split * CW + tid], tot, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0) {
            uint32_t* ctr = counters + (b * gridDim.x + chunk);
            const uint32_t prev =
                __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            is_last = (prev == (uint32_t)(n_split - 1));
            if (is_last) __hip_atomic_store(ctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        if (!is_last) return;
        if (tid < CW && c < n_vis) {
            float s = 0.f;
#pragma unroll 8
            for (int i = 0; i < n_split; ++i)
                s += __hip_atomic_load(&pslot[(size_t)i * CW + tid], __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
            put(s * inv_rows);
        }
        if (!FUSED) return;
    }
    // ---- fused tail: this chunk of sample b is complete; the last chunk's workgroup finishes b
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) {
        const uint32_t prev = __hip_atomic_fetch_add(&fused.sample_counters[b], 1u, __ATOMIC_RELAXED,
                                                     __HIP_MEMORY_SCOPE_AGENT);
        is_last = (prev == gridDim.x - 1);
        if (is_last)
            __hip_atomic_store(&fused.sample_counters[b], 0u, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (!is_last) return;
    finish_sample<true>(sal + (size_t)b * n_vis, fused, b, dyn_lds);
}

static void salience_shape(int B, int R, int n_vis, int vec, int* chunks, int* n_split,
                           int* rows_per_split) {
    const int cw = SAL_LPR * vec;
    *chunks = (n_vis + cw - 1) / cw;
    // aim for ~2048 blocks, at least 2 passes of the 16 row-groups each
    long blocks = (long)B * *chunks;
    int split = (int)((2048 + blocks - 1) / blocks);
    const int max_split = (R + 2 * SAL_GROUPS - 1) / (2 * SAL_GROUPS);
    if (split > max_split) split = max_split;
    if (split < 1) split = 1;
    *rows_per_split = (R + split - 1) / split;
    *n_split = (R + *rows_per_split - 1) / *rows_per_split;
}

size_t salience_scratch_bytes(int B, int H, int Nq, int n_vis) {
    // worst case over VEC in {1,4}: chunks*CW <= n_vis + 63, n_split <= R/32 + 1
    const size_t R = (size_t)H * Nq;
    return align_up((size_t)B * (size_t)(n_vis + 64) * (R / (2 * SAL_GROUPS) + 2) * 4, 256);
}

// mean_rows: the row count the sums are divided by; 0 means the R = H*Nq rows read.  (When the
// rows are already sums over a tile of queries, the caller passes the original row count.)
static int launch_salience_any(const float* attn, int B, int H, int Nq, int S, int n_vis,
                               float* sal, float* partial, uint32_t* counters,
                               const FusedPrune* fused, int mean_rows, hipStream_t st) {
    const int R = H * Nq;
    const bool vec4 = (S % 4 == 0) && ((reinterpret_cast<uintptr_t>(attn) & 15) == 0);
    int chunks, n_split, rps;
    salience_shape(B, R, n_vis, vec4 ? 4 : 1, &chunks, &n_split, &rps);
    // counters: [0, B*chunks) chunk arrivals, then B sample arrivals (first half of the area)
    if ((long)B * chunks + B > kCounterWords / 2) return MVLA_EUNSUPPORTED;
    dim3 grid(chunks, n_split, B);
    const float inv_rows = 1.0f / (float)(mean_rows > 0 ? mean_rows : R);
    FusedPrune f{};
    size_t lds = 0;
    if (fused) {
        f = *fused;
        f.sample_counters = counters + (size_t)B * chunks;
        lds = (size_t)max(f.n2 + f.n3, 1) * 4;   // selection keys of both segments
    }
    // (the fused variants keep the keys of both segments in LDS: up to 128 KiB, above the default
    // limit of a kernel, which is raised once per device)
#define MVLA_SAL(V, F)                                                                          \
    do {                                                                                        \
        auto kern = salience_kernel<V, F>;                                                      \
        if (F) {                                                                                \
            static bool lds_set[kMaxDevices] = {};                                              \
            int dev = 0;                                                                        \
            MVLA_HIP_CHECK(hipGetDevice(&dev));                                                 \
            if (dev < 0 || dev >= kMaxDevices || !lds_set[dev]) {                               \
                MVLA_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),         \
                                                   hipFuncAttributeMaxDynamicSharedMemorySize,  \
                                                   2 * SEL_MAX_N * 4));                         \
                if (dev >= 0 && dev < kMaxDevices) lds_set[dev] = true;                         \
            }                                                                                   \
        }                                                                                       \
        hipLaunchKernelGGL(kern, grid, dim3(SAL_THREADS), lds, st, attn, R, S, n_vis, rps,      \
                           n_split, inv_rows, sal, partial, counters, f);                       \
    } while (0)
    if (vec4) {
        if (fused) MVLA_SAL(4, true); else MVLA_SAL(4, false);
    } else {
        if (fused) MVLA_SAL(1, true); else MVLA_SAL(1, false);
    }
#undef MVLA_SAL
    MVLA_HIP_CHECK(hipGetLastError());
    return MVLA_OK;
}

int launch_salience(const float* attn, int B, int H, int Nq, int S, int n_vis, float* sal,
                    float* partial, uint32_t* counters, int mean_rows, hipStream_t st) {
    return launch_salience_any(attn, B, H, Nq, S, n_vis, sal, partial, counters, nullptr, mean_rows,
                               st);
}

int launch_prune_fused(const float* attn, int B, int H, int Nq, int S, int n2, int n3, int n_text,
                       int k_total, int min2, int min3, float* sal, int32_t* k2k3,
                       int32_t* kept_idx, float* partial, uint32_t* counters, int mean_rows,
                       hipStream_t st) {
    FusedPrune f{n2, n3, n_text, k_total, min2, min3, k2k3, kept_idx, nullptr};
    return launch_salience_any(attn, B, H, Nq, S, n2 + n3, sal, partial, counters, &f, mean_rows,
                               st);
}

// ---------------------------------------------------------------------------
// Salience without a context or workspace, for callers that cannot allocate
// device memory (code under graph capture, serving loops): the row-split
// partial sums and the arrival counters live in a fixed array of this module.
// Every GPU holds its own copy of the array until the process ends.
// ---------------------------------------------------------------------------
constexpr size_t kStaticCounterBytes = size_t(kCounterWords / 2) * 4;   // 32 KiB of arrival counters
constexpr size_t kStaticPartialBytes = size_t(16) << 20;                // 16 MiB of partial sums
static __device__ __align__(256) unsigned char scratch[kStaticCounterBytes + kStaticPartialBytes];
// device address of `scratch` on each GPU (the array's name is only a host-side handle)
static void* g_scratch_addr[kMaxDevices] = {};

__global__ void clear_words_kernel(uint32_t* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

}  // namespace mvla

extern "C" int mvla_salience_noalloc(void* hip_stream, const float* attn, int B, int H, int Nq, int S,
                                     int n_vis, float* sal) {
    using namespace mvla;
    if (!attn || !sal) return MVLA_EINVAL;
    if (B <= 0 || H <= 0 || Nq <= 0 || S <= 0 || n_vis <= 0 || n_vis > S) return MVLA_EINVAL;
    if ((reinterpret_cast<uintptr_t>(attn) & 3) || (reinterpret_cast<uintptr_t>(sal) & 3))
        return MVLA_EINVAL;
    // the fixed scratch bounds the shape: partial sums and one counter per (sample, column chunk)
    const bool vec4 = (S % 4 == 0) && ((reinterpret_cast<uintptr_t>(attn) & 15) == 0);
    int chunks, n_split, rps;
    salience_shape(B, H * Nq, n_vis, vec4 ? 4 : 1, &chunks, &n_split, &rps);
    const long n_counters = (long)B * chunks + B;
    if (salience_scratch_bytes(B, H, Nq, n_vis) > kStaticPartialBytes ||
        n_counters > (long)(kStaticCounterBytes / 4))
        return MVLA_ELIMIT;
    int dev = 0;
    MVLA_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return MVLA_EUNSUPPORTED;
    if (!g_scratch_addr[dev]) {   // once per device, with that device current
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return MVLA_EHIP;
        g_scratch_addr[dev] = p;
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    uint32_t* counters = static_cast<uint32_t*>(g_scratch_addr[dev]);
    float* partial = reinterpret_cast<float*>(static_cast<char*>(g_scratch_addr[dev]) + kStaticCounterBytes);
    // the array keeps whatever the last call left: the counters this call uses start at zero
    // (a kernel, not a memset, so that the call can be recorded into a graph)
    hipLaunchKernelGGL(clear_words_kernel, dim3((unsigned)((n_counters + 255) / 256)), dim3(256), 0, st,
                       counters, (int)n_counters);
    MVLA_HIP_CHECK(hipGetLastError());
    return launch_salience(attn, B, H, Nq, S, n_vis, sal, partial, counters, 0, st);
}

namespace mvla {

// ---------------------------------------------------------------------------
// Modality budget (paper Eq. 5): fp64 masses per sample, integer split.
// ---------------------------------------------------------------------------
constexpr int BUD_THREADS = 256;

// Workgroup barrier for data that is exchanged through LDS only: it waits for this wave's LDS
// operations, not for its outstanding global stores.  (__syncthreads() waits for those too --
// a full write round trip whenever budget or index stores are in flight, several times per
// sample in the tail of the fused kernel.)
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ inline double block_sum_f64(double v, double* sh) {
    // fixed-shape tree: wave shuffle then 4 partials in LDS
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    lds_barrier();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    lds_barrier();
    double t = 0.0;
    for (int w = 0; w < BUD_THREADS / 64; ++w) t += sh[w];
    return t;
}

__device__ inline void budget_split(double a2, double a3, int n2, int n3, int k_total, int min2,
                                    int min3, int* k2_out, double* m2_out) {
    const double tot = a2 + a3;
    const double m2 = tot > 0.0 ? a2 / tot : (double)n2 / (double)(n2 + n3);
    int k2 = (int)floor((double)k_total * m2 + 0.5);
    const int lo = max(min2, k_total - n3);
    const int hi = min(n2, k_total - min3);
    k2 = min(max(k2, lo), hi);
    *k2_out = k2;
    *m2_out = m2;
}

__global__ __launch_bounds__(BUD_THREADS) void budget_kernel(const float* __restrict__ sal, int n2,
                                                             int n3, int k_total, int min2,
                                                             int min3, int32_t* __restrict__ k2k3,
                                                             float* __restrict__ mass) {
    __shared__ double sh[BUD_THREADS / 64];
    const int b = blockIdx.x;
    const float* s = sal + (size_t)b * (n2 + n3);
    double a2 = 0.0, a3 = 0.0;
    for (int i = threadIdx.x; i < n2; i += BUD_THREADS) a2 += (double)s[i];
    for (int i = threadIdx.x; i < n3; i += BUD_THREADS) a3 += (double)s[n2 + i];
    a2 = block_sum_f64(a2, sh);
    a3 = block_sum_f64(a3, sh);
    if (threadIdx.x == 0) {
        int k2;
        double m2;
        budget_split(a2, a3, n2, n3, k_total, min2, min3, &k2, &m2);
        k2k3[2 * b] = k2;
        k2k3[2 * b + 1] = k_total - k2;
        if (mass) {
            mass[2 * b] = (float)m2;
            mass[2 * b + 1] = (float)(1.0 - m2);
        }
    }
}

int launch_budget(const float* sal, int B, int n2, int n3, int k_total, int min2, int min3,
                  int32_t* k2k3, float* mass, hipStream_t st) {
    hipLaunchKernelGGL(budget_kernel, dim3(B), dim3(BUD_THREADS), 0, st, sal, n2, n3, k_total,
                       min2, min3, k2k3, mass);
    MVLA_HIP_CHECK(hipGetLastError());
    return MVLA_OK;
}

// ---------------------------------------------------------------------------
// Per-modality top-k.  One workgroup per (sample, segment); the segment's
// scores sit in LDS as order-preserving 32-bit keys.  Four 8-bit radix passes
// find the K-th largest key T exactly; tokens with key > T are kept, and of
// those with key == T the lowest-indexed (K - #greater).  Each thread owns a
// contiguous index range, so a block prefix sum of its keep counts gives
// output slots that are already in ascending index order -- no sort.
// ---------------------------------------------------------------------------

__device__ inline uint32_t sal_key(float x) {
    uint32_t u = __float_as_uint(x);
    if (u == 0x80000000u) u = 0u;  // -0 ranks with +0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// inclusive prefix sum over SEL_THREADS values (one per thread), result per thread
__device__ inline uint32_t block_scan_incl(uint32_t v, uint32_t* wsum) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = __shfl_up(v, o);
        if (lane >= o) v += t;
    }
    lds_barrier();
    if (lane == 63) wsum[wave] = v;
    lds_barrier();
    uint32_t add = 0;
    for (int w = 0; w < wave; ++w) add += wsum[w];
    return v + add;
}

// Short segments (at most one token per thread; used up to SEL_SMALL_N): thread i ranks key i
// directly -- the keys above it plus the equal keys at a lower index -- and keeps it when that
// rank is below k.  No threshold search: n comparisons per thread instead of four histogram
// passes with their scans.  Every lane reads the same key in a step (an LDS broadcast).
// Threads are in index order, so the keep flags' prefix count is the output slot.
__device__ __forceinline__ void select_small(const uint32_t* keys /*LDS [n]*/, int n, int k, int idx_offset,
                             int32_t* __restrict__ out, uint32_t* wsum /*LDS [4]*/) {
    const int i = threadIdx.x, lane = i & 63, wave = i >> 6;
    lds_barrier();   // the keys are in LDS
    const uint32_t my = i < n ? keys[i] : 0u;
    // keys before i count when >= my, keys after i when > my, i.e. >= my + 1 (a key of all ones
    // is a NaN, invalid input: its threshold wraps and the token is dropped)
    const uint32_t my1 = my + 1u;
    const int w0 = min(wave * 64, n), w1 = min(w0 + 64, n);   // the indices this wave's lanes hold
    int rank = 0;
    // 32 keys per batch, so that the LDS reads of a batch are in flight together (read one by
    // one, their latency is all the loop does); batches below or above the wave's own indices
    // compare against one threshold
    constexpr int BATCH = 32;
    for (int j = 0; j < n; j += BATCH) {
        uint32_t v[BATCH];
        const bool full = j + BATCH <= n;
        if (full) {
#pragma unroll
            for (int u = 0; u < BATCH; ++u) v[u] = keys[j + u];
        } else {
#pragma unroll
            for (int u = 0; u < BATCH; ++u) v[u] = j + u < n ? keys[j + u] : 0u;
        }
        if (j + BATCH <= w0) {
#pragma unroll
            for (int u = 0; u < BATCH; ++u) rank += v[u] >= my;
        } else if (j >= w1 && full) {
#pragma unroll
            for (int u = 0; u < BATCH; ++u) rank += v[u] >= my1;
        } else {
#pragma unroll
            for (int u = 0; u < BATCH; ++u)
                rank += (j + u < n) && v[u] >= (j + u < i ? my : my1);
        }
    }
    const bool keep = i < n && rank < k;
    const unsigned long long bal = __ballot(keep);
    if (lane == 0) wsum[wave] = (uint32_t)__popcll(bal);
    lds_barrier();
    uint32_t slot = (uint32_t)__popcll(bal & ((1ull << lane) - 1ull));
    for (int w = 0; w < wave; ++w) slot += wsum[w];
    if (keep) out[slot] = idx_offset + i;
}

// Selection among n keys that already sit in LDS (written by this workgroup; the first barrier
// below orders those writes before the reads).
__device__ __forceinline__ void select_from_keys(const uint32_t* keys /*LDS [n]*/, int n, int k, int idx_offset,
                                 int32_t* __restrict__ out, uint32_t* hist /*LDS [256]*/,
                                 uint32_t* wsum /*LDS [4]*/, uint32_t* bcast /*LDS [4]*/) {
    const int tid = threadIdx.x;
    if (k <= 0) return;
    if (k > n) k = n;
    if (n <= SEL_SMALL_N) {
        select_small(keys, n, k, idx_offset, out, wsum);
        return;
    }
    uint32_t prefix = 0, prefix_mask = 0;
    uint32_t remaining = (uint32_t)k;  // rank (1-based, from the top) of T among matching keys
    for (int shift = 24; shift >= 0; shift -= 8) {
        hist[tid] = 0;
        lds_barrier();
        for (int i = tid; i < n; i += SEL_THREADS) {
            const uint32_t key = keys[i];
            if ((key & prefix_mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
        }
        lds_barrier();
        // suffix counts from the top digit down: thread t looks at digit 255-t
        const uint32_t mine = hist[255 - tid];
        const uint32_t incl = block_scan_incl(mine, wsum);
        const uint32_t excl = incl - mine;
        if (excl < remaining && remaining <= incl) {
            bcast[0] = (uint32_t)(255 - tid);
            bcast[1] = remaining - excl;
        }
        lds_barrier();
        prefix |= bcast[0] << shift;
        prefix_mask |= 255u << shift;
        remaining = bcast[1];
        lds_barrier();
    }
    const uint32_t T = prefix;
    const uint32_t need_eq = remaining;  // how many keys equal to T are kept
    const int per = (n + SEL_THREADS - 1) / SEL_THREADS;
    const int i0 = min(n, tid * per), i1 = min(n, i0 + per);
    uint32_t gt = 0, eq = 0;
    for (int i = i0; i < i1; ++i) {
        const uint32_t key = keys[i];
        gt += key > T;
        eq += key == T;
    }
    const uint32_t gt_before = block_scan_incl(gt, wsum) - gt;
    const uint32_t eq_before = block_scan_incl(eq, wsum) - eq;
    uint32_t eq_rank = eq_before;
    uint32_t slot = gt_before + min(eq_before, need_eq);
    for (int i = i0; i < i1; ++i) {
        const uint32_t key = keys[i];
        bool keep = key > T;
        if (key == T) {
            keep = eq_rank < need_eq;
            ++eq_rank;
        }
        if (keep) out[slot++] = idx_offset + i;
    }
}

__device__ __forceinline__ void select_segment(const float* __restrict__ seg, int n, int k, int idx_offset,
                               int32_t* __restrict__ out, uint32_t* keys /*LDS [n]*/,
                               uint32_t* hist, uint32_t* wsum, uint32_t* bcast) {
    for (int i = threadIdx.x; i < n; i += SEL_THREADS) keys[i] = sal_key(seg[i]);
    select_from_keys(keys, n, k, idx_offset, out, hist, wsum, bcast);
}

__global__ __launch_bounds__(SEL_THREADS) void select_kernel(const float* __restrict__ sal,
                                                             const int32_t* __restrict__ k2k3,
                                                             int n2, int n3, int n_text,
                                                             int k_total,
                                                             int32_t* __restrict__ kept_idx) {
    extern __shared__ uint32_t keys[];
    __shared__ uint32_t hist[256];
    __shared__ uint32_t wsum[SEL_THREADS / 64];
    __shared__ uint32_t bcast[4];
    const int b = blockIdx.y, which = blockIdx.x;
    int32_t* row = kept_idx + (size_t)b * (k_total + n_text);
    // clamp a malformed budget row into the feasible range
    int k2 = k2k3[2 * b];
    k2 = min(max(k2, max(0, k_total - n3)), min(n2, k_total));
    const int k3 = k_total - k2;
    if (which == 0) {
        select_segment(sal + (size_t)b * (n2 + n3), n2, k2, 0, row, keys, hist, wsum, bcast);
    } else if (which == 1) {
        select_segment(sal + (size_t)b * (n2 + n3) + n2, n3, k3, n2, row + k2, keys, hist,
                              wsum, bcast);
    } else {
        for (int i = threadIdx.x; i < n_text; i += SEL_THREADS) row[k_total + i] = n2 + n3 + i;
    }
}

// Budget and selection of one sample by one workgroup (tail of the fused kernel).  Same
// summation order as budget_kernel, same selection as select_kernel.
template <bool COHERENT>
__device__ __forceinline__ void finish_sample(const float* sal_b, const FusedPrune& f, int b,
                                              uint32_t* keys) {
    __shared__ double sh_d[BUD_THREADS / 64];
    __shared__ uint32_t hist[256];
    __shared__ uint32_t wsum[SEL_THREADS / 64];
    __shared__ uint32_t bcast[4];
    __shared__ int sh_k2;
    auto ld = [&](int i) {
        return COHERENT ? __hip_atomic_load(&sal_b[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                        : sal_b[i];
    };
    // one pass over the sample's scores feeds both the masses and the selection keys of both
    // segments (keys [0, n2) and [n2, n2 + n3) of the LDS array)
    double a2 = 0.0, a3 = 0.0;
    for (int i = threadIdx.x; i < f.n2; i += BUD_THREADS) {
        const float v = ld(i);
        a2 += (double)v;
        keys[i] = sal_key(v);
    }
    for (int i = threadIdx.x; i < f.n3; i += BUD_THREADS) {
        const float v = ld(f.n2 + i);
        a3 += (double)v;
        keys[f.n2 + i] = sal_key(v);
    }
    a2 = block_sum_f64(a2, sh_d);
    a3 = block_sum_f64(a3, sh_d);
    if (threadIdx.x == 0) {
        int k2;
        double m2;
        budget_split(a2, a3, f.n2, f.n3, f.k_total, f.min2, f.min3, &k2, &m2);
        f.k2k3[2 * b] = k2;
        f.k2k3[2 * b + 1] = f.k_total - k2;
        sh_k2 = k2;
    }
    lds_barrier();
    const int k2 = sh_k2;
    int32_t* row = f.kept_idx + (size_t)b * (f.k_total + f.n_text);
    select_from_keys(keys, f.n2, k2, 0, row, hist, wsum, bcast);
    lds_barrier();
    select_from_keys(keys + f.n2, f.n3, f.k_total - k2, f.n2, row + k2, hist, wsum, bcast);
    for (int i = threadIdx.x; i < f.n_text; i += SEL_THREADS)
        row[f.k_total + i] = f.n2 + f.n3 + i;
}

int launch_select(const float* sal, const int32_t* k2k3, int B, int n2, int n3, int n_text,
                  int k_total, int32_t* kept_idx, hipStream_t st) {
    if (n2 > SEL_MAX_N || n3 > SEL_MAX_N) return MVLA_EUNSUPPORTED;
    const size_t lds = (size_t)max(max(n2, n3), 1) * 4;
    hipLaunchKernelGGL(select_kernel, dim3(3, B), dim3(SEL_THREADS), lds, st, sal, k2k3, n2, n3,
                       n_text, k_total, kept_idx);
    MVLA_HIP_CHECK(hipGetLastError());
    return MVLA_OK;
}

// ---------------------------------------------------------------------------
// Gather-compaction (paper Sec. 4.4 / Eq. 10): copy kept rows and their
// position ids.  One workgroup per output row, 16 bytes per lane per access.
// ---------------------------------------------------------------------------
constexpr int CMP_THREADS = 256;

__global__ __launch_bounds__(CMP_THREADS) void compact_kernel(
    const uint4* __restrict__ h, const int32_t* __restrict__ pos,
    const int32_t* __restrict__ kept_idx, int S, int S_out, int row_vec /* D*2/16 */,
    uint4* __restrict__ h_out, int32_t* __restrict__ pos_out) {
    const int i = blockIdx.x, b = blockIdx.y;
    int src = kept_idx[(size_t)b * S_out + i];
    src = min(max(src, 0), S - 1);
    const uint4* from = h + ((size_t)b * S + src) * row_vec;
    uint4* to = h_out + ((size_t)b * S_out + i) * row_vec;
    int c = threadIdx.x;
    for (; c + CMP_THREADS < row_vec; c += 2 * CMP_THREADS) {
        const uint4 a = from[c];
        const uint4 d = from[c + CMP_THREADS];
        to[c] = a;
        to[c + CMP_THREADS] = d;
    }
    for (; c < row_vec; c += CMP_THREADS) to[c] = from[c];
    if (threadIdx.x == 0) pos_out[(size_t)b * S_out + i] = pos[(size_t)b * S + src];
}

int launch_compact(const bf16_t* h, const int32_t* pos, const int32_t* kept_idx, int B, int S,
                   int S_out, int D, bf16_t* h_out, int32_t* pos_out, hipStream_t st) {
    if (S_out == 0 || B == 0) return MVLA_OK;
    hipLaunchKernelGGL(compact_kernel, dim3(S_out, B), dim3(CMP_THREADS), 0, st,
                       reinterpret_cast<const uint4*>(h), pos, kept_idx, S, S_out, D / 8,
                       reinterpret_cast<uint4*>(h_out), pos_out);
    MVLA_HIP_CHECK(hipGetLastError());
    return MVLA_OK;
}

// ---------------------------------------------------------------------------
// Per-patch modality indicators of the semantic stage (paper Sec. 3.2,
// Eqs. 4-6): the 3D attention vector of a patch (over the head x query rows)
// is split into its projection on the 2D vector and the orthogonal rest; the
// outputs are the L1 shares |a2| / (|a2|+|a3|) and |a3_ortho| / (|a2|+|a3|).
// One workgroup handles 8 patches of one sample with 32 row-groups (a thread
// owns a patch and every 32nd row; small patch groups keep the launch wide at
// batch 1); pass 1 accumulates <a2,a2>, <a2,a3>, |a2|, |a3|, pass 2 the L1 norm
// of the residual (second read served by the L2).
// ---------------------------------------------------------------------------
constexpr int DEC_THREADS = 256;
constexpr int DEC_PP = 8;                       // patches per workgroup
constexpr int DEC_RG = DEC_THREADS / DEC_PP;    // row groups

__global__ __launch_bounds__(DEC_THREADS) void decompose_kernel(const float* __restrict__ attn,
                                                                int R, int S, int n_patch,
                                                                float* __restrict__ m2d,
                                                                float* __restrict__ m3d) {
    __shared__ float red[4][DEC_RG][DEC_PP];
    __shared__ float coef[DEC_PP];
    const int lp = threadIdx.x % DEC_PP, g = threadIdx.x / DEC_PP;
    const int b = blockIdx.y, p = blockIdx.x * DEC_PP + lp;
    const bool live = p < n_patch;
    const float* base = attn + (size_t)b * R * S;
    float s22 = 0.f, s23 = 0.f, l2 = 0.f, l3 = 0.f;
    if (live) {
#pragma unroll 4
        for (int r = g; r < R; r += DEC_RG) {
            const float a2 = base[(size_t)r * S + p], a3 = base[(size_t)r * S + n_patch + p];
            s22 += a2 * a2;
            s23 += a2 * a3;
            l2 += fabsf(a2);
            l3 += fabsf(a3);
        }
    }
    red[0][g][lp] = s22;
    red[1][g][lp] = s23;
    red[2][g][lp] = l2;
    red[3][g][lp] = l3;
    __syncthreads();
    float den = 0.f, n2 = 0.f;
    if (g == 0) {
        float t[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            t[q] = 0.f;
            for (int w = 0; w < DEC_RG; ++w) t[q] += red[q][w][lp];
        }
        coef[lp] = t[0] > 0.f ? t[1] / t[0] : 0.f;
        n2 = t[2];
        den = t[2] + t[3];
    }
    __syncthreads();
    const float c = coef[lp];
    float lo = 0.f;
    if (live) {
#pragma unroll 4
        for (int r = g; r < R; r += DEC_RG) {
            const float a2 = base[(size_t)r * S + p], a3 = base[(size_t)r * S + n_patch + p];
            lo += fabsf(a3 - c * a2);
        }
    }
    red[0][g][lp] = lo;
    __syncthreads();
    if (g == 0 && live) {
        float t = 0.f;
        for (int w = 0; w < DEC_RG; ++w) t += red[0][w][lp];
        m2d[(size_t)b * n_patch + p] = den > 0.f ? n2 / den : 0.f;
        m3d[(size_t)b * n_patch + p] = den > 0.f ? t / den : 0.f;
    }
}

int launch_decompose(const float* attn, int B, int H, int Nq, int S, int n_patch, float* m2d,
                     float* m3d, hipStream_t st) {
    hipLaunchKernelGGL(decompose_kernel, dim3((n_patch + DEC_PP - 1) / DEC_PP, B), dim3(DEC_THREADS),
                       0, st, attn, H * Nq, S, n_patch, m2d, m3d);
    MVLA_HIP_CHECK(hipGetLastError());
    return MVLA_OK;
}

// ---------------------------------------------------------------------------
// Action-iteration smoothing of an indicator (paper Sec. 4.3 Eq. 7, Sec. 4.4
// Eqs. 8-9): observation at the cold start, running mean while the window
// fills, exponential moving average afterwards.  w_prev and w_new are the two
// weights of the step, computed on the host in fp64 and rounded to fp32.
// ---------------------------------------------------------------------------
__global__ void smooth_kernel(const float* __restrict__ x_t, float* __restrict__ x_hat, size_t n,
                              float w_prev, float w_new, int cold) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float x = x_t[i];
    x_hat[i] = cold ? x : w_prev * x_hat[i] + w_new * x;
}

int launch_smooth(const float* x_t, float* x_hat, size_t n, int t, int k, double beta,
                  hipStream_t st) {
    if (n == 0) return MVLA_OK;
    double wp, wn;
    if (t < k) {
        wp = (double)(t - 1) / (double)t;
        wn = 1.0 / (double)t;
    } else {
        wp = beta;
        wn = 1.0 - beta;
    }
    hipLaunchKernelGGL(smooth_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, x_t,
                       x_hat, n, (float)wp, (float)wn, t == 1 ? 1 : 0);
    MVLA_HIP_CHECK(hipGetLastError());
    return MVLA_OK;
}

}  // namespace mvla
