// Rates this device sustains on the simplest possible kernels, for quoting a roofline
// fraction against what the part delivers as well as against its datasheet: a streaming read,
// a streaming copy, a loop of bf16 matrix-core instructions on register operands, and the
// cost of an empty launch.  Measurement only; nothing of the method is computed here.
#include "common.h"
#include "mfma.h"

namespace mvla {

constexpr int PROBE_THREADS = 256;

// The two streaming shapes below are the fastest of a sweep on this part (loads in flight per
// lane 4 / 8, plain and non-temporal, grid-strided and contiguous per workgroup, 1 Ki .. 64 Ki
// workgroups over 2 GiB): reads 6.2 - 6.6 TB/s, copies 5.3 - 5.4 TB/s (read + written).
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

// grid-stride read of n 16-byte words, eight non-temporal loads in flight per lane; the xor of
// everything read is stored only if it has a value it cannot have (keeps the loads alive
// without a store stream)
constexpr int PROBE_U = 8;
__global__ __launch_bounds__(PROBE_THREADS) void probe_read_kernel(const u32x4_t* __restrict__ src,
                                                                   size_t n, uint32_t* sink) {
    const size_t stride = (size_t)gridDim.x * PROBE_THREADS;
    size_t i = (size_t)blockIdx.x * PROBE_THREADS + threadIdx.x;
    uint32_t acc = 0;
    for (; i + (PROBE_U - 1) * stride < n; i += PROBE_U * stride) {
        u32x4_t v[PROBE_U];
#pragma unroll
        for (int u = 0; u < PROBE_U; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < PROBE_U; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < n; i += stride) {
        const u32x4_t a = src[i];
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    if (acc == 0x9e3779b9u && sink) *sink = acc;
}

// every workgroup copies its own contiguous run of words, eight loads then eight stores per lane
__global__ __launch_bounds__(PROBE_THREADS) void probe_copy_kernel(const u32x4_t* __restrict__ src,
                                                                   u32x4_t* __restrict__ dst, size_t n) {
    const size_t per = (n + gridDim.x - 1) / gridDim.x;
    const size_t lo = (size_t)blockIdx.x * per, hi = lo + per < n ? lo + per : n;
    size_t i = lo + threadIdx.x;
    for (; i + (PROBE_U - 1) * PROBE_THREADS < hi; i += PROBE_U * PROBE_THREADS) {
        u32x4_t v[PROBE_U];
#pragma unroll
        for (int u = 0; u < PROBE_U; ++u) v[u] = src[i + u * PROBE_THREADS];
#pragma unroll
        for (int u = 0; u < PROBE_U; ++u) dst[i + u * PROBE_THREADS] = v[u];
    }
    for (; i < hi; i += PROBE_THREADS) dst[i] = src[i];
}

// Every wave takes 4 + 4 operand fragments from `operands` (whatever values lie there: zeros,
// or random bf16) and runs `iters` rounds of the 16 independent 32x32x16 products of a 128x128
// register tile, the shape of the projection kernel's inner loop without any memory traffic.
__global__ __launch_bounds__(PROBE_THREADS) void probe_mfma_kernel(const uint4* __restrict__ operands,
                                                                   int iters, float* sink) {
    const int lane = threadIdx.x & 63;
    uint4 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = operands[(size_t)(i * 64 + lane)];
        b[i] = operands[(size_t)((4 + i) * 64 + lane)];
    }
    f32x16_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] = mfma32(b[j], a[i], acc[i][j]);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) s += acc[i][j][v];
    if (s == 1.2345e30f && sink) *sink = s;
}

__global__ void probe_empty_kernel() {}

int launch_probe_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t st) {
    const size_t n = bytes / 16;
    const unsigned grid = (unsigned)(n / (PROBE_THREADS * PROBE_U) < 65536 ? n / (PROBE_THREADS * PROBE_U) + 1
                                                                            : 65536);
    hipLaunchKernelGGL(probe_read_kernel, dim3(grid), dim3(PROBE_THREADS), 0, st,
                       static_cast<const u32x4_t*>(src), n, sink);
    MVLA_HIP_CHECK(hipGetLastError());
    return MVLA_OK;
}
int launch_probe_copy(const void* src, void* dst, size_t bytes, hipStream_t st) {
    hipLaunchKernelGGL(probe_copy_kernel, dim3(8192), dim3(PROBE_THREADS), 0, st,
                       static_cast<const u32x4_t*>(src), static_cast<u32x4_t*>(dst), bytes / 16);
    MVLA_HIP_CHECK(hipGetLastError());
    return MVLA_OK;
}
// one workgroup of four waves (one per SIMD) per compute unit
int launch_probe_mfma(const void* operands, int n_cu, int iters, float* sink, hipStream_t st) {
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(n_cu), dim3(PROBE_THREADS), 0, st,
                       static_cast<const uint4*>(operands), iters, sink);
    MVLA_HIP_CHECK(hipGetLastError());
    return MVLA_OK;
}
int launch_probe_empty(hipStream_t st) {
    hipLaunchKernelGGL(probe_empty_kernel, dim3(1), dim3(64), 0, st);
    MVLA_HIP_CHECK(hipGetLastError());
    return MVLA_OK;
}

}  // namespace mvla
