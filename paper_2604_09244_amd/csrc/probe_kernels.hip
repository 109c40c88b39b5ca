// Rates this device sustains on the simplest possible kernels, for quoting a roofline
// fraction against what the part delivers as well as against its datasheet: a streaming read,
// a streaming copy, a loop of bf16 matrix-core instructions on register operands, and the
// cost of an empty launch.  Measurement only; nothing of the method is computed here.
#include "common.h"
#include "mfma.h"

namespace mvla {

constexpr int PROBE_THREADS = 256;

// grid-stride read of n 16-byte words; the xor of everything read is stored only if it has a
// value it cannot have (keeps the loads alive without a store stream)
__global__ __launch_bounds__(PROBE_THREADS) void probe_read_kernel(const uint4* __restrict__ src,
                                                                   size_t n, uint32_t* sink) {
    const size_t stride = (size_t)gridDim.x * PROBE_THREADS;
    size_t i = (size_t)blockIdx.x * PROBE_THREADS + threadIdx.x;
    uint32_t acc = 0;
    for (; i + 3 * stride < n; i += 4 * stride) {
        const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^
               d.z ^ d.w;
    }
    for (; i < n; i += stride) {
        const uint4 a = src[i];
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    if (acc == 0x9e3779b9u && sink) *sink = acc;
}

__global__ __launch_bounds__(PROBE_THREADS) void probe_copy_kernel(const uint4* __restrict__ src,
                                                                   uint4* __restrict__ dst, size_t n) {
    const size_t stride = (size_t)gridDim.x * PROBE_THREADS;
    size_t i = (size_t)blockIdx.x * PROBE_THREADS + threadIdx.x;
    for (; i + 3 * stride < n; i += 4 * stride) {
        const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        dst[i] = a;
        dst[i + stride] = b;
        dst[i + 2 * stride] = c;
        dst[i + 3 * stride] = d;
    }
    for (; i < n; i += stride) dst[i] = src[i];
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
    hipLaunchKernelGGL(probe_read_kernel, dim3(256 * 16), dim3(PROBE_THREADS), 0, st,
                       static_cast<const uint4*>(src), bytes / 16, sink);
    MVLA_HIP_CHECK(hipGetLastError());
    return MVLA_OK;
}
int launch_probe_copy(const void* src, void* dst, size_t bytes, hipStream_t st) {
    hipLaunchKernelGGL(probe_copy_kernel, dim3(256 * 16), dim3(PROBE_THREADS), 0, st,
                       static_cast<const uint4*>(src), static_cast<uint4*>(dst), bytes / 16);
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
