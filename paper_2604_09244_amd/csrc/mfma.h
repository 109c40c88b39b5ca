// gfx950 matrix-core helpers: operand types and LDS tile addressing.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// v_mfma_f32_32x32x16_bf16: D[32x32] += A[32x16] * B[16x32].
//   A operand: lane l holds row (l % 32), k = 8*(l/32) .. 8*(l/32)+7
//   B operand: lane l holds col (l % 32), k = 8*(l/32) .. 8*(l/32)+7
//   D: lane l holds col (l % 32); register v holds row 8*(v/4) + 4*(l/32) + (v%4)
__device__ __forceinline__ f32x16_t mfma32(const uint4& a, const uint4& b, f32x16_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

__device__ __forceinline__ int mfma32_row(int v, int lane) {
    return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
}

__device__ __forceinline__ float bf16_to_f32(uint16_t h) {
    return __uint_as_float((uint32_t)h << 16);
}
// fp32 -> bf16, round-to-nearest-even, through the gfx950 pack-convert instruction
// (v_cvt_pk_bf16_f32)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ uint16_t f32_to_bf16(float f) { return (uint16_t)pack_bf16x2(f, 0.f); }

// LDS tiles hold rows of 64 bf16 (128 bytes = eight 16-byte chunks).  Chunk c
// of row r lives at slot r*8 + (c ^ (r & 7)), which spreads the 32 rows a
// fragment load touches over all banks.
__device__ __forceinline__ int lds_slot(int row, int chunk) {
    return row * 8 + (chunk ^ (row & 7));
}
