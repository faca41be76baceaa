// Shared device helpers for the gfx950 SVD-Attention kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace solar {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

__host__ __device__ inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// bf16 bit pattern -> float (exact).
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// D = A(16x4) * B(4x16) + C in float.  Lane l supplies A[l%16][l/16] and
// B[l/16][l%16]; it receives D[4*(l/16)+t][l%16] in component t.
__device__ __forceinline__ v4f mfma16x16x4(float a, float b, v4f c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// D = A(16x32) * B(32x16) + C, bf16 inputs, float accumulate.  Lane l supplies
// eight consecutive k-slots of row l%16 of A and of column l%16 of B (slot group
// l/16); D is laid out as for mfma16x16x4.
__device__ __forceinline__ v4f mfma16x16x32bf16(v4u a, v4u b, v4f c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, a),
                                                   __builtin_bit_cast(v8bf, b), c, 0, 0, 0);
}

__device__ __forceinline__ float wave_xor_max(float v, int mask) {
    return fmaxf(v, __shfl_xor(v, mask));
}

// Valid length of user b clamped to [0, N].
__device__ __forceinline__ int user_len(const int32_t* lengths, int b, int N) {
    int len = lengths ? lengths[b] : N;
    return len < 0 ? 0 : (len > N ? N : len);
}

}  // namespace solar
