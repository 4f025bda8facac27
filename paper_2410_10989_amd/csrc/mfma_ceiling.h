// Measurement aid, not part of the path: a loop of v_mfma_f32_32x32x16_bf16 and nothing
// else (no global memory, no LDS), one wavefront per SIMD with 16 accumulator tiles like
// the product kernel.  What the matrix pipes sustain depends on how many operand bits
// toggle from one MFMA to the next (the chip lowers its clock under that load), so the
// loop can be run on zeros, on one fixed pair of fragments, or on 4 A x 4 B fragments of
// normal deviates in the order of one K sub-step of the product kernel; the last is the
// ceiling a product of such data can reach, whatever feeds it.
#pragma once
#include "flce_device.h"

namespace flce {

__device__ __forceinline__ uint32_t mc_hash(uint32_t x) {
    x ^= x >> 16;
    x *= 0x7feb352du;
    x ^= x >> 15;
    x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

// pattern 0: zero operands, 1: one A and one B fragment for all MFMAs, 2: 4 A x 4 B.
// A ~ N(0, 1), B ~ N(0, std_b^2), rounded to bf16.  out: gridDim.x * 256 floats.
template <int PATTERN>
__global__ __launch_bounds__(256) void mfma_ceiling_kernel(float* __restrict__ out, int iters,
                                                           float std_b) {
    bf16x8 a[4], b[4];
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t h = mc_hash(threadIdx.x * 977u + blockIdx.x * 131071u + s * 64u + i);
            const float u1 = ((h & 0xffffu) + 1) * (1.0f / 65537.0f), u2 = (h >> 16) * (1.0f / 65536.0f);
            const float r = __builtin_sqrtf(-2.0f * __builtin_logf(u1));
            a[s][i] = from_f32<bf16_t>(PATTERN == 0 ? 0.0f : r * __builtin_cosf(6.2831853f * u2));
            b[s][i] = from_f32<bf16_t>(PATTERN == 0 ? 0.0f : r * __builtin_sinf(6.2831853f * u2) * std_b);
        }
    f32x16 acc[16];
#pragma unroll
    for (int n = 0; n < 16; ++n)
#pragma unroll
        for (int g = 0; g < 16; ++g) acc[n][g] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int n = 0; n < 16; ++n) {
            constexpr bool MANY = PATTERN == 2;
            acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[MANY ? (n & 3) : 0], a[MANY ? (n >> 2) : 0],
                                                             acc[n], 0, 0, 0);
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) asm volatile("" : "+v"(a[s]), "+v"(b[s]));   // keep the loop as written
    }
    float sum = 0.0f;
#pragma unroll
    for (int n = 0; n < 16; ++n)
#pragma unroll
        for (int g = 0; g < 16; ++g) sum += acc[n][g];
    out[blockIdx.x * 256 + threadIdx.x] = sum;
}

}  // namespace flce
