// Layout helpers: tiled transpose through LDS, fp32 -> storage-type cast.
#pragma once
#include "flce_device.h"

namespace flce {

// out[c][r] = in[r][c] for r < R, c < Cc.  64 x 64 tile, 256 threads; tiles are numbered
// along grid x, row of tiles by row of tiles.
template <typename T>
__global__ __launch_bounds__(256) void transpose_kernel(const T* __restrict__ in, int64_t ldin,
                                                        T* __restrict__ out, int64_t ldout, int R,
                                                        int Cc) {
    __shared__ T tile[64][64 + 2];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int tiles_c = (Cc + 63) / 64;
    const int r0 = (int)(blockIdx.x / tiles_c) * 64, c0 = (int)(blockIdx.x % tiles_c) * 64;
#pragma unroll 4
    for (int i = ty; i < 64; i += 4) {
        const int r = r0 + i, c = c0 + tx;
        if (r < R && c < Cc) tile[i][tx] = in[(int64_t)r * ldin + c];
    }
    __syncthreads();
#pragma unroll 4
    for (int i = ty; i < 64; i += 4) {
        const int c = c0 + i, r = r0 + tx;
        if (r < R && c < Cc) out[(int64_t)c * ldout + r] = tile[tx][i];
    }
}

// out[i] = sum_s part[s][i] in the fixed order s = 0, 1, ...: the reduction of split-K
// partial results (n elements each, split_stride elements apart).
// With ADD the previous content of out is added as well (dX summed over heads).
// VEC4: four elements per thread and access (n, split_stride and the pointers' element
// offsets are multiples of 4); the additions per element are the same either way.
// dyn_nsplit (optional): the number of ranges when only the device knows it.
template <typename T, bool ADD, bool VEC4>
__global__ void splitk_reduce_kernel(const float* __restrict__ part, int64_t split_stride, int nsplit,
                                     T* __restrict__ out, int64_t n, const int* __restrict__ dyn_nsplit) {
    if (dyn_nsplit) nsplit = *dyn_nsplit;
    if constexpr (VEC4) {
        typedef float f32x4v __attribute__((ext_vector_type(4)));
        for (int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4; i < n;
             i += (int64_t)gridDim.x * blockDim.x * 4) {
            f32x4v v = *reinterpret_cast<const f32x4v*>(part + i);
            if constexpr (ADD) {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] += to_f32(out[i + e]);
            }
            for (int s = 1; s < nsplit; ++s) v += *reinterpret_cast<const f32x4v*>(part + (int64_t)s * split_stride + i);
            if constexpr (sizeof(T) == 4) {
                *reinterpret_cast<f32x4v*>(out + i) = v;
            } else {
                typedef uint32_t u32x2v __attribute__((ext_vector_type(2)));
                const bf16x2 p0 = {from_f32<bf16_t>(v[0]), from_f32<bf16_t>(v[1])};
                const bf16x2 p1 = {from_f32<bf16_t>(v[2]), from_f32<bf16_t>(v[3])};
                const u32x2v q = {__builtin_bit_cast(uint32_t, p0), __builtin_bit_cast(uint32_t, p1)};
                *reinterpret_cast<u32x2v*>(out + i) = q;
            }
        }
    } else {
        for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
             i += (int64_t)gridDim.x * blockDim.x) {
            float v = part[i];
            if constexpr (ADD) v += to_f32(out[i]);
            for (int s = 1; s < nsplit; ++s) v += part[(int64_t)s * split_stride + i];
            out[i] = from_f32<T>(v);
        }
    }
}

template <typename T>
__global__ void cast_from_f32_kernel(const float* __restrict__ in, T* __restrict__ out, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x)
        out[i] = from_f32<T>(in[i]);
}

}  // namespace flce
