// Layout helpers: tiled transpose through LDS, fp32 -> storage-type cast.
#pragma once
#include "flce_device.h"

namespace flce {

// out[c][r] = in[r][c] for r < R, c < Cc.  64 x 64 tile, 256 threads.
template <typename T>
__global__ __launch_bounds__(256) void transpose_kernel(const T* __restrict__ in, int64_t ldin,
                                                        T* __restrict__ out, int64_t ldout, int R,
                                                        int Cc) {
    __shared__ T tile[64][64 + 2];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
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

// out[r][c] = sum_s part[s][r][c] in the fixed order s = 0, 1, ...: the reduction
// of split-K partial results (row stride ld for both).
// With ADD the previous content of out is added as well (dX summed over heads).
template <typename T, bool ADD>
__global__ void splitk_reduce_kernel(const float* __restrict__ part, int64_t split_stride, int nsplit,
                                     T* __restrict__ out, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x) {
        float v = part[i];
        if constexpr (ADD) v += to_f32(out[i]);
        for (int s = 1; s < nsplit; ++s) v += part[(int64_t)s * split_stride + i];
        out[i] = from_f32<T>(v);
    }
}

template <typename T>
__global__ void cast_from_f32_kernel(const float* __restrict__ in, T* __restrict__ out, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x)
        out[i] = from_f32<T>(in[i]);
}

}  // namespace flce
