// RMSNorm in front of the output projection (paper section 3.2, RMSNorm
// paragraph, Eq. RMSNorm-forward / RMSNorm-backward), row by row:
//
//     rms = sqrt(sum_j x_j^2 / n + eps),  xhat = x / rms,  y = xhat * gamma
//     dx     = (1/rms) * (dy*gamma - [xhat . (dy*gamma) / n] * xhat)
//     dgamma = sum over rows of dy * xhat
//
// All arithmetic in fp32 on values widened from the storage type; y and dx are
// rounded once when stored.  dgamma is summed without atomics: the backward
// kernel runs RN_SLOTS workgroups, workgroup p owns rows p, p + RN_SLOTS, ... and
// row p of an fp32 partial buffer [RN_SLOTS x n]; a second kernel adds the
// partial rows in fixed order.  The kernels are bandwidth bound and touch
// O(rows * n) bytes, which is negligible next to the three products.
//
// Two forms of each kernel: the vector form (rows of up to 4 * 256 16-byte vectors,
// 16-byte aligned) keeps a row in registers, reads it once with 16-byte accesses and
// keeps a workgroup's dgamma sums in registers over all its rows; the scalar form
// takes any row length.
#pragma once
#include "flce_device.h"
#include "rowreduce.h"

namespace flce {

constexpr int RN_THREADS = 256;
constexpr int RN_SLOTS = 512;

// Sum over the 256 threads of a workgroup, the same value returned to every thread.
__device__ __forceinline__ float rn_block_sum(float v, float* red) {
    v = wave_sum(v);
    __syncthreads();   // red may still be read from a previous call
    if ((threadIdx.x & (WAVE - 1)) == 0) red[threadIdx.x / WAVE] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

// One workgroup per output row: y = x / rms(x) * gamma, rstd[row] = 1 / rms(x).
// With idx / live (a compacted chunk) output row i reads input row idx[i], and
// workgroups past the chunk's *live rows return.
template <typename T>
__global__ __launch_bounds__(RN_THREADS) void rmsnorm_fwd_kernel(const T* __restrict__ x,
                                                                 const T* __restrict__ gamma,
                                                                 float eps, int n,
                                                                 T* __restrict__ y,
                                                                 float* __restrict__ rstd,
                                                                 const int* __restrict__ idx,
                                                                 const int* __restrict__ live) {
    __shared__ float red[RN_THREADS / WAVE];
    if (live && (int)blockIdx.x >= *live) return;
    const int64_t base = (int64_t)(idx ? idx[blockIdx.x] : (int)blockIdx.x) * n;
    const int64_t obase = (int64_t)blockIdx.x * n;
    float ss = 0.f;
    for (int j = threadIdx.x; j < n; j += RN_THREADS) {
        const float v = to_f32(x[base + j]);
        ss += v * v;
    }
    ss = rn_block_sum(ss, red);
    const float r = 1.0f / sqrtf(ss / (float)n + eps);
    if (threadIdx.x == 0) rstd[blockIdx.x] = r;
    for (int j = threadIdx.x; j < n; j += RN_THREADS)
        y[obase + j] = from_f32<T>(to_f32(x[base + j]) * r * to_f32(gamma[j]));
}

// Workgroup p: rows p, p + RN_SLOTS, ... of this chunk.  dx is written; the
// workgroup's own row of `partial` accumulates dy * xhat (column j always by the
// same thread, so there is no race and the order of additions is fixed).
// With idx / live (a compacted chunk) dy and rstd are indexed by the chunk's row i, x and
// dx by row idx[i], and only *live rows exist.
template <typename T>
__global__ __launch_bounds__(RN_THREADS) void rmsnorm_bwd_kernel(
    const T* __restrict__ x, const T* __restrict__ gamma, const float* __restrict__ rstd,
    const T* __restrict__ dy, int rows, int n, T* __restrict__ dx, float* __restrict__ partial,
    const int* __restrict__ idx, const int* __restrict__ live) {
    __shared__ float red[RN_THREADS / WAVE];
    float* mine = partial + (int64_t)blockIdx.x * n;
    if (live) rows = min(rows, *live);
    for (int row = blockIdx.x; row < rows; row += RN_SLOTS) {
        const int64_t base = (int64_t)(idx ? idx[row] : row) * n;
        const int64_t cbase = (int64_t)row * n;
        const float r = rstd[row];
        float dot = 0.f;
        for (int j = threadIdx.x; j < n; j += RN_THREADS)
            dot += (to_f32(x[base + j]) * r) * (to_f32(dy[cbase + j]) * to_f32(gamma[j]));
        dot = rn_block_sum(dot, red) / (float)n;
        for (int j = threadIdx.x; j < n; j += RN_THREADS) {
            const float xh = to_f32(x[base + j]) * r;
            const float d = to_f32(dy[cbase + j]);
            dx[base + j] = from_f32<T>(r * (d * to_f32(gamma[j]) - dot * xh));
            mine[j] += d * xh;
        }
    }
}

// Vector form of rmsnorm_fwd_kernel: n is a multiple of the vector width, thread t holds
// vectors t, t + 256, ... (NV of them: n <= NV * 256 vectors).
template <typename T, int NV>
__global__ __launch_bounds__(RN_THREADS) void rmsnorm_fwd_vec_kernel(
    const T* __restrict__ x, const T* __restrict__ gamma, float eps, int n, T* __restrict__ y,
    float* __restrict__ rstd, const int* __restrict__ idx, const int* __restrict__ live) {
    constexpr int N = RowVec<T>::N;
    __shared__ float red[RN_THREADS / WAVE];
    if (live && (int)blockIdx.x >= *live) return;
    const int nvec = n / N;
    const u32x4* xr = reinterpret_cast<const u32x4*>(x + (int64_t)(idx ? idx[blockIdx.x] : (int)blockIdx.x) * n);
    u32x4* yr = reinterpret_cast<u32x4*>(y + (int64_t)blockIdx.x * n);
    const u32x4* gr = reinterpret_cast<const u32x4*>(gamma);
    float xv[NV][N];
    float ss = 0.f;
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        const int v = threadIdx.x + k * RN_THREADS;
        if (v < nvec) {
            RowVec<T>::unpack(xr[v], xv[k]);
#pragma unroll
            for (int e = 0; e < N; ++e) ss += xv[k][e] * xv[k][e];
        }
    }
    ss = rn_block_sum(ss, red);
    const float r = 1.0f / sqrtf(ss / (float)n + eps);
    if (threadIdx.x == 0) rstd[blockIdx.x] = r;
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        const int v = threadIdx.x + k * RN_THREADS;
        if (v < nvec) {
            float g[N], o[N];
            RowVec<T>::unpack(gr[v], g);
#pragma unroll
            for (int e = 0; e < N; ++e) o[e] = xv[k][e] * r * g[e];
            yr[v] = RowVec<T>::pack(o);
        }
    }
}

// Vector form of rmsnorm_bwd_kernel (same layout as the forward form): gamma and the
// workgroup's dgamma sums stay in registers over all its rows; the sums are added to
// the workgroup's partial row once, at the end.
template <typename T, int NV>
__global__ __launch_bounds__(RN_THREADS) void rmsnorm_bwd_vec_kernel(
    const T* __restrict__ x, const T* __restrict__ gamma, const float* __restrict__ rstd,
    const T* __restrict__ dy, int rows, int n, T* __restrict__ dx, float* __restrict__ partial,
    const int* __restrict__ idx, const int* __restrict__ live) {
    constexpr int N = RowVec<T>::N;
    __shared__ float red[RN_THREADS / WAVE];
    const int nvec = n / N;
    const u32x4* gr = reinterpret_cast<const u32x4*>(gamma);
    float gv[NV][N], acc[NV][N];
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        const int v = threadIdx.x + k * RN_THREADS;
#pragma unroll
        for (int e = 0; e < N; ++e) {
            gv[k][e] = 0.f;
            acc[k][e] = 0.f;
        }
        if (v < nvec) RowVec<T>::unpack(gr[v], gv[k]);
    }
    if (live) rows = min(rows, *live);
    for (int row = blockIdx.x; row < rows; row += RN_SLOTS) {
        const int64_t base = (int64_t)(idx ? idx[row] : row) * n;
        const u32x4* xr = reinterpret_cast<const u32x4*>(x + base);
        const u32x4* dr = reinterpret_cast<const u32x4*>(dy + (int64_t)row * n);
        u32x4* outr = reinterpret_cast<u32x4*>(dx + base);
        const float r = rstd[row];
        float xh[NV][N], d[NV][N];
        float dot = 0.f;
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            const int v = threadIdx.x + k * RN_THREADS;
            if (v < nvec) {
                RowVec<T>::unpack(xr[v], xh[k]);
                RowVec<T>::unpack(dr[v], d[k]);
#pragma unroll
                for (int e = 0; e < N; ++e) {
                    xh[k][e] *= r;
                    dot += xh[k][e] * (d[k][e] * gv[k][e]);
                }
            }
        }
        dot = rn_block_sum(dot, red) / (float)n;
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            const int v = threadIdx.x + k * RN_THREADS;
            if (v < nvec) {
                float o[N];
#pragma unroll
                for (int e = 0; e < N; ++e) {
                    o[e] = r * (d[k][e] * gv[k][e] - dot * xh[k][e]);
                    acc[k][e] += d[k][e] * xh[k][e];
                }
                outr[v] = RowVec<T>::pack(o);
            }
        }
    }
    float* mine = partial + (int64_t)blockIdx.x * n;
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        const int v = threadIdx.x + k * RN_THREADS;
        if (v < nvec) {
#pragma unroll
            for (int e = 0; e < N; ++e) mine[v * N + e] += acc[k][e];
        }
    }
}

__global__ void fill_zero_kernel(float* __restrict__ p, int64_t count) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count;
         i += (int64_t)gridDim.x * blockDim.x)
        p[i] = 0.f;
}

// dgamma[j] = sum_p partial[p][j].  A workgroup of 64 x 4 threads owns 64 columns: thread
// (c, q) adds rows q, q + 4, ... of column c in order, then the four sums are added in
// the order q = 0, 1, 2, 3: a fixed order, and 4 n / 256 workgroups instead of n / 256.
constexpr int RN_DG_COLS = 64, RN_DG_PARTS = 4;
template <typename T>
__global__ __launch_bounds__(RN_DG_COLS * RN_DG_PARTS) void rmsnorm_dgamma_kernel(
    const float* __restrict__ partial, int n, T* __restrict__ dgamma) {
    __shared__ float sums[RN_DG_PARTS][RN_DG_COLS];
    const int c = threadIdx.x % RN_DG_COLS, q = threadIdx.x / RN_DG_COLS;
    const int j = blockIdx.x * RN_DG_COLS + c;
    float s = 0.f;
    if (j < n)
        for (int p = q; p < RN_SLOTS; p += RN_DG_PARTS) s += partial[(int64_t)p * n + j];
    sums[q][c] = s;
    __syncthreads();
    if (q == 0 && j < n) dgamma[j] = from_f32<T>(((sums[0][c] + sums[1][c]) + sums[2][c]) + sums[3][c]);
}

}  // namespace flce
