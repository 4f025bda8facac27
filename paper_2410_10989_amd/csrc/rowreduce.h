// Row-wise softmax cross entropy with the gradient written over the logits
// (paper section 3.2, CE paragraph: online softmax, in-place dlogits).
//
// One workgroup per row.  Sweep 1 keeps a running (max, sum of exp) pair per
// thread and merges the pairs across the wavefront and the workgroup; the loss
// of the row is lse - z[target] ("safe log": log is only taken of a sum that is
// at least 1).  Sweep 2 rewrites the row as (exp(z - lse) - onehot) / N, or as
// zeros for an ignored row.  N arrives through the device header as 1/N.
#pragma once
#include "flce_device.h"

namespace flce {

constexpr int RR_THREADS = 256;

struct MaxSum {
    float m, s;
};
__device__ __forceinline__ MaxSum ms_merge(MaxSum a, MaxSum b) {
    const float m = fmaxf(a.m, b.m);
    // exp(-inf - finite) = 0 handles empty partners; both -inf cannot occur for
    // the partner that holds at least one element, guard it anyway
    const float sa = (a.m == -INFINITY) ? 0.f : a.s * __expf(a.m - m);
    const float sb = (b.m == -INFINITY) ? 0.f : b.s * __expf(b.m - m);
    return {m, sa + sb};
}
__device__ __forceinline__ void ms_push(MaxSum& a, float x) {
    if (x > a.m) {
        a.s = a.s * __expf(a.m - x) + 1.f;   // a.m = -inf gives 0 * 0 + 1
        a.m = x;
    } else {
        a.s += __expf(x - a.m);
    }
}

template <typename T, bool VEC16>
__global__ __launch_bounds__(RR_THREADS) void ce_rows_inplace_kernel(
    T* __restrict__ Z, int64_t ldz, const int64_t* __restrict__ targets, int V,
    int64_t ignore_index, const DeviceHeader* __restrict__ hdr, float* __restrict__ row_loss) {
    constexpr int VEC = 16 / sizeof(T);
    const int row = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    T* z = Z + (int64_t)row * ldz;
    const int64_t t = targets[row];
    const bool valid = (t != ignore_index);

    __shared__ MaxSum part[RR_THREADS / WAVE];
    __shared__ float s_lse;

    const int nvec = VEC16 ? V / VEC : 0;
    float lse = 0.f;
    if (valid) {
        MaxSum a = {-INFINITY, 0.f};
        if constexpr (VEC16) {
            for (int i = tid; i < nvec; i += RR_THREADS) {
                u32x4 raw = reinterpret_cast<const u32x4*>(z)[i];
                const T* e = reinterpret_cast<const T*>(&raw);
#pragma unroll
                for (int j = 0; j < VEC; ++j) ms_push(a, to_f32(e[j]));
            }
        }
        for (int v = nvec * VEC + tid; v < V; v += RR_THREADS) ms_push(a, to_f32(z[v]));
#pragma unroll
        for (int o = WAVE / 2; o > 0; o >>= 1) {
            MaxSum b = {__shfl_xor(a.m, o, WAVE), __shfl_xor(a.s, o, WAVE)};
            a = ms_merge(a, b);
        }
        if (lane == 0) part[wave] = a;
        __syncthreads();
        if (tid == 0) {
            MaxSum r = part[0];
            for (int w = 1; w < RR_THREADS / WAVE; ++w) r = ms_merge(r, part[w]);
            const float l = r.m + logf(r.s);
            s_lse = l;
            row_loss[row] = l - to_f32(z[t]);
        }
        __syncthreads();   // z[target] is read before anybody overwrites the row
        lse = s_lse;
    } else if (tid == 0) {
        row_loss[row] = 0.f;
    }

    const float inv_n = hdr->inv_n;
    const int tcol = valid ? (int)t : -1;
    if constexpr (VEC16) {
        for (int i = tid; i < nvec; i += RR_THREADS) {
            u32x4 raw = {0u, 0u, 0u, 0u};
            if (valid) {
                raw = reinterpret_cast<const u32x4*>(z)[i];
                T* e = reinterpret_cast<T*>(&raw);
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    float g = __expf(to_f32(e[j]) - lse) * inv_n;
                    if (i * VEC + j == tcol) g -= inv_n;
                    e[j] = from_f32<T>(g);
                }
            }
            reinterpret_cast<u32x4*>(z)[i] = raw;
        }
    }
    for (int v = nvec * VEC + tid; v < V; v += RR_THREADS) {
        float g = 0.f;
        if (valid) {
            g = __expf(to_f32(z[v]) - lse) * inv_n;
            if (v == tcol) g -= inv_n;
        }
        z[v] = from_f32<T>(g);
    }
}

// Variant for long rows: one workgroup of 1024 threads per row keeps the first
// 1024 * RC_NV 16-byte vectors of the row (128 K bf16 logits) in registers between
// the two sweeps, so that part of the row is read from HBM once instead of twice;
// what is beyond is swept twice as above.  All of a thread's loads are issued
// before the first is consumed.  16 wavefronts per CU keep the per-thread ALU phases
// short (a variant with 4 wavefronts per CU and the whole row cached was slower
// than two sweeps).  Used for rows of 128-256 KB, where it measures 6-12 % faster.
constexpr int RC_THREADS = 1024;
constexpr int RC_NV = 16;

template <typename T>
__global__ __launch_bounds__(RC_THREADS) void ce_rows_cached_kernel(
    T* __restrict__ Z, int64_t ldz, const int64_t* __restrict__ targets, int V,
    int64_t ignore_index, const DeviceHeader* __restrict__ hdr, float* __restrict__ row_loss) {
    constexpr int VEC = 16 / sizeof(T);
    const int row = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    T* z = Z + (int64_t)row * ldz;
    const int64_t t = targets[row];
    const bool valid = (t != ignore_index);
    const int nvec = V / VEC;                 // full vectors; the tail is handled by scalars
    u32x4* zv = reinterpret_cast<u32x4*>(z);

    __shared__ MaxSum part[RC_THREADS / WAVE];
    __shared__ float s_lse;

    if (!valid) {                              // uniform per workgroup
        const u32x4 zero = {0u, 0u, 0u, 0u};
        for (int i = tid; i < nvec; i += RC_THREADS) zv[i] = zero;
        for (int v = nvec * VEC + tid; v < V; v += RC_THREADS) z[v] = from_f32<T>(0.f);
        if (tid == 0) row_loss[row] = 0.f;
        return;
    }

    u32x4 keep[RC_NV];
#pragma unroll
    for (int k = 0; k < RC_NV; ++k) {
        const int i = tid + k * RC_THREADS;
        if (i < nvec) keep[k] = zv[i];
    }
    MaxSum a = {-INFINITY, 0.f};
#pragma unroll
    for (int k = 0; k < RC_NV; ++k) {
        const int i = tid + k * RC_THREADS;
        if (i < nvec) {
            const T* e = reinterpret_cast<const T*>(&keep[k]);
#pragma unroll
            for (int j = 0; j < VEC; ++j) ms_push(a, to_f32(e[j]));
        }
    }
    for (int i = tid + RC_NV * RC_THREADS; i < nvec; i += RC_THREADS) {   // beyond the cache
        u32x4 raw = zv[i];
        const T* e = reinterpret_cast<const T*>(&raw);
#pragma unroll
        for (int j = 0; j < VEC; ++j) ms_push(a, to_f32(e[j]));
    }
    for (int v = nvec * VEC + tid; v < V; v += RC_THREADS) ms_push(a, to_f32(z[v]));
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) {
        MaxSum b = {__shfl_xor(a.m, o, WAVE), __shfl_xor(a.s, o, WAVE)};
        a = ms_merge(a, b);
    }
    if (lane == 0) part[wave] = a;
    __syncthreads();
    if (tid == 0) {
        MaxSum r = part[0];
        for (int w = 1; w < RC_THREADS / WAVE; ++w) r = ms_merge(r, part[w]);
        const float l = r.m + logf(r.s);
        s_lse = l;
        row_loss[row] = l - to_f32(z[t]);
    }
    __syncthreads();   // z[target] is read before anybody overwrites the row
    const float lse = s_lse;
    const float inv_n = hdr->inv_n;
    const int tcol = (int)t;
    auto rewrite = [&](u32x4 raw, int i) {
        T* e = reinterpret_cast<T*>(&raw);
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
            float g = __expf(to_f32(e[j]) - lse) * inv_n;
            if (i * VEC + j == tcol) g -= inv_n;
            e[j] = from_f32<T>(g);
        }
        zv[i] = raw;
    };
#pragma unroll
    for (int k = 0; k < RC_NV; ++k) {
        const int i = tid + k * RC_THREADS;
        if (i < nvec) rewrite(keep[k], i);
    }
    for (int i = tid + RC_NV * RC_THREADS; i < nvec; i += RC_THREADS) rewrite(zv[i], i);
    for (int v = nvec * VEC + tid; v < V; v += RC_THREADS) {
        float g = __expf(to_f32(z[v]) - lse) * inv_n;
        if (v == tcol) g -= inv_n;
        z[v] = from_f32<T>(g);
    }
}

// Adds the per-row losses of one launch to the running sum, in a fixed order
// (one workgroup, fixed strides), so repeated runs give the same bits.
__global__ __launch_bounds__(256) void loss_accumulate_kernel(const float* __restrict__ row_loss,
                                                              int rows, DeviceHeader* hdr) {
    __shared__ double part[4];
    double s = 0.0;
    for (int i = threadIdx.x; i < rows; i += 256) s += (double)row_loss[i];
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) hdr->loss_sum += (part[0] + part[1]) + (part[2] + part[3]);
}

// Counts the valid rows and resets the running loss.  Integer sum: exact in any order.
// `weight` scales every gradient of this head (1 for a single head).
__global__ __launch_bounds__(1024) void count_valid_kernel(const int64_t* __restrict__ targets,
                                                           int64_t BT, int64_t ignore_index,
                                                           float weight, DeviceHeader* hdr) {
    __shared__ int part[16];
    int c = 0;
    for (int64_t i = threadIdx.x; i < BT; i += 1024) c += (targets[i] != ignore_index);
    c = wave_sum(c);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) {
        int n = 0;
        for (int w = 0; w < 16; ++w) n += part[w];
        hdr->n_valid = n;
        hdr->inv_n = n > 0 ? weight / (float)n : 0.f;
        hdr->loss_sum = 0.0;
    }
}

// loss = sum over heads of weight_j * (mean loss of head j); head_losses (optional)
// receives the unweighted means.  One header per head; WeightsT is a struct of
// floats w[] passed by value.
template <typename WeightsT>
__global__ void finalize_loss_kernel(const DeviceHeader* hdr, int n_heads, WeightsT weights,
                                     float* loss, float* __restrict__ head_losses) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        double total = 0.0;
        for (int j = 0; j < n_heads; ++j) {
            const double mean =
                hdr[j].n_valid > 0 ? hdr[j].loss_sum / (double)hdr[j].n_valid : 0.0;
            if (head_losses) head_losses[j] = (float)mean;
            total += (double)weights.w[j] * mean;
        }
        *loss = (float)total;
    }
}

}  // namespace flce
