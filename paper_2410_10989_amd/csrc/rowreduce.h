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
    float m, s;   // running maximum and sum of exp(z - m)
};
__device__ __forceinline__ MaxSum ms_merge(MaxSum a, MaxSum b) {
    const float m = fmaxf(a.m, b.m);
    // exp(-inf - finite) = 0 handles empty partners; both -inf cannot occur for
    // the partner that holds at least one element, guard it anyway
    const float sa = (a.m == -INFINITY) ? 0.f : a.s * __expf(a.m - m);
    const float sb = (b.m == -INFINITY) ? 0.f : b.s * __expf(b.m - m);
    return {m, sa + sb};
}

// The arithmetic per logit decides the speed of these kernels as much as the memory
// traffic does (a CU retires 64 plain and 16 transcendental lane operations per
// cycle), so both sweeps work on whole 16-byte vectors and exponentials are taken as
// exp2(fma(z, log2 e, c)): one multiply-add and one v_exp_f32 per logit.
constexpr float RR_LOG2E = 1.4426950408889634f;

template <typename T> struct RowVec;
template <> struct RowVec<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void unpack(const u32x4& raw, float (&f)[4]) {
#pragma unroll
        for (int w = 0; w < 4; ++w) f[w] = __uint_as_float(raw[w]);
    }
    static __device__ __forceinline__ u32x4 pack(const float (&f)[4]) {
        u32x4 r;
#pragma unroll
        for (int w = 0; w < 4; ++w) r[w] = __float_as_uint(f[w]);
        return r;
    }
};
template <> struct RowVec<bf16_t> {
    static constexpr int N = 8;
    // a bf16 is the upper half of the float with the same value
    static __device__ __forceinline__ void unpack(const u32x4& raw, float (&f)[8]) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            f[2 * w] = __uint_as_float(raw[w] << 16);
            f[2 * w + 1] = __uint_as_float(raw[w] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ u32x4 pack(const float (&f)[8]) {
        u32x4 r;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const bf16x2 p = {(bf16_t)f[2 * w], (bf16_t)f[2 * w + 1]};   // round to nearest even
            r[w] = __builtin_bit_cast(uint32_t, p);
        }
        return r;
    }
};

// exp(z - ref).  bf16 logits: exp2(fma(z, log2 e, -ref log2 e)), the rounding of the
// constant (half an ulp of |ref| log2 e) is far below what bf16 resolves.  fp32
// logits: the difference is taken first, which stays exact for large |z|.
template <typename T> struct RowExp;
template <> struct RowExp<bf16_t> {
    float c;
    __device__ __forceinline__ explicit RowExp(float ref) : c(-ref * RR_LOG2E) {}
    __device__ __forceinline__ float operator()(float z) const {
        return __builtin_amdgcn_exp2f(fmaf(z, RR_LOG2E, c));
    }
};
template <> struct RowExp<float> {
    float ref;
    __device__ __forceinline__ explicit RowExp(float r) : ref(r) {}
    __device__ __forceinline__ float operator()(float z) const {
        return __builtin_amdgcn_exp2f((z - ref) * RR_LOG2E);
    }
};

// Online softmax update with N logits at once: one rescale of the running sum per
// vector instead of one decision per logit.
template <typename T, int N>
__device__ __forceinline__ void ms_push_vec(MaxSum& a, const float (&f)[N]) {
    float vm = f[0];
#pragma unroll
    for (int j = 1; j < N; ++j) vm = fmaxf(vm, f[j]);
    const float m_new = fmaxf(a.m, vm);
    // a row may start with -inf logits: keep the reference finite
    const RowExp<T> ex((m_new == -INFINITY) ? 0.f : m_new);
    float s = a.s * ex(a.m);   // a.m = -inf: s was 0 and stays 0
#pragma unroll
    for (int j = 0; j < N; ++j) s += ex(f[j]);
    a.m = m_new;
    a.s = s;
}
template <typename T>
__device__ __forceinline__ void ms_push(MaxSum& a, float x) {
    const float f[1] = {x};
    ms_push_vec<T, 1>(a, f);
}

// (softmax - onehot) / N of one vector: exp(z - lse) * inv_n; the one-hot term only
// touches the vector that holds the target column.
template <typename T>
__device__ __forceinline__ u32x4 ce_gradient_vec(const u32x4& raw, int i, int tcol,
                                                 const RowExp<T>& ex, float inv_n) {
    constexpr int N = RowVec<T>::N;
    float f[N];
    RowVec<T>::unpack(raw, f);
#pragma unroll
    for (int j = 0; j < N; ++j) f[j] = ex(f[j]) * inv_n;
    if (i == tcol / N) {
#pragma unroll
        for (int j = 0; j < N; ++j)
            if (j == tcol % N) f[j] -= inv_n;
    }
    return RowVec<T>::pack(f);
}
template <typename T>
__device__ __forceinline__ T ce_gradient_one(T z, int v, int tcol, const RowExp<T>& ex, float inv_n) {
    float g = ex(to_f32(z)) * inv_n;
    if (v == tcol) g -= inv_n;
    return from_f32<T>(g);
}

// Merges the per-thread pairs of a workgroup of NW wavefronts; thread 0 then holds
// the row's log-sum-exp, publishes it and the row's loss.  Ends with a barrier, so
// z[target] has been read before any thread overwrites the row.
template <typename T, int NW>
__device__ __forceinline__ float row_lse(MaxSum a, const T* z, int64_t t, int row,
                                         float* __restrict__ row_loss, MaxSum* part, float* s_lse) {
    const int lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x / WAVE;
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) {
        MaxSum b = {__shfl_xor(a.m, o, WAVE), __shfl_xor(a.s, o, WAVE)};
        a = ms_merge(a, b);
    }
    if (lane == 0) part[wave] = a;
    __syncthreads();
    if (threadIdx.x == 0) {
        MaxSum r = part[0];
        for (int w = 1; w < NW; ++w) r = ms_merge(r, part[w]);
        const float l = r.m + logf(r.s);
        *s_lse = l;
        row_loss[row] = l - to_f32(z[t]);
    }
    __syncthreads();
    return *s_lse;
}

template <typename T, bool VEC16>
__global__ __launch_bounds__(RR_THREADS) void ce_rows_inplace_kernel(
    T* __restrict__ Z, int64_t ldz, const int64_t* __restrict__ targets, int V, int zero_pad,
    int64_t ignore_index, const DeviceHeader* __restrict__ hdr, float* __restrict__ row_loss,
    const int* __restrict__ live) {
    constexpr int VEC = RowVec<T>::N;
    const int row = blockIdx.x;
    const int tid = threadIdx.x;
    if (live && row >= *live) {   // past the chunk's live rows (uniform per workgroup)
        if (tid == 0) row_loss[row] = 0.f;
        return;
    }
    T* z = Z + (int64_t)row * ldz;
    const int64_t t = targets[row];
    const bool valid = (t != ignore_index);
    u32x4* zv = reinterpret_cast<u32x4*>(z);

    __shared__ MaxSum part[RR_THREADS / WAVE];
    __shared__ float s_lse;

    const int nvec = VEC16 ? V / VEC : 0;
    if (tid < zero_pad) z[V + tid] = from_f32<T>(0.f);   // zero_pad < 64
    if (!valid) {   // uniform per workgroup
        const u32x4 zero = {0u, 0u, 0u, 0u};
        for (int i = tid; i < nvec; i += RR_THREADS) zv[i] = zero;
        for (int v = nvec * VEC + tid; v < V; v += RR_THREADS) z[v] = from_f32<T>(0.f);
        if (tid == 0) row_loss[row] = 0.f;
        return;
    }

    MaxSum a = {-INFINITY, 0.f};
    if constexpr (VEC16) {
        for (int i = tid; i < nvec; i += RR_THREADS) {
            float f[VEC];
            RowVec<T>::unpack(zv[i], f);
            ms_push_vec<T, VEC>(a, f);
        }
    }
    for (int v = nvec * VEC + tid; v < V; v += RR_THREADS) ms_push<T>(a, to_f32(z[v]));
    const float lse = row_lse<T, RR_THREADS / WAVE>(a, z, t, row, row_loss, part, &s_lse);

    const float inv_n = hdr->inv_n;
    const RowExp<T> ex(lse);
    const int tcol = (int)t;
    if constexpr (VEC16) {
        for (int i = tid; i < nvec; i += RR_THREADS)
            zv[i] = ce_gradient_vec<T>(zv[i], i, tcol, ex, inv_n);
    }
    for (int v = nvec * VEC + tid; v < V; v += RR_THREADS)
        z[v] = ce_gradient_one<T>(z[v], v, tcol, ex, inv_n);
}

// Variant that keeps the row in registers: one workgroup of THREADS threads per row holds
// the first THREADS * NV 16-byte vectors of the row between the two sweeps, so that part
// of the row is read from HBM once instead of twice; what is beyond is swept twice as
// above.  All of a thread's loads are issued before the first is consumed.  Three shapes
// are used: 256 threads x 12 vectors for rows up to 48 KB and 512 threads x 12 vectors up
// to 96 KB, where several workgroups fit a CU and overlap one another's memory, reduction
// and barrier phases (6.3-6.7 TB/s of algorithmic traffic on 32 .. 96 KB rows of bf16,
// 4096 rows, kernel alone); 1024 threads x 16 vectors (256 KB) beyond, where 16 wavefronts
// keep the per-thread ALU phases short (5.0-5.4 TB/s; a variant with 4 wavefronts per CU
// and the whole row cached was slower than two sweeps).  At these rates the arithmetic
// (about 16 lane operations per logit) takes as long as the memory traffic.
constexpr int RC_THREADS = 1024;
constexpr int RC_NV = 16;
constexpr int RM_THREADS = 512;   // rows up to 96 KB
constexpr int RM_NV = 12;
constexpr int RS_THREADS = 256;   // rows up to 48 KB
constexpr int RS_NV = 12;

template <typename T, int THREADS, int NV>
__global__ __launch_bounds__(THREADS) void ce_rows_cached_kernel(
    T* __restrict__ Z, int64_t ldz, const int64_t* __restrict__ targets, int V, int zero_pad,
    int64_t ignore_index, const DeviceHeader* __restrict__ hdr, float* __restrict__ row_loss,
    const int* __restrict__ live) {
    constexpr int VEC = RowVec<T>::N;
    const int row = blockIdx.x;
    const int tid = threadIdx.x;
    if (live && row >= *live) {   // past the chunk's live rows (uniform per workgroup)
        if (tid == 0) row_loss[row] = 0.f;
        return;
    }
    T* z = Z + (int64_t)row * ldz;
    const int64_t t = targets[row];
    const bool valid = (t != ignore_index);
    const int nvec = V / VEC;                 // full vectors; the tail is handled by scalars
    u32x4* zv = reinterpret_cast<u32x4*>(z);

    __shared__ MaxSum part[THREADS / WAVE];
    __shared__ float s_lse;

    if (tid < zero_pad) z[V + tid] = from_f32<T>(0.f);   // zero_pad < 64
    if (!valid) {                              // uniform per workgroup
        const u32x4 zero = {0u, 0u, 0u, 0u};
        for (int i = tid; i < nvec; i += THREADS) zv[i] = zero;
        for (int v = nvec * VEC + tid; v < V; v += THREADS) z[v] = from_f32<T>(0.f);
        if (tid == 0) row_loss[row] = 0.f;
        return;
    }

    u32x4 keep[NV];
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        const int i = tid + k * THREADS;
        if (i < nvec) keep[k] = zv[i];
    }
    MaxSum a = {-INFINITY, 0.f};
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        const int i = tid + k * THREADS;
        if (i < nvec) {
            float f[VEC];
            RowVec<T>::unpack(keep[k], f);
            ms_push_vec<T, VEC>(a, f);
        }
        // one vector at a time: interleaving several would spill the cached row
        __builtin_amdgcn_sched_barrier(0);
    }
    for (int i = tid + NV * THREADS; i < nvec; i += THREADS) {   // beyond the cache
        float f[VEC];
        RowVec<T>::unpack(zv[i], f);
        ms_push_vec<T, VEC>(a, f);
    }
    for (int v = nvec * VEC + tid; v < V; v += THREADS) ms_push<T>(a, to_f32(z[v]));
    const float lse = row_lse<T, THREADS / WAVE>(a, z, t, row, row_loss, part, &s_lse);

    const float inv_n = hdr->inv_n;
    const RowExp<T> ex(lse);
    const int tcol = (int)t;
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        const int i = tid + k * THREADS;
        // hide the value's history: otherwise the unpacked floats of sweep 1 are kept
        // for reuse here, which does not fit the register file and spills
        asm volatile("" : "+v"(keep[k]));
        if (i < nvec) zv[i] = ce_gradient_vec<T>(keep[k], i, tcol, ex, inv_n);
        __builtin_amdgcn_sched_barrier(0);
    }
    for (int i = tid + NV * THREADS; i < nvec; i += THREADS)
        zv[i] = ce_gradient_vec<T>(zv[i], i, tcol, ex, inv_n);
    for (int v = nvec * VEC + tid; v < V; v += THREADS)
        z[v] = ce_gradient_one<T>(z[v], v, tcol, ex, inv_n);
}

// Adds the per-row losses of one launch to the running sum, in a fixed order
// (one workgroup, fixed strides), so repeated runs give the same bits.  With
// `mean_out` the mean over the valid rows is written there as well (the last
// launch of a single-head call: saves the separate finalize launch).
__global__ __launch_bounds__(256) void loss_accumulate_kernel(const float* __restrict__ row_loss,
                                                              int rows, DeviceHeader* hdr,
                                                              float* __restrict__ mean_out) {
    __shared__ double part[4];
    double s = 0.0;
    for (int i = threadIdx.x; i < rows; i += 256) s += (double)row_loss[i];
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        const double total = hdr->loss_sum + ((part[0] + part[1]) + (part[2] + part[3]));
        hdr->loss_sum = total;
        if (mean_out) *mean_out = hdr->n_valid > 0 ? (float)(total / (double)hdr->n_valid) : 0.f;
    }
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
