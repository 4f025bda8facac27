// Rows whose target is ignore_index take no part in the result: their loss is not
// counted, their dlogits are zero, so they add nothing to dW and their dX row is
// zero.  Instead of projecting them and multiplying zeros, the chunk loop runs over
// the VALID rows: chunk c gathers the next (at most) C valid rows of the batch into a
// dense block, all three products and the row kernel run on the block, and dX is
// scattered back; ignored rows of dX are zeroed once.  Where a chunk ends in the
// batch and how many live rows it holds is known on the device only: a two-word
// device array carries the row cursor and the live row count from kernel to kernel
// ("dynamic rows"), so the host never waits and the launches are sized for the worst
// case (no row ignored).  Every output element is computed by the same arithmetic as
// without compaction; only dW sums the same non-zero terms in other groups of K.
#pragma once
#include "flce_device.h"

namespace flce {

constexpr int CP_THREADS = 1024;
constexpr int CP_PER = 8;   // consecutive rows per thread and round

// live rows of a part: clamp(*live - sub, 0, cap)
__device__ __forceinline__ int dyn_live_rows(const int* live, int sub, int cap) {
    return min(cap, max(0, *live - sub));
}

// One workgroup.  Collects the next valid rows of the batch, at most `cap`, starting at
// the row cursor dyn[0] (at row 0 when `first`):
//   idx[i] = row of the i-th collected row (ascending), tv[i] = its target
//   dyn[1] = number of rows collected, dyn[0] = the row after the last one looked at
__global__ __launch_bounds__(CP_THREADS) void compact_chunk_kernel(
    const int64_t* __restrict__ targets, int BT, int64_t ignore_index, int cap, int first,
    int* __restrict__ idx, int64_t* __restrict__ tv, int* __restrict__ dyn) {
    __shared__ int wave_total[CP_THREADS / WAVE];
    __shared__ int s_next;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid / WAVE;
    int cursor = first ? 0 : dyn[0];
    int found = 0;
    while (cursor < BT && found < cap) {   // uniform: every thread sees the same values
        const int r0 = min(BT, cursor + tid * CP_PER), r1 = min(BT, r0 + CP_PER);
        int c = 0;
        for (int r = r0; r < r1; ++r) c += (targets[r] != ignore_index);
        int incl = c;   // inclusive prefix sum over the workgroup
#pragma unroll
        for (int o = 1; o < WAVE; o <<= 1) {
            const int up = __shfl_up(incl, o, WAVE);
            if (lane >= o) incl += up;
        }
        if (tid == 0) s_next = -1;
        __syncthreads();   // also: wave_total and s_next of the previous round are no longer read
        if (lane == WAVE - 1) wave_total[wave] = incl;
        __syncthreads();
        int base = 0, total = 0;
        for (int w = 0; w < CP_THREADS / WAVE; ++w) {
            if (w < wave) base += wave_total[w];
            total += wave_total[w];
        }
        int at = found + base + incl - c;
        for (int r = r0; r < r1; ++r) {
            const int64_t t = targets[r];
            if (t != ignore_index) {
                if (at < cap) {
                    idx[at] = r;
                    tv[at] = t;
                    if (at == cap - 1) s_next = r + 1;   // the chunk is full after this row
                }
                ++at;
            }
        }
        __syncthreads();
        if (found + total >= cap) {
            found = cap;
            cursor = s_next;
        } else {
            found += total;
            cursor = min(BT, cursor + CP_THREADS * CP_PER);
        }
    }
    if (tid == 0) {
        dyn[0] = cursor;
        dyn[1] = found;
    }
}

// out[i][:] = in[idx[i]][:] for the live rows i; one workgroup per row, rows are n
// 16-byte vectors long.
__global__ __launch_bounds__(256) void gather_rows_kernel(const u32x4* __restrict__ in,
                                                          const int* __restrict__ idx,
                                                          const int* __restrict__ live, int n,
                                                          u32x4* __restrict__ out) {
    const int i = blockIdx.x;
    if (i >= *live) return;
    const u32x4* src = in + (int64_t)idx[i] * n;
    u32x4* dst = out + (int64_t)i * n;
    for (int v = threadIdx.x; v < n; v += 256) dst[v] = src[v];
}

// The way back: out[idx[i]][:] = in[i][:] for the live rows i.  With ADD
// the row is added to what out holds (fp32 add, one rounding).  One workgroup per
// row; n elements per row, n % VEC == 0.
template <typename T, bool ADD>
__global__ __launch_bounds__(256) void scatter_rows_kernel(const T* __restrict__ in,
                                                           const int* __restrict__ idx,
                                                           const int* __restrict__ live, int n,
                                                           T* __restrict__ out) {
    constexpr int VEC = 16 / sizeof(T);
    const int i = blockIdx.x;
    if (i >= *live) return;
    u32x4* dst = reinterpret_cast<u32x4*>(out + (int64_t)idx[i] * n);
    const u32x4* from = reinterpret_cast<const u32x4*>(in + (int64_t)i * n);
    const int nv = n / VEC;
    for (int v = threadIdx.x; v < nv; v += 256) {
        u32x4 a = from[v];
        if constexpr (ADD) {
            u32x4 b = dst[v];
            T* ea = reinterpret_cast<T*>(&a);
            const T* eb = reinterpret_cast<const T*>(&b);
#pragma unroll
            for (int j = 0; j < VEC; ++j) ea[j] = from_f32<T>(to_f32(ea[j]) + to_f32(eb[j]));
        }
        dst[v] = a;
    }
}

// Rows with an ignored target get a zero gradient.  Workgroups stride over the rows of
// the batch.
template <typename T>
__global__ __launch_bounds__(256) void zero_ignored_rows_kernel(const int64_t* __restrict__ targets,
                                                                int64_t BT, int64_t ignore_index,
                                                                int n, T* __restrict__ out) {
    constexpr int VEC = 16 / sizeof(T);
    const u32x4 zero = {0u, 0u, 0u, 0u};
    for (int64_t r = blockIdx.x; r < BT; r += gridDim.x) {
        if (targets[r] != ignore_index) continue;   // uniform per workgroup
        u32x4* dst = reinterpret_cast<u32x4*>(out + r * n);
        for (int v = threadIdx.x; v < n / VEC; v += 256) dst[v] = zero;
    }
}

}  // namespace flce
