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
#include "scheduler.h"

namespace flce {

constexpr int CP_THREADS = 1024;
constexpr int CP_PER = 8;   // consecutive rows per thread and round

// live rows of a part: clamp(*live - sub, 0, cap)
__device__ __forceinline__ int dyn_live_rows(const int* live, int sub, int cap) {
    return min(cap, max(0, *live - sub));
}

// Words of the device array that carries the chunk loop's state from kernel to kernel.
enum { DYN_CURSOR = 0,      // first batch row the next chunk looks at
       DYN_LIVE = 1,        // rows of the current chunk
       DYN_FIRST_LIVE = 2,  // index of the first chunk launch that holds rows
       DYN_DX_RANGES = 3 }; // K ranges of the current chunk's dX product

// One workgroup; launch `c` of `nchunks`, each sized for `C` rows.  The N valid rows of
// the batch (N = hdr->n_valid, counted before the loop) are dealt evenly to the LAST
// n = max(1, ceil(N / C)) launches, ceil_256(ceil(N / n)) rows each (the last one takes
// what is left), so no launch ends up with a handful of rows and a batch with many
// ignored rows runs fewer chunks: launches before the first live one hold no rows, and
// the dW product, which keeps fp32 partial sums from the first live chunk to the last
// launch, skips them altogether.  The last launch is always live (with N = 0 it holds
// zero rows and writes a zero dW).  For a live launch this collects the next valid rows
// of the batch starting at the row cursor:
//   idx[i] = row of the i-th collected row (ascending), tv[i] = its target
//   dyn[DYN_LIVE] = rows collected, dyn[DYN_CURSOR] = the row after the last one looked at
//   dyn[DYN_DX_RANGES] = K ranges of the dX product for that many rows (dx_tiles_n tile
//   columns, dx_ksteps K steps, at most dx_max_ranges ranges)
__global__ __launch_bounds__(CP_THREADS) void compact_chunk_kernel(
    const int64_t* __restrict__ targets, int BT, int64_t ignore_index, int C, int c, int nchunks,
    const DeviceHeader* __restrict__ hdr, int dx_tiles_n, int dx_ksteps, int dx_max_ranges,
    int* __restrict__ idx, int64_t* __restrict__ tv, int* __restrict__ dyn) {
    __shared__ int wave_total[CP_THREADS / WAVE];
    __shared__ int s_next;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid / WAVE;
    const int n_valid = hdr->n_valid;
    const int n_live = max(1, (n_valid + C - 1) / C);
    const int first_live = nchunks - n_live;
    const int quota = min(C, ((n_valid + n_live - 1) / n_live + 255) / 256 * 256);
    const int cap = c < first_live ? 0 : quota;
    int cursor = c == 0 ? 0 : dyn[DYN_CURSOR];
    int found = 0;
    while (cursor < BT && found < cap) {   // uniform: every thread sees the same values
        const int r0 = min(BT, cursor + tid * CP_PER), r1 = min(BT, r0 + CP_PER);
        int n = 0;
        for (int r = r0; r < r1; ++r) n += (targets[r] != ignore_index);
        int incl = n;   // inclusive prefix sum over the workgroup
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
        int at = found + base + incl - n;
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
        dyn[DYN_CURSOR] = cursor;
        dyn[DYN_LIVE] = found;
        dyn[DYN_FIRST_LIVE] = first_live;
        dyn[DYN_DX_RANGES] = dx_max_ranges > 1
            ? choose_ksplit((int64_t)((found + 255) / 256) * dx_tiles_n, dx_ksteps, dx_max_ranges) : 1;
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
