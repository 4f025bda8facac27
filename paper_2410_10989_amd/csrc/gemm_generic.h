// Guarded "NT" matrix product on the matrix cores, any shape, any alignment:
//     C[M x N] (+)= A[M x K] * B[N x K]^T        (A, B row-major, K contiguous)
// Both operands are K-contiguous, which is the layout the MFMA operand
// registers want.  This kernel is the correct-everywhere path: it serves the
// fp32 storage type (true fp32 products on v_mfma_f32_32x32x2_f32) and every
// bf16 shape the tuned kernel does not take (ragged or unaligned).
//
// A launch can cut K into ranges (grid z), each writing a partial result of its own:
// products with few output tiles and a long K (dX of a small batch) fill the chip
// that way; the partial results are summed in a fixed order by splitk_reduce_kernel.
//
// Workgroup: 256 threads = 4 wavefronts in a 2 x 2 arrangement; macro tile
// 128 x 128, K step 64 bytes per row; each wavefront owns a 64 x 64 quadrant
// as 2 x 2 MFMA 32 x 32 tiles with fp32 accumulators.
#pragma once
#include "flce_device.h"

namespace flce {

constexpr int GG_BM = 128, GG_BN = 128, GG_THREADS = 256;
constexpr int GG_ROW_BYTES = 64;   // K bytes of one tile row
constexpr int GG_LDS_ROW = 80;     // padded LDS row stride in bytes

template <typename T> struct GGTraits;
template <> struct GGTraits<bf16_t> {
    static constexpr int VEC = 8;      // elements per 16-byte vector
    static constexpr int BK = 32;      // elements per tile row
    static constexpr int KSTEP = 16;   // K per MFMA
};
template <> struct GGTraits<float> {
    static constexpr int VEC = 4;
    static constexpr int BK = 16;
    static constexpr int KSTEP = 2;
};

// 16 bytes of one operand row starting at element k (k is a multiple of VEC),
// zero beyond the matrix.  ALIGNED: K % VEC == 0, ld % VEC == 0, base 16-byte
// aligned, so a vector is entirely inside or entirely outside the row.
template <typename T, bool ALIGNED>
__device__ __forceinline__ u32x4 gg_load16(const T* base, int64_t ld, int row, int rows, int k,
                                           int K) {
    u32x4 r = {0u, 0u, 0u, 0u};
    if (row >= rows || k >= K) return r;
    const T* p = base + (int64_t)row * ld + k;
    if constexpr (ALIGNED) {
        r = *reinterpret_cast<const u32x4*>(p);
    } else {
        constexpr int VEC = GGTraits<T>::VEC;
        T tmp[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) tmp[e] = (k + e < K) ? p[e] : from_f32<T>(0.f);
        r = *reinterpret_cast<u32x4*>(tmp);
    }
    return r;
}

template <typename T, typename OutT, bool ALIGNED, bool ACCUM>
__global__ __launch_bounds__(GG_THREADS) void gemm_nt_generic(const T* __restrict__ A, int64_t lda,
                                                              const T* __restrict__ B, int64_t ldb,
                                                              OutT* __restrict__ C, int64_t ldc,
                                                              int M, int N, int K, int k_per,
                                                              int64_t split_stride) {
    using TR = GGTraits<T>;
    __shared__ __attribute__((aligned(16))) unsigned char lds_a[GG_BM * GG_LDS_ROW];
    __shared__ __attribute__((aligned(16))) unsigned char lds_b[GG_BN * GG_LDS_ROW];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    // tiles are numbered along grid x, row of tiles by row of tiles (grid y is limited to 65535)
    const int tiles_n = (N + GG_BN - 1) / GG_BN;
    const int m0 = (int)(blockIdx.x / tiles_n) * GG_BM, n0 = (int)(blockIdx.x % tiles_n) * GG_BN;
    // K range of this workgroup: blockIdx.z counts ranges of k_per elements (a multiple of
    // the K step), each with a result matrix of its own, split_stride elements apart
    const int k_begin = blockIdx.z * k_per;
    K = min(K, k_begin + k_per);
    C += (int64_t)blockIdx.z * split_stride;

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int g = 0; g < 16; ++g) acc[i][j][g] = 0.f;

    // staging: 128 rows x 4 vectors per operand tile, 2 vectors per thread
    const int ld_row = tid >> 2, ld_vec = tid & 3;

    for (int k0 = k_begin; k0 < K; k0 += TR::BK) {
        u32x4 ra[2], rb[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int r = ld_row + h * 64;
            ra[h] = gg_load16<T, ALIGNED>(A, lda, m0 + r, M, k0 + ld_vec * TR::VEC, K);
            rb[h] = gg_load16<T, ALIGNED>(B, ldb, n0 + r, N, k0 + ld_vec * TR::VEC, K);
        }
        __syncthreads();   // previous tile fully consumed
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int r = ld_row + h * 64;
            *reinterpret_cast<u32x4*>(lds_a + r * GG_LDS_ROW + ld_vec * 16) = ra[h];
            *reinterpret_cast<u32x4*>(lds_b + r * GG_LDS_ROW + ld_vec * 16) = rb[h];
        }
        __syncthreads();

        const int frow = lane & 31, fk = lane >> 5;
        if constexpr (sizeof(T) == 2) {
#pragma unroll
            for (int kk = 0; kk < TR::BK / TR::KSTEP; ++kk) {
                bf16x8 fa[2], fb[2];
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    fa[i] = *reinterpret_cast<const bf16x8*>(
                        lds_a + (wm * 64 + i * 32 + frow) * GG_LDS_ROW + kk * 32 + fk * 16);
                    fb[i] = *reinterpret_cast<const bf16x8*>(
                        lds_b + (wn * 64 + i * 32 + frow) * GG_LDS_ROW + kk * 32 + fk * 16);
                }
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j],
                                                                            0, 0, 0);
            }
        } else {
#pragma unroll
            for (int kk = 0; kk < TR::BK / TR::KSTEP; ++kk) {
                float fa[2], fb[2];
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    fa[i] = *reinterpret_cast<const float*>(
                        lds_a + (wm * 64 + i * 32 + frow) * GG_LDS_ROW + (kk * 2 + fk) * 4);
                    fb[i] = *reinterpret_cast<const float*>(
                        lds_b + (wn * 64 + i * 32 + frow) * GG_LDS_ROW + (kk * 2 + fk) * 4);
                }
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i], fb[j], acc[i][j], 0,
                                                                         0, 0);
            }
        }
    }

    // accumulator register g of lane l holds row 8*(g/4) + 4*(l/32) + g%4,
    // column l%32 of its 32 x 32 tile
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = n0 + wn * 64 + j * 32 + (lane & 31);
#pragma unroll
            for (int g = 0; g < 16; ++g) {
                const int row = m0 + wm * 64 + i * 32 + 8 * (g >> 2) + 4 * (lane >> 5) + (g & 3);
                if (row < M && col < N) {
                    OutT* p = C + (int64_t)row * ldc + col;
                    float v = acc[i][j][g];
                    if constexpr (ACCUM) v += to_f32(*p);
                    *p = from_f32<OutT>(v);
                }
            }
        }
}

}  // namespace flce
