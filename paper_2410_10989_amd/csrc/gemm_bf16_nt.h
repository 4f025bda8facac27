// Tuned bf16 "NT" matrix product for gfx950:
//     C[M x N] (+)= A[M x K] * B[N x K]^T     (A, B row-major bf16, K contiguous)
// fp32 accumulation on v_mfma_f32_32x32x16_bf16.  All three products of the
// fused linear cross-entropy path (logits, dX, dW) are brought into this form.
//
// Shape of the kernel
//  - workgroup = 256 threads = 4 wavefronts (2 x 2); macro tile 256 x 256, K step
//    64; each wavefront owns 128 x 128 = 4 x 4 MFMA tiles, i.e. 256 fp32
//    accumulator registers per lane (one wavefront per SIMD, full register file).
//  - global -> registers -> LDS, two LDS stages of 64 KB (of the CU's 160 KB):
//    while the matrix cores work on stage t, the tile t+1 sitting in registers is
//    written to the other stage and the loads of tile t+2 are issued; one
//    workgroup barrier per K step.  Loads are buffer loads: the descriptor's
//    byte range makes rows beyond M / N read as zero, offsets stay 32-bit.
//  - LDS rows are 128 B (64 bf16); the eight 16-byte pieces of a row are XOR
//    swizzled with the row number so that ds_read_b128 of one K piece over 32
//    consecutive rows (the MFMA operand pattern) spreads over all banks.
//  - operand fragments are double buffered in registers across the four K=16
//    sub-steps and across the barrier, so LDS latency hides behind MFMAs.
//  - workgroup id -> tile: ids are dealt round-robin to the 8 XCDs, so id%8
//    selects the XCD and each XCD walks its own contiguous span of a grouped
//    (8 tile rows at a time) tile order; tiles that run together on one XCD
//    share A and B panels in that XCD's L2.
// Requirements (checked on the host): K % 64 == 0, lda % 8 == 0, ldb % 8 == 0,
// A and B 16-byte aligned, 256 * ld * 2 bytes < 2^31.  M and N are arbitrary.
#pragma once
#include "flce_device.h"

namespace flce {

constexpr int FG_BM = 256, FG_BN = 256, FG_BK = 64, FG_THREADS = 256;
constexpr int FG_TILE_BYTES = FG_BM * FG_BK * 2;    // one operand, one stage: 32 KB
constexpr int FG_STAGE_BYTES = 2 * FG_TILE_BYTES;   // A + B
constexpr int FG_LDS_BYTES = 2 * FG_STAGE_BYTES;    // two stages: 128 KB
constexpr int FG_GROUP_M = 8;
constexpr int FG_XCDS = 8;

struct FGArgs {
    const bf16_t* A;
    int64_t lda;
    const bf16_t* B;
    int64_t ldb;
    void* C;
    int64_t ldc;
    int M, N, K;
    int tiles_m, tiles_n;
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t fg_make_rsrc(const void* base, uint32_t bytes) {
    // raw buffer, no stride: offsets >= bytes read as zero
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

template <typename OutT, bool ACCUM, int SWS>
__global__ __launch_bounds__(FG_THREADS) void gemm_bf16_nt_256(FGArgs a) {
    __shared__ __attribute__((aligned(16))) unsigned char smem[FG_LDS_BYTES];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // ---- workgroup id -> tile (XCD aware, grouped order) ----
    const int total = a.tiles_m * a.tiles_n;
    const int per_xcd = (int)gridDim.x / FG_XCDS;
    const int seq = ((int)blockIdx.x % FG_XCDS) * per_xcd + (int)blockIdx.x / FG_XCDS;
    if (seq >= total) return;
    const int group_size = FG_GROUP_M * a.tiles_n;
    const int grp = seq / group_size;
    const int first_m = grp * FG_GROUP_M;
    const int gm = min(FG_GROUP_M, a.tiles_m - first_m);
    const int rem = seq - grp * group_size;
    const int pm = first_m + rem % gm, pn = rem / gm;
    const int m0 = pm * FG_BM, n0 = pn * FG_BN;

    // ---- global side ----
    const int rows_a = min(FG_BM, a.M - m0), rows_b = min(FG_BN, a.N - n0);
    const __amdgpu_buffer_rsrc_t rsrc_a =
        fg_make_rsrc(a.A + (int64_t)m0 * a.lda, (uint32_t)rows_a * (uint32_t)a.lda * 2u);
    const __amdgpu_buffer_rsrc_t rsrc_b =
        fg_make_rsrc(a.B + (int64_t)n0 * a.ldb, (uint32_t)rows_b * (uint32_t)a.ldb * 2u);
    const int ld_row = tid >> 3, ld_piece = tid & 7;
    int off_a[8], off_b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        off_a[i] = (ld_row + 32 * i) * (int)a.lda * 2 + ld_piece * 16;
        off_b[i] = (ld_row + 32 * i) * (int)a.ldb * 2 + ld_piece * 16;
    }

    // ---- LDS side ----
    const int wr = ld_row * 128 + ((ld_piece ^ ((ld_row >> SWS) & 7)) << 4);
    const int frow = lane & 31, fhalf = lane >> 5;
    const int fsw = (frow >> SWS) & 7;
    int rd_a[4], rd_b[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        const int piece = ((kk << 1) | fhalf) ^ fsw;
        rd_a[kk] = (wm * 128 + frow) * 128 + (piece << 4);
        rd_b[kk] = FG_TILE_BYTES + (wn * 128 + frow) * 128 + (piece << 4);
    }

    u32x4 ra[8], rb[8];
    auto gload = [&](int kt) {
        const int soff = kt * (FG_BK * 2);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            ra[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_a, off_a[i], soff, 0);
            rb[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_b, off_b[i], soff, 0);
        }
    };
    auto lds_store = [&](int stage) {
        unsigned char* base = smem + stage * FG_STAGE_BYTES + wr;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            *reinterpret_cast<u32x4*>(base + i * 4096) = ra[i];
            *reinterpret_cast<u32x4*>(base + FG_TILE_BYTES + i * 4096) = rb[i];
        }
    };
    bf16x8 fa[2][4], fb[2][4];
    auto read_frags = [&](int stage, int kk, int buf) {
        const unsigned char* base = smem + stage * FG_STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            fa[buf][i] = *reinterpret_cast<const bf16x8*>(base + rd_a[kk] + i * 4096);
            fb[buf][i] = *reinterpret_cast<const bf16x8*>(base + rd_b[kk] + i * 4096);
        }
    };

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int g = 0; g < 16; ++g) acc[i][j][g] = 0.f;
    auto mma = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] =
                    __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[buf][i], fb[buf][j], acc[i][j], 0, 0, 0);
    };

    const int nk = a.K / FG_BK;
    gload(0);
    lds_store(0);
    if (nk > 1) gload(1);
    __syncthreads();
    read_frags(0, 0, 0);

    for (int t = 0; t < nk; ++t) {
        const int cur = t & 1, nxt = cur ^ 1;
        read_frags(cur, 1, 1);
        if (t + 1 < nk) lds_store(nxt);   // tile t+1 waits in registers
        if (t + 2 < nk) gload(t + 2);
        mma(0);
        read_frags(cur, 2, 0);
        mma(1);
        read_frags(cur, 3, 1);
        mma(0);
        __syncthreads();                  // stage nxt written, stage cur fully read
        if (t + 1 < nk) read_frags(nxt, 0, 0);
        mma(1);
    }

    // ---- epilogue: accumulator register g of lane l is row 8*(g/4)+4*(l/32)+g%4,
    // column l%32 of its 32 x 32 tile ----
    OutT* C = static_cast<OutT*>(a.C);
    const bool full = (rows_a == FG_BM) && (rows_b == FG_BN);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int col = n0 + wn * 128 + j * 32 + frow;
#pragma unroll
            for (int g = 0; g < 16; ++g) {
                const int row = m0 + wm * 128 + i * 32 + 8 * (g >> 2) + 4 * fhalf + (g & 3);
                if (full || (row < a.M && col < a.N)) {
                    OutT* p = C + (int64_t)row * a.ldc + col;
                    float v = acc[i][j][g];
                    if constexpr (ACCUM) v += to_f32(*p);
                    *p = from_f32<OutT>(v);
                }
            }
        }
}

}  // namespace flce
