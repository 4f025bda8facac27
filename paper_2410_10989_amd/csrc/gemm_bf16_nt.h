// Tuned bf16 "NT" matrix product for gfx950:
//     C[M x N] (+)= A[M x K] * B[N x K]^T     (A, B row-major bf16, K contiguous)
// fp32 accumulation on v_mfma_f32_32x32x16_bf16.  All three products of the
// fused linear cross-entropy path (logits, dX, dW) are brought into this form.
//
// Shape of the kernel
//  - workgroup = 256 threads = 4 wavefronts (2 x 2); macro tile 256 x 256, K step
//    64; each wavefront owns 128 x 128 = 4 x 4 MFMA tiles, i.e. 256 fp32
//    accumulator registers per lane (one wavefront per SIMD, full register file).
//  - global -> LDS directly (buffer_load_dwordx4 ... lds), two LDS stages of
//    64 KB (of the CU's 160 KB): while the matrix cores work on stage t, tile t+1
//    streams into the other stage; one workgroup barrier per K step.  The buffer
//    descriptor's byte range makes rows beyond M / N read as zero, offsets stay
//    32-bit, and no vector registers or LDS write instructions are spent on
//    staging.
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
// A and B 16-byte aligned, (256 * ld + K + 256) * 2 bytes < 2^31 for lda and ldb,
// 256 * ldc * sizeof(C element) < 2^31.  M and N are arbitrary.
#pragma once
#include <type_traits>

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

    // ---- global side: direct-to-LDS buffer loads ----
    // One wavefront-wide load moves 64 x 16 bytes straight into LDS at
    // M0 + lane * 16, i.e. 8 consecutive tile rows of 128 bytes.  Lane l therefore
    // owns the physical position (row l/8, piece l%8) and fetches the logical
    // piece (l%8) ^ swizzle(row) from global memory.  Wavefront w fills rows
    // 8w..8w+7 of every 32-row group; 8 loads per operand per K step.
    const int rows_a = min(FG_BM, a.M - m0), rows_b = min(FG_BN, a.N - n0);
    const __amdgpu_buffer_rsrc_t rsrc_a =
        fg_make_rsrc(a.A + (int64_t)m0 * a.lda, (uint32_t)rows_a * (uint32_t)a.lda * 2u);
    const __amdgpu_buffer_rsrc_t rsrc_b =
        fg_make_rsrc(a.B + (int64_t)n0 * a.ldb, (uint32_t)rows_b * (uint32_t)a.ldb * 2u);
    const int ld_row = tid >> 3;                                   // 0..31
    const int ld_piece = (tid & 7) ^ ((ld_row >> SWS) & 7);        // logical piece fetched
    int off_a[8], off_b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        off_a[i] = (ld_row + 32 * i) * (int)a.lda * 2 + ld_piece * 16;
        off_b[i] = (ld_row + 32 * i) * (int)a.ldb * 2 + ld_piece * 16;
    }
    const int uwave = __builtin_amdgcn_readfirstlane(wave);
    typedef __attribute__((address_space(3))) void* lds_ptr_t;
    // quad r < 8: A rows 32r.., r >= 8: B rows 32(r-8)..
    auto gload = [&](int stage, int kt, int r_lo, int r_hi) {
        const int soff = kt * (FG_BK * 2);
#pragma unroll
        for (int r = r_lo; r < r_hi; ++r) {
            unsigned char* dst = smem + stage * FG_STAGE_BYTES + (r >> 3) * FG_TILE_BYTES +
                                 (r & 7) * 4096 + uwave * 1024;
            if (r < 8)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, (lds_ptr_t)dst, 16, off_a[r], soff, 0, 0);
            else
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_b, (lds_ptr_t)dst, 16, off_b[r - 8], soff, 0, 0);
        }
    };

    // ---- LDS side: MFMA operand fragments ----
    const int frow = lane & 31, fhalf = lane >> 5;
    const int fsw = (frow >> SWS) & 7;
    int rd_a[4], rd_b[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        const int piece = ((kk << 1) | fhalf) ^ fsw;
        rd_a[kk] = (wm * 128 + frow) * 128 + (piece << 4);
        rd_b[kk] = FG_TILE_BYTES + (wn * 128 + frow) * 128 + (piece << 4);
    }
    // Fragment order a0 b0 b1 b2 b3 a1 a2 a3 = the order the MFMAs below need them.
    bf16x8 fa[2][4], fb[2][4];
    auto read_frags = [&](int stage, int kk, auto buf) {
        constexpr int Bf = decltype(buf)::value;
        const unsigned char* base = smem + stage * FG_STAGE_BYTES;
        fa[Bf][0] = *reinterpret_cast<const bf16x8*>(base + rd_a[kk]);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            fb[Bf][j] = *reinterpret_cast<const bf16x8*>(base + rd_b[kk] + j * 4096);
#pragma unroll
        for (int i = 1; i < 4; ++i)
            fa[Bf][i] = *reinterpret_cast<const bf16x8*>(base + rd_a[kk] + i * 4096);
    };

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int g = 0; g < 16; ++g) acc[i][j][g] = 0.f;
    auto mma = [&](auto buf) {
        constexpr int Bf = decltype(buf)::value;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[Bf][i], fb[Bf][j], acc[i][j],
                                                                    0, 0, 0);
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;

    // Instruction-mix hints for the backend scheduler.  Per K step a wavefront
    // issues 64 MFMAs, 32 LDS reads and 16 direct-to-LDS loads; the memory
    // instructions are spread between the MFMAs instead of issued in bursts.
    constexpr int SG_MFMA = 0x008, SG_VMEM = 0x010, SG_DS_RD = 0x100;
#define FG_SLOT(mask)                                        \
    __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 0);     \
    __builtin_amdgcn_sched_group_barrier((mask), 1, 0);
#define FG_PHASE(n_ld)                                                  \
    _Pragma("unroll") for (int q_ = 0; q_ < 8; ++q_) {                  \
        FG_SLOT(SG_DS_RD)                                               \
        if (q_ < (n_ld)) { FG_SLOT(SG_VMEM) }                           \
        else { __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 0); }   \
    }

    // One K step on the tile in LDS stage `cur`; tile t+1 streams into the other
    // stage meanwhile and has to be complete at the barrier.  A tile beyond the
    // last one is loaded but never consumed (the descriptor returns zeros past
    // its range), which keeps the steady state free of branches.
    const int nk = a.K / FG_BK;
    gload(0, 0, 0, 16);
    __syncthreads();
    read_frags(0, 0, I0{});
    gload(1, 1, 0, 8);
    for (int t = 0; t < nk; ++t) {
        const int cur = t & 1, nxt = cur ^ 1;
        // K sub-step 0 (fragments of sub-step 1 arrive meanwhile)
        read_frags(cur, 1, I1{});
        gload(nxt, t + 1, 8, 16);
        mma(I0{});
        // K sub-step 1
        read_frags(cur, 2, I0{});
        mma(I1{});
        // K sub-step 2
        read_frags(cur, 3, I1{});
        mma(I0{});
        FG_PHASE(8)
        FG_PHASE(0)
        FG_PHASE(0)
        __syncthreads();   // stage nxt complete (loads drained), stage cur read by everyone
        // K sub-step 3 runs on fragments already in registers while the first
        // fragments of the next stage arrive and the loads of tile t+2 start
        read_frags(nxt, 0, I0{});
        gload(cur, t + 2, 0, 8);
        mma(I1{});
        FG_PHASE(8)
    }
#undef FG_PHASE
#undef FG_SLOT
    // the loads of the tiles past the end still target LDS: let them land before
    // the workgroup can retire and its LDS be handed to another one
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    // ---- epilogue.  Accumulator register g of lane l is row 8*(g/4)+4*(l/32)+g%4,
    // column l%32 of its 32 x 32 tile.  Stores go through a buffer descriptor that
    // covers the tile's valid rows (rows past M are dropped by the range check);
    // the part of the address that is the same for the whole wavefront travels in
    // a scalar register, so no per-element 64-bit address arithmetic is needed. ----
    constexpr int ES = (int)sizeof(OutT);
    const int ldc = (int)a.ldc;
    const __amdgpu_buffer_rsrc_t rsrc_c = fg_make_rsrc(
        static_cast<OutT*>(a.C) + (int64_t)m0 * a.ldc, (uint32_t)rows_a * (uint32_t)ldc * (uint32_t)ES);
    const int uwm = __builtin_amdgcn_readfirstlane(wm), uwn = __builtin_amdgcn_readfirstlane(wn);
    const int lane_off = (4 * fhalf * ldc + frow) * ES;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int col0 = n0 + uwn * 128 + j * 32;
        if (col0 + frow < a.N) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row0 = uwm * 128 + i * 32;
                if constexpr (ACCUM) {
                    static_assert(!ACCUM || ES == 4, "accumulation is into fp32");
                    float old[16];
#pragma unroll
                    for (int g = 0; g < 16; ++g) {
                        const int soff = ((row0 + 8 * (g >> 2) + (g & 3)) * ldc + col0) * ES;
                        old[g] = __uint_as_float(
                            __builtin_amdgcn_raw_buffer_load_b32(rsrc_c, lane_off, soff, 0));
                    }
#pragma unroll
                    for (int g = 0; g < 16; ++g) acc[i][j][g] += old[g];
                }
#pragma unroll
                for (int g = 0; g < 16; ++g) {
                    const int soff = ((row0 + 8 * (g >> 2) + (g & 3)) * ldc + col0) * ES;
                    const float v = acc[i][j][g];
                    if constexpr (ES == 4) {
                        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), rsrc_c, lane_off, soff,
                                                              0);
                    } else {
                        __builtin_amdgcn_raw_buffer_store_b16(
                            __builtin_bit_cast(unsigned short, from_f32<bf16_t>(v)), rsrc_c, lane_off,
                            soff, 0);
                    }
                }
            }
        }
    }
}

}  // namespace flce
