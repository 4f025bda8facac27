// Tuned bf16 "NT" matrix product for gfx950:
//     C[M x N] (+)= A[M x K] * B[N x K]^T     (A, B row-major bf16, K contiguous)
// fp32 accumulation on v_mfma_f32_32x32x16_bf16.  All three products of the
// fused linear cross-entropy path (logits, dX, dW) are brought into this form.
//
// Shape of the kernel
//  - workgroup = 256 threads = 4 wavefronts (2 x 2); macro tile 256 x 256, K step
//    64; each wavefront owns 128 x 128 = 4 x 4 MFMA tiles, i.e. 256 fp32
//    accumulator registers per lane (one wavefront per SIMD, full register file).
//  - global -> LDS directly (buffer_load_dwordx4 ... lds): no vector registers
//    and no LDS write instructions are spent on staging.  The buffer descriptor's
//    byte range makes rows beyond M / N read as zero and keeps offsets 32-bit.
//  - the whole 160 KB LDS of the CU is a ring of five 32 KB slots, each holding
//    the A tile or the B tile (256 rows x 64 bf16) of one K step, filled in the
//    order A0 B0 A1 B1 A2 ...  While step t is multiplied, B(t+1) and A(t+2)
//    stream in, so the loads run up to two steps ahead and the memory pipe is
//    fed continuously instead of in one burst per step; one workgroup barrier
//    per K step, which waits for all but the youngest slot (s_waitcnt vmcnt(8)).
//    What limits this kernel next to the matrix pipe is L2 bandwidth: a 256 x 256
//    tile needs 128 B per row and step from L2, 16 TB/s at 2 PFLOP/s.
//  - LDS rows are 128 B (64 bf16); the eight 16-byte pieces of a row are XOR
//    swizzled with (row / 2) % 8 so that ds_read_b128 of one K piece over
//    consecutive rows (the MFMA operand pattern) spreads over all banks.
//  - operand fragments are double buffered in registers across the four K=16
//    sub-steps; the last sub-step of a tile runs behind the barrier while the
//    first fragments of the next tile arrive.
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
constexpr int FG_TILE_BYTES = FG_BM * FG_BK * 2;    // one operand tile of one K step: 32 KB
constexpr int FG_SLOTS = 5;                         // ring of operand-tile slots
constexpr int FG_LDS_BYTES = FG_SLOTS * FG_TILE_BYTES;   // 160 KB: the whole LDS of a CU
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

template <typename OutT, bool ACCUM>
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
    const int ld_piece = (tid & 7) ^ ((ld_row >> 1) & 7);        // logical piece fetched
    int off_a[8], off_b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        off_a[i] = (ld_row + 32 * i) * (int)a.lda * 2 + ld_piece * 16;
        off_b[i] = (ld_row + 32 * i) * (int)a.ldb * 2 + ld_piece * 16;
    }
    const int uwave = __builtin_amdgcn_readfirstlane(wave);
    typedef __attribute__((address_space(3))) void* lds_ptr_t;
    // The ring: operand tiles are loaded in the order A0 B0 A1 B1 A2 ... and item
    // number n lives in slot n % 5.  8 loads per wavefront fill one slot.
    auto gload_a = [&](int kt, int slot) {
        const int soff = kt * (FG_BK * 2);
        unsigned char* dst = smem + slot * FG_TILE_BYTES + uwave * 1024;
#pragma unroll
        for (int r = 0; r < 8; ++r)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, (lds_ptr_t)(dst + r * 4096), 16, off_a[r],
                                                     soff, 0, 0);
    };
    auto gload_b = [&](int kt, int slot) {
        const int soff = kt * (FG_BK * 2);
        unsigned char* dst = smem + slot * FG_TILE_BYTES + uwave * 1024;
#pragma unroll
        for (int r = 0; r < 8; ++r)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_b, (lds_ptr_t)(dst + r * 4096), 16, off_b[r],
                                                     soff, 0, 0);
    };

    // ---- LDS side: MFMA operand fragments ----
    // lane l of a fragment: tile row l%32, K piece 2*kk + l/32 (8 bf16 = 16 bytes)
    const int frow = lane & 31, fhalf = lane >> 5;
    const int fsw = (frow >> 1) & 7;
    int rd_a[4], rd_b[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        const int piece = ((kk << 1) | fhalf) ^ fsw;
        rd_a[kk] = (wm * 128 + frow) * 128 + (piece << 4);
        rd_b[kk] = (wn * 128 + frow) * 128 + (piece << 4);
    }
    // Fragment order a0 b0 b1 b2 b3 a1 a2 a3 = the order the MFMAs below need them.
    bf16x8 fa[2][4], fb[2][4];
    auto read_frags = [&](int slot_a, int slot_b, int kk, auto buf) {
        constexpr int Bf = decltype(buf)::value;
        const unsigned char* pa = smem + slot_a * FG_TILE_BYTES + rd_a[kk];
        const unsigned char* pb = smem + slot_b * FG_TILE_BYTES + rd_b[kk];
        fa[Bf][0] = *reinterpret_cast<const bf16x8*>(pa);
#pragma unroll
        for (int j = 0; j < 4; ++j) fb[Bf][j] = *reinterpret_cast<const bf16x8*>(pb + j * 4096);
#pragma unroll
        for (int i = 1; i < 4; ++i) fa[Bf][i] = *reinterpret_cast<const bf16x8*>(pa + i * 4096);
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

    // Workgroup barrier of the pipeline.  Loads complete in order and every
    // wavefront issues 8 per slot, so "at most 8 outstanding" means everything
    // but the youngest slot (the A tile two steps ahead) has landed.  All LDS
    // reads of the step are complete as well, so its two slots can be refilled.
    auto pipeline_barrier = [&]() {
        asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    };

    // One K step.  PH = t % 5 fixes the slots: A(t) in (2 PH) % 5, B(t) in
    // (2 PH + 1) % 5; B(t+1) refills the slot A(t-1) left, A(t+2) the slot B(t-1)
    // left.  The fourth K=16 sub-step of a tile is multiplied at the start of the
    // next step, behind the barrier, while the new fragments arrive.  Tiles past
    // the end are loaded but never consumed (the descriptor returns zeros past
    // its range), which keeps the steady state free of branches.
    auto step = [&](auto phase, int t) {
        constexpr int PH = decltype(phase)::value;
        constexpr int SA = (2 * PH) % 5, SB = (2 * PH + 1) % 5;
        constexpr int SB1 = (2 * PH + 3) % 5, SA2 = (2 * PH + 4) % 5;
        read_frags(SA, SB, 0, I0{});
        gload_b(t + 1, SB1);
        mma(I1{});                       // sub-step 3 of the previous tile
        read_frags(SA, SB, 1, I1{});
        gload_a(t + 2, SA2);
        mma(I0{});
        read_frags(SA, SB, 2, I0{});
        mma(I1{});
        read_frags(SA, SB, 3, I1{});
        mma(I0{});
        pipeline_barrier();
    };

    const int nk = a.K / FG_BK;
    gload_a(0, 0);
    gload_b(0, 1);
    gload_a(1, 2);
#pragma unroll
    for (int i = 0; i < 4; ++i) {        // the first step has no previous sub-step: add zero
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            fa[1][i][e] = (bf16_t)0.f;
            fb[1][i][e] = (bf16_t)0.f;
        }
    }
    pipeline_barrier();
    int t = 0;
    for (; t + 5 <= nk; t += 5) {
        step(std::integral_constant<int, 0>{}, t);
        step(std::integral_constant<int, 1>{}, t + 1);
        step(std::integral_constant<int, 2>{}, t + 2);
        step(std::integral_constant<int, 3>{}, t + 3);
        step(std::integral_constant<int, 4>{}, t + 4);
    }
    if (t < nk) step(std::integral_constant<int, 0>{}, t++);
    if (t < nk) step(std::integral_constant<int, 1>{}, t++);
    if (t < nk) step(std::integral_constant<int, 2>{}, t++);
    if (t < nk) step(std::integral_constant<int, 3>{}, t++);
    mma(I1{});
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
