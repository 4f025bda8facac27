// Tuned bf16 matrix product for gfx950, fp32 accumulation on
// v_mfma_f32_32x32x16_bf16:
//     C[M x N] = (Cin +) sum_k a(m,k) * b(n,k)          (Cin: fp32 or bf16, optional)
// where each operand is given either K-contiguous ("row" form: a(m,k) = A[m*lda + k])
// or K-major ("column" form: a(m,k) = A[k*lda + m]).  All three products of the
// fused linear cross-entropy path run on it without transposed copies:
//     logits  Z  = X_c W^T      A = X_c row form,  B = W   row form
//     dX_c       = G W          A = G   row form,  B = W   column form (K = V)
//     dW        += G^T X_c      A = G   column form, B = X_c column form (K = chunk rows)
//
// Shape of the kernel
//  - workgroup = 256 threads = 4 wavefronts (2 x 2); macro tile 256 x 256, K step
//    64; each wavefront owns 128 x 128 = 4 x 4 MFMA tiles, i.e. 256 fp32
//    accumulator registers per lane (one wavefront per SIMD, full register file).
//  - global -> LDS directly (buffer_load_dwordx4 ... lds): no vector registers
//    and no LDS write instructions are spent on staging.  The buffer descriptor's
//    byte range makes reads past the operand return zero and keeps offsets 32-bit.
//  - the whole 160 KB LDS of the CU is a ring of five 32 KB slots, each holding
//    the A tile or the B tile of one K step, filled in the order A0 B0 A1 B1 A2 ...
//    While step t is multiplied, B(t+1) and A(t+2) stream in, so the loads run up
//    to two steps ahead and the memory pipe is fed continuously; one workgroup
//    barrier per K step, which waits for all but the youngest slot
//    (s_waitcnt vmcnt(8)).  Next to the matrix pipe the limit is L2 bandwidth:
//    a 256 x 256 tile pulls 64 KB per K step from L2, 16 TB/s at 2 PFLOP/s.
//  - row-form tiles sit in LDS as 256 rows of 128 B whose eight 16-byte pieces are
//    XOR swizzled with (row / 2) % 8, so that ds_read_b128 of one K piece over
//    consecutive rows (the MFMA operand pattern) spreads over all banks.
//  - column-form tiles sit in LDS as 64 K rows of 512 B (the layout they have in
//    memory) whose eight 64-byte chunks are XOR swizzled with a function of the K
//    row; fragments are fetched with ds_read_b64_tr_b16, the transposing LDS read:
//    inside each group of 16 lanes it turns 4 K rows x 16 columns into 16 lanes x
//    4 consecutive K values, which is the MFMA operand layout.
//  - operand fragments are double buffered in registers across the four K=16
//    sub-steps; the last sub-step of a tile runs behind the barrier while the
//    first fragments of the next tile arrive.  The LDS reads are issued as inline
//    assembly with explicit s_waitcnt: the compiler would otherwise put a full
//    vmcnt(0) in front of every transposing read (it cannot tell that the read
//    does not alias an in-flight direct-to-LDS load), and it clusters reads
//    instead of issuing one per MFMA.  The instruction order of the steady state
//    is pinned with sched_barrier: MFMA, LDS read(s) or one load, MFMA, ...
//  - workgroup id -> tile: ids are dealt round-robin to the 8 XCDs, so id%8
//    selects the XCD and each XCD walks its own contiguous span of a grouped
//    (8 tile rows at a time) tile order; tiles that run together on one XCD
//    share A and B panels in that XCD's L2.
//  - epilogue through LDS: the MFMAs take the B fragment first and the A fragment
//    second, so a lane's accumulators are four consecutive columns of one row per
//    register quad; each wavefront stages 32 x 128 values at a time in its own LDS
//    region and writes 16 bytes of output per lane, whole row segments per
//    instruction (the memory pipe charges per store instruction).
// With ksplit > 1 the K range is cut into ksplit pieces computed by different
// workgroups; piece s writes its partial result to C + s * split_stride (fp32), and a
// separate fixed-order reduction adds the pieces (used when M x N has fewer tiles
// than the chip has CUs, as for dX with its very long K = V).
// Requirements (checked on the host): leading dimensions % 8 == 0, A and B 16-byte
// aligned, the byte extent of one tile below 2^30 (row form: 256 * ld * 2 + 128,
// column form: 64 * ld * 2 + 512; operands themselves may be of any size),
// 256 * ldc * sizeof(element) < 2^31 for C and Cin.  M and N are arbitrary: tile rows /
// columns past them hold zeros or stale values and only feed outputs that are never
// stored.  K is arbitrary for a column-form operand (its K rows past K lie outside the
// descriptor's range and read as zero); a row-form operand needs K % 64 == 0, or rows
// that are allocated up to the next multiple of 64 and hold zeros there (the dlogits
// chunk is kept that way); the last K step then multiplies zeros.
#pragma once
#include <type_traits>

#include "flce_device.h"
#include "scheduler.h"

namespace flce {

constexpr int FG_BM = 256, FG_BN = 256, FG_BK = 64, FG_THREADS = 256;
constexpr int FG_TILE_BYTES = FG_BM * FG_BK * 2;    // one operand tile of one K step: 32 KB
constexpr int FG_SLOTS = 5;                         // ring of operand-tile slots
constexpr int FG_LDS_BYTES = FG_SLOTS * FG_TILE_BYTES;   // 160 KB: the whole LDS of a CU
// Tile order (FGArgs::group_m, group_cols, xcd_interleave).  The 32 tiles an XCD runs at a time
// are group_m tile rows x 32 / group_m tile columns (or the other way round), and with
// xcd_interleave the 8 XCDs run 8 such rounds that follow one another in the order.  What the
// launches use, measured per product at the Llama-3 and Gemma-2 heads (launch times, one box,
// other settings as adopted):
//   logits  groups of 4 tile COLUMNS (4 panels of W, each visited in one stretch, against 8
//           panels of the chunk's X rows), interleaved: 5.84 ms; groups of 8 tile rows, not
//           interleaved (the order before): 6.02; 4 columns not interleaved 5.88; 8 columns 5.85;
//           16 columns 5.99; 2 rows 6.6; 1 row 7.7  (Gemma-2: 5.12 against 5.39 ms)
//   dX      groups of 4 tile rows, interleaved: 5.88 ms; not interleaved 5.94; 8 rows 5.91 / 5.98;
//           column groups no better
//   dW      groups of 4 tile rows, interleaved: 6.04 ms; not interleaved 6.13; 8 rows not
//           interleaved (the order before) 6.25; 16 rows 6.65; column groups no better
// The operands that are expensive to fetch (W in the logits product, the chunk of logit
// gradients read in column form in the dW product: 512-byte pieces 2 ldz bytes apart) want many
// CUs on the same panel at the same time and few visits of it over the launch.
constexpr int FG_GROUP_TILES = 4;
constexpr int FG_XCDS = 8;

struct FGArgs {
    const bf16_t* A;
    int64_t lda;
    const bf16_t* B;
    int64_t ldb;
    void* C;
    int64_t ldc;
    const void* Cin;    // optional addend, fp32 or bf16 (may alias C when of C's type)
    int64_t ldcin;
    int M, N, K;
    int tiles_m, tiles_n;
    int ksplit;            // K is cut into this many ranges (>= 1), one workgroup per tile and range
    int64_t split_stride;  // elements between the partial results of consecutive K ranges in C
    // Row count known on the device only (a chunk's number of non-ignored rows): when
    // dyn_rows is not null, min(*dyn_rows, static size) replaces M
    // (dyn_is_k = 0) or K (dyn_is_k = 1, column-form operands only).  The grid is
    // launched for the static size; workgroups of tiles past the dynamic M return at once.
    const int* dyn_rows;
    int dyn_is_k;
    // Number of K ranges known on the device only: when not null, *dyn_ksplit (at most
    // ksplit, which sizes the grid) replaces ksplit.
    const int* dyn_ksplit;
    // Chunk launches that may turn out empty: when first_live is not null, this launch
    // (number `launch`) returns at once if launch < *first_live, and the addend Cin is
    // taken as zero (not read) unless launch > *first_live.
    const int* first_live;
    int launch;
    // Tiles of the last, partly filled round cut along K (see tail_plan): from position
    // tail_begin of an XCD's tile span on, the next tail_r tiles are computed as tail_s K
    // ranges each by tail_r * tail_s workgroups, which write fp32 partial blocks of 256 x
    // 256 to tail_part; fg_tail_reduce_kernel adds them up and writes C.  tail_s <= 1: off.
    int tail_begin, tail_r, tail_s;
    float* tail_part;
    // Tile order: group_m tile rows at a time, column by column inside such a group (the 32
    // tiles an XCD runs at a time then share group_m A panels and 32 / group_m B panels).
    int group_m;
    // group_cols = 1: the same order with rows and columns exchanged (groups of group_m tile
    // COLUMNS, row by row inside a group): every B panel is then visited in one stretch.
    int group_cols;
    // xcd_interleave = 1: the full rounds of 32 tiles are dealt to the XCDs round-robin (round j
    // to XCD j % 8) instead of as one contiguous span per XCD, so that at any time the 8 XCDs
    // work on 256 consecutive tiles of the order: neighbours that share operand panels beyond
    // the XCDs' own L2s.  The last, partial round of every XCD is dealt as before.
    int xcd_interleave;
};

constexpr size_t FG_TAIL_BLOCK_FLOATS = (size_t)FG_BM * FG_BN;   // one fp32 partial block of a tail tile
static_assert(FG_TAIL_BLOCK_FLOATS * sizeof(float) == TAIL_BLOCK_BYTES && FG_XCDS == TAIL_XCDS, "planner and kernel agree on the tail blocks");

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) void* fg_lds_ptr;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t fg_make_rsrc(const void* base, uint32_t bytes) {
    // raw buffer, no stride: offsets >= bytes read as zero / are not written
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

// One GEMM operand: where its tiles come from in global memory, where they land
// in LDS, and how MFMA fragments (32 rows x 16 K, lane l = row l%32, K values
// 8*(l/32) .. +7) are read back.  KM = false: row form, KM = true: column form.
template <bool KM>
struct FgOperand {
    // The buffer descriptor covers the operand from K step kt_base on; the loads of K
    // step kt add (kt - kt_base) * kstep as scalar offset.  All offsets are 32-bit, so
    // the descriptor is moved forward every seg_steps K steps (a rarely taken uniform
    // branch; for most operands never), which lets operands be of any size.
    const unsigned char* base0;   // first byte of K step kt_base of this workgroup's tiles
    int64_t bytes;                // bytes from base0 to the end of the operand's valid range
    __amdgpu_buffer_rsrc_t rsrc;
    int kt_base, seg_steps;
    int off[8];   // per-lane byte offset of each of the 8 loads a wavefront issues per tile
    int kstep;    // bytes between consecutive K steps
    int rd[4];    // per-lane LDS byte offsets of the fragment reads

    // base/ld: the matrix; r0: first row (row form) or column (column form) of this
    // tile; extent: number of rows / columns of the matrix; sub: which 128-wide half
    // of the tile this wavefront multiplies.
    __device__ __forceinline__ void init(const bf16_t* base, int64_t ld, int r0, int extent, int K,
                                         int tid, int sub) {
        const int lane = tid & 63, wave = tid >> 6;
        const int ildb = (int)ld * 2;   // leading dimension in bytes
        if constexpr (!KM) {
            // a wavefront-wide load = 8 consecutive tile rows of 128 B; lane l owns the
            // physical position (row l/8, piece l%8) and fetches the logical piece
            // (l%8) ^ swizzle(row); wavefront w fills rows 8w..8w+7 of every 32-row group
            const int rows = min(FG_BM, extent - r0);
            base0 = reinterpret_cast<const unsigned char*>(base + (int64_t)r0 * ld);
            bytes = (int64_t)rows * ildb;
            const int ld_row = tid >> 3;
            const int piece = (tid & 7) ^ ((ld_row >> 1) & 7);
#pragma unroll
            for (int r = 0; r < 8; ++r) off[r] = (ld_row + 32 * r) * ildb + piece * 16;
            kstep = FG_BK * 2;
            const int frow = lane & 31, fhalf = lane >> 5, fsw = (frow >> 1) & 7;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                rd[kk] = (sub * 128 + frow) * 128 + ((((kk << 1) | fhalf) ^ fsw) << 4);
        } else {
            // a wavefront-wide load = 2 consecutive K rows of 512 B; load r of wavefront
            // w covers K rows 8r + 2w and 8r + 2w + 1; lane l owns the physical 16-byte
            // piece l%32 of row l/32 and fetches the logical 64-byte chunk
            // (piece / 4) ^ f(k), f(k) = k%4 + 4 * ((k/8) % 2)
            base0 = reinterpret_cast<const unsigned char*>(base + r0);
            bytes = ((int64_t)K * ld - r0) * 2;
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const int k = 8 * r + 2 * wave + (lane >> 5);
                const int f = (k & 3) | (((k >> 3) & 1) << 2);
                const int chunk = ((lane & 31) >> 2) ^ f;
                off[r] = k * ildb + chunk * 64 + (lane & 3) * 16;
            }
            kstep = FG_BK * ildb;
            // transposing read: group g = l/16 of the wavefront reads K rows
            // 8*(g/2) + {0..3} (+4 for the second read), columns 16*(g%2) + 0..15 of the
            // 32-wide fragment; source lane s = l%16 supplies row s/4, columns 4*(s%4)..+3
            const int g = lane >> 4, s = lane & 15;
            const int f = (s >> 2) | ((g >> 1) << 2);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                rd[i] = (8 * (g >> 1) + (s >> 2)) * 512 + (((sub * 4 + i) ^ f) * 64) + 32 * (g & 1) +
                        8 * (s & 3);
        }
    }

    __device__ __forceinline__ void make_rsrc() {
        const int64_t left = bytes < 0 ? 0 : (bytes > 0xFFFFFFFFll ? 0xFFFFFFFFll : bytes);
        rsrc = fg_make_rsrc(base0, (uint32_t)left);
    }
    // K step 0 of the loads below is K step k_begin of the matrix
    __device__ __forceinline__ void start_at(int k_begin) {
        base0 += (int64_t)k_begin * kstep;
        bytes -= (int64_t)k_begin * kstep;
        kt_base = 0;
        seg_steps = max(1, (1 << 30) / kstep);
        make_rsrc();
    }
    // call before the first load of K step kt (kt never decreases)
    __device__ __forceinline__ void before_step(int kt) {
        if (kt - kt_base >= seg_steps) {
            base0 += (int64_t)seg_steps * kstep;
            bytes -= (int64_t)seg_steps * kstep;
            kt_base += seg_steps;
            make_rsrc();
        }
    }

    // start the 8 loads of this wavefront for K step kt into ring slot `slot`
    __device__ __forceinline__ void load(unsigned char* smem, int slot, int kt, int uwave) {
        before_step(kt);
        const int soff = (kt - kt_base) * kstep;
        unsigned char* dst = smem + slot * FG_TILE_BYTES + uwave * 1024;
#pragma unroll
        for (int r = 0; r < 8; ++r)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (fg_lds_ptr)(dst + r * 4096), 16, off[r], soff,
                                                     0, 0);
    }

    // start one of the 8 loads of this wavefront for K step kt into ring slot `slot`
    __device__ __forceinline__ void load_one(unsigned char* smem, int slot, int kt, int uwave, int r) const {
        unsigned char* dst = smem + slot * FG_TILE_BYTES + uwave * 1024 + r * 4096;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (fg_lds_ptr)dst, 16, off[r], (kt - kt_base) * kstep,
                                                 0, 0);
    }
};

// Registers an in-flight fragment lands in.  The reads are asynchronous inline
// assembly: nothing may touch these registers until fg_wait has run.
template <bool KM> struct FgRaw;
template <> struct FgRaw<false> { bf16x8 v; };
template <> struct FgRaw<true> { s16x4 lo, hi; };

// Issue the LDS read(s) of fragment I (32-row block) of K sub-step KK; `slot_addr`
// is the LDS byte address of the ring slot.
template <int KK, int I>
__device__ __forceinline__ void fg_issue(FgRaw<false>& r, const FgOperand<false>& op, unsigned slot_addr) {
    const unsigned addr = slot_addr + (unsigned)op.rd[KK];
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r.v) : "v"(addr), "n"(I * 4096));
}
template <int KK, int I>
__device__ __forceinline__ void fg_issue(FgRaw<true>& r, const FgOperand<true>& op, unsigned slot_addr) {
    const unsigned addr = slot_addr + (unsigned)op.rd[I];
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r.lo) : "v"(addr), "n"(KK * 8192));
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r.hi) : "v"(addr), "n"(KK * 8192 + 2048));
}

// Wait until every LDS read issued so far has returned.  The registers are tied
// to the asm statements so that nothing that uses them is moved above the wait.
__device__ __forceinline__ void fg_tie(FgRaw<false> (&r)[4]) {
    asm volatile("" : "+v"(r[0].v), "+v"(r[1].v), "+v"(r[2].v), "+v"(r[3].v));
}
__device__ __forceinline__ void fg_tie(FgRaw<true> (&r)[4]) {
    asm volatile("" : "+v"(r[0].lo), "+v"(r[0].hi), "+v"(r[1].lo), "+v"(r[1].hi), "+v"(r[2].lo),
                 "+v"(r[2].hi), "+v"(r[3].lo), "+v"(r[3].hi));
}
template <bool AKM, bool BKM>
__device__ __forceinline__ void fg_wait(FgRaw<AKM> (&ra)[4], FgRaw<BKM> (&rb)[4]) {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    fg_tie(ra);
    fg_tie(rb);
}
__device__ __forceinline__ bf16x8 fg_value(const FgRaw<false>& r) { return r.v; }
__device__ __forceinline__ bf16x8 fg_value(const FgRaw<true>& r) {
    const s16x8 both = __builtin_shufflevector(r.lo, r.hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
}
__device__ __forceinline__ void fg_zero(FgRaw<false>& r) {
#pragma unroll
    for (int e = 0; e < 8; ++e) r.v[e] = (bf16_t)0.f;
}
__device__ __forceinline__ void fg_zero(FgRaw<true>& r) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        r.lo[e] = 0;
        r.hi[e] = 0;
    }
}

template <typename InT> struct FgInSize { static constexpr int value = (int)sizeof(InT); };
template <> struct FgInSize<void> { static constexpr int value = 4; };

// Writes a workgroup's 256 x 256 tile of fp32 accumulators out.  The MFMAs are fed the B
// fragment first and the A fragment second, so accumulator register g of lane l is ROW
// l%32, column 8*(g/4)+4*(l/32)+g%4 of its 32 x 32 tile: four consecutive columns per group
// of four registers.  Written straight from the registers, a store instruction would touch
// 32 different rows.  The memory pipe's cost is per instruction (about 9 cycles of the CU's
// address unit per wavefront-wide store, whatever it carries: measured), so the tile goes
// through LDS instead, which is free by then: each wavefront stages 32 rows x 128 columns of
// its 128 x 128 sub-tile as fp32 in its own LDS region, reads them back row-major, 16 bytes
// of output per lane (4 fp32 or 8 bf16 consecutive columns), adds the addend (loaded with
// the same wide, row-contiguous accesses, one pass ahead) and stores 16 bytes per lane: 16
// or 8 times fewer memory instructions, each writing whole row segments.  Loads and stores go
// through buffer descriptors that cover the tile's valid rows (rows past them are dropped by
// the range check).  OutT: element type of C; InT: of the addend (void: none).
template <typename OutT, typename InT>
struct FgOut {
    static constexpr bool HAS_IN = !std::is_void<InT>::value;
    static constexpr int IS = FgInSize<InT>::value;
    static constexpr int ES = (int)sizeof(OutT);
    static constexpr int EW = 16 / ES;                 // output elements per lane and access: 4 or 8
    static constexpr int LANES_PER_ROW = 128 / EW;     // 32 or 16
    static constexpr int ROWS_PER_ACCESS = 64 / LANES_PER_ROW;   // rows one wavefront-wide access covers: 2 or 4
    static constexpr int PITCH = 128 + 4;              // fp32 words per staged row: 16 lanes' 16-byte writes of one column group hit 64 different banks
    static constexpr int NACC = 32 / ROWS_PER_ACCESS;  // accesses per 32-row pass: 16 or 8
    static constexpr int INW = HAS_IN ? EW * IS / 4 : 1;   // dwords of addend per lane and access

    __amdgpu_buffer_rsrc_t rsrc_c, rsrc_in;
    int ldc, ldcin, uwm, colw, orow, ocol, lane_off, lane_off_in, frow, fhalf;
    bool col_ok;
    float* stage;
    // Two buffers: a pass's addend is requested one pass ahead, the first one before the last
    // MFMAs of the K loop, so that the memory latency (a few thousand cycles: the addend comes
    // from HBM) is not waited for in every pass.
    uint32_t old2[HAS_IN ? 2 : 1][NACC][INW];

    // c_tile / cin_tile: first element of the tile's first row (column 0 of the matrix);
    // rows: valid rows of the tile; col0: the tile's first column; n_cols: columns of the matrix
    // (written in groups of EW: its rows must be allocated up to n_cols rounded up to EW).
    __device__ __forceinline__ void init(void* c_tile, int ldc_, const void* cin_tile, int ldcin_, bool use_in,
                                         int rows, int col0, int n_cols, unsigned char* smem, int lane,
                                         int uwave, int uwm_, int uwn) {
        ldc = ldc_;
        ldcin = ldcin_;
        uwm = uwm_;
        frow = lane & 31;
        fhalf = lane >> 5;
        rsrc_c = fg_make_rsrc(c_tile, (uint32_t)rows * (uint32_t)ldc * (uint32_t)ES);
        rsrc_in = rsrc_c;
        if constexpr (HAS_IN)   // a range of zero bytes makes every addend load return zero without touching memory
            rsrc_in = fg_make_rsrc(cin_tile, use_in ? (uint32_t)rows * (uint32_t)ldcin * (uint32_t)IS : 0u);
        stage = reinterpret_cast<float*>(smem + uwave * (FG_LDS_BYTES / 4));   // 40 KB per wavefront
        // output mapping of the lane: row (inside a group of ROWS_PER_ACCESS) and first column
        orow = lane / LANES_PER_ROW;
        ocol = (lane % LANES_PER_ROW) * EW;
        colw = col0 + uwn * 128;                       // first column of the wavefront's sub-tile
        col_ok = colw + ocol < ((n_cols + EW - 1) / EW) * EW;
        lane_off = (orow * ldc + ocol) * ES;
        lane_off_in = (orow * ldcin + ocol) * IS;
    }

    // Addend of pass `pass` (rows 32 pass .. + 31 of the wavefront's sub-tile) into buffer B.
    template <int B>
    __device__ __forceinline__ void load_addend(int pass) {
        if constexpr (HAS_IN) {
            const int row0 = uwm * 128 + pass * 32;
#pragma unroll
            for (int k = 0; k < NACC; ++k) {
                const int soff = ((row0 + k * ROWS_PER_ACCESS) * ldcin + colw) * IS;
                if constexpr (INW == 4) {
                    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc_in, lane_off_in, soff, 0);
#pragma unroll
                    for (int e = 0; e < 4; ++e) old2[B][k][e] = v[e];
                } else if constexpr (INW == 8) {
                    const u32x4 v0 = __builtin_amdgcn_raw_buffer_load_b128(rsrc_in, lane_off_in, soff, 0);
                    const u32x4 v1 = __builtin_amdgcn_raw_buffer_load_b128(rsrc_in, lane_off_in + 16, soff, 0);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        old2[B][k][e] = v0[e];
                        old2[B][k][4 + e] = v1[e];
                    }
                } else {   // 8 bf16 = 4 dwords, or 4 bf16 = 2 dwords
                    static_assert(INW == 2, "addend width");
                    const auto v = __builtin_amdgcn_raw_buffer_load_b64(rsrc_in, lane_off_in, soff, 0);
                    old2[B][k][0] = v[0];
                    old2[B][k][1] = v[1];
                }
            }
        }
    }

    // The four passes; load_addend<0>(0) has been issued before.
    __device__ __forceinline__ void write(f32x16 (&acc)[4][4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {                          // pass: rows 32 i .. 32 i + 31 of the sub-tile
            const int row0 = uwm * 128 + i * 32;
            // the next pass's addend is requested before this pass is staged: it arrives while this
            // pass goes through LDS
            if (i == 0) load_addend<1>(1);
            if (i == 1) load_addend<0>(2);
            if (i == 2) load_addend<1>(3);
            uint32_t (&old)[NACC][INW] = old2[HAS_IN ? (i & 1) : 0];
            // stage the pass: the lane holds row frow and, per group of four registers, the four
            // consecutive columns 32 j + 8 (g/4) + 4 fhalf .. + 3: one 16-byte LDS write per group
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    // read the elements into scalars first: a bit_cast applied directly
                    // to an accumulator vector element is miscompiled by this toolchain
                    const float v0 = acc[i][j][4 * g4], v1 = acc[i][j][4 * g4 + 1], v2 = acc[i][j][4 * g4 + 2],
                                v3 = acc[i][j][4 * g4 + 3];
                    const f32x4 q = {v0, v1, v2, v3};
                    *reinterpret_cast<f32x4*>(stage + frow * PITCH + 32 * j + 8 * g4 + 4 * fhalf) = q;
                }
            // The region is private to the wavefront and LDS executes a wavefront's accesses in
            // order: no workgroup barrier is needed, only that the compiler keeps the order (a
            // barrier of the usual kind would also wait for the global stores of the previous
            // pass to be acknowledged: measured 1 000 cycles per pass).
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int k = 0; k < NACC; ++k) {
                const float* src = stage + (k * ROWS_PER_ACCESS + orow) * PITCH + ocol;
                float v[EW];
#pragma unroll
                for (int e = 0; e < EW; e += 4) {
                    const f32x4 q = *reinterpret_cast<const f32x4*>(src + e);
#pragma unroll
                    for (int u = 0; u < 4; ++u) v[e + u] = q[u];
                }
                if constexpr (HAS_IN) {
#pragma unroll
                    for (int e = 0; e < EW; ++e) {
                        if constexpr (IS == 4) v[e] += __uint_as_float(old[k][e]);
                        else v[e] += __uint_as_float((e & 1) ? (old[k][e >> 1] & 0xffff0000u) : (old[k][e >> 1] << 16));
                    }
                }
                const int soff = ((row0 + k * ROWS_PER_ACCESS) * ldc + colw) * ES;
                u32x4 out;
                if constexpr (ES == 4) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) out[e] = __float_as_uint(v[e]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const bf16x2 p2 = {from_f32<bf16_t>(v[2 * e]), from_f32<bf16_t>(v[2 * e + 1])};
                        out[e] = __builtin_bit_cast(uint32_t, p2);
                    }
                }
                if (col_ok) __builtin_amdgcn_raw_buffer_store_b128(out, rsrc_c, lane_off, soff, 0);
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // reads done before the next pass rewrites the region
        }
    }
};

// What a launch's device-side values resolve to (shared by the product kernel and the
// reduction of its tail blocks).
struct FgResolved {
    int M, K, ksplit;
    bool skip, use_in;
};
__device__ __forceinline__ FgResolved fg_resolve(const FGArgs& a, bool has_in) {
    FgResolved r{a.M, a.K, a.ksplit, false, has_in};
    if (a.first_live) {
        const int fl = *a.first_live;   // uniform: a scalar load
        r.skip = a.launch < fl;
        r.use_in = has_in && a.launch > fl;
    }
    if (a.dyn_rows) {
        const int n = *a.dyn_rows;
        if (a.dyn_is_k) r.K = min(r.K, n); else r.M = min(r.M, n);
    }
    if (a.dyn_ksplit) r.ksplit = min(r.ksplit, max(1, *a.dyn_ksplit));
    return r;
}

// Position in_xcd of XCD xcd's tile list -> number in the launch's tile sequence (see
// FGArgs::xcd_interleave and xcd_tile_number).
__device__ __forceinline__ int fg_seq(const FGArgs& a, int xcd, int in_xcd, int per_xcd) {
    return a.xcd_interleave ? xcd_tile_number(xcd, in_xcd, per_xcd) : xcd * per_xcd + in_xcd;
}

// Tile number `seq` of the grouped order (group_m tile rows at a time, column by column
// inside a group) -> first row and column of the tile.
__device__ __forceinline__ void fg_tile_origin(int seq, int tiles_m, int tiles_n, int group_m, int group_cols,
                                               int& m0, int& n0) {
    // (rows and columns change places for the column-grouped order)
    const int major = group_cols ? tiles_n : tiles_m, minor = group_cols ? tiles_m : tiles_n;
    const int group_size = group_m * minor;
    const int grp = seq / group_size;
    const int first = grp * group_m;
    const int g = min(group_m, major - first);
    const int rem = seq - grp * group_size;
    const int in_major = first + rem % g, in_minor = rem / g;
    m0 = (group_cols ? in_minor : in_major) * FG_BM;
    n0 = (group_cols ? in_major : in_minor) * FG_BN;
}


// InT: element type of the addend Cin (float or bf16_t), void for no addend.
template <typename OutT, typename InT, bool A_KM, bool B_KM>
__global__ __launch_bounds__(FG_THREADS) void gemm_bf16_256(FGArgs a) {
    constexpr bool HAS_IN = !std::is_void<InT>::value;
    constexpr int IS = FgInSize<InT>::value;
    __shared__ __attribute__((aligned(16))) unsigned char smem[FG_LDS_BYTES];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // ---- workgroup id -> (K range, tile) (XCD aware, grouped order) ----
    const FgResolved rs = fg_resolve(a, HAS_IN);
    if (rs.skip) return;
    const int M = rs.M, K = rs.K, ksplit = rs.ksplit;
    const bool use_in = rs.use_in;
    // The tile sequence covers the live rows only (a dynamic M can be smaller than the M the
    // grid was sized for): the live tiles are dealt evenly to the XCDs, and the workgroups
    // that are left over have the highest ids, are dispatched last and return at once.
    const int tiles_m = (M + FG_BM - 1) / FG_BM;
    const int tiles = tiles_m * a.tiles_n;
    const int total = tiles * ksplit;
    const int per_xcd = (total + FG_XCDS - 1) / FG_XCDS;
    const int xcd = (int)blockIdx.x % FG_XCDS;
    int in_xcd = (int)blockIdx.x / FG_XCDS;
    // a tile of the last round that is cut along K: range tail_i of tail_n, partial block tail_blk
    int tail_i = 0, tail_n = 1, tail_blk = 0;
    if (a.tail_s > 1 && in_xcd >= a.tail_begin) {
        const int u = in_xcd - a.tail_begin;
        if (u >= a.tail_r * a.tail_s) return;
        const int slot = u % a.tail_r;
        in_xcd = a.tail_begin + slot;
        tail_i = u / a.tail_r;
        tail_n = a.tail_s;
        tail_blk = (xcd * a.tail_r + slot) * a.tail_s + tail_i;
    }
    if (in_xcd >= per_xcd) return;
    const int seq_all = fg_seq(a, xcd, in_xcd, per_xcd);
    if (seq_all >= total) return;
    const int split = seq_all / tiles;
    int m0, n0;
    fg_tile_origin(seq_all - split * tiles, tiles_m, a.tiles_n, a.group_m, a.group_cols, m0, n0);

    FgOperand<A_KM> opa;
    FgOperand<B_KM> opb;
    opa.init(a.A, a.lda, m0, M, K, tid, wm);
    opb.init(a.B, a.ldb, n0, a.N, K, tid, wn);
    const int uwave = __builtin_amdgcn_readfirstlane(wave);

    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int g = 0; g < 16; ++g) acc[i][j][g] = 0.f;

    // two register buffers of in-flight fragments (4 of A, 4 of B each)
    FgRaw<A_KM> raw_a[2][4];
    FgRaw<B_KM> raw_b[2][4];

    // Workgroup barrier of the pipeline.  Loads complete in order and every
    // wavefront issues 8 per slot, so "at most 8 outstanding" means everything
    // but the youngest slot (the A tile two steps ahead) has landed.  All LDS
    // reads of the step are complete as well, so its two slots can be refilled.
    auto pipeline_barrier = [&]() {
        asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    };

    // One quarter of a K step: the 16 MFMAs of one K=16 sub-step on the fragments in
    // register buffer MB, interleaved with the 8 fragment reads of sub-step KK of the
    // tile in slots (SA, SB) into buffer 1-MB (one fragment per MFMA, in the order
    // a0 b0 b1 b2 b3 a1 a2 a3 in which the next quarter consumes them), and with 4 of
    // the 16 loads of the step, one behind every fourth MFMA (DMA = 1: loads R0..R0+3
    // of the B tile of step kt into slot SD, DMA = 2: of the A tile).  Loads issued in
    // bursts fill the memory pipe's queue and stall the wavefront, and with it the
    // matrix pipe: measured 500 extra cycles for 8 back-to-back loads.
    auto quarter = [&](auto mb_, auto kk_, auto sa_, auto sb_, auto dma_, auto sd_, auto r0_, int kt) {
        constexpr int MB = decltype(mb_)::value, RB = 1 - MB, KK = decltype(kk_)::value;
        constexpr int SA = decltype(sa_)::value, SB = decltype(sb_)::value;
        constexpr int DMA = decltype(dma_)::value, SD = decltype(sd_)::value, R0 = decltype(r0_)::value;
        if constexpr (DMA == 1 && R0 == 0) opb.before_step(kt);
        if constexpr (DMA == 2 && R0 == 0) opa.before_step(kt);
        fg_wait(raw_a[MB], raw_b[MB]);
        bf16x8 fa[4], fb[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            fa[i] = fg_value(raw_a[MB][i]);
            fb[i] = fg_value(raw_b[MB][i]);
        }
        const unsigned sa_addr = lds0 + SA * FG_TILE_BYTES, sb_addr = lds0 + SB * FG_TILE_BYTES;
        __builtin_amdgcn_sched_barrier(0);
#define FG_MFMA(q) \
        acc[(q) >> 2][(q) & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[(q) & 3], fa[(q) >> 2], acc[(q) >> 2][(q) & 3], 0, 0, 0)
#define FG_DMA(n)                                                          \
        if constexpr (DMA == 1) opb.load_one(smem, SD, kt, uwave, R0 + (n));   \
        if constexpr (DMA == 2) opa.load_one(smem, SD, kt, uwave, R0 + (n))
#define FG_END __builtin_amdgcn_sched_barrier(0)
        FG_MFMA(0);  fg_issue<KK, 0>(raw_a[RB][0], opa, sa_addr); FG_END;
        FG_MFMA(1);  fg_issue<KK, 0>(raw_b[RB][0], opb, sb_addr); FG_END;
        FG_MFMA(2);  fg_issue<KK, 1>(raw_b[RB][1], opb, sb_addr); FG_DMA(0); FG_END;
        FG_MFMA(3);  fg_issue<KK, 2>(raw_b[RB][2], opb, sb_addr); FG_END;
        FG_MFMA(4);  fg_issue<KK, 3>(raw_b[RB][3], opb, sb_addr); FG_END;
        FG_MFMA(5);  fg_issue<KK, 1>(raw_a[RB][1], opa, sa_addr); FG_END;
        FG_MFMA(6);  fg_issue<KK, 2>(raw_a[RB][2], opa, sa_addr); FG_DMA(1); FG_END;
        FG_MFMA(7);  fg_issue<KK, 3>(raw_a[RB][3], opa, sa_addr); FG_END;
        FG_MFMA(8);  FG_END;
        FG_MFMA(9);  FG_END;
        FG_MFMA(10); FG_DMA(2); FG_END;
        FG_MFMA(11); FG_END;
        FG_MFMA(12); FG_END;
        FG_MFMA(13); FG_END;
        FG_MFMA(14); FG_DMA(3); FG_END;
        FG_MFMA(15); FG_END;
#undef FG_MFMA
#undef FG_DMA
#undef FG_END
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    using I3 = std::integral_constant<int, 3>;

    // One K step.  PH = t % 5 fixes the slots: A(t) in (2 PH) % 5, B(t) in
    // (2 PH + 1) % 5; B(t+1) refills the slot A(t-1) left, A(t+2) the slot B(t-1)
    // left.  The fourth K=16 sub-step of a tile is multiplied in the first quarter
    // of the next step, behind the barrier, while the new fragments arrive.  Tiles
    // past the end are loaded but never consumed (the descriptor returns zeros
    // past its range), which keeps the steady state free of branches.
    auto step = [&](auto phase, int t) {
        constexpr int PH = decltype(phase)::value;
        using SA = std::integral_constant<int, (2 * PH) % 5>;
        using SB = std::integral_constant<int, (2 * PH + 1) % 5>;
        using SB1 = std::integral_constant<int, (2 * PH + 3) % 5>;
        using SA2 = std::integral_constant<int, (2 * PH + 4) % 5>;
        using I4 = std::integral_constant<int, 4>;
        quarter(I1{}, I0{}, SA{}, SB{}, I1{}, SB1{}, I0{}, t + 1);   // MFMA: sub-step 3 of tile t-1
        quarter(I0{}, I1{}, SA{}, SB{}, I1{}, SB1{}, I4{}, t + 1);   // MFMA: sub-step 0
        quarter(I1{}, I2{}, SA{}, SB{}, I2{}, SA2{}, I0{}, t + 2);   // MFMA: sub-step 1
        quarter(I0{}, I3{}, SA{}, SB{}, I2{}, SA2{}, I4{}, t + 2);   // MFMA: sub-step 2
        pipeline_barrier();
    };

    // K steps [k_begin, k_begin + nk) belong to this workgroup
    const int steps_all = (K + FG_BK - 1) / FG_BK;
    // (a launch cut into K ranges as a whole, ksplit > 1, has no tail ranges: tail_n = 1)
    const int kr_i = tail_n > 1 ? tail_i : split, kr_n = tail_n > 1 ? tail_n : ksplit;
    const int k_begin = (int)((int64_t)steps_all * kr_i / kr_n);
    const int nk = (int)((int64_t)steps_all * (kr_i + 1) / kr_n) - k_begin;
    opa.start_at(k_begin);
    opb.start_at(k_begin);
    opa.load(smem, 0, 0, uwave);
    opb.load(smem, 1, 0, uwave);
    opa.load(smem, 2, 1, uwave);
#pragma unroll
    for (int i = 0; i < 4; ++i) {        // the first step has no previous sub-step: add zero
        fg_zero(raw_a[1][i]);
        fg_zero(raw_b[1][i]);
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
    // Where the tile goes: to C (plus addend), or, for a K range of a tail tile, to its fp32
    // partial block (256 x 256, dense).  The first addend slice is requested before the last
    // MFMAs.
    const int uwm = __builtin_amdgcn_readfirstlane(wm), uwn = __builtin_amdgcn_readfirstlane(wn);
    FgOut<OutT, InT> out;
    FgOut<float, void> part;
    if (tail_n > 1) {
        part.init(a.tail_part + (size_t)tail_blk * FG_TAIL_BLOCK_FLOATS, FG_BN, nullptr, 0, false, FG_BM, 0, FG_BN,
                  smem, lane, uwave, uwm, uwn);
    } else {
        out.init(static_cast<OutT*>(a.C) + (int64_t)split * a.split_stride + (int64_t)m0 * a.ldc, (int)a.ldc,
                 HAS_IN ? static_cast<const unsigned char*>(a.Cin) + (int64_t)m0 * a.ldcin * IS : nullptr,
                 (int)a.ldcin, use_in, min(FG_BM, M - m0), n0, a.N, smem, lane, uwave, uwm, uwn);
        out.template load_addend<0>(0);
    }
    {   // sub-step 3 of the last tile
        fg_wait(raw_a[1], raw_b[1]);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    fg_value(raw_b[1][j]), fg_value(raw_a[1][i]), acc[i][j], 0, 0, 0);
    }
    // The loads of the tiles past the end still target LDS: let them land, for every
    // wavefront of the workgroup, before LDS is reused below (and before the workgroup can
    // retire and its LDS be handed to another one).
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");

    // ---- epilogue (see FgOut) ----
    if (tail_n > 1) part.write(acc); else out.write(acc);
}

// Second step of a launch whose last round was cut along K: adds the tail_s fp32 partial
// blocks of every tail tile in the fixed order 0, 1, ..., adds the addend, and writes the
// tile to C.  Same arguments as the product launch; grid = FG_XCDS * tail_r tiles x 8
// slabs of 32 rows, 256 threads: a thread owns 4 consecutive columns of 4 rows of its slab.
template <typename OutT, typename InT>
__global__ __launch_bounds__(256) void fg_tail_reduce_kernel(FGArgs a) {
    constexpr bool HAS_IN = !std::is_void<InT>::value;
    const FgResolved rs = fg_resolve(a, HAS_IN);
    if (rs.skip || a.tail_s <= 1) return;
    const int tiles_m = (rs.M + FG_BM - 1) / FG_BM;
    const int tiles = tiles_m * a.tiles_n;            // launches with tail ranges have ksplit = 1
    const int per_xcd = (tiles + FG_XCDS - 1) / FG_XCDS;
    const int tile_id = (int)blockIdx.x / 8, slab = (int)blockIdx.x % 8;
    const int xcd = tile_id / a.tail_r, slot = tile_id % a.tail_r;
    const int in_xcd = a.tail_begin + slot;
    if (in_xcd >= per_xcd) return;
    const int seq = fg_seq(a, xcd, in_xcd, per_xcd);
    if (seq >= tiles) return;
    int m0, n0;
    fg_tile_origin(seq, tiles_m, a.tiles_n, a.group_m, a.group_cols, m0, n0);
    const float* blk = a.tail_part + (size_t)((xcd * a.tail_r + slot) * a.tail_s) * FG_TAIL_BLOCK_FLOATS;
    const int c4 = ((int)threadIdx.x % 64) * 4;       // first of the thread's 4 columns inside the tile
    const int col = n0 + c4;
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        const int r = slab * 32 + p * 4 + (int)threadIdx.x / 64;   // row inside the tile
        const int row = m0 + r;
        if (row >= rs.M || col >= a.N) continue;
        f32x4 v = *reinterpret_cast<const f32x4*>(blk + (size_t)r * FG_BN + c4);
        for (int t = 1; t < a.tail_s; ++t)
            v += *reinterpret_cast<const f32x4*>(blk + (size_t)t * FG_TAIL_BLOCK_FLOATS + (size_t)r * FG_BN + c4);
        OutT* dst = static_cast<OutT*>(a.C) + (int64_t)row * a.ldc + col;
        if constexpr (HAS_IN) {
            if (rs.use_in) {
                const InT* src = static_cast<const InT*>(a.Cin) + (int64_t)row * a.ldcin + col;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (col + e < a.N) v[e] += to_f32(src[e]);
            }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (col + e < a.N) dst[e] = from_f32<OutT>(v[e]);
    }
}

}  // namespace flce
