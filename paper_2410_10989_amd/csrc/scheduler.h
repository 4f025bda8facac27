// Host-side chunk scheduler and workspace layout.  Pure integer arithmetic, no
// HIP calls, so it can be exercised on a machine without a GPU.
//
// The method bounds memory by projecting only a chunk of C rows at a time
// (paper section 3.2, FLCE paragraph).  Here C is set by a byte budget for the
// chunk's logits instead of the paper's power-of-two rule: on this chip each
// chunk re-reads W twice and read-modify-writes the fp32 dW accumulator, so C
// has to stay in the thousands for the products to remain compute bound.
#pragma once
#include <stddef.h>
#include <stdint.h>

#include <algorithm>

#if defined(__HIPCC__)
#define FLCE_HD __host__ __device__
#else
#define FLCE_HD
#endif

namespace flce {

constexpr int64_t CHUNK_ALIGN = 256;   // chunk rows are a multiple of the GEMM macro tile

// A launch of one workgroup per 256 x 256 tile runs in rounds of as many tiles as the chip
// has CUs (one tile per CU at a time: a tile takes the whole LDS), dealt to the 8 XCDs in
// equal spans.  When the last round holds only r <= 16 tiles per XCD, half or more of the
// CUs would idle through it, so each of those tiles is cut into s = 32 / r K ranges instead
// (at most 8, each at least 16 K steps long): the round takes 1 / s of a tile's time plus a
// small reduction of fp32 partial blocks.  s = 1: the launch is left as it is.  `total` =
// tiles of the launch, ksteps = K steps (of 64) per tile; begin = position inside an XCD's
// span of its first tail tile.
constexpr int TAIL_XCDS = 8, TAIL_CUS_PER_XCD = 32;
constexpr size_t TAIL_BLOCK_BYTES = (size_t)256 * 256 * sizeof(float);
struct TailPlan {
    int begin, r, s;
};
inline TailPlan tail_plan(int64_t total, int64_t ksteps) {
    TailPlan t{0, 0, 1};
    const int64_t per_xcd = (total + TAIL_XCDS - 1) / TAIL_XCDS;
    const int r = (int)(per_xcd % TAIL_CUS_PER_XCD);
    if (per_xcd < TAIL_CUS_PER_XCD || r == 0 || r > TAIL_CUS_PER_XCD / 2) return t;
    int s = TAIL_CUS_PER_XCD / r;
    if (s > 8) s = 8;
    while (s > 1 && ksteps / s < 16) --s;
    if (s <= 1) return t;
    t.begin = (int)(per_xcd - r);
    t.r = r;
    t.s = s;
    return t;
}
// How a launch's tiles, numbered 0 .. total-1 in its tile order, are dealt to the 8 XCDs
// (workgroup id % 8 is the XCD, id / 8 the position in_xcd in that XCD's list of
// per_xcd = ceil(total / 8) = 32 F + r tiles): the 8 F full rounds of 32 consecutive numbers
// go round-robin (round j to XCD j % 8, so that at any time the XCDs work on 256 consecutive
// tiles), the numbers from 256 F on, at most r per XCD, are dealt in 8 runs of r: these are the
// tiles tail_plan cuts.  Numbers >= total (the last XCDs' lists can be short) mean "no tile".
FLCE_HD inline int xcd_tile_number(int xcd, int in_xcd, int per_xcd) {
    const int full = per_xcd / TAIL_CUS_PER_XCD * TAIL_CUS_PER_XCD;   // 32 F
    if (in_xcd < full)
        return ((in_xcd / TAIL_CUS_PER_XCD) * TAIL_XCDS + xcd) * TAIL_CUS_PER_XCD + in_xcd % TAIL_CUS_PER_XCD;
    return full * TAIL_XCDS + xcd * (per_xcd - full) + (in_xcd - full);
}
// bytes of partial blocks such a launch needs (0 when it is not cut)
inline size_t tail_partial_bytes(int64_t total, int64_t ksteps) {
    const TailPlan t = tail_plan(total, ksteps);
    return t.s > 1 ? (size_t)TAIL_XCDS * t.r * t.s * TAIL_BLOCK_BYTES : 0;
}

inline int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }
inline size_t elem_size(int dtype) { return dtype == 0 ? 4 : 2; }

struct Plan {
    int64_t C = 0;         // rows per chunk (last chunk may hold fewer)
    int64_t nchunks = 0;
    int64_t ldz = 0;       // row stride of the logits chunk, elements
    int64_t ldc = 0;       // row stride of the row-transposed scratch, elements
    bool fp32_dw_acc = false;   // dW is accumulated in an fp32 scratch across chunks
    // which products can run on the tuned bf16 kernel straight from X, W and the
    // logits chunk; the others need transposed copies and the guarded kernel
    bool fast_logits = false, fast_dx = false, fast_dw_full = false, fast_dw_last = false;
    int dx_ksplit = 1;     // K ranges of the dX product (K = V), > 1 when C x H has few tiles
    // every product of every chunk runs on the tuned kernel: chunks are compacted, i.e.
    // rows with an ignored target are left out of the products (see compact.h)
    bool compact = false;
    // byte offsets into the workspace
    size_t off_hdr = 0, off_row_loss = 0, off_z = 0, off_gt = 0, off_wt = 0, off_xt = 0,
           off_dwacc = 0, off_dxpart = 0, off_xg = 0, off_dxg = 0, off_idx = 0, off_tv = 0,
           off_dyn = 0, off_tail = 0, total = 0;
    size_t tail_bytes = 0;   // room at off_tail
};

// How many K ranges to cut a product with `tiles` output tiles and `ksteps` K steps
// into, so that tiles * ranges fills whole rounds of the chip's 256 CUs (one tile per
// CU at a time).  288 tiles, for example, run as two rounds at 56 % occupancy; cut
// into 8 ranges they are 9 full rounds.  Prefers few ranges (each costs an fp32
// partial result: a larger count must fill the rounds better by more than 2 % of the
// chip, and more than 8 are only taken while they fill a first round) and keeps ranges
// at least 64 K steps long; with many rounds the tail does not
// matter and the answer is 1.  Integer arithmetic only: the host and the device (which
// knows the live row count of a compacted chunk) must agree on the answer.
FLCE_HD inline int choose_ksplit(int64_t tiles, int64_t ksteps, int max_ranges) {
    constexpr int64_t CUS = 256, MIN_STEPS = 64;
    int best = 1;
    int64_t best_work = 0, best_rounded = 1;   // occupancy of the best choice = best_work / best_rounded
    for (int s = 1; s <= 16 && s <= max_ranges && ksteps / s >= MIN_STEPS; ++s) {
        const int64_t work = tiles * s;
        if (s > 8 && work > CUS) break;   // more than 8 ranges only to fill a first round
        const int64_t rounded = ((work + CUS - 1) / CUS) * CUS;
        // work / rounded > best_work / best_rounded + 1/50
        if (rounded > 0 && 50 * work * best_rounded > (50 * best_work + best_rounded) * rounded) {
            best_work = work;
            best_rounded = rounded;
            best = s;
        }
    }
    return best;
}

// The fp32 partial results of a cut dX product (ranges x rows x H) may take half as much
// memory as the logits chunk, not more.
inline int max_dx_ranges(size_t budget_bytes, int64_t rows, int64_t H) {
    const size_t one = (size_t)rows * (size_t)H * sizeof(float);
    const size_t n = one ? budget_bytes / 2 / one : 1;
    return (int)std::max<size_t>(1, std::min<size_t>(n, 16));
}

// K ranges of the dX product (rows x H output, K = V).  The tuned kernel works on
// 256 x 256 tiles and K steps of 64; the guarded kernel on 128 x 128 tiles, where a
// range is at least 256 elements long.
inline int dx_ranges(bool tuned, int64_t rows, int64_t H, int64_t V, size_t budget_bytes) {
    if (tuned)
        return choose_ksplit(((rows + 255) / 256) * ((H + 255) / 256), (V + 63) / 64,
                             max_dx_ranges(budget_bytes, round_up(rows, 256), H));
    return choose_ksplit(((rows + 127) / 128) * ((H + 127) / 128), V / 4,
                         max_dx_ranges(budget_bytes, round_up(rows, 128), H));
}

// Limits of the tuned kernel's 32-bit offsets inside one tile (see gemm_bf16_nt.h).
inline bool fits_row_form(int64_t ld, int64_t) { return 256 * ld * 2 + 128 < ((int64_t)1 << 30); }
inline bool fits_col_form(int64_t ld, int64_t) { return 64 * ld * 2 + 512 < ((int64_t)1 << 30); }

// Byte offsets of the workspace for a plan whose chunking (C, nchunks, rows of the last
// chunk) is decided; `dxpart_floor` is a lower bound for the K-range partials.
inline void lay_out(Plan& p, int64_t H, int64_t V, int dtype, int64_t rows_last, size_t budget_bytes,
                    bool allow_compact, size_t dxpart_floor) {
    const size_t es = elem_size(dtype);
    p.ldc = round_up(p.C, 64);
    p.fp32_dw_acc = (dtype != 0) && p.nchunks > 1;
    p.fast_logits = p.fast_dx = p.fast_dw_full = p.fast_dw_last = false;
    if (dtype != 0) {
        const bool out_ok = 256 * H * 4 < ((int64_t)1 << 31);
        p.fast_logits = (H % 64 == 0) && fits_row_form(H, H) && 256 * p.ldz * 2 < ((int64_t)1 << 31);
        // K of the dX product is V: the dlogits rows are padded with zeros to ldz, W is read
        // K-major; K of the dW product is the chunk's row count, both operands K-major: any
        // V and any row count do
        p.fast_dx = (H % 8 == 0) && fits_row_form(p.ldz, V) && fits_col_form(H, V) && out_ok;
        auto dw_ok = [&](int64_t rows) {
            return (H % 8 == 0) && fits_col_form(p.ldz, rows) && fits_col_form(H, rows) && out_ok;
        };
        p.fast_dw_full = (p.nchunks > 1) ? dw_ok(p.C) : dw_ok(rows_last);
        p.fast_dw_last = dw_ok(rows_last);
    }
    {
        const int64_t rows = p.nchunks > 1 ? p.C : rows_last;
        p.dx_ksplit = dx_ranges(p.fast_dx, rows, H, V, budget_bytes);
    }
    p.compact = allow_compact && p.fast_logits && p.fast_dx && p.fast_dw_full && p.fast_dw_last;
    const bool need_wt = !p.fast_dx;
    const bool need_gt = !(p.fast_dw_full && p.fast_dw_last);

    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += (bytes + 255) / 256 * 256;
        return at;
    };
    p.off_hdr = take(256);
    p.off_row_loss = take((size_t)p.C * sizeof(float));
    p.off_z = take((size_t)p.C * p.ldz * es);
    p.off_gt = take(need_gt ? (size_t)V * p.ldc * es : 0);
    p.off_wt = take(need_wt ? (size_t)H * p.ldz * es : 0);
    p.off_xt = take(need_gt ? (size_t)H * p.ldc * es : 0);
    p.off_dwacc = take(p.fp32_dw_acc ? (size_t)V * H * sizeof(float) : 0);
    const size_t dxpart = p.dx_ksplit > 1 ? (size_t)p.dx_ksplit * p.C * H * sizeof(float) : 0;
    p.off_dxpart = take(std::max(dxpart, dxpart_floor));
    // a chunk of gathered input rows and of their gradient (also the normalised rows and
    // their gradient when an RMSNorm runs in front), index maps of the compaction
    p.off_xg = take((size_t)p.C * H * es);
    p.off_dxg = take((size_t)p.C * H * es);
    p.off_idx = take(p.compact ? (size_t)p.C * sizeof(int32_t) : 0);
    p.off_tv = take(p.compact ? (size_t)p.C * sizeof(int64_t) : 0);
    p.off_dyn = take(256);
    // fp32 partial blocks of the dW product's last, partly filled round of tiles when it is cut
    // along K (tail_plan; a shorter last chunk has fewer K steps and never needs more)
    const int64_t dw_tiles = ((V + 255) / 256) * ((H + 255) / 256);
    p.tail_bytes = (p.fast_dw_full && p.fast_dw_last) ? tail_partial_bytes(dw_tiles, (p.C + 63) / 64) : 0;
    p.off_tail = take(p.tail_bytes);
    p.total = off;
}

// budget_bytes bounds one chunk of logits.  A batch whose WHOLE logits fit in
// single_bytes (>= budget_bytes) runs as one chunk whatever the budget says: the
// automatic rule passes the chunk budget plus the size of the fp32 dW partial sums,
// which only several chunks need, so that one chunk is taken whenever it needs no more
// memory than the chunked plan would (and it is always faster: no second pass over W,
// no fp32 round trip of dW).  worst_case_bt: the plan with the largest workspace any BT
// can lead to (BT is ignored).
inline Plan make_plan(int64_t BT, int64_t H, int64_t V, int dtype, size_t budget_bytes,
                      bool worst_case_bt = false, bool allow_compact = true, size_t single_bytes = 0) {
    Plan p;
    const size_t es = elem_size(dtype);
    p.ldz = round_up(V, 64);
    const size_t row_bytes = (size_t)p.ldz * es;
    int64_t cmax = (int64_t)(budget_bytes / row_bytes);
    cmax = cmax / CHUNK_ALIGN * CHUNK_ALIGN;
    if (cmax < CHUNK_ALIGN) cmax = CHUNK_ALIGN;
    const int64_t single_max = std::max<int64_t>(cmax, (int64_t)(single_bytes / row_bytes));   // rows
    if (worst_case_bt) {
        // the bound has to hold for every chunk size the scheduler can pick: the number of
        // K ranges of the dX product depends on the row count through its tile count
        auto dxpart_over = [&](bool tuned, int64_t upto) {
            size_t m = 0;
            for (int64_t c = 128; c <= upto; c += 128) {
                const int ks = dx_ranges(tuned, c, H, V, budget_bytes);
                if (ks > 1) m = std::max(m, (size_t)ks * c * H * sizeof(float));
            }
            return m;
        };
        // several chunks, the last one ragged (the most expensive case) ...
        p.C = cmax;
        p.nchunks = 2;
        lay_out(p, H, V, dtype, 1, budget_bytes, allow_compact, 0);
        lay_out(p, H, V, dtype, 1, budget_bytes, allow_compact, dxpart_over(p.fast_dx, cmax));
        // ... or the largest batch that still runs as one chunk
        Plan q;
        q.ldz = p.ldz;
        q.C = single_max;
        q.nchunks = 1;
        lay_out(q, H, V, dtype, single_max, budget_bytes, allow_compact, 0);
        lay_out(q, H, V, dtype, single_max, budget_bytes, allow_compact, dxpart_over(q.fast_dx, single_max));
        return q.total > p.total ? q : p;
    }
    int64_t rows_last;
    if (BT <= single_max) {
        p.C = BT;
        p.nchunks = 1;
        rows_last = BT;
    } else {
        p.nchunks = (BT + cmax - 1) / cmax;
        p.C = round_up((BT + p.nchunks - 1) / p.nchunks, CHUNK_ALIGN);   // even out the chunks
        p.nchunks = (BT + p.C - 1) / p.C;
        rows_last = BT - (p.nchunks - 1) * p.C;
    }
    lay_out(p, H, V, dtype, rows_last, budget_bytes, allow_compact, 0);
    return p;
}

// Paper's rule: chunk = 2^ceil(log2(ceil(BT / ceil(V / H)))).
inline int64_t paper_chunk_rows(int64_t BT, int64_t H, int64_t V) {
    const int64_t inc = (V + H - 1) / H;
    const int64_t c = (BT + inc - 1) / inc;
    int64_t p2 = 1;
    while (p2 < c) p2 <<= 1;
    return p2;
}

}  // namespace flce
