// C ABI of the fused linear cross-entropy library for gfx950: argument checks,
// chunk loop, workspace handling, kernel launches.  Declarations and the
// meaning of every argument are in include/flce.h.
#include <hip/hip_runtime.h>
#include <atomic>
#include <mutex>
#include <vector>

#include "../../include/flce.h"
#include "compact.h"
#include "flce_device.h"
#include "gemm_bf16_nt.h"
#include "gemm_generic.h"
#include "mfma_ceiling.h"
#include "misc_kernels.h"
#include "rmsnorm.h"
#include "rowreduce.h"
#include "scheduler.h"

using namespace flce;

// Scratch of flce_cross_entropy_inplace_noalloc: the device header and one loss per
// row, in the image of the code object instead of allocated memory.  Every GPU the
// library runs on holds its own copy at its own address until the process ends.  In
// host code this name is only a handle for hipGetSymbolAddress, never an address.
constexpr size_t CE_NOALLOC_BYTES = 256 + (size_t)FLCE_CE_NOALLOC_MAX_ROWS * sizeof(float);
static __device__ __align__(256) unsigned char scratch[CE_NOALLOC_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
constexpr int64_t MAX_DIM = (int64_t)1 << 30;      // per-dimension limit, keeps int tile math safe
constexpr int64_t CE_ROWS_PER_LAUNCH = 65536;
constexpr int64_t MAX_GRID_X = 0x7fffffff;        // workgroups along grid x
constexpr size_t AUTO_BUDGET_BYTES = (size_t)1 << 30;
constexpr int64_t AUTO_BUDGET_MIN_ROWS = 4096;

struct DeviceWorkspace {
    void* lent = nullptr;
    size_t lent_bytes = 0;
    void* own = nullptr;
    size_t own_bytes = 0;
};

std::mutex g_mutex;
DeviceWorkspace g_ws[MAX_DEVICES];
void* g_scratch_ptr[MAX_DEVICES] = {};   // device address of `scratch` on each device, once looked up
// Process-wide settings: read by every call, written by the setters (any thread).
std::atomic<size_t> g_budget{0};   // 0 = the automatic rule of effective_budget()
std::atomic<bool> g_compact{true};

// What a call's plan depends on besides the shape: the process-wide settings, or the
// options a caller passes with the call.
struct Settings {
    size_t budget;   // 0 = the automatic rule
    bool compact;
    void* ws = nullptr;   // the call's own workspace (flce_options), null = the device's shared one
    size_t ws_bytes = 0;
};
Settings global_settings() { return {g_budget.load(), g_compact.load()}; }

// The byte budget of the logits chunk: what the caller set, or by default 1 GiB but at
// least 4096 rows of logits.  Every chunk costs one more pass over W and an fp32
// read-modify-write of the dW partial sums (16 V H bytes) whatever its row count, which
// is about 433 / C of the chunk's product time on this chip: 10 % at 4096 rows.
size_t effective_budget(const Settings& st, int64_t V, int dtype) {
    if (st.budget) return st.budget;
    const size_t rows_bytes = (size_t)AUTO_BUDGET_MIN_ROWS * (size_t)round_up(V, 64) * elem_size(dtype);
    return rows_bytes > AUTO_BUDGET_BYTES ? rows_bytes : AUTO_BUDGET_BYTES;
}

// Up to how many bytes of logits a batch runs as ONE chunk.  With an explicit budget:
// the budget.  Automatic rule: the chunk budget plus the fp32 dW partial sums that only
// a chunked run needs (bf16 storage), i.e. one chunk whenever that takes no more memory
// than chunking would; it is also the faster plan.
size_t single_chunk_bytes(const Settings& st, int64_t H, int64_t V, int dtype) {
    const size_t b = effective_budget(st, V, dtype);
    if (st.budget || dtype == FLCE_F32) return b;
    return b + (size_t)V * (size_t)H * sizeof(float);
}

Plan plan_for(const Settings& st, int64_t BT, int64_t H, int64_t V, int dtype, bool worst_case_bt = false) {
    return make_plan(BT, H, V, dtype, effective_budget(st, V, dtype), worst_case_bt, st.compact,
                     single_chunk_bytes(st, H, V, dtype));
}
Plan plan_for(int64_t BT, int64_t H, int64_t V, int dtype, bool worst_case_bt = false) {
    return plan_for(global_settings(), BT, H, V, dtype, worst_case_bt);
}

// ---- optional per-kernel timing (benchmarks only) ----
struct TimingRecord {
    hipEvent_t start, stop;
    int kind;
};
constexpr int MAX_TIMING_RECORDS = 8192;
std::atomic<bool> g_timing_on{false};
std::vector<TimingRecord> g_records;   // guarded by g_mutex

struct ScopedKernelTimer {
    hipStream_t stream;
    bool active = false;
    TimingRecord rec{};
    ScopedKernelTimer(int kind, hipStream_t s) : stream(s) {   // kind < 0: never timed
        if (kind < 0 || !g_timing_on.load()) return;
        {
            std::lock_guard<std::mutex> lock(g_mutex);
            if ((int)g_records.size() >= MAX_TIMING_RECORDS) return;
        }
        if (hipEventCreate(&rec.start) != hipSuccess) return;
        if (hipEventCreate(&rec.stop) != hipSuccess) {
            (void)hipEventDestroy(rec.start);
            return;
        }
        rec.kind = kind;
        active = (hipEventRecord(rec.start, stream) == hipSuccess);
    }
    ~ScopedKernelTimer() {
        if (!active) return;
        (void)hipEventRecord(rec.stop, stream);
        std::lock_guard<std::mutex> lock(g_mutex);
        g_records.push_back(rec);
    }
};

#define HIP_TRY(expr)                          \
    do {                                       \
        if ((expr) != hipSuccess) {            \
            (void)hipGetLastError();           \
            return FLCE_ERR_HIP;               \
        }                                      \
    } while (0)

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

int acquire_workspace(size_t need, char** out) {
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return FLCE_ERR_ARG;
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceWorkspace& w = g_ws[dev];
    if (w.lent) {
        if (w.lent_bytes < need) return FLCE_ERR_WORKSPACE;
        *out = static_cast<char*>(w.lent);
        return FLCE_OK;
    }
    if (w.own_bytes < need) {
        if (w.own) {
            HIP_TRY(hipDeviceSynchronize());
            HIP_TRY(hipFree(w.own));
            w.own = nullptr;
            w.own_bytes = 0;
        }
        if (hipMalloc(&w.own, need) != hipSuccess) {
            (void)hipGetLastError();
            w.own = nullptr;
            return FLCE_ERR_WORKSPACE;
        }
        w.own_bytes = need;
    }
    *out = static_cast<char*>(w.own);
    return FLCE_OK;
}

// C[M x N] (+)= A[M x K] * B[N x K]^T on the generic guarded kernel.  With ksplit > 1
// K is cut into ksplit ranges and range z writes its partial result to
// C + z * split_stride (no accumulation then).
template <typename T, typename OutT>
int launch_gemm_generic(int kind, const T* A, int64_t lda, const T* B, int64_t ldb, OutT* C,
                        int64_t ldc, int64_t M, int64_t N, int64_t K, bool accum, hipStream_t s,
                        int ksplit = 1, int64_t split_stride = 0) {
    if (M <= 0 || N <= 0) return FLCE_OK;
    if (ksplit > 1 && accum) return FLCE_ERR_SHAPE;
    ScopedKernelTimer timer(kind, s);
    constexpr int VEC = GGTraits<T>::VEC;
    constexpr int BK = GGTraits<T>::BK;
    const bool al = (K % VEC == 0) && (lda % VEC == 0) && (ldb % VEC == 0) && aligned(A, 16) &&
                    aligned(B, 16);
    const int64_t k_per = round_up((K + ksplit - 1) / ksplit, BK);
    const int64_t tiles = ((N + GG_BN - 1) / GG_BN) * ((M + GG_BM - 1) / GG_BM);
    if (tiles > MAX_GRID_X) return FLCE_ERR_SHAPE;   // check_launch_limits refuses such shapes up front
    dim3 grid((unsigned)tiles, 1, (unsigned)ksplit);
    dim3 block(GG_THREADS);
#define GG_LAUNCH(AL, AC)                                                                       \
    hipLaunchKernelGGL((gemm_nt_generic<T, OutT, AL, AC>), grid, block, 0, s, A, lda, B, ldb, C, \
                       ldc, (int)M, (int)N, (int)K, (int)k_per, split_stride)
    if (al) {
        if (accum) GG_LAUNCH(true, true); else GG_LAUNCH(true, false);
    } else {
        if (accum) GG_LAUNCH(false, true); else GG_LAUNCH(false, false);
    }
#undef GG_LAUNCH
    HIP_TRY(hipGetLastError());
    return FLCE_OK;
}

// What only the device knows about a product launch of a compacted chunk (see FGArgs).
struct FastDyn {
    const int* rows = nullptr;      // live rows: replaces M (is_k = 0) or K (is_k = 1)
    int is_k = 0;
    const int* ksplit = nullptr;    // number of K ranges, at most the launch's ksplit
    const int* first_live = nullptr;
    int launch = 0;
};

// Tuned bf16 kernel (see gemm_bf16_nt.h for what A_KM / B_KM / InT mean).  The
// caller has checked the shape limits (Plan::fast_*).  tail_part: tail_bytes of
// room for fp32 partial blocks; when that is enough for the launch's tail_plan (and the
// launch is not cut into K ranges as a whole and its tile count is known here), the tiles
// of a poorly filled last round are cut along K and summed by a second, small launch.
template <typename OutT, typename InT, bool A_KM, bool B_KM>
int launch_gemm_fast(int kind, const bf16_t* A, int64_t lda, const bf16_t* B, int64_t ldb, OutT* C,
                     int64_t ldc, const InT* Cin, int64_t ldcin, int64_t M, int64_t N, int64_t K,
                     hipStream_t s, int ksplit = 1, int64_t split_stride = 0, const FastDyn& d = FastDyn{},
                     float* tail_part = nullptr, size_t tail_bytes = 0) {
    if (M <= 0 || N <= 0 || K <= 0) return FLCE_OK;
    if (!aligned(A, 16) || !aligned(B, 16)) return FLCE_ERR_ARG;
    ScopedKernelTimer timer(kind, s);
    FGArgs a{A, lda, B, ldb, C, ldc, Cin, ldcin, (int)M, (int)N, (int)K,
             (int)((M + FG_BM - 1) / FG_BM), (int)((N + FG_BN - 1) / FG_BN), ksplit, split_stride,
             d.rows, d.is_k, d.ksplit, d.first_live, d.launch, 0, 0, 1, tail_part,
             FG_GROUP_TILES, kind == FLCE_KIND_LOGITS_GEMM ? 1 : 0, 1};
    const int64_t total = (int64_t)a.tiles_m * a.tiles_n * ksplit;
    if (total >= ((int64_t)1 << 30)) return FLCE_ERR_SHAPE;   // the kernel counts tiles in 32 bits
    int64_t wgs_per_xcd = (total + FG_XCDS - 1) / FG_XCDS;
    const bool m_static = !(d.rows && !d.is_k);   // a dynamic M changes the tile count on the device
    if (tail_part && ksplit == 1 && !d.ksplit && m_static) {
        const TailPlan t = tail_plan(total, (K + FG_BK - 1) / FG_BK);
        if (t.s > 1 && (size_t)FG_XCDS * t.r * t.s * TAIL_BLOCK_BYTES <= tail_bytes) {
            a.tail_begin = t.begin;
            a.tail_r = t.r;
            a.tail_s = t.s;
            wgs_per_xcd = (int64_t)t.begin + (int64_t)t.r * t.s;
        }
    }
    const dim3 grid((unsigned)(wgs_per_xcd * FG_XCDS));
    hipLaunchKernelGGL((gemm_bf16_256<OutT, InT, A_KM, B_KM>), grid, dim3(FG_THREADS), 0, s, a);
    HIP_TRY(hipGetLastError());
    if (a.tail_s > 1) {
        hipLaunchKernelGGL((fg_tail_reduce_kernel<OutT, InT>), dim3((unsigned)(FG_XCDS * a.tail_r * 8)), dim3(256),
                           0, s, a);
        HIP_TRY(hipGetLastError());
    }
    return FLCE_OK;
}

template <typename T>
int launch_transpose(const T* in, int64_t ldin, T* out, int64_t ldout, int64_t R, int64_t Cc,
                     hipStream_t s) {
    if (R <= 0 || Cc <= 0) return FLCE_OK;
    ScopedKernelTimer timer(FLCE_KIND_OTHER, s);
    const int64_t tiles = ((Cc + 63) / 64) * ((R + 63) / 64);
    if (tiles > MAX_GRID_X) return FLCE_ERR_SHAPE;
    dim3 grid((unsigned)tiles);
    hipLaunchKernelGGL((transpose_kernel<T>), grid, dim3(256), 0, s, in, ldin, out, ldout, (int)R,
                       (int)Cc);
    HIP_TRY(hipGetLastError());
    return FLCE_OK;
}

// zero_pad: columns V .. V + zero_pad - 1 of every row are set to zero as well (the
// padding of the workspace's dlogits chunk, which the dX product reads as part of K).
template <typename T>
int launch_ce_rows(T* Z, int64_t ldz, const int64_t* targets, int64_t rows, int64_t V,
                   int zero_pad, int64_t ignore_index, DeviceHeader* hdr, float* row_loss,
                   hipStream_t s, const int* n_rows = nullptr, bool timed = true, float* mean_out = nullptr) {
    const bool vec = aligned(Z, 16) && ((ldz * sizeof(T)) % 16 == 0);
    ScopedKernelTimer timer(timed ? FLCE_KIND_CE_ROWS : -1, s);
    // Rows of whole 16-byte vectors take the kernel that keeps the row in registers between
    // its two sweeps, in the shape that fits the row: 256 threads x 12 vectors up to 48 KB,
    // 512 x 12 up to 96 KB, 1024 x 16 beyond (the first 256 KB cached).  Measured, 4096 rows
    // of bf16, kernel alone, TB/s of algorithmic traffic: 5.3 at 16 KB rows, 6.3-6.7 from
    // 32 KB to 96 KB, 5.0-5.4 from 128 KB to 256 KB; two plain sweeps: 3.4-4.7.
    const int64_t row_bytes = V * (int64_t)sizeof(T);
#define CE_CACHED(TH, NV)                                                                              \
    hipLaunchKernelGGL((ce_rows_cached_kernel<T, TH, NV>), dim3((unsigned)rows), dim3(TH), 0, s, Z, ldz, \
                       targets, (int)V, zero_pad, ignore_index, hdr, row_loss, n_rows)
    if (vec && row_bytes > 98304) CE_CACHED(RC_THREADS, RC_NV);
    else if (vec && row_bytes > 49152) CE_CACHED(RM_THREADS, RM_NV);
    else if (vec) CE_CACHED(RS_THREADS, RS_NV);
#undef CE_CACHED
    else
        hipLaunchKernelGGL((ce_rows_inplace_kernel<T, false>), dim3((unsigned)rows),
                           dim3(RR_THREADS), 0, s, Z, ldz, targets, (int)V, zero_pad, ignore_index,
                           hdr, row_loss, n_rows);
    HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(loss_accumulate_kernel, dim3(1), dim3(256), 0, s, row_loss, (int)rows, hdr, mean_out);
    HIP_TRY(hipGetLastError());
    return FLCE_OK;
}

#define FLCE_TRY(expr)                 \
    do {                               \
        const int rc_ = (expr);        \
        if (rc_ != FLCE_OK) return rc_; \
    } while (0)

constexpr int MAX_HEADS = 16;   // headers of all heads share the 256-byte header slot
static_assert(MAX_HEADS * sizeof(DeviceHeader) <= 256, "header slot too small");

struct HeadWeights {
    float w[MAX_HEADS];
};

// RMSNorm in front of the projection: the chunk loop normalises each chunk of the
// raw hidden states just before its logits product (into the chunk buffer that
// otherwise holds gathered rows) and turns the chunk's dX into the gradient of the
// raw hidden states right after.
template <typename T>
struct NormCtx {
    const T* gamma;
    float eps;
    float* rstd;     // [C]
    float* partial;  // [RN_SLOTS x H] fp32 partial sums of dgamma, zero before the loop
    T* dh;           // [BT x H] out
};

// Sum of the K-range partial results of a dX product into dXc (+= with add).
template <typename T>
int launch_splitk_reduce(const float* part, int64_t split_stride, int nsplit, T* out, int64_t n,
                         bool add, hipStream_t s, const int* dyn_nsplit = nullptr) {
    ScopedKernelTimer timer(FLCE_KIND_DX_GEMM, s);
    const bool vec = (n % 4 == 0) && (split_stride % 4 == 0) && aligned(part, 16) &&
                     aligned(out, 4 * sizeof(T));
    const dim3 grid(2048), block(256);
#define SK_LAUNCH(ADD, VEC) \
    hipLaunchKernelGGL((splitk_reduce_kernel<T, ADD, VEC>), grid, block, 0, s, part, split_stride, nsplit, out, n, dyn_nsplit)
    if (vec) {
        if (add) SK_LAUNCH(true, true); else SK_LAUNCH(false, true);
    } else {
        if (add) SK_LAUNCH(true, false); else SK_LAUNCH(false, false);
    }
#undef SK_LAUNCH
    HIP_TRY(hipGetLastError());
    return FLCE_OK;
}

// Which form of the RMSNorm kernels a row length takes: 1, 2 or 4 16-byte vectors per
// thread (rows of whole vectors, at most 1024 of them, 16-byte aligned operands; the
// workspace buffers always are), or 0 for the scalar form.
template <typename T>
int rmsnorm_vectors_per_thread(int64_t H, const void* x, const void* gamma, const void* dh) {
    constexpr int N = 16 / (int)sizeof(T);
    if (H % N != 0 || !aligned(x, 16) || !aligned(gamma, 16) || !aligned(dh, 16)) return 0;
    const int64_t nvec = H / N;
    return nvec <= RN_THREADS ? 1 : nvec <= 2 * RN_THREADS ? 2 : nvec <= 4 * RN_THREADS ? 4 : 0;
}

// One head: count its valid rows, then run the chunk loop.  Gradients are scaled by
// weight / N_valid.  With dx_add the head's dX is added to what dX already holds
// (rounded to the storage type once per head), otherwise dX is overwritten.
template <typename T>
int run_head(const T* X, const T* W, const int64_t* targets, int64_t BT, int64_t H, int64_t V,
             int64_t ignore_index, float weight, DeviceHeader* hdr, bool dx_add, T* dX, T* dW,
             unsigned flags, const Plan& p, char* ws, hipStream_t s,
             const NormCtx<T>* norm = nullptr) {
    constexpr bool BF16 = (sizeof(T) == 2);
    const bool want_dx = !(flags & FLCE_SKIP_DX), want_dw = !(flags & FLCE_SKIP_DW);
    float* row_loss = reinterpret_cast<float*>(ws + p.off_row_loss);
    T* Z = reinterpret_cast<T*>(ws + p.off_z);
    T* GT = reinterpret_cast<T*>(ws + p.off_gt);
    T* WT = reinterpret_cast<T*>(ws + p.off_wt);
    T* XT = reinterpret_cast<T*>(ws + p.off_xt);
    float* dWacc = reinterpret_cast<float*>(ws + p.off_dwacc);
    T* Xg = reinterpret_cast<T*>(ws + p.off_xg);     // gathered (or normalised) rows of the chunk
    T* dXg = reinterpret_cast<T*>(ws + p.off_dxg);   // their gradient
    int* idx = reinterpret_cast<int*>(ws + p.off_idx);
    int64_t* tv = reinterpret_cast<int64_t*>(ws + p.off_tv);
    int* dyn = reinterpret_cast<int*>(ws + p.off_dyn);   // [0] row cursor, [1] live rows of the chunk
    float* tail = reinterpret_cast<float*>(ws + p.off_tail);   // partial blocks of the dW product's last round
    constexpr int VEC = 16 / (int)sizeof(T);

    hipLaunchKernelGGL(count_valid_kernel, dim3(1), dim3(1024), 0, s, targets, BT, ignore_index,
                       weight, hdr);
    HIP_TRY(hipGetLastError());
    if (want_dx && !p.fast_dx) FLCE_TRY(launch_transpose<T>(W, H, WT, p.ldz, V, H, s));   // WT[H x V]
    if (p.compact && want_dx && !dx_add) {   // rows without a target: zero gradient
        ScopedKernelTimer timer(FLCE_KIND_OTHER, s);
        hipLaunchKernelGGL((zero_ignored_rows_kernel<T>), dim3((unsigned)(BT < 8192 ? BT : 8192)),
                           dim3(256), 0, s, targets, BT, ignore_index, (int)H, norm ? norm->dh : dX);
        HIP_TRY(hipGetLastError());
    }

    bool dw_needs_cast = false;
    for (int64_t c = 0; c < p.nchunks; ++c) {
        const int64_t r0 = c * p.C;
        const bool last = (c == p.nchunks - 1);
        // Compacted: the chunk is the next rows of the batch that have a target, wherever they
        // are, at most C of them (the valid rows are dealt evenly to the last launches, see
        // compact_chunk_kernel); Xc, Z and dXc hold *n_live rows (a device value), the launches
        // below are sized for C rows, and idx maps the chunk's rows to batch rows.  Otherwise
        // the chunk is rows r0 .. r0 + rows - 1 of the batch.
        const int64_t rows = p.compact ? p.C : ((BT - r0 < p.C) ? BT - r0 : p.C);
        const int* n_live = p.compact ? dyn + DYN_LIVE : nullptr;
        const int* row_map = p.compact ? idx : nullptr;
        const T* Xin = p.compact ? X : X + r0 * H;   // what the chunk's row indices refer to
        const T* Xc = Xin;
        const int64_t* tc = targets + r0;
        FastDyn dyn_m, dyn_dx, dyn_dw;   // logits (M = live rows), dX (M and K ranges), dW (K = live rows)
        if (p.compact) {
            ScopedKernelTimer timer(FLCE_KIND_OTHER, s);
            hipLaunchKernelGGL(compact_chunk_kernel, dim3(1), dim3(CP_THREADS), 0, s, targets, (int)BT,
                               ignore_index, (int)p.C, (int)c, (int)p.nchunks, hdr,
                               (int)((H + FG_BN - 1) / FG_BN), (int)((V + FG_BK - 1) / FG_BK),
                               p.dx_ksplit, idx, tv, dyn);
            HIP_TRY(hipGetLastError());
            tc = tv;
            dyn_m.rows = dyn_dx.rows = dyn_dw.rows = n_live;
            dyn_dw.is_k = 1;
            dyn_dx.ksplit = dyn + DYN_DX_RANGES;
            dyn_dw.first_live = dyn + DYN_FIRST_LIVE;
            dyn_dw.launch = (int)c;
        }
        if (norm) {   // X holds the raw hidden states: normalise the chunk's rows
            ScopedKernelTimer timer(FLCE_KIND_OTHER, s);
#define RN_FWD(KERNEL)                                                                           \
    hipLaunchKernelGGL((KERNEL), dim3((unsigned)rows), dim3(RN_THREADS), 0, s, Xin, norm->gamma, \
                       norm->eps, (int)H, Xg, norm->rstd, row_map, n_live)
            switch (rmsnorm_vectors_per_thread<T>(H, Xin, norm->gamma, norm->dh)) {
                case 1: RN_FWD((rmsnorm_fwd_vec_kernel<T, 1>)); break;
                case 2: RN_FWD((rmsnorm_fwd_vec_kernel<T, 2>)); break;
                case 4: RN_FWD((rmsnorm_fwd_vec_kernel<T, 4>)); break;
                default: RN_FWD((rmsnorm_fwd_kernel<T>)); break;
            }
#undef RN_FWD
            HIP_TRY(hipGetLastError());
            Xc = Xg;
        } else if (p.compact) {
            ScopedKernelTimer timer(FLCE_KIND_OTHER, s);
            hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)rows), dim3(256), 0, s,
                               reinterpret_cast<const u32x4*>(X), idx, n_live, (int)(H / VEC),
                               reinterpret_cast<u32x4*>(Xg));
            HIP_TRY(hipGetLastError());
            Xc = Xg;
        }

        // logits of the chunk: Z = X_c W^T
        if (BF16 && p.fast_logits) {
            if constexpr (BF16)
                FLCE_TRY((launch_gemm_fast<bf16_t, void, false, false>(
                    FLCE_KIND_LOGITS_GEMM, Xc, H, W, H, Z, p.ldz, nullptr, 0, rows, V, H, s, 1, 0, dyn_m)));
        } else {
            FLCE_TRY((launch_gemm_generic<T, T>(FLCE_KIND_LOGITS_GEMM, Xc, H, W, H, Z, p.ldz, rows, V, H,
                                                false, s)));
        }

        // loss and in-place dlogits
        FLCE_TRY(launch_ce_rows<T>(Z, p.ldz, tc, rows, V, (int)(p.ldz - V), ignore_index, hdr,
                                   row_loss, s, n_live));

        // dX_c (+)= G W
        if (want_dx) {
            // where the product writes: straight into dX, or into the chunk buffer when the rows
            // still have to be scattered back or to pass through the RMSNorm backward
            const bool staged = p.compact || norm;
            T* dXc = staged ? dXg : dX + r0 * H;
            const bool add_in_gemm = dx_add && !staged;
            if (BF16 && p.fast_dx) {
                if constexpr (BF16) {
                    if (p.dx_ksplit > 1) {
                        // few output tiles, very long K: K ranges -> fp32 partials -> fixed-order sum
                        float* part = reinterpret_cast<float*>(ws + p.off_dxpart);
                        FLCE_TRY((launch_gemm_fast<float, void, false, true>(
                            FLCE_KIND_DX_GEMM, Z, p.ldz, W, H, part, H, nullptr, 0, rows, H, V, s,
                            p.dx_ksplit, p.C * H, dyn_dx)));
                        FLCE_TRY(launch_splitk_reduce<bf16_t>(part, p.C * H, p.dx_ksplit, dXc, rows * H,
                                                              add_in_gemm, s, dyn_dx.ksplit));
                    } else if (add_in_gemm) {
                        FLCE_TRY((launch_gemm_fast<bf16_t, bf16_t, false, true>(
                            FLCE_KIND_DX_GEMM, Z, p.ldz, W, H, dXc, H, dXc, H, rows, H, V, s)));
                    } else {
                        FLCE_TRY((launch_gemm_fast<bf16_t, void, false, true>(
                            FLCE_KIND_DX_GEMM, Z, p.ldz, W, H, dXc, H, nullptr, 0, rows, H, V, s, 1, 0,
                            dyn_m)));
                    }
                }
            } else {
                if (p.dx_ksplit > 1) {
                    float* part = reinterpret_cast<float*>(ws + p.off_dxpart);
                    FLCE_TRY((launch_gemm_generic<T, float>(FLCE_KIND_DX_GEMM, Z, p.ldz, WT, p.ldz, part,
                                                            H, rows, H, V, false, s, p.dx_ksplit,
                                                            p.C * H)));
                    FLCE_TRY(launch_splitk_reduce<T>(part, p.C * H, p.dx_ksplit, dXc, rows * H, add_in_gemm,
                                                     s));
                } else {
                    FLCE_TRY((launch_gemm_generic<T, T>(FLCE_KIND_DX_GEMM, Z, p.ldz, WT, p.ldz, dXc, H,
                                                        rows, H, V, add_in_gemm, s)));
                }
            }
            if (norm) {
                ScopedKernelTimer timer(FLCE_KIND_OTHER, s);
#define RN_BWD(KERNEL)                                                                              \
    hipLaunchKernelGGL((KERNEL), dim3(RN_SLOTS), dim3(RN_THREADS), 0, s, Xin, norm->gamma,           \
                       norm->rstd, dXg, (int)rows, (int)H, p.compact ? norm->dh : norm->dh + r0 * H, \
                       norm->partial, row_map, n_live)
                switch (rmsnorm_vectors_per_thread<T>(H, Xin, norm->gamma, norm->dh)) {
                    case 1: RN_BWD((rmsnorm_bwd_vec_kernel<T, 1>)); break;
                    case 2: RN_BWD((rmsnorm_bwd_vec_kernel<T, 2>)); break;
                    case 4: RN_BWD((rmsnorm_bwd_vec_kernel<T, 4>)); break;
                    default: RN_BWD((rmsnorm_bwd_kernel<T>)); break;
                }
#undef RN_BWD
                HIP_TRY(hipGetLastError());
            } else if (p.compact) {
                ScopedKernelTimer timer(FLCE_KIND_OTHER, s);
                if (dx_add)
                    hipLaunchKernelGGL((scatter_rows_kernel<T, true>), dim3((unsigned)rows), dim3(256), 0,
                                       s, static_cast<const T*>(dXg), idx, n_live, (int)H, dX);
                else
                    hipLaunchKernelGGL((scatter_rows_kernel<T, false>), dim3((unsigned)rows), dim3(256), 0,
                                       s, static_cast<const T*>(dXg), idx, n_live, (int)H, dX);
                HIP_TRY(hipGetLastError());
            }
        }

        // dW (+)= G^T X_c   (K = the chunk's rows; in a compacted chunk K = *n_live)
        if (want_dw) {
            const bool fast = BF16 && (last ? p.fast_dw_last : p.fast_dw_full);
            if (fast) {
                if constexpr (BF16) {
                    if (p.nchunks == 1) {
                        FLCE_TRY((launch_gemm_fast<bf16_t, void, true, true>(
                            FLCE_KIND_DW_GEMM, Z, p.ldz, Xc, H, dW, H, nullptr, 0, V, H, rows, s, 1, 0,
                            dyn_dw, tail, p.tail_bytes)));
                    } else if (c == 0) {
                        FLCE_TRY((launch_gemm_fast<float, void, true, true>(
                            FLCE_KIND_DW_GEMM, Z, p.ldz, Xc, H, dWacc, H, nullptr, 0, V, H, rows, s, 1, 0,
                            dyn_dw, tail, p.tail_bytes)));
                    } else if (!last) {
                        FLCE_TRY((launch_gemm_fast<float, float, true, true>(
                            FLCE_KIND_DW_GEMM, Z, p.ldz, Xc, H, dWacc, H, dWacc, H, V, H, rows, s, 1, 0,
                            dyn_dw, tail, p.tail_bytes)));
                    } else {   // last chunk: add the fp32 partial sums and write dW in bf16
                        FLCE_TRY((launch_gemm_fast<bf16_t, float, true, true>(
                            FLCE_KIND_DW_GEMM, Z, p.ldz, Xc, H, dW, H, dWacc, H, V, H, rows, s, 1, 0,
                            dyn_dw, tail, p.tail_bytes)));
                    }
                }
            } else {
                // guarded path: GT[V x rows] times XT[H x rows]^T
                FLCE_TRY(launch_transpose<T>(Z, p.ldz, GT, p.ldc, rows, V, s));
                FLCE_TRY(launch_transpose<T>(Xc, H, XT, p.ldc, rows, H, s));
                if (p.fp32_dw_acc) {
                    FLCE_TRY((launch_gemm_generic<T, float>(FLCE_KIND_DW_GEMM, GT, p.ldc, XT, p.ldc,
                                                            dWacc, H, V, H, rows, c > 0, s)));
                    dw_needs_cast = last;
                } else {
                    FLCE_TRY((launch_gemm_generic<T, T>(FLCE_KIND_DW_GEMM, GT, p.ldc, XT, p.ldc, dW, H,
                                                        V, H, rows, c > 0, s)));
                }
            }
        }
    }
    if (want_dw && dw_needs_cast) {
        ScopedKernelTimer timer(FLCE_KIND_OTHER, s);
        hipLaunchKernelGGL((cast_from_f32_kernel<T>), dim3(2048), dim3(256), 0, s, dWacc, dW,
                           V * H);
        HIP_TRY(hipGetLastError());
    }
    return FLCE_OK;
}

// All heads one after the other on the same stream and the same workspace; then
// loss = sum_j weight_j * mean loss of head j.
template <typename T>
int run_heads(const T* X, const void* const* W, const int64_t* const* targets, const float* weights,
              int n_heads, int64_t BT, int64_t H, int64_t V, int64_t ignore_index, float* loss,
              float* head_losses, T* dX, void* const* dW, unsigned flags, const Plan& p, char* ws,
              hipStream_t s) {
    DeviceHeader* hdr = reinterpret_cast<DeviceHeader*>(ws + p.off_hdr);
    const bool want_dw = !(flags & FLCE_SKIP_DW);
    HeadWeights hw{};
    for (int j = 0; j < n_heads; ++j) {
        hw.w[j] = weights ? weights[j] : 1.0f;
        FLCE_TRY(run_head<T>(X, static_cast<const T*>(W[j]), targets[j], BT, H, V, ignore_index,
                             hw.w[j], hdr + j, j > 0, dX, want_dw ? static_cast<T*>(dW[j]) : nullptr,
                             flags, p, ws, s));
    }
    hipLaunchKernelGGL(finalize_loss_kernel, dim3(1), dim3(64), 0, s, hdr, n_heads, hw, loss,
                       head_losses);
    HIP_TRY(hipGetLastError());
    return FLCE_OK;
}

int check_dims(int64_t BT, int64_t H, int64_t V, int dtype) {
    if (dtype != FLCE_F32 && dtype != FLCE_BF16) return FLCE_ERR_DTYPE;
    if (BT <= 0 || H <= 0 || V <= 0 || BT > MAX_DIM || H > MAX_DIM || V > MAX_DIM)
        return FLCE_ERR_SHAPE;
    return FLCE_OK;
}

// Launch-size limits of the kernels a plan uses, checked before anything is launched: the
// guarded product and the transposes number their tiles along grid x, the row kernels and
// the row copies take one workgroup per row of a chunk.
int check_launch_limits(const Plan& p, int64_t H, int64_t V) {
    auto tiles = [](int64_t r, int64_t c, int64_t t) { return ((r + t - 1) / t) * ((c + t - 1) / t); };
    if (p.C > MAX_GRID_X) return FLCE_ERR_SHAPE;
    const bool all_fast = p.fast_logits && p.fast_dx && p.fast_dw_full && p.fast_dw_last;
    if (!all_fast) {
        const int64_t worst = std::max(std::max(tiles(p.C, V, 128), tiles(V, H, 128)),
                                       std::max(tiles(V, H, 64), tiles(p.C, V, 64)));
        if (worst > MAX_GRID_X) return FLCE_ERR_SHAPE;
    }
    return FLCE_OK;
}

struct NormLayout {
    size_t off_rstd, off_partial, total;
};
NormLayout norm_layout(const Plan& p, int64_t H) {
    NormLayout l{};
    size_t off = p.total;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += (bytes + 255) / 256 * 256;
        return at;
    };
    l.off_rstd = take((size_t)p.C * sizeof(float));
    l.off_partial = take((size_t)RN_SLOTS * H * sizeof(float));
    l.total = off;
    return l;
}

template <typename T>
int run_rmsnorm_head(const T* h, const T* gamma, float eps, const T* W, const int64_t* targets,
                     int64_t BT, int64_t H, int64_t V, int64_t ignore_index, float* loss, T* dh,
                     T* dgamma, T* dW, unsigned flags, const Plan& p, const NormLayout& l, char* ws,
                     hipStream_t s) {
    const bool want_dx = !(flags & FLCE_SKIP_DX);
    NormCtx<T> n{gamma, eps, reinterpret_cast<float*>(ws + l.off_rstd),
                 reinterpret_cast<float*>(ws + l.off_partial), dh};
    DeviceHeader* hdr = reinterpret_cast<DeviceHeader*>(ws + p.off_hdr);
    if (want_dx) {
        hipLaunchKernelGGL(fill_zero_kernel, dim3(256), dim3(256), 0, s, n.partial,
                           (int64_t)RN_SLOTS * H);
        HIP_TRY(hipGetLastError());
    }
    FLCE_TRY(run_head<T>(h, W, targets, BT, H, V, ignore_index, 1.0f, hdr, false, nullptr, dW, flags, p,
                         ws, s, &n));
    if (want_dx) {
        hipLaunchKernelGGL((rmsnorm_dgamma_kernel<T>), dim3((unsigned)((H + RN_DG_COLS - 1) / RN_DG_COLS)),
                           dim3(RN_DG_COLS * RN_DG_PARTS), 0, s, n.partial, (int)H, dgamma);
        HIP_TRY(hipGetLastError());
    }
    HeadWeights one{};
    one.w[0] = 1.0f;
    hipLaunchKernelGGL(finalize_loss_kernel, dim3(1), dim3(64), 0, s, hdr, 1, one, loss,
                       static_cast<float*>(nullptr));
    HIP_TRY(hipGetLastError());
    return FLCE_OK;
}

// Argument checks shared by the two stand-alone cross-entropy entry points.
int check_ce_args(const void* Z, const int64_t* targets, int64_t BT, int64_t V, int64_t ldz,
                  int64_t ignore_index, int dtype, const float* loss) {
    FLCE_TRY(check_dims(BT, 1, V, dtype));
    if (!Z || !targets || !loss) return FLCE_ERR_NULL;
    if (ldz < V || ldz > MAX_DIM * 4) return FLCE_ERR_SHAPE;
    if (!aligned(Z, elem_size(dtype)) || !aligned(targets, 8) || !aligned(loss, 4))
        return FLCE_ERR_ALIGN;
    if (ignore_index >= 0 && ignore_index < V) return FLCE_ERR_ARG;
    return FLCE_OK;
}

// Stand-alone cross entropy on logits Z, `step` rows per launch, with the device header
// and the per-row losses (`step` floats) in memory the caller of this function provides.
int run_ce_inplace(void* Z, const int64_t* targets, int64_t BT, int64_t V, int64_t ldz,
                   int64_t ignore_index, int dtype, float* loss, DeviceHeader* hdr, float* row_loss,
                   int64_t step, bool timed, hipStream_t s) {
    hipLaunchKernelGGL(count_valid_kernel, dim3(1), dim3(1024), 0, s, targets, BT, ignore_index,
                       1.0f, hdr);
    HIP_TRY(hipGetLastError());
    for (int64_t r0 = 0; r0 < BT; r0 += step) {
        const int64_t rows = (BT - r0 < step) ? BT - r0 : step;
        float* mean_out = (r0 + rows == BT) ? loss : nullptr;   // the last launch also writes the mean
        if (dtype == FLCE_F32)
            FLCE_TRY(launch_ce_rows<float>(static_cast<float*>(Z) + r0 * ldz, ldz, targets + r0,
                                           rows, V, 0, ignore_index, hdr, row_loss, s, nullptr, timed, mean_out));
        else
            FLCE_TRY(launch_ce_rows<bf16_t>(static_cast<bf16_t*>(Z) + r0 * ldz, ldz, targets + r0,
                                            rows, V, 0, ignore_index, hdr, row_loss, s, nullptr, timed, mean_out));
    }
    return FLCE_OK;
}

// flce_multihead_fwd_bwd with the settings given (the process-wide ones, or a call's options)
int multihead_fwd_bwd(const Settings& st, const void* X, const void* const* W, const int64_t* const* targets,
                      const float* weights, int n_heads, int64_t BT, int64_t H, int64_t V,
                      int64_t ignore_index, int dtype, float* loss, float* head_losses, void* dX,
                      void* const* dW, unsigned flags, void* stream) {
    FLCE_TRY(check_dims(BT, H, V, dtype));
    if (n_heads < 1 || n_heads > MAX_HEADS) return FLCE_ERR_ARG;
    if (flags & ~(unsigned)(FLCE_SKIP_DX | FLCE_SKIP_DW)) return FLCE_ERR_ARG;
    const bool want_dx = !(flags & FLCE_SKIP_DX), want_dw = !(flags & FLCE_SKIP_DW);
    if (!X || !W || !targets || !loss || (want_dx && !dX) || (want_dw && !dW)) return FLCE_ERR_NULL;
    if (!aligned(X, 16) || (want_dx && !aligned(dX, 16)) || !aligned(loss, 4) ||
        (head_losses && !aligned(head_losses, 4)))
        return FLCE_ERR_ALIGN;
    for (int j = 0; j < n_heads; ++j) {
        if (!W[j] || !targets[j] || (want_dw && !dW[j])) return FLCE_ERR_NULL;
        if (!aligned(W[j], 16) || !aligned(targets[j], 8) || (want_dw && !aligned(dW[j], 16)))
            return FLCE_ERR_ALIGN;
        if (weights && !(weights[j] == weights[j] && weights[j] - weights[j] == 0.0f))
            return FLCE_ERR_ARG;   // NaN or infinite weight
        for (int k = 0; want_dw && k < j; ++k)
            if (dW[k] == dW[j]) return FLCE_ERR_ARG;   // every head needs a dW of its own
    }
    if (ignore_index >= 0 && ignore_index < V) return FLCE_ERR_ARG;   // would shadow a class

    const Plan p = plan_for(st, BT, H, V, dtype);
    FLCE_TRY(check_launch_limits(p, H, V));
    char* ws = static_cast<char*>(st.ws);
    if (ws) {
        if (!aligned(ws, 256)) return FLCE_ERR_ALIGN;
        if (st.ws_bytes < p.total) return FLCE_ERR_WORKSPACE;
    } else {
        FLCE_TRY(acquire_workspace(p.total, &ws));
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dtype == FLCE_F32)
        return run_heads<float>(static_cast<const float*>(X), W, targets, weights, n_heads, BT, H, V,
                                ignore_index, loss, head_losses, static_cast<float*>(dX), dW, flags,
                                p, ws, s);
    return run_heads<bf16_t>(static_cast<const bf16_t*>(X), W, targets, weights, n_heads, BT, H, V,
                             ignore_index, loss, head_losses, static_cast<bf16_t*>(dX), dW, flags, p,
                             ws, s);
}

}  // namespace

extern "C" {

int flce_multihead_fwd_bwd(const void* X, const void* const* W, const int64_t* const* targets,
                           const float* weights, int n_heads, int64_t BT, int64_t H, int64_t V,
                           int64_t ignore_index, int dtype, float* loss, float* head_losses, void* dX,
                           void* const* dW, unsigned flags, void* stream) {
    return multihead_fwd_bwd(global_settings(), X, W, targets, weights, n_heads, BT, H, V, ignore_index,
                             dtype, loss, head_losses, dX, dW, flags, stream);
}

void flce_default_options(flce_options* opt) {
    if (!opt) return;
    const Settings st = global_settings();
    opt->size = sizeof(flce_options);
    opt->logits_budget_bytes = st.budget;
    opt->row_compaction = st.compact ? 1 : 0;
    opt->flags = 0u;
    opt->workspace = nullptr;
    opt->workspace_bytes = 0;
}

// The settings a call's options stand for; FLCE_ERR_ARG for a struct this library cannot read.
static int settings_from(const flce_options* opt, Settings* st, unsigned* flags) {
    *st = global_settings();
    *flags = 0u;
    if (!opt) return FLCE_OK;
    if (opt->size != sizeof(flce_options)) return FLCE_ERR_ARG;
    if (opt->row_compaction != 0 && opt->row_compaction != 1) return FLCE_ERR_ARG;
    st->budget = opt->logits_budget_bytes;
    st->compact = opt->row_compaction != 0;
    st->ws = opt->workspace;
    st->ws_bytes = opt->workspace ? opt->workspace_bytes : 0;
    *flags = opt->flags;
    return FLCE_OK;
}

int flce_fwd_bwd_opt(const void* X, const void* W, const int64_t* targets, int64_t BT, int64_t H,
                     int64_t V, int64_t ignore_index, int dtype, float* loss, void* dX, void* dW,
                     const flce_options* opt, void* stream) {
    Settings st;
    unsigned flags;
    FLCE_TRY(settings_from(opt, &st, &flags));
    const void* Ws[1] = {W};
    const int64_t* ts[1] = {targets};
    void* dWs[1] = {dW};
    return multihead_fwd_bwd(st, X, Ws, ts, nullptr, 1, BT, H, V, ignore_index, dtype, loss, nullptr, dX,
                             dWs, flags, stream);
}

size_t flce_workspace_bytes_opt(int64_t BT, int64_t H, int64_t V, int dtype, const flce_options* opt) {
    Settings st;
    unsigned flags;
    if (check_dims(BT, H, V, dtype) != FLCE_OK || settings_from(opt, &st, &flags) != FLCE_OK) return 0;
    return plan_for(st, BT, H, V, dtype).total;
}

int flce_rmsnorm_fwd_bwd(const void* h, const void* gamma, float eps, const void* W,
                         const int64_t* targets, int64_t BT, int64_t H, int64_t V,
                         int64_t ignore_index, int dtype, float* loss, void* dh, void* dgamma,
                         void* dW, unsigned flags, void* stream) {
    FLCE_TRY(check_dims(BT, H, V, dtype));
    if (flags & ~(unsigned)(FLCE_SKIP_DX | FLCE_SKIP_DW)) return FLCE_ERR_ARG;
    const bool want_dx = !(flags & FLCE_SKIP_DX), want_dw = !(flags & FLCE_SKIP_DW);
    if (!h || !gamma || !W || !targets || !loss || (want_dx && (!dh || !dgamma)) || (want_dw && !dW))
        return FLCE_ERR_NULL;
    if (!aligned(h, 16) || !aligned(W, 16) || !aligned(gamma, elem_size(dtype)) ||
        (want_dx && (!aligned(dh, 16) || !aligned(dgamma, elem_size(dtype)))) ||
        (want_dw && !aligned(dW, 16)) || !aligned(targets, 8) || !aligned(loss, 4))
        return FLCE_ERR_ALIGN;
    if (ignore_index >= 0 && ignore_index < V) return FLCE_ERR_ARG;
    if (!(eps >= 0.0f) || eps - eps != 0.0f) return FLCE_ERR_ARG;   // negative, NaN or infinite

    const Plan p = plan_for(BT, H, V, dtype);
    FLCE_TRY(check_launch_limits(p, H, V));
    const NormLayout l = norm_layout(p, H);
    char* ws = nullptr;
    FLCE_TRY(acquire_workspace(l.total, &ws));
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dtype == FLCE_F32)
        return run_rmsnorm_head<float>(static_cast<const float*>(h), static_cast<const float*>(gamma),
                                       eps, static_cast<const float*>(W), targets, BT, H, V,
                                       ignore_index, loss, static_cast<float*>(dh),
                                       static_cast<float*>(dgamma), static_cast<float*>(dW), flags, p,
                                       l, ws, s);
    return run_rmsnorm_head<bf16_t>(static_cast<const bf16_t*>(h), static_cast<const bf16_t*>(gamma),
                                    eps, static_cast<const bf16_t*>(W), targets, BT, H, V,
                                    ignore_index, loss, static_cast<bf16_t*>(dh),
                                    static_cast<bf16_t*>(dgamma), static_cast<bf16_t*>(dW), flags, p,
                                    l, ws, s);
}

size_t flce_rmsnorm_workspace_bytes(int64_t BT, int64_t H, int64_t V, int dtype) {
    if (check_dims(BT, H, V, dtype) != FLCE_OK) return 0;
    return norm_layout(plan_for(BT, H, V, dtype), H).total;
}

int flce_fwd_bwd_ex(const void* X, const void* W, const int64_t* targets, int64_t BT, int64_t H,
                    int64_t V, int64_t ignore_index, int dtype, float* loss, void* dX, void* dW,
                    unsigned flags, void* stream) {
    const void* Ws[1] = {W};
    const int64_t* ts[1] = {targets};
    void* dWs[1] = {dW};
    return flce_multihead_fwd_bwd(X, Ws, ts, nullptr, 1, BT, H, V, ignore_index, dtype, loss, nullptr,
                                  dX, dWs, flags, stream);
}

int flce_fwd_bwd(const void* X, const void* W, const int64_t* targets, int64_t BT, int64_t H,
                 int64_t V, int64_t ignore_index, int dtype, float* loss, void* dX, void* dW,
                 void* stream) {
    return flce_fwd_bwd_ex(X, W, targets, BT, H, V, ignore_index, dtype, loss, dX, dW, 0u, stream);
}

int flce_cross_entropy_inplace(void* Z, const int64_t* targets, int64_t BT, int64_t V, int64_t ldz,
                               int64_t ignore_index, int dtype, float* loss, void* stream) {
    FLCE_TRY(check_ce_args(Z, targets, BT, V, ldz, ignore_index, dtype, loss));
    const int64_t step = BT < CE_ROWS_PER_LAUNCH ? BT : CE_ROWS_PER_LAUNCH;
    char* ws = nullptr;
    FLCE_TRY(acquire_workspace(256 + (size_t)step * sizeof(float), &ws));
    return run_ce_inplace(Z, targets, BT, V, ldz, ignore_index, dtype, loss,
                          reinterpret_cast<DeviceHeader*>(ws), reinterpret_cast<float*>(ws + 256), step,
                          true, static_cast<hipStream_t>(stream));
}

int flce_cross_entropy_inplace_noalloc(void* Z, const int64_t* targets, int64_t BT, int64_t V,
                                       int64_t ldz, int64_t ignore_index, int dtype, float* loss,
                                       void* stream) {
    FLCE_TRY(check_ce_args(Z, targets, BT, V, ldz, ignore_index, dtype, loss));
    if (BT > FLCE_CE_NOALLOC_MAX_ROWS) return FLCE_ERR_TOO_LARGE;
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return FLCE_ERR_ARG;
    char* ptr = nullptr;
    {
        // first call on this device: ask the runtime where this device's copy of the array is
        std::lock_guard<std::mutex> lock(g_mutex);
        if (!g_scratch_ptr[dev]) {
            void* p = nullptr;
            HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
            if (!p) return FLCE_ERR_HIP;
            g_scratch_ptr[dev] = p;
        }
        ptr = static_cast<char*>(g_scratch_ptr[dev]);
    }
    // The header is reset by the counting kernel and every row's loss slot is written by the
    // row kernel before it is summed, so nothing of the previous call's contents is read.
    return run_ce_inplace(Z, targets, BT, V, ldz, ignore_index, dtype, loss,
                          reinterpret_cast<DeviceHeader*>(ptr), reinterpret_cast<float*>(ptr + 256), BT,
                          false, static_cast<hipStream_t>(stream));
}

size_t flce_workspace_bytes(int64_t BT, int64_t H, int64_t V, int dtype) {
    if (check_dims(BT, H, V, dtype) != FLCE_OK) return 0;
    return plan_for(BT, H, V, dtype).total;
}

size_t flce_workspace_bytes_max(int64_t H, int64_t V, int dtype) {
    if (check_dims(1, H, V, dtype) != FLCE_OK) return 0;
    return plan_for(0, H, V, dtype, true).total;
}

int flce_set_workspace(void* ws, size_t bytes) {
    if (ws && !aligned(ws, 256)) return FLCE_ERR_ALIGN;
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return FLCE_ERR_ARG;
    std::lock_guard<std::mutex> lock(g_mutex);
    g_ws[dev].lent = ws;
    g_ws[dev].lent_bytes = ws ? bytes : 0;
    return FLCE_OK;
}

int flce_release_workspace(void) {
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return FLCE_ERR_ARG;
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceWorkspace& w = g_ws[dev];
    if (w.own) {
        HIP_TRY(hipDeviceSynchronize());
        HIP_TRY(hipFree(w.own));
        w.own = nullptr;
        w.own_bytes = 0;
    }
    return FLCE_OK;
}

int flce_set_logits_budget_bytes(size_t bytes) {
    g_budget.store(bytes);
    return FLCE_OK;
}

size_t flce_get_logits_budget_bytes(void) { return g_budget.load(); }

int flce_set_row_compaction(int on) {
    g_compact.store(on != 0);
    return FLCE_OK;
}

int flce_get_row_compaction(void) { return g_compact.load() ? 1 : 0; }

int64_t flce_chunk_rows(int64_t BT, int64_t H, int64_t V, int dtype) {
    if (check_dims(BT, H, V, dtype) != FLCE_OK) return 0;
    return plan_for(BT, H, V, dtype).C;
}

int64_t flce_num_chunks(int64_t BT, int64_t H, int64_t V, int dtype) {
    if (check_dims(BT, H, V, dtype) != FLCE_OK) return 0;
    return plan_for(BT, H, V, dtype).nchunks;
}

size_t flce_logits_budget_for_workspace(int64_t BT, int64_t H, int64_t V, int dtype, size_t max_workspace_bytes) {
    if (check_dims(BT, H, V, dtype) != FLCE_OK) return 0;
    Settings st = global_settings();
    const size_t row_bytes = (size_t)round_up(V, 64) * elem_size(dtype);
    // the workspace grows with the rows per chunk apart from small steps in the dX partial
    // results, so the first fit from the top is the largest
    for (int64_t c = round_up(BT, CHUNK_ALIGN); c >= CHUNK_ALIGN; c -= CHUNK_ALIGN) {
        st.budget = (size_t)c * row_bytes;
        const Plan p = plan_for(st, BT, H, V, dtype);
        if (p.total <= max_workspace_bytes && check_launch_limits(p, H, V) == FLCE_OK) return st.budget;
    }
    return 0;
}

int flce_dx_k_ranges(int64_t BT, int64_t H, int64_t V, int dtype) {
    if (check_dims(BT, H, V, dtype) != FLCE_OK) return 0;
    return plan_for(BT, H, V, dtype).dx_ksplit;
}

int64_t flce_paper_chunk_rows(int64_t BT, int64_t H, int64_t V) {
    if (BT <= 0 || H <= 0 || V <= 0) return 0;
    return paper_chunk_rows(BT, H, V);
}

size_t flce_full_logits_bytes(int64_t BT, int64_t V, int dtype) {
    if (BT <= 0 || V <= 0 || (dtype != FLCE_F32 && dtype != FLCE_BF16)) return 0;
    return (size_t)BT * (size_t)V * elem_size(dtype);
}

int flce_mfma_ceiling_launch(int pattern, int workgroups, int iters, float std_b, float* out,
                             size_t out_floats, void* stream) {
    if (!out) return FLCE_ERR_NULL;
    if (pattern < 0 || pattern > 2 || workgroups <= 0 || workgroups > 65536 || iters <= 0 ||
        (int64_t)workgroups * iters > ((int64_t)1 << 26) || !(std_b >= 0.0f) ||
        out_floats < (size_t)workgroups * 256)
        return FLCE_ERR_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)workgroups), block(256);
    if (pattern == 0) hipLaunchKernelGGL((mfma_ceiling_kernel<0>), grid, block, 0, s, out, iters, std_b);
    if (pattern == 1) hipLaunchKernelGGL((mfma_ceiling_kernel<1>), grid, block, 0, s, out, iters, std_b);
    if (pattern == 2) hipLaunchKernelGGL((mfma_ceiling_kernel<2>), grid, block, 0, s, out, iters, std_b);
    HIP_TRY(hipGetLastError());
    return FLCE_OK;
}

int flce_timing_enable(int on) {
    g_timing_on.store(on != 0);
    return FLCE_OK;
}

int flce_timing_collect(double* total_ms, int64_t* launches) {
    if (!total_ms || !launches) return FLCE_ERR_NULL;
    std::lock_guard<std::mutex> lock(g_mutex);
    for (int k = 0; k < FLCE_NUM_KINDS; ++k) {
        total_ms[k] = 0.0;
        launches[k] = 0;
    }
    int rc = FLCE_OK;
    for (TimingRecord& r : g_records) {
        float ms = 0.f;
        if (hipEventSynchronize(r.stop) == hipSuccess &&
            hipEventElapsedTime(&ms, r.start, r.stop) == hipSuccess) {
            total_ms[r.kind] += ms;
            launches[r.kind] += 1;
        } else {
            (void)hipGetLastError();
            rc = FLCE_ERR_HIP;
        }
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    g_records.clear();
    return rc;
}

const char* flce_status_string(int status) {
    switch (status) {
        case FLCE_OK: return "ok";
        case FLCE_ERR_NULL: return "a required pointer is NULL";
        case FLCE_ERR_SHAPE: return "BT, H, V or a stride is out of range";
        case FLCE_ERR_DTYPE: return "unknown dtype";
        case FLCE_ERR_ALIGN: return "a pointer misses its required alignment";
        case FLCE_ERR_WORKSPACE: return "workspace too small or allocation failed";
        case FLCE_ERR_HIP: return "a HIP runtime call or kernel launch failed";
        case FLCE_ERR_ARG: return "invalid argument";
        case FLCE_ERR_TOO_LARGE: return "problem larger than the fixed scratch of the allocation-free entry point";
        default: return "unknown status";
    }
}

}  // extern "C"
