/*
 * flce.h - C ABI of the MI355X (gfx950) fused linear cross-entropy library.
 *
 * One call computes, for hidden states X[BT x H], an output-projection weight
 * W[V x H] and integer targets[BT],
 *
 *     logits   z_i = W x_i                                  (never stored whole)
 *     loss       L = -(1/N) sum_{i valid} log softmax(z_i)[t_i]
 *     dX_i         = W^T g_i,      dW = sum_i g_i x_i^T,
 *     g_i          = (softmax(z_i) - onehot(t_i)) / N  for valid i, 0 otherwise,
 *
 * where a row is valid when t_i != ignore_index and N is the number of valid
 * rows.  This is the paper's FusedLinearCrossEntropy (section 3.2, FLCE
 * paragraph and Eq. FLCE-backward) on top of its CrossEntropy kernel (CE
 * paragraph, Eq. CE-forward / CE-backward): rows are processed in chunks, each
 * chunk's logits are turned into their gradient in place, and only one chunk
 * of logits exists at any time.  Deviation from the paper's remark on mean
 * reduction: every gradient is divided by the global N (counted on the device
 * before the chunk loop), so the result does not depend on the chunk size.
 *
 * Conventions
 *  - All matrices are dense row-major; X, W, dX, dW, loss, targets are DEVICE
 *    pointers owned by the caller.  X, W, dX, dW must be 16-byte aligned,
 *    targets 8-byte, loss 4-byte.  Inputs are not modified.  dX, dW and loss
 *    are fully overwritten (rows of dX whose target is ignored become 0).
 *  - dtype selects the storage type of X, W, dX, dW (flce_dtype).  Products
 *    accumulate in fp32; the reduction math is fp32; loss is fp32.
 *  - Any BT, H, V >= 1 (each below 2^30) are accepted, except shapes whose
 *    kernels would exceed the launch limits (more than 2^31 - 1 tiles of 64 x 64
 *    in one matrix on the guarded path: FLCE_ERR_SHAPE, like every argument
 *    error before anything is launched).  bf16 problems with
 *    H % 64 == 0 run entirely on the tuned matrix-core kernel, whatever BT and V
 *    are; other H and fp32 storage run on slower, fully guarded kernels and need
 *    more workspace (transposed copies); the results meet the same bars.
 *  - Targets must lie in [0, V) or equal ignore_index; anything else is a
 *    precondition violation (not detected: checking would need a host sync).
 *  - N == 0 gives loss = 0, dX = 0, dW = 0.
 *  - The upstream gradient of the loss is 1.  There is no bias term.
 *  - Every call is asynchronous: all work is enqueued on `stream` (a
 *    hipStream_t, NULL = the default stream) and the function returns without
 *    synchronising.  Argument errors are found on the host before anything is
 *    launched.  Functions return an flce_status and never throw or abort.
 *  - Scratch memory ("workspace") lives on the device.  Either the caller
 *    lends a buffer with flce_set_workspace, or the library allocates one per
 *    device on first use and keeps it (growing it if a later call needs more;
 *    growing synchronises the device).  Calls that overlap in time on the same
 *    device share the workspace and therefore race: serialise them on one
 *    stream, or give each call a workspace of its own (flce_options).
 *  - Once the workspace is large enough (after a first call of the same size, or
 *    with a lent buffer) a call consists of kernel launches on `stream` only: no
 *    allocation, no memset, no synchronisation.  It can therefore be recorded
 *    into a HIP graph by stream capture and replayed (not while
 *    flce_timing_enable is on).
 */
#ifndef FLCE_H
#define FLCE_H

#include <stddef.h>
#include <stdint.h>

#if defined(__GNUC__)
#define FLCE_API __attribute__((visibility("default")))
#else
#define FLCE_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { FLCE_F32 = 0, FLCE_BF16 = 1 } flce_dtype;

typedef enum {
    FLCE_OK = 0,
    FLCE_ERR_NULL = 1,      /* a required pointer is NULL                     */
    FLCE_ERR_SHAPE = 2,     /* BT, H or V is not positive / too large         */
    FLCE_ERR_DTYPE = 3,     /* dtype is not an flce_dtype                     */
    FLCE_ERR_ALIGN = 4,     /* a pointer misses its alignment                 */
    FLCE_ERR_WORKSPACE = 5, /* lent workspace too small, or allocation failed */
    FLCE_ERR_HIP = 6,       /* a HIP runtime call or kernel launch failed     */
    FLCE_ERR_ARG = 7,       /* any other invalid argument                     */
    FLCE_ERR_TOO_LARGE = 8  /* more rows than an allocation-free entry point's fixed scratch holds */
} flce_status;

/* Flags for flce_fwd_bwd_ex: skip one of the two gradients (a frozen backbone
 * needs no dX, a frozen head needs no dW).  The skipped output may be NULL. */
enum { FLCE_SKIP_DX = 1, FLCE_SKIP_DW = 2 };

/*
 * The whole hot path: loss, dX and dW (paper section 3.2, FLCE paragraph).
 *   X        device, [BT x H] dtype          in
 *   W        device, [V x H]  dtype          in
 *   targets  device, [BT] int64              in
 *   loss     device, 1 float                 out (mean over valid rows)
 *   dX       device, [BT x H] dtype          out
 *   dW       device, [V x H]  dtype          out
 *   stream   hipStream_t
 */
FLCE_API int flce_fwd_bwd(const void* X, const void* W, const int64_t* targets, int64_t BT, int64_t H,
                 int64_t V, int64_t ignore_index, int dtype, float* loss, void* dX, void* dW,
                 void* stream);

/* Same, with FLCE_SKIP_* flags (paper section 4.2, Medusa paragraph: extra
 * heads trained on a frozen backbone need no hidden-state gradient). */
FLCE_API int flce_fwd_bwd_ex(const void* X, const void* W, const int64_t* targets, int64_t BT, int64_t H,
                    int64_t V, int64_t ignore_index, int dtype, float* loss, void* dX, void* dW,
                    unsigned flags, void* stream);

/*
 * The same call with its settings passed along instead of taken from the
 * process-wide setters below (flce_set_logits_budget_bytes,
 * flce_set_row_compaction), for callers that run several configurations side by
 * side or from several threads.  (Paper section 3.2, FLCE paragraph: the chunk
 * size is the method's one tuning knob.)
 *   size                 must be sizeof(flce_options) (FLCE_ERR_ARG otherwise)
 *   logits_budget_bytes  bytes one chunk of logits may take, 0 = the automatic rule
 *   row_compaction       0 or 1
 *   flags                FLCE_SKIP_*
 *   workspace            device buffer (256-byte aligned) that THIS call uses as its
 *                        scratch memory instead of the device's shared workspace, or
 *                        NULL for the shared one; owned by the caller, who keeps it
 *                        alive until the call's work on the stream has finished
 *   workspace_bytes      its size: at least flce_workspace_bytes_opt of the same
 *                        arguments (FLCE_ERR_WORKSPACE otherwise; FLCE_ERR_ALIGN for
 *                        a misaligned buffer)
 * Calls that bring their own workspace share nothing on the device, so they may
 * overlap on one GPU (different streams, different threads) as long as their
 * workspaces and outputs are distinct.
 * flce_default_options fills a struct with the current process-wide settings,
 * flags = 0 and no workspace.  opt == NULL means exactly that.
 * flce_workspace_bytes_opt is flce_workspace_bytes for such a call (0 for bad
 * arguments).
 */
typedef struct {
    size_t size;
    size_t logits_budget_bytes;
    int row_compaction;
    unsigned flags;
    void* workspace;
    size_t workspace_bytes;
} flce_options;
FLCE_API void flce_default_options(flce_options* opt);
FLCE_API int flce_fwd_bwd_opt(const void* X, const void* W, const int64_t* targets, int64_t BT, int64_t H,
                     int64_t V, int64_t ignore_index, int dtype, float* loss, void* dX, void* dW,
                     const flce_options* opt, void* stream);
FLCE_API size_t flce_workspace_bytes_opt(int64_t BT, int64_t H, int64_t V, int dtype, const flce_options* opt);

/*
 * Several output heads on the same hidden states (paper section 4.2, Medusa
 * paragraph: extra decoding heads, head j trained to predict the token j + 1
 * positions further on, each with a cross-entropy loss of its own, all sharing
 * the backbone's hidden states).  For heads j = 0 .. n_heads-1 with weights W[j]
 * and targets[j]:
 *
 *     loss_j  = mean CE of head j over ITS valid rows (as in flce_fwd_bwd)
 *     loss    = sum_j weights[j] * loss_j
 *     dW[j]   = d loss / d W[j]        dX = d loss / d X = sum_j (head j's dX)
 *
 * None of the heads' logits is stored whole: the heads run one after the other
 * through the same chunk loop and the same workspace, so peak extra memory is
 * that of a single head.  dX is summed in its storage type: head 0 writes it,
 * every later head's rows are added to the stored rows in fp32 and rounded (with
 * row compaction, see flce_set_row_compaction, the head's rows are themselves
 * rounded once before that addition).
 *
 *   W, targets, dW   HOST arrays of n_heads DEVICE pointers ([V x H] dtype,
 *                    [BT] int64, [V x H] dtype); read before the call returns.
 *                    The dW[j] must be distinct buffers.
 *   weights          HOST array of n_heads finite floats, NULL = all 1
 *   n_heads          1 .. 16
 *   loss             device, 1 float          out (weighted sum)
 *   head_losses      device, n_heads floats   out (unweighted loss_j), may be NULL
 *   flags            FLCE_SKIP_DX: dX may be NULL;  FLCE_SKIP_DW: dW may be NULL
 * Shifting the targets per head (and marking the rows that run off the end of a
 * sequence with ignore_index) is the caller's job.  With n_heads = 1 and
 * weights = NULL this is flce_fwd_bwd_ex.
 */
FLCE_API int flce_multihead_fwd_bwd(const void* X, const void* const* W, const int64_t* const* targets,
                           const float* weights, int n_heads, int64_t BT, int64_t H, int64_t V,
                           int64_t ignore_index, int dtype, float* loss, float* head_losses,
                           void* dX, void* const* dW, unsigned flags, void* stream);

/*
 * RMSNorm in front of the projection, fused into the same call (paper section
 * 3.2, RMSNorm paragraph, Eq. RMSNorm-forward / RMSNorm-backward, followed by
 * the FLCE paragraph).  For raw hidden states h[BT x H] and a scale gamma[H]:
 *
 *     x_i    = h_i / sqrt(mean_j h_ij^2 + eps) * gamma        (row by row)
 *     loss, dW as flce_fwd_bwd on X = x
 *     dh     = gradient of the loss w.r.t. h      dgamma = gradient w.r.t. gamma
 *
 * The normalised rows and their gradient exist only one chunk at a time in the
 * workspace, so peak extra memory stays independent of BT.  x is rounded to
 * dtype once (after the multiplication by gamma) before it enters the products.
 *   h, dh        device, [BT x H] dtype     in / out
 *   gamma,dgamma device, [H] dtype          in / out
 *   eps          finite, >= 0
 *   flags        FLCE_SKIP_DX: neither dh nor dgamma is computed (both may be
 *                NULL); FLCE_SKIP_DW: dW may be NULL
 * Everything else as flce_fwd_bwd.
 */
FLCE_API int flce_rmsnorm_fwd_bwd(const void* h, const void* gamma, float eps, const void* W,
                         const int64_t* targets, int64_t BT, int64_t H, int64_t V,
                         int64_t ignore_index, int dtype, float* loss, void* dh, void* dgamma,
                         void* dW, unsigned flags, void* stream);
FLCE_API size_t flce_rmsnorm_workspace_bytes(int64_t BT, int64_t H, int64_t V, int dtype);

/*
 * Stand-alone cross entropy on given logits (paper section 3.2, CE paragraph):
 * Z[BT x V] (device, dtype, row stride ldz elements, ldz >= V) is replaced in
 * place by dL/dZ; loss receives the mean over valid rows.  Needs no workspace
 * beyond a few kilobytes.
 */
FLCE_API int flce_cross_entropy_inplace(void* Z, const int64_t* targets, int64_t BT, int64_t V,
                               int64_t ldz, int64_t ignore_index, int dtype, float* loss,
                               void* stream);

/*
 * flce_cross_entropy_inplace for callers that cannot allocate device memory: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same kernels, same results bit for bit, but the device header and
 * the per-row losses live in a fixed array inside the library's device image
 * (256 + 4 * FLCE_CE_NOALLOC_MAX_ROWS bytes = 262 400 bytes on every GPU the library
 * is used on, held until the process ends) instead of the workspace, so the call
 * allocates and frees nothing and ignores flce_set_workspace and flce_timing_enable.
 *   BT > FLCE_CE_NOALLOC_MAX_ROWS returns FLCE_ERR_TOO_LARGE before anything is launched.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU
 * (different streams, different threads) race; serialise them on one stream.  The
 * array keeps the previous call's contents; the kernels overwrite every slot they
 * read, nothing needs clearing.  The first call on a device looks the array's device
 * address up (hipGetSymbolAddress): make one call outside stream capture first.
 */
#define FLCE_CE_NOALLOC_MAX_ROWS 65536
FLCE_API int flce_cross_entropy_inplace_noalloc(void* Z, const int64_t* targets, int64_t BT, int64_t V,
                                       int64_t ldz, int64_t ignore_index, int dtype, float* loss,
                                       void* stream);

/* Bytes of device scratch flce_fwd_bwd uses for this problem.  For fixed H, V
 * and dtype it does not grow with BT once BT exceeds one chunk:
 * flce_workspace_bytes(BT, ...) <= flce_workspace_bytes_max(...). */
FLCE_API size_t flce_workspace_bytes(int64_t BT, int64_t H, int64_t V, int dtype);
FLCE_API size_t flce_workspace_bytes_max(int64_t H, int64_t V, int dtype);

/* Lend a device buffer (256-byte aligned) as workspace for the current device;
 * ws == NULL returns to library-owned allocation.  The library never frees a
 * lent buffer. */
FLCE_API int flce_set_workspace(void* ws, size_t bytes);

/* Free the library-owned workspace of the current device (synchronises). */
FLCE_API int flce_release_workspace(void);

/* Chunk scheduler (paper section 3.2, FLCE paragraph: chunked logits bound the
 * memory).  The logits chunk [C x V] is sized to fit this many bytes.  0 (the
 * default) selects the automatic rule: 1 GiB, but at least 4096 rows of logits
 * (each chunk re-reads W twice and read-modify-writes the fp32 dW partial sums,
 * which only pays off over a few thousand rows); and a batch whose WHOLE logits
 * take no more than that budget plus the V x H fp32 partial sums a chunked run
 * needs is not chunked at all (no more memory than chunking, and faster).  A
 * non-zero value is taken literally: chunks of at most that many bytes, one chunk
 * only when the whole logits fit in it.  The getter returns the setting
 * (0 = automatic). */
FLCE_API int flce_set_logits_budget_bytes(size_t bytes);
FLCE_API size_t flce_get_logits_budget_bytes(void);

/* Row compaction (default on).  Rows whose target is ignore_index add nothing to
 * the loss or to dW and have a zero dX row, so each chunk first gathers its other
 * rows into a dense block, runs the products and the row kernel on that block
 * only, and scatters dX back; the chunk's live row count stays on the device (no
 * host synchronisation).  The results are the same (dW sums the same non-zero
 * terms in other groups); the time of a chunk shrinks with its share of ignored
 * rows, in steps of the 256-row tiles.  The valid rows are dealt evenly to as few
 * of the chunk launches as can hold them (the last ones); launches before them do
 * no work, so a batch with many ignored rows runs fewer chunks.  Only problems that run entirely on the
 * tuned kernel are compacted.  Off: every row is projected; for batches known to
 * have no ignored row that saves the gather and scatter copies (about 0.5 % of
 * the time at V = 128K, 1 % at V = 32K). */
FLCE_API int flce_set_row_compaction(int on);
FLCE_API int flce_get_row_compaction(void);

/* Rows per chunk C and number of chunks the scheduler picks (host only). */
FLCE_API int64_t flce_chunk_rows(int64_t BT, int64_t H, int64_t V, int dtype);
FLCE_API int64_t flce_num_chunks(int64_t BT, int64_t H, int64_t V, int dtype);

/* The largest logits budget (a whole number of 256-row steps, for
 * flce_set_logits_budget_bytes or flce_options) whose plan for this problem needs at
 * most max_workspace_bytes of workspace under the current row compaction setting, for
 * callers who have a fixed amount of memory to give; 0 if not even 256-row chunks
 * fit (or the arguments are bad).  Fewer rows per chunk cost time: every chunk
 * re-reads W twice and passes over the fp32 dW partial sums (paper section 3.2, FLCE
 * paragraph: the chunk size trades memory for speed).  Host only. */
FLCE_API size_t flce_logits_budget_for_workspace(int64_t BT, int64_t H, int64_t V, int dtype,
                                                 size_t max_workspace_bytes);

/* Number of K ranges (K = V) the dX product of one chunk is cut into so that its
 * output tiles fill whole rounds of the chip's CUs; 1 = not cut (host only). */
FLCE_API int flce_dx_k_ranges(int64_t BT, int64_t H, int64_t V, int dtype);

/* The paper's own chunk-size rule, 2^ceil(log2(ceil(BT / ceil(V/H)))), for
 * reference and reporting; the scheduler above does not use it. */
FLCE_API int64_t flce_paper_chunk_rows(int64_t BT, int64_t H, int64_t V);

/* Bytes of the full logits tensor BT x V that is never materialised. */
FLCE_API size_t flce_full_logits_bytes(int64_t BT, int64_t V, int dtype);

/*
 * Per-kernel timing for benchmarks (not for production loops).  While enabled,
 * every kernel launch of flce_fwd_bwd / flce_cross_entropy_inplace is bracketed
 * by HIP events on the call's own stream and booked under an flce_kernel_kind.
 * flce_timing_collect waits for the recorded events, adds up milliseconds and
 * launch counts per kind into the caller's HOST arrays (FLCE_NUM_KINDS entries
 * each) and clears the records.  At most 8192 launches are kept between two
 * collects; later ones are not recorded.
 */
typedef enum {
    FLCE_KIND_LOGITS_GEMM = 0, /* Z_c = X_c W^T                      */
    FLCE_KIND_CE_ROWS = 1,     /* loss + in-place dlogits             */
    FLCE_KIND_DX_GEMM = 2,     /* dX_c = G_c W                        */
    FLCE_KIND_DW_GEMM = 3,     /* dW += G_c^T X_c                     */
    FLCE_KIND_OTHER = 4,       /* count, transposes, casts, finalize  */
    FLCE_NUM_KINDS = 5
} flce_kernel_kind;
FLCE_API int flce_timing_enable(int on);
FLCE_API int flce_timing_collect(double* total_ms, int64_t* launches);

/* Measurement aid, not part of the path (benchmarks report it beside the product
 * kernels' rate): enqueues on `stream` one launch of `workgroups` workgroups (4
 * wavefronts each, one per SIMD: 256 fill the chip) that execute iters * 16
 * v_mfma_f32_32x32x16_bf16 per wavefront on register operands and touch no memory
 * but `out` (device, at least workgroups * 256 floats, overwritten with checksums).
 * pattern 0: zero operands; 1: one fixed pair of fragments; 2: 4 A x 4 B fragments
 * per wavefront in the order of a K sub-step of the product kernel, A ~ N(0,1),
 * B ~ N(0, std_b^2), rounded to bf16.  Work: workgroups * 4 * iters * 16 * 32768
 * flops.  The sustained rate depends on the pattern because the chip lowers its
 * clock as more operand bits toggle; pattern 2 is the ceiling for products of such
 * data.  FLCE_ERR_ARG for sizes out of range: workgroups <= 65536 and workgroups *
 * iters <= 2^26, which bounds a launch to about 0.1 s. */
FLCE_API int flce_mfma_ceiling_launch(int pattern, int workgroups, int iters, float std_b, float* out,
                                      size_t out_floats, void* stream);

FLCE_API const char* flce_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* FLCE_H */
