/*
 * lora_mi355x.h -- C ABI of the multi-LoRA batched linear layer for MI355X (gfx950).
 *
 * The layer is the "unmerged" LoRA linear of the paper (section 2.2: the
 * backbone product and the adapter product are computed separately and their
 * results gathered; section 4.4 and section 5: the shared backbone stays
 * read-only and the adapter computation is kept distinct), for a batch in
 * which every request carries its own adapter on one resident backbone:
 *
 *     Y[t,:] = X[t,:] W0 + s_a (X[t,:] A_a) B_a ,   a = adapter of row t's request
 *     Y[t,:] = X[t,:] W0                            for requests with adapter -1
 *
 * Conventions
 *   - Plain C, no exceptions, no mutable global state (the one file-scope
 *     object is the scratch array of lora_linear_static()).  Every function returns an int:
 *     LORA_OK (0) or a negative lora_status; lora_strerror() names it.
 *   - "host" / "device" is stated for every pointer.  The library never
 *     allocates device memory and never synchronises the stream unless a
 *     function says so: plan storage and workspace are caller-provided device
 *     buffers (e.g. a torch tensor's data_ptr()).
 *   - W0, X, A_a, B_a are const: no kernel ever writes them.  W0 is used in the
 *     layout its owner keeps it in (it may be memory shared by another process,
 *     section 4.4), never re-laid-out or copied.
 *   - Storage layouts (row-major; "ld" = row stride in elements):
 *         X   [T, ldx]   rows of a request contiguous, requests in submission order
 *         W0  [N, ldw]   nn.Linear.weight, i.e. W0[k,n] of the formula at W0[n*ldw + k]
 *         A_a [r_a, K]   A_a[k,j] of the formula at A_a[j*K + k]
 *         B_a [N, r_a]   B_a[j,n] of the formula at B_a[n*r_a + j]
 *         Y   [T, ldy]
 *   - dtype LORA_DTYPE_BF16: all five tensors bf16, fp32 accumulation; above
 *     128 rows the intermediate s_a (X A_a) is rounded once to bf16 before the
 *     second product (up to 128 rows it stays fp32).  dtype LORA_DTYPE_F32:
 *     everything fp32.
 *   - Run-to-run results are bitwise reproducible (no floating-point atomics).
 *   - Thread safety: a ctx may be shared by threads as long as calls that use
 *     the same plan_buf / workspace / Y are ordered by the caller; lora_plan()
 *     takes an internal lock for its pinned staging ring.
 */
#ifndef LORA_MI355X_H
#define LORA_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lora_ctx lora_ctx;

/* A hipStream_t, passed as an opaque pointer so that this header needs no HIP
 * header (torch.cuda.current_stream().cuda_stream is this value). */
typedef void *lora_stream_t;

typedef enum lora_dtype { LORA_DTYPE_F32 = 0, LORA_DTYPE_BF16 = 1 } lora_dtype;

typedef enum lora_status {
    LORA_OK = 0,
    LORA_ERR_INVALID_ARG = -1,           /* null pointer, negative size, unknown dtype/option   */
    LORA_ERR_BAD_ADAPTER_ID = -2,        /* request adapter id outside [-1, n_adapters)         */
    LORA_ERR_LENGTH_MISMATCH = -3,       /* negative token count, or sum of counts != T         */
    LORA_ERR_ADAPTER_NOT_RESIDENT = -4,  /* a used adapter has rank 0 (or null weights)         */
    LORA_ERR_RANK_TOO_LARGE = -5,        /* a used adapter's rank exceeds r_max                 */
    LORA_ERR_WORKSPACE_TOO_SMALL = -6,   /* plan_buf or workspace smaller than *_bytes() says   */
    LORA_ERR_ALIGNMENT = -7,             /* pointer not 16-byte aligned / stride not 16-byte    */
    LORA_ERR_SHAPE = -8,                 /* K, N, ld*, rank violate the stated requirements     */
    LORA_ERR_HIP = -9,                   /* a HIP call failed; see lora_last_hip_error()        */
    LORA_ERR_PLAN = -10                  /* plan not built by this library / built with errors  */
} lora_status;

/* Limits (checked, never silently clamped). */
#define LORA_MAX_REQUESTS 65536   /* requests per batch                                  */
#define LORA_MAX_ADAPTERS 65536   /* adapter slots in a table                            */
#define LORA_MAX_RANK 512         /* rank of one adapter; ranks are multiples of 8       */
#define LORA_STATIC_SCRATCH_BYTES (32u << 20) /* workspace limit of lora_linear_static()     */

/*
 * Adapter pointer table.  A table, not one packed tensor, because adapters are
 * loaded and evicted one at a time and may have different ranks (sections 4.1
 * and 4.3 of the paper: artifacts, adapters included, come and go
 * independently).  The struct itself lives on the HOST; A, B and scale point to
 * DEVICE arrays of n_adapters entries; A[a] / B[a] are DEVICE pointers to that
 * adapter's weights (16-byte aligned), or NULL for a slot that is not resident.
 * The caller owns everything and may edit entries between calls (stream-ordered).
 * The ranks are not part of the table: a rank belongs to the adapter, not to one
 * projection's weights, so the rank array (and r_max, the row stride of the
 * intermediate) is an argument of lora_plan*(), which fixes them for every
 * projection and layer that uses the plan; a table entry must then point at
 * weights of that rank.
 */
typedef struct lora_adapter_table_t {
    int32_t n_adapters;
    int32_t reserved;
    const void *const *A; /* device: [n_adapters] device pointers, A[a] -> [rank[a], K] */
    const void *const *B; /* device: [n_adapters] device pointers, B[a] -> [N, rank[a]] */
    const float *scale;   /* device: [n_adapters] fp32 s_a                               */
} lora_adapter_table_t;

/*
 * Segment table ("plan"): token rows grouped by adapter.  Plain data, filled by
 * lora_plan*(): device pointers into the caller's plan_buf plus host copies of
 * the sizes.  Valid until plan_buf is freed or reused; one plan serves every
 * projection and layer of the same batch.
 *
 * Row order: rows are sorted stably by adapter id (ascending; rows without an
 * adapter last).  "slot" = position in that order.
 */
typedef struct lora_plan_t {
    int64_t T;              /* token rows                                                   */
    int32_t n_req;
    int32_t n_adapters;
    int32_t r_max;          /* row stride of the intermediate V, >= every used rank         */
    int32_t seg_cap;        /* capacity of the seg_* arrays                                 */
    int32_t ext_cap;        /* capacity of ext_rec                                          */
    int32_t magic;
    int32_t unit_rows;      /* most rows of a work unit: 64, or 16 in a plan of few rows and segments */
    const int32_t *perm;        /* device [T]        slot -> row index of X / Y             */
    const int32_t *row_seg;     /* device [T]        slot -> segment                        */
    const int32_t *row_adapter; /* device [T]        row (original order) -> adapter id     */
    const int32_t *row_ext;     /* device [T]        row -> (first column of its adapter on the concatenated rank axis / 8) << 7 | rank / 8 */
    const int32_t *seg_adapter; /* device [seg_cap]  adapter id of the segment (-1 = none)  */
    const int32_t *seg_indptr;  /* device [seg_cap+1] first slot of the segment             */
    const int32_t *seg_rank;    /* device [seg_cap]  rank (0 for the no-adapter segment)    */
    const int32_t *seg_ext;     /* device [seg_cap+1] exclusive prefix sum of seg_rank      */
    const int32_t *seg_unit;    /* device [seg_cap+1] prefix sum of ceil(rows/unit_rows) (work list) */
    const int32_t *unit_rec;    /* device [(T/16+seg_cap+8)*4] work units: adapter, rank (| 1<<16: segment of >= 64 rows), first slot, rows */
    const int32_t *ext_rec;     /* device [ext_cap*4] per 8 ranks: adapter, rank<<16|j0, slot_lo, slot_hi */
    const int32_t *tok_off;     /* device [n_req+1]  first row of every request             */
    int32_t *scalars;           /* device [8]: n_seg, build status, ext_total, n_units, T, evicted flag */
} lora_plan_t;

typedef struct lora_linear_desc {
    int32_t dtype;          /* lora_dtype */
    int32_t K;              /* d_in:  multiple of 8, > 0                                    */
    int32_t N;              /* d_out: > 0                                                   */
    int32_t flags;          /* must be 0                                                    */
    const void *X;          /* device [T, ldx]                                              */
    int64_t ldx;            /* >= K, multiple of 8 (bf16) or 4 (fp32); X smaller than 4 GiB*/
    const void *W0;         /* device [N, ldw], const, externally owned                     */
    int64_t ldw;            /* >= K, multiple of 8 (bf16) or 4 (fp32); < 4 Mi elements     */
    void *Y;                /* device [T, ldy]; must not alias X, W0 or the adapters        */
    int64_t ldy;            /* >= N, multiple of 8 (bf16) or 4 (fp32)                       */
    const lora_adapter_table_t *tbl; /* host pointer; NULL = backbone product only         */
    void *workspace;        /* device, 256-byte aligned, lora_linear_workspace_bytes() big  */
    size_t workspace_bytes;
} lora_linear_desc;

/* ---- context ----------------------------------------------------------- */

/* Creates a context on device `device_ordinal` (host int).  It caches device
 * properties, owns a small pinned host staging ring used by lora_plan(), and
 * does the per-device set-up of the kernels (dynamic-LDS grants; the address
 * of lora_linear_static()'s scratch on that device), so that no later call
 * has to: create contexts outside stream capture.  *out is set to NULL on
 * failure.  Errors: INVALID_ARG, HIP. */
int lora_ctx_create(lora_ctx **out, int device_ordinal);
int lora_ctx_destroy(lora_ctx *ctx);

/* Overrides of the built-in kernel choices, for tests and measurements:
 * "gemm_variant" (0 tile 128x128, 1 256x128, 3 64x64,
 * 4 the decode path (bf16, up to 128 rows), 5 256x256 on 4 waves,
 * 9 128x192, 10 256x192, 11 256x224), "decode_waves" (waves per workgroup of
 * the decode path's streaming kernel: 8..12), "decode_max_rows" (0: never
 * the decode path), "plan_variant" (1: never the one-lane-per-request
 * plan kernels), "plan_fused_rows" (most rows for which one workgroup builds
 * the whole plan), "expand_split" (0 / 1: adapter term always computed inside
 * the GEMM / by the separate expand kernel whenever the workspace has room
 * for it), "gemm_split_k" (0: never split the tiled GEMM along K),
 * "shrink_rank_block" (8 / 16 / 32 / 64).  value < 0 restores the
 * built-in choice.  Results never depend on them beyond fp32 summation order.
 * Not thread-safe against concurrent calls on the same ctx.  Errors:
 * INVALID_ARG for an unknown name or a value the option does not take. */
int lora_ctx_set_option(lora_ctx *ctx, const char *name, int value);

/* ---- step a1: segment / indptr builder ---------------------------------- */

/* Pure host check of a batch (all pointers HOST; adapter_rank has n_adapters
 * entries, 0 = not resident).  Checks, in this order: argument sanity
 * (INVALID_ARG), ids in [-1, n_adapters) (BAD_ADAPTER_ID), counts >= 0 and
 * summing to T_expected without overflow (LENGTH_MISMATCH), every used
 * adapter resident (ADAPTER_NOT_RESIDENT), rank a multiple of 8 (SHAPE) and
 * <= r_max (RANK_TOO_LARGE).  Touches no GPU.  Optional outputs (may be
 * NULL): number of segments and total rank over the used adapters. */
int lora_plan_validate(const int32_t *req_adapter, const int32_t *req_ntok, int32_t n_req,
                       const int32_t *adapter_rank, int32_t n_adapters, int32_t r_max,
                       int64_t T_expected, int32_t *n_seg_out, int64_t *ext_total_out);

/* Bytes of device memory a plan for such a batch needs (0 on invalid sizes). */
size_t lora_plan_bytes(int32_t n_req, int64_t T, int32_t n_adapters, int32_t r_max);

/* Builds the plan from HOST request arrays (the batcher is CPU code: section
 * 4.2, the batching scheduler forms per-function batches on the controller).
 * Validates as lora_plan_validate() before touching the GPU, copies the three
 * small arrays through the context's pinned ring (they may be freed on
 * return) and builds every T-sized array on the device, in plan_buf (DEVICE,
 * 256-byte aligned, >= lora_plan_bytes()).  Asynchronous on `stream`; may
 * block only when the pinned ring is full (4 plans in flight).  T == 0 is
 * valid.  Errors: as lora_plan_validate, plus WORKSPACE_TOO_SMALL, ALIGNMENT, HIP. */
int lora_plan(lora_ctx *ctx, const int32_t *req_adapter, const int32_t *req_ntok, int32_t n_req,
              const int32_t *adapter_rank, int32_t n_adapters, int32_t r_max, int64_t T_expected,
              void *plan_buf, size_t plan_buf_bytes, lora_stream_t stream, lora_plan_t *out);

/* Same, with req_adapter, req_ntok and adapter_rank already resident on the
 * DEVICE (read when the stream reaches the build kernels; keep them alive
 * until then).  Nothing is validated on the host beyond sizes; the device
 * records the first lora_status it finds in the plan's status word, and every
 * kernel that later consumes such a plan does nothing.  Query it with
 * lora_plan_status(). */
int lora_plan_device(lora_ctx *ctx, const int32_t *req_adapter, const int32_t *req_ntok, int32_t n_req,
                     const int32_t *adapter_rank, int32_t n_adapters, int32_t r_max, int64_t T_expected,
                     void *plan_buf, size_t plan_buf_bytes, lora_stream_t stream, lora_plan_t *out);

/* Synchronises `stream` and returns the plan's device-side status: the
 * negative lora_status recorded by the build if it failed (every kernel given
 * such a plan does nothing); else ADAPTER_NOT_RESIDENT if a layer kernel since
 * the build met a NULL table entry of an adapter the batch uses (that call
 * left the adapter term of those rows out -- their Y is the backbone product
 * or undefined -- and every other row, projection and later call is
 * unaffected; the flag stays set until the plan is rebuilt); else LORA_OK.
 * *n_seg_out (HOST, may be NULL) receives the number of segments. */
int lora_plan_status(lora_ctx *ctx, const lora_plan_t *plan, lora_stream_t stream, int32_t *n_seg_out);

/* ---- steps a2-a4: the layer --------------------------------------------- */

/* Device bytes lora_linear needs in desc->workspace for T rows, K inputs, N
 * outputs and V row stride r_max.  It holds the intermediate V = s_a X A_a
 * ([T, r_max]) and, for decode-sized bf16 batches (T <= 128), the fp32 partial
 * sums of the slices the contraction axis is cut into (about
 * ceil(K / 512) * (N + T * r_max) * 4 bytes per 16 rows of the batch).  One
 * workspace may serve calls of different shapes as long as it is big enough
 * for each and the calls do not overlap in time.  Returns 0 for invalid
 * arguments. */
size_t lora_linear_workspace_bytes(int64_t T, int32_t K, int32_t N, int32_t r_max, int32_t dtype);

/* The workspace size that lets every batch take its fastest path: the size
 * above plus room for the adapter term in fp32 ([T, N]; bf16 batches of any
 * size, fp32 ones of more than 128 rows).  Batches of many small segments,
 * and decode-sized batches with much adapter work, then compute that term
 * in a weight-streaming kernel of its own and the GEMM (or the decode path's
 * reduction) adds it before the single rounding of Y; with a smaller
 * workspace the term is computed inside the GEMM / the reduction (same
 * result within the rounding of the intermediate V and fp32 summation order).  For batches of 129 to
 * 1024 rows whose output tiles would leave most of the chip idle (and larger
 * ones with K >= 10240 into few columns) it also has
 * room for the fp32 partial outputs of a GEMM split along K (2 to 8 copies
 * of [T, N]; a second launch sums them in a fixed order, adds the adapter
 * term and rounds Y once).  Returns 0 for invalid arguments. */
size_t lora_linear_workspace_bytes_preferred(int64_t T, int32_t K, int32_t N, int32_t r_max, int32_t dtype);

/* a2, shrink: V[row, :r_a] = s_a * X[row, :] A_a for every row with an
 * adapter, written to the workspace (bf16 for the bf16 path, fp32 for fp32).
 * It is the first of the layer's two stages whatever the batch: for
 * decode-sized bf16 batches (T <= 128, unless the output is so wide that the
 * tiled path is cheaper) the launch streams W0 and the used A_a against X
 * once, slice by slice of the contraction axis, and leaves fp32 partial sums
 * of both X W0 and X A_a in the workspace, so call it even when desc->tbl is
 * NULL.
 * Asynchronous on `stream`.  No-op when T == 0. */
int lora_shrink(lora_ctx *ctx, const lora_plan_t *plan, const lora_linear_desc *desc, lora_stream_t stream);

/* a3 + a4, base GEMM with the adapter term added before the single rounding and
 * store of Y: Y[row, :] = X[row, :] W0 + V[row, :r_a] B_a, V (and the copy of
 * X) taken from the workspace as lora_shrink() left them for the same plan,
 * desc->X and K (decode-sized bf16 batches: sums the partial sums lora_shrink()
 * left, adds V B_a in fp32 -- V never rounded -- and stores Y; with much
 * adapter work and a workspace of the preferred size V is reduced and rounded
 * to bf16 by a launch of its own and the term comes from the weight-streaming
 * kernel below).  Otherwise two forms, same result up
 * to fp32 summation order: the expand
 * as extra K-steps of the GEMM's own MFMA loop (always, with a workspace of the
 * minimal size; and for segments of 64 rows and more up to rank 64), or -- with
 * a workspace of the preferred size and many small segments -- a
 * weight-streaming kernel of its own that leaves the term in fp32 in the
 * workspace ([T, N], written and read once), which the GEMM's epilogue adds to
 * its fp32 accumulators.  Batches whose tiles would leave
 * most of the chip idle split the GEMM along K as well (see
 * lora_linear_workspace_bytes_preferred).  Either way every element of Y is
 * rounded and written exactly once. */
int lora_gemm_expand(lora_ctx *ctx, const lora_plan_t *plan, const lora_linear_desc *desc, lora_stream_t stream);

/* The whole layer: lora_shrink() then lora_gemm_expand() on `stream`.  Returns
 * after enqueueing.  Errors (all found before the first launch): INVALID_ARG,
 * PLAN, SHAPE, ALIGNMENT, WORKSPACE_TOO_SMALL; HIP if a launch fails. */
int lora_linear(lora_ctx *ctx, const lora_plan_t *plan, const lora_linear_desc *desc, lora_stream_t stream);

/* lora_linear() for callers that cannot allocate or bring a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): desc->workspace must be NULL and desc->workspace_bytes 0; the
 * kernels use a static device array of LORA_STATIC_SCRATCH_BYTES that the
 * library's code object holds on every GPU it runs on until the process ends.
 * No allocation, no memset, no synchronisation: launches only.  Problems whose
 * lora_linear_workspace_bytes() exceeds LORA_STATIC_SCRATCH_BYTES are rejected
 * with WORKSPACE_TOO_SMALL.  All calls on one GPU share that array (it keeps
 * the last call's contents; nothing in it needs to start at zero): calls that
 * overlap in time on one GPU race -- order them on one stream.  Same result as
 * lora_linear() with a workspace of LORA_STATIC_SCRATCH_BYTES.  Other errors:
 * as lora_linear(). */
int lora_linear_static(lora_ctx *ctx, const lora_plan_t *plan, const lora_linear_desc *desc, lora_stream_t stream);

/* Several projections of the SAME activations in one call -- fused QKV, gate + up
 * of a decoder layer (all seven of which carry LoRA here): descs (HOST array
 * of n HOST pointers, 1 <= n <= LORA_MAX_MULTI) share X, ldx, K, dtype and the
 * plan; each has its own W0, N, Y, adapter table and workspace (of its own
 * lora_linear_workspace_bytes[_preferred]).  Computes what n calls of
 * lora_linear compute (same formula per projection; fp32 summation order may
 * differ, as between tile shapes); every kernel runs as one launch whose grid
 * holds the work of all projections (decode-sized batches: unless one of the
 * projections has much adapter work or takes the tiled path -- then projection
 * by projection).
 * Errors: those of lora_linear for any desc; INVALID_ARG also for n out of
 * range, descs that differ in X / ldx / K / dtype, or two descs with the same Y
 * or workspace. */
#define LORA_MAX_MULTI 4
int lora_linear_multi(lora_ctx *ctx, const lora_plan_t *plan, const lora_linear_desc *const *descs, int32_t n,
                      lora_stream_t stream);

/* Profiling mode, for benchmarks: between lora_profile_begin() and
 * lora_profile_end() every kernel the library launches through `ctx` is
 * bracketed by its own pair of HIP events (at most max_launches per kernel
 * kind; later launches run untimed).  lora_profile_end() synchronises `stream`
 * and writes, for the LORA_PROFILE_KINDS kernel kinds in the order {plan
 * segments, plan fill, first layer kernel (shrink; for decode-sized batches
 * the weight-streaming kernel), second layer kernel (GEMM with the fused
 * expand; for decode-sized batches the reduction + expand), separate expand
 * kernel}, the average execution time in microseconds into
 * avg_us[LORA_PROFILE_KINDS] (HOST) and the number of timed launches into
 * counts[LORA_PROFILE_KINDS] (HOST).  Errors: INVALID_ARG, HIP. */
#define LORA_PROFILE_KINDS 5
int lora_profile_begin(lora_ctx *ctx, int max_launches);
int lora_profile_end(lora_ctx *ctx, lora_stream_t stream, double *avg_us, int32_t *counts);

/* Name of the GEMM kernel variant lora_gemm_expand() would launch for this
 * problem ("decode_tb4", "tile_128x128", ...), for reports.  Host only. */
const char *lora_gemm_kernel_name(lora_ctx *ctx, int64_t T, int32_t K, int32_t N, int32_t dtype);

/* ---- the shared backbone across processes (section 4.4, section 5) -------- */

/* The backbone's tensors live in ONE process (the "backbone function") and every LoRA function
 * process maps them read-only, zero-copy, through an inter-process memory handle; W0 of
 * lora_linear_desc is such a mapped pointer.  These four calls are that plumbing (the paper's
 * IPC-handle plugin): the holder allocates a region of its own (a whole device allocation, which
 * is what a handle names; keep each below 2 GiB), fills it, exports the handle as
 * LORA_IPC_HANDLE_BYTES opaque bytes that it passes to the other processes by any means; they
 * open it, use the returned DEVICE pointer as W0 for as long as they like, and close it.  The
 * mapping costs no copy and no device memory beyond the driver's bookkeeping.  The library never
 * writes through W0.  All four: device `device_ordinal` of the calling process; errors
 * INVALID_ARG, HIP. */
#define LORA_IPC_HANDLE_BYTES 64
int lora_backbone_alloc(int device_ordinal, size_t bytes, void **dev_ptr_out);
int lora_backbone_free(int device_ordinal, void *dev_ptr);
int lora_backbone_export(int device_ordinal, const void *dev_ptr, unsigned char handle_out[LORA_IPC_HANDLE_BYTES]);
int lora_backbone_open(int device_ordinal, const unsigned char handle[LORA_IPC_HANDLE_BYTES], void **dev_ptr_out);
int lora_backbone_close(int device_ordinal, void *dev_ptr);

/* ---- errors ------------------------------------------------------------- */
const char *lora_strerror(int status);
/* The hipError_t (as int) of the last failing HIP call on this thread, 0 if none. */
int lora_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LORA_MI355X_H */
