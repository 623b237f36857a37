/*
 * lora_sched.h -- C ABI of the two host-side schedulers that sit directly around the multi-LoRA
 * linear layer of lora_mi355x.h: the adaptive batching scheduler that forms the batches the
 * layer's segment builder consumes (paper section 4.2, equations 2-5), and the greedy
 * value-density residency policy that decides which adapters (and other artifacts) stay in GPU
 * memory and which are offloaded when memory is needed (sections 4.1 and 4.3, equations 1, 6, 7).
 *
 * Everything here is host code: no GPU call, no device pointer.  All times are milliseconds as
 * doubles on a clock of the caller's choosing (the schedulers never read a clock themselves, so
 * they are deterministic and testable with simulated time).  Every function returns 0 or a
 * negative lora_sched_status.  Objects are not thread-safe: serialise calls per object.
 */
#ifndef LORA_SCHED_H
#define LORA_SCHED_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum lora_sched_status {
    LORA_SCHED_OK = 0,
    LORA_SCHED_ERR_INVALID_ARG = -1, /* null pointer, index out of range, non-finite or negative time / size */
    LORA_SCHED_ERR_CAPACITY = -2     /* an output array is too small for the result */
} lora_sched_status;

/* ======================= adaptive batching (section 4.2) ===================================== */

/* One serverless function = one LoRA adapter on the shared backbone.  Its batch of b requests
 * needs T(b) = t0_ms + alpha_ms * (b - 1) to produce the first token (equation 2; t0 and alpha
 * come from offline profiling) and must do so within slo_ms of a request's arrival. */
typedef struct lora_function_profile {
    double t0_ms;      /* > 0 */
    double alpha_ms;   /* >= 0 */
    double slo_ms;     /* > 0 */
    int32_t adapter;   /* adapter id handed to lora_plan for this function's requests (-1: none) */
    int32_t max_batch; /* 0: B = the largest b with T(b) <= slo_ms (at least 1); > 0: that, capped */
} lora_function_profile;

typedef struct lora_batcher lora_batcher;

/* One dispatched batch.  request ids / token counts are written to the arrays the caller passes
 * to lora_batcher_poll, at [first, first + n). */
typedef struct lora_batch {
    int32_t function;
    int32_t adapter;
    int32_t n;           /* requests in the batch */
    int32_t first;       /* offset of its requests in the output arrays */
    double wait_ms;      /* w: how long its oldest request has waited at dispatch */
    double margin_ms;    /* deadline margin (equation 5) at dispatch: slo - (w + M * T(n)) */
    double t_batch_ms;   /* T(n) (equation 2) */
} lora_batch;

int lora_batcher_create(lora_batcher **out, const lora_function_profile *functions, int32_t n_functions);
int lora_batcher_destroy(lora_batcher *b);

/* The batch size limit B_i of a function (section 4.2: "the maximum batch size within the SLO"). */
int lora_batcher_max_batch(const lora_batcher *b, int32_t function, int32_t *out);

/* The function's current batch size setting N_i, 1 <= N_i <= B_i (initially max(1, B_i / 2)): a
 * batch closes when it holds N_i requests, and N_i fixes the batch delay of equation 3,
 * d_i = slo - T(N_i) -- the smaller the batch size, the longer the scheduler waits.  The paper
 * leaves the choice of N_i to an adjustment loop it does not describe; here the caller sets it. */
int lora_batcher_set_batch_size(lora_batcher *b, int32_t function, int32_t n);
int lora_batcher_batch_size(const lora_batcher *b, int32_t function, int32_t *out);
int lora_batcher_delay(const lora_batcher *b, int32_t function, double *delay_ms_out);

/* A request for `function` with n_tokens prompt tokens arrives at now_ms.  Times passed to one
 * batcher must not decrease.  *request_id_out (may be NULL) receives its id: 0, 1, 2, ... in
 * order of submission. */
int lora_batcher_submit(lora_batcher *b, int32_t function, int32_t n_tokens, double now_ms, int64_t *request_id_out);

/* Dispatch decision at now_ms with `running` batches already executing on the GPU.
 * Fill or expire (section 4.2, local level): a function's forming batch is its oldest
 * min(queued, N_i) requests; it is READY when it holds N_i requests or when its oldest request
 * has waited the batch delay d_i (equation 3).  Global level: with M = running + 1 batches
 * sharing the GPU a batch of b requests takes M * T(b) (equation 4) and its deadline margin is
 * slo - (w + M * T(b)) (equation 5), w = now - arrival of its oldest request.  Ready batches are
 * dispatched in order of increasing margin (ties: lower function index), at most max_batches of
 * them; the others keep collecting requests.
 *
 * Outputs (HOST arrays of the caller): batches[max_batches]; request_ids / req_adapter /
 * req_ntok [max_requests], the dispatched requests in dispatch order -- req_adapter and req_ntok
 * are exactly the arrays lora_plan() takes for the multi-LoRA batch made of all dispatched
 * batches.  *n_batches_out, *n_requests_out receive the counts.  If the next ready batch does
 * not fit max_requests it stays queued (CAPACITY is returned only if nothing at all fits). */
int lora_batcher_poll(lora_batcher *b, double now_ms, int32_t running, int32_t max_batches, lora_batch *batches,
                      int32_t max_requests, int64_t *request_ids, int32_t *req_adapter, int32_t *req_ntok,
                      int32_t *n_batches_out, int32_t *n_requests_out);

/* Earliest time at which some batch is ready (now_ms if one already is); +inf (HUGE_VAL) if
 * every queue is empty.  Between now and that time nothing can be dispatched
 * unless a request arrives. */
int lora_batcher_next_event(const lora_batcher *b, double now_ms, int32_t running, double *t_out);

int lora_batcher_queued(const lora_batcher *b, int32_t function, int32_t *out);

/* ======================= artifact residency: pre-loading and offloading ======================= */

/* Artifact kinds of a function (section 4.1) and the places one can be pre-loaded in. */
typedef enum lora_artifact_kind { LORA_ART_LIBRARY = 0, LORA_ART_BACKBONE = 1, LORA_ART_ADAPTER = 2, LORA_ART_KERNEL = 3 } lora_artifact_kind;
typedef enum lora_place { LORA_PLACE_NONE = 0, LORA_PLACE_CONTAINER = 1, LORA_PLACE_GPU = 2 } lora_place;

/* One artifact of one function.  value = loading delay saved x request arrival rate (section
 * 4.1); value density = value / bytes.  Backbones are shared: artifacts of kind BACKBONE with
 * the same share_id are ONE object (placed, counted and valued once per place; the values of the
 * functions that share it add up).  Libraries pre-load in the container only, kernels on the GPU
 * only, backbones and adapters in either (the GPU copy is the one inference uses). */
typedef struct lora_artifact {
    int32_t function;
    int32_t kind;       /* lora_artifact_kind */
    int32_t share_id;   /* BACKBONE: which backbone; others: ignored */
    int32_t pinned;     /* offloading only: != 0 -- in use by an invoked function, never offloaded */
    double bytes;       /* > 0 */
    double value;       /* >= 0 */
} lora_artifact;

/* Pre-loading decision (equation 1, greedy by value density under the constraints of section
 * 4.1): candidates are (artifact, place) pairs; they are taken in order of decreasing density
 * (ties: lower artifact index, container before GPU) whenever capacity and precedence allow, and
 * the scan restarts after every placement until none fits --
 *   capacity:   bytes placed in the container <= container_bytes, on the GPU <= gpu_bytes;
 *   precedence: a backbone or adapter needs its function's library in the container first; on
 *               the GPU an adapter needs its function's backbone on the GPU (coupling), a kernel
 *               needs its function's backbone and adapter on the GPU;
 *   an artifact is placed at most once per place; a GPU placement does not need the container copy.
 * place_out[n] (HOST) receives a bit mask per artifact: bit 0 container, bit 1 GPU.  Shared
 * backbones: every artifact of the share gets the same mask.  *value_out (may be NULL): the
 * objective of equation 1 reached. */
int lora_preload_greedy(const lora_artifact *artifacts, int32_t n, double container_bytes, double gpu_bytes,
                        uint8_t *place_out, double *value_out);

/* Offloading decision (equations 6-7, same greedy): need_bytes must be freed on the GPU.
 * on_gpu[n] says which artifacts are there now.  Models (backbones, adapters) and kernels that
 * are not pinned are removed in order of increasing value density (ties: higher artifact index
 * first) until the bytes freed reach need_bytes; a backbone goes only after every adapter and
 * kernel that depends on it on the GPU has gone or been chosen, an adapter only after its
 * function's kernel.  evict_out[n] (HOST) receives 1 for the artifacts to remove.  *freed_out
 * and *value_lost_out (may be NULL) receive the totals.  Returns LORA_SCHED_ERR_CAPACITY (with
 * the best effort in the outputs) if even removing everything allowed frees less than need_bytes. */
int lora_offload_greedy(const lora_artifact *artifacts, int32_t n, const uint8_t *on_gpu, double need_bytes,
                        uint8_t *evict_out, double *freed_out, double *value_lost_out);

const char *lora_sched_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* LORA_SCHED_H */
