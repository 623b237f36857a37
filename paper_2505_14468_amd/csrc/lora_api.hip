// Host side of the C ABI: argument validation, plan storage layout, kernel selection and launch.
// Every check that can be made without the GPU is made before the first HIP call.
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>

#include "../../include/lora_mi355x.h"
#include "kernels.h"

using namespace lora;

static_assert(LORA_ERR_BAD_ADAPTER_ID == kErrBadAdapterId, "status codes out of sync");
static_assert(LORA_ERR_LENGTH_MISMATCH == kErrLengthMismatch, "status codes out of sync");
static_assert(LORA_ERR_ADAPTER_NOT_RESIDENT == kErrNotResident, "status codes out of sync");
static_assert(LORA_ERR_RANK_TOO_LARGE == kErrRankTooLarge, "status codes out of sync");
static_assert(LORA_ERR_SHAPE == kErrShape, "status codes out of sync");
static_assert(LORA_MAX_MULTI == kMaxGemmSets, "projection limit out of sync");
static_assert(LORA_MAX_RANK == kMaxRank, "rank limit out of sync");

// Scratch of lora_linear_static(): the layer's workspace for callers that cannot bring or allocate one.  One copy
// per GPU, at its own address (looked up once per context, on that context's device), held until the process ends.
static __device__ __align__(256) unsigned char scratch[LORA_STATIC_SCRATCH_BYTES];

namespace {

thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e) {
    g_last_hip_error = (int)e;
    (void)hipGetLastError();  // clear the sticky error so that the caller's next HIP call is not blamed
    return LORA_ERR_HIP;
}
#define LORA_HIP(call)                           \
    do {                                         \
        hipError_t e_ = (call);                  \
        if (e_ != hipSuccess) return hip_fail(e_); \
    } while (0)

enum ProfKind { kProfPlanSegments = 0, kProfPlanFill = 1, kProfShrink = 2, kProfGemm = 3, kProfExpand = 4, kProfKinds = 5 };
static_assert(kProfKinds == LORA_PROFILE_KINDS, "profile kinds out of sync");

constexpr int kRingSlots = 4;
constexpr size_t kRingSlotInts = 2 * (size_t)LORA_MAX_REQUESTS + LORA_MAX_ADAPTERS;

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace

struct lora_ctx {
    int device = 0;
    int num_cu = 256;
    unsigned char *static_scratch = nullptr;  // this device's copy of `scratch`
    // pinned staging ring for lora_plan's small host arrays
    int32_t *ring = nullptr;
    hipEvent_t ring_event[kRingSlots] = {};
    bool ring_used[kRingSlots] = {};
    int ring_next = 0;
    std::mutex ring_mutex;
    // tuning overrides (-1 = heuristic)
    int opt_gemm_variant = -1;
    int opt_decode_waves = -1;
    int opt_decode_max_rows = -1;
    int opt_plan_fused_rows = -1;
    int opt_shrink_rank_block = -1;
    int opt_plan_variant = -1;
    int opt_expand_split = -1;
    int opt_gemm_split_k = -1;
    // profiling mode: event pairs recorded tightly around each kernel
    bool prof_on = false;
    int prof_cap = 0;
    int prof_used[kProfKinds] = {};
    hipEvent_t *prof_start[kProfKinds] = {};
    hipEvent_t *prof_stop[kProfKinds] = {};
};

namespace {

// Sets the context's device for the duration of a call and restores the caller's.
struct DeviceGuard {
    int prev = -1;
    bool changed = false;
    hipError_t err = hipSuccess;
    explicit DeviceGuard(int dev) {
        err = hipGetDevice(&prev);
        if (err == hipSuccess && prev != dev) {
            err = hipSetDevice(dev);
            changed = err == hipSuccess;
        }
    }
    ~DeviceGuard() {
        if (changed) (void)hipSetDevice(prev);
    }
};

// Next event pair of a kernel kind while profiling (null otherwise, or when the pairs ran out).
bool next_timer(lora_ctx *ctx, int kind, KernelTimer *out) {
    if (!ctx->prof_on || ctx->prof_used[kind] >= ctx->prof_cap) return false;
    const int i = ctx->prof_used[kind]++;
    out->start = ctx->prof_start[kind][i];
    out->stop = ctx->prof_stop[kind][i];
    return true;
}

void free_profiler(lora_ctx *ctx) {
    for (int k = 0; k < kProfKinds; ++k) {
        for (int i = 0; i < ctx->prof_cap; ++i) {
            if (ctx->prof_start[k] && ctx->prof_start[k][i]) (void)hipEventDestroy(ctx->prof_start[k][i]);
            if (ctx->prof_stop[k] && ctx->prof_stop[k][i]) (void)hipEventDestroy(ctx->prof_stop[k][i]);
        }
        delete[] ctx->prof_start[k];
        delete[] ctx->prof_stop[k];
        ctx->prof_start[k] = ctx->prof_stop[k] = nullptr;
        ctx->prof_used[k] = 0;
    }
    ctx->prof_cap = 0;
    ctx->prof_on = false;
}

// ---- plan storage layout ------------------------------------------------------------------------
struct PlanLayout {
    size_t staged, tok_off, req_dst, hist, cursor, key_seg, perm, row_seg, row_adapter, row_ext, seg_adapter, seg_indptr, seg_rank, seg_ext,
        seg_unit, unit_rec, ext_rec, scalars, total_bytes;
    int32_t seg_cap, ext_cap;
};

bool plan_sizes_ok(int32_t n_req, int64_t T, int32_t n_adapters, int32_t r_max) {
    return n_req >= 0 && n_req <= LORA_MAX_REQUESTS && n_adapters >= 0 && n_adapters <= LORA_MAX_ADAPTERS && T >= 0 &&
           T <= (int64_t)INT32_MAX - 65536 && r_max >= 0 && r_max <= LORA_MAX_RANK && (r_max & 7) == 0;
}

PlanLayout plan_layout(int32_t n_req, int64_t T, int32_t n_adapters, int32_t r_max) {
    PlanLayout L;
    size_t off = 0;  // in int32 units; every section starts on a 256-byte boundary
    auto take = [&](size_t n) {
        size_t o = off;
        off = align_up(off + n, 64);
        return o;
    };
    const size_t R = (size_t)n_req, A = (size_t)n_adapters;
    L.seg_cap = n_adapters + 1;
    const size_t used_max = R < A ? R : A;
    L.ext_cap = (int32_t)(used_max * (size_t)(r_max / 8));
    L.staged = take(2 * R + A);
    L.tok_off = take(R + 1);
    L.req_dst = take(R);
    L.hist = take(A + 1);
    L.cursor = take(A + 1);
    L.key_seg = take(A + 1);
    L.perm = take((size_t)T);
    L.row_seg = take((size_t)T);
    L.row_adapter = take((size_t)T);
    L.row_ext = take((size_t)T);
    L.seg_adapter = take((size_t)L.seg_cap);
    L.seg_indptr = take((size_t)L.seg_cap + 1);
    L.seg_rank = take((size_t)L.seg_cap);
    L.seg_ext = take((size_t)L.seg_cap + 1);
    L.seg_unit = take((size_t)L.seg_cap + 1);
    // (room for either unit size, and for the shrink grid, padded to eight units, to read the records of its padding)
    L.unit_rec = take(((size_t)T / kShrinkRowsSmall + (size_t)L.seg_cap + 8) * 4);
    L.ext_rec = take((size_t)L.ext_cap * 4);
    L.scalars = take(8);
    L.total_bytes = off * sizeof(int32_t);
    return L;
}

int validate_batch(const int32_t *req_adapter, const int32_t *req_ntok, int32_t n_req, const int32_t *adapter_rank,
                   int32_t n_adapters, int32_t r_max, int64_t T_expected, int32_t *n_seg_out, int64_t *ext_total_out) {
    if (!plan_sizes_ok(n_req, T_expected, n_adapters, r_max)) return LORA_ERR_INVALID_ARG;
    if (n_req > 0 && (!req_adapter || !req_ntok)) return LORA_ERR_INVALID_ARG;
    if (n_adapters > 0 && !adapter_rank) return LORA_ERR_INVALID_ARG;
    for (int32_t i = 0; i < n_req; ++i)
        if (req_adapter[i] < -1 || req_adapter[i] >= n_adapters) return LORA_ERR_BAD_ADAPTER_ID;
    int64_t sum = 0;
    for (int32_t i = 0; i < n_req; ++i) {
        if (req_ntok[i] < 0) return LORA_ERR_LENGTH_MISMATCH;
        sum += req_ntok[i];
    }
    if (sum != T_expected) return LORA_ERR_LENGTH_MISMATCH;
    // used adapters: O(R) marks in a bitmap on the stack-free heap (n_adapters <= 65536 -> 8 KiB)
    const size_t words = ((size_t)n_adapters + 1 + 63) / 64;
    uint64_t *used = new (std::nothrow) uint64_t[words ? words : 1]();
    if (!used) return LORA_ERR_INVALID_ARG;
    bool any_none = false;
    for (int32_t i = 0; i < n_req; ++i) {
        if (req_ntok[i] == 0) continue;
        if (req_adapter[i] < 0)
            any_none = true;
        else
            used[req_adapter[i] >> 6] |= 1ull << (req_adapter[i] & 63);
    }
    int rc = LORA_OK;
    int32_t n_seg = any_none ? 1 : 0;
    int64_t ext = 0;
    for (int32_t a = 0; a < n_adapters && rc == LORA_OK; ++a) {
        if (!(used[a >> 6] >> (a & 63) & 1ull)) continue;
        const int32_t r = adapter_rank[a];
        if (r <= 0)
            rc = LORA_ERR_ADAPTER_NOT_RESIDENT;
        else if (r & 7)
            rc = LORA_ERR_SHAPE;
        else if (r > r_max)
            rc = LORA_ERR_RANK_TOO_LARGE;
        ++n_seg;
        ext += r;
    }
    delete[] used;
    if (rc != LORA_OK) return rc;
    if (n_seg_out) *n_seg_out = n_seg;
    if (ext_total_out) *ext_total_out = ext;
    return LORA_OK;
}

int build_plan(lora_ctx *ctx, const int32_t *req_adapter_dev, const int32_t *req_ntok_dev, const int32_t *rank_dev,
               int32_t n_req, int32_t n_adapters, int32_t r_max, int64_t T, const PlanLayout &L, int32_t *base,
               hipStream_t stream, lora_plan_t *out) {
    PlanBuildArgs a;
    a.req_adapter = req_adapter_dev;
    a.req_ntok = req_ntok_dev;
    a.rank = rank_dev;
    a.n_req = n_req;
    a.n_adapters = n_adapters;
    a.r_max = r_max;
    a.T = (int32_t)T;
    a.seg_cap = L.seg_cap;
    a.ext_cap = L.ext_cap;
    // Work units of 16 rows while that keeps their number within one workgroup per CU (decode batches, small mixed
    // batches: the long segments then spread over the chip instead of holding a few CUs four times as long), of 64
    // rows otherwise (a unit of 64 rows reads its adapter once for four times the rows).
    const int64_t seg_bound = std::min<int64_t>(std::min<int64_t>(n_req, n_adapters), T);
    const bool small_units = T / kShrinkRowsSmall + seg_bound <= (int64_t)ctx->num_cu;
    a.unit_rows = small_units ? kShrinkRowsSmall : kShrinkRows;
    a.unit_shift = small_units ? 4 : 6;
    a.tok_off = base + L.tok_off;
    a.req_dst = base + L.req_dst;
    a.hist = base + L.hist;
    a.cursor = base + L.cursor;
    a.key_seg = base + L.key_seg;
    a.perm = base + L.perm;
    a.row_seg = base + L.row_seg;
    a.row_adapter = base + L.row_adapter;
    a.row_ext = base + L.row_ext;
    a.seg_adapter = base + L.seg_adapter;
    a.seg_indptr = base + L.seg_indptr;
    a.seg_rank = base + L.seg_rank;
    a.seg_ext = base + L.seg_ext;
    a.seg_unit = base + L.seg_unit;
    a.unit_rec = base + L.unit_rec;
    a.ext_rec = base + L.ext_rec;
    a.scalars = base + L.scalars;
    // One workgroup builds the whole plan (per-row arrays included) up to 4096 rows, up to 8192 for batches of at
    // most 64 requests (the one-lane-per-request kernel leaves its workgroup more time for the rows); beyond that
    // the per-row arrays are filled by a second, grid-wide kernel.
    const int fused_rows = ctx->opt_plan_fused_rows >= 0 ? ctx->opt_plan_fused_rows : (n_req <= 64 ? 8192 : 4096);
    const bool fuse = T <= fused_rows && L.ext_cap <= 8192;
    KernelTimer timers[2];
    const bool timed = next_timer(ctx, kProfPlanSegments, &timers[0]) && (fuse || next_timer(ctx, kProfPlanFill, &timers[1]));
    LORA_HIP(launch_plan_build(a, fuse, ctx->opt_plan_variant > 0 ? ctx->opt_plan_variant : 0, stream, timed ? timers : nullptr));

    out->T = T;
    out->n_req = n_req;
    out->n_adapters = n_adapters;
    out->r_max = r_max;
    out->seg_cap = L.seg_cap;
    out->ext_cap = L.ext_cap;
    out->magic = kPlanMagic;
    out->unit_rows = a.unit_rows;
    out->perm = a.perm;
    out->row_seg = a.row_seg;
    out->row_adapter = a.row_adapter;
    out->row_ext = a.row_ext;
    out->seg_adapter = a.seg_adapter;
    out->seg_indptr = a.seg_indptr;
    out->seg_rank = a.seg_rank;
    out->seg_ext = a.seg_ext;
    out->seg_unit = a.seg_unit;
    out->unit_rec = a.unit_rec;
    out->ext_rec = a.ext_rec;
    out->tok_off = a.tok_off;
    out->scalars = a.scalars;
    return LORA_OK;
}

int check_plan_buf(const void *plan_buf, size_t plan_buf_bytes, const PlanLayout &L, lora_plan_t *out) {
    if (!out) return LORA_ERR_INVALID_ARG;
    if (!plan_buf) return LORA_ERR_INVALID_ARG;
    if (((uintptr_t)plan_buf & 255u) != 0) return LORA_ERR_ALIGNMENT;
    if (plan_buf_bytes < L.total_bytes) return LORA_ERR_WORKSPACE_TOO_SMALL;
    return LORA_OK;
}

// ---- kernel selection ---------------------------------------------------------------------------------
int decode_tblk(int64_t T) { return T <= 16 ? 1 : T <= 32 ? 2 : T <= 64 ? 4 : T <= 96 ? 6 : 8; }

struct GemmChoice {
    int variant;
    int tblk;   // decode path only: 16-row blocks of the batch
    int waves;  // decode path only: waves (16-row weight blocks) per workgroup of the streaming kernel
};

// Geometry of the decode path's launches and workspace: blocks of 16 weight rows (extension rows first, by an upper
// bound of how many ranks the batch can use), slices of 512 along K.
struct DecodeGeom {
    int tblk, nbw, nbe_cap, ks;
    size_t p_bytes;
};
DecodeGeom decode_geom(int64_t T, int32_t K, int32_t N, int64_t ext_rows_bound) {
    DecodeGeom g;
    g.tblk = decode_tblk(T);
    g.nbw = (N + 15) / 16;
    g.nbe_cap = (int)((ext_rows_bound + 15) / 16);
    g.ks = (K / 8 + 63) / 64;
    g.p_bytes = (size_t)(g.nbe_cap + g.nbw) * (size_t)g.ks * (size_t)g.tblk * 1024;
    return g;
}

// A decode-sized batch takes the decode path unless the tiled GEMM is clearly cheaper: towards 128 rows and wide
// outputs the partial tiles of the K slices (T x N x 4 bytes per slice, written and read) outgrow the weights.
// Both sides are fits to measured layer times in microseconds (bf16, with adapters): the decode path moves its bytes
// at ~3.6 TB/s behind ~8 us of fixed cost; the tiled path (64x64 tiles, shrink and expand launches ~15 us) is bound
// by its chain of K stages or by the weights at ~3 TB/s.  4096 -> 11008: decode up to 96 rows (52.8 vs 55.4 us), tiled
// from 112 (56.4 vs 59.8); 5120 -> 13824: tiled from 72 rows (65 vs 73 us); 4096 -> 4096 and 11008 -> 4096: decode
// throughout (28 vs 43 us, 63 vs 93 us at 128 rows).
bool decode_path_cheaper(int64_t T, int32_t K, int32_t N) {
    const double w_mb = 2.0e-6 * (double)K * (double)N;
    const double p_mb = 1.024e-3 * (double)((N + 15) / 16) * (double)((K / 8 + 63) / 64) * (double)decode_tblk(T);
    const double t_decode = 8.0 + (w_mb + 2.0 * p_mb) / 3.6;
    const double t_tiled = 15.0 + std::max(29.0 * (double)K / 4096.0, w_mb / 3.0 + 6.0);
    return t_decode <= 1.08 * t_tiled;
}

// (ns / n_sets: the output widths of the projections one tiled launch covers; the decode path is chosen per projection,
// with n_sets == 1, and covers several projections with its own launches)
GemmChoice choose_gemm_sets(const lora_ctx *ctx, int64_t T, int32_t K, const int32_t *ns, int n_sets, int32_t dtype) {
    GemmChoice c{kGemmTile128x128, 0, kDecodeMinWaves};
    const int max_rows = ctx && ctx->opt_decode_max_rows >= 0 ? ctx->opt_decode_max_rows : kDecodeMaxRows;
    int forced = ctx ? ctx->opt_gemm_variant : -1;
    const bool fits = dtype == LORA_DTYPE_BF16 && T <= kDecodeMaxRows && n_sets == 1;
    if (forced == kGemmDecode && !fits) forced = -1;
    const bool decode = forced == kGemmDecode || (forced < 0 && fits && T <= max_rows && decode_path_cheaper(T, K, ns[0]));
    if (decode) {
        c.variant = kGemmDecode;
        c.tblk = decode_tblk(T);
        // (waves per workgroup of the streaming kernel: chosen at launch, when the plan's bound of extension rows is known)
        return c;
    }
    if (forced >= 0 && forced != kGemmDecode) {
        c.variant = forced;
        return c;
    }
    const int cus = ctx ? ctx->num_cu : 256;
    // Time model: rounds of one tile per CU, a tile costing its area over its MFMA efficiency (measured per
    // round at K = 4096: 256x256 104 us, 256x224 100 us, 256x192 88 us, 256x128 64 us, 128x192 51 us, 128x128 34 us, all on 4 waves).
    struct Cand {
        int variant, bm, bn;
        double eff;
    };
    const Cand cands[] = {{kGemmTile256x256w4, 256, 256, 1.00},
                          {kGemmTile256x128, 256, 128, 0.81},
                          {kGemmTile256x224, 256, 224, 0.905},
                          {kGemmTile256x192, 256, 192, 0.89},
                          {kGemmTile128x192, 128, 192, 0.77},
                          {kGemmTile128x128, 128, 128, 0.77},
                          {kGemmTile64x64, 64, 64, 0.45}};
    double best = 0.0;
    bool have = false;
    for (const Cand &cd : cands) {
        int64_t tiles_n = 0;
        for (int i = 0; i < n_sets; ++i) tiles_n += (ns[i] + cd.bn - 1) / cd.bn;
        const int64_t tiles = ((T + cd.bm - 1) / cd.bm) * tiles_n;
        const int64_t rounds = (tiles + cus - 1) / cus;
        const double cost = (double)rounds * cd.bm * cd.bn / cd.eff;
        if (!have || cost < best) {
            best = cost;
            have = true;
            c.variant = cd.variant;
        }
    }
    return c;
}

GemmChoice choose_gemm(const lora_ctx *ctx, int64_t T, int32_t K, int32_t N, int32_t dtype) {
    return choose_gemm_sets(ctx, T, K, &N, 1, dtype);
}

struct WorkspaceLayout {
    size_t v_off, p_off, p_bytes, total;          // total: what every call needs
    size_t d_off, d_bytes, ldd, total_preferred;  // fp32 adapter term of the separate expand kernel (optional)
    size_t sk_off, sk_bytes;                      // partial outputs of a GEMM split along K (optional, inside total_preferred)
};

// Batches whose tiles alone would leave most CUs idle: the tiled GEMM is split along K as well, its fp32 partial
// outputs summed by a second launch.  Depends on the shape alone (the workspace is sized from it).
struct SplitK {
    int s, k_chunk, variant;
};
SplitK choose_split_k(int64_t T, int32_t K, int32_t N, int32_t dtype) {
    SplitK r{1, 0, kGemmTile128x128};
    if (T <= kDecodeMaxRows) return r;  // (the decode path, or a batch too small to matter)
    const int stage = dtype == LORA_DTYPE_BF16 ? 64 : 32;
    int64_t s = 0;
    if (T <= 1024) {
        // Mid-sized batches on 128x128 tiles.  Worth it while the tiles alone leave most of the chip idle (measured at
        // 4096 -> 4096: 129 rows 46.7 -> 37.8 us per layer, 256 rows 48.5 -> 42.7, 512 rows no gain; 11008 -> 4096, 512
        // rows: 126 -> 108 us; at 4096 -> 11008, 172 tiles and more, the partial outputs cost more than the idle CUs:
        // 72 -> 84 us).
        const int64_t tiles = ((T + 127) / 128) * (((int64_t)N + 127) / 128);
        if (tiles > 128 || (tiles > 96 && K < 8192)) return r;
        s = (384 + tiles - 1) / tiles;  // about one and a half workgroups per CU (two of them fit one)
    } else {
        // A long contraction axis into few columns (a down projection at a thousand-odd rows): 256x256 tiles, as many
        // stretches of K as make one round of workgroups.  Measured per layer, 11008 -> 4096: 1100 rows 169 -> 154 us,
        // 1216 rows 171 -> 157; with two stretches (1536 and 2048 rows: 192 -> 190, 198 -> 218) and at 8192 -> 4096 (three
        // stretches, 1216 rows: 130 -> 130) the partial outputs cost what the idle CUs did, or more.
        const int64_t tiles = ((T + 255) / 256) * (((int64_t)N + 255) / 256);
        if (tiles > 85 || K < 10240) return r;
        s = 256 / tiles;  // (the part's 256 CUs: the workspace size must not depend on the context)
        r.variant = kGemmTile256x256w4;
    }
    s = std::min<int64_t>(s, 8);
    s = std::min<int64_t>(s, K / (16 * stage));  // at least 16 stages per split
    if (s < 2) return SplitK{1, 0, kGemmTile128x128};
    r.k_chunk = (int)(((K + s - 1) / s + stage - 1) / stage * stage);
    r.s = (K + r.k_chunk - 1) / r.k_chunk;
    if (r.s < 2) r = SplitK{1, 0, kGemmTile128x128};
    return r;
}

WorkspaceLayout workspace_layout(int64_t T, int32_t K, int32_t N, int32_t r_max, int32_t dtype) {
    WorkspaceLayout w;
    const size_t es = dtype == LORA_DTYPE_BF16 ? 2 : 4;
    w.v_off = 0;
    size_t off = align_up((size_t)T * (size_t)r_max * es, 256);
    // decode-sized bf16 batches: the partial tiles of the K slices (any batch of T rows uses at most T * r_max ranks)
    w.p_off = off;
    w.p_bytes = (dtype == LORA_DTYPE_BF16 && T > 0 && T <= kDecodeMaxRows) ? decode_geom(T, K, N, T * (int64_t)r_max).p_bytes : 0;
    off = align_up(off + w.p_bytes, 256);
    w.total = off < 256 ? 256 : off;
    w.ldd = align_up((size_t)N, 8);  // (the GEMM's epilogue reads whole 8-column pieces of a row)
    w.d_off = w.total;
    // (also for decode-sized bf16 batches: the decode path hands batches with much adapter work to the expand kernel)
    w.d_bytes = (T > kDecodeMaxRows || (dtype == LORA_DTYPE_BF16 && T > 0)) ? (size_t)T * w.ldd * sizeof(float) : 0;
    w.sk_off = align_up(w.d_off + w.d_bytes, 256);
    const SplitK sk = choose_split_k(T, K, N, dtype);
    w.sk_bytes = sk.s > 1 ? (size_t)sk.s * (size_t)T * w.ldd * sizeof(float) : 0;
    w.total_preferred = align_up(w.sk_off + w.sk_bytes, 256);
    return w;
}

// (check_ws = false: the entry point that brings its own workspace; d->workspace is then not looked at)
int check_linear(const lora_ctx *ctx, const lora_plan_t *plan, const lora_linear_desc *d, bool need_ctx = true, bool check_ws = true) {
    if (!plan || !d) return LORA_ERR_INVALID_ARG;
    if (plan->magic != kPlanMagic || plan->T < 0 || !plan->scalars) return LORA_ERR_PLAN;
    if (plan->unit_rows != kShrinkRows && plan->unit_rows != kShrinkRowsSmall) return LORA_ERR_PLAN;
    if (d->dtype != LORA_DTYPE_BF16 && d->dtype != LORA_DTYPE_F32) return LORA_ERR_INVALID_ARG;
    if (d->flags != 0) return LORA_ERR_INVALID_ARG;
    const int ce = d->dtype == LORA_DTYPE_BF16 ? 8 : 4;
    if (d->K <= 0 || d->N <= 0 || (d->K & 7) != 0) return LORA_ERR_SHAPE;
    if (d->ldx < d->K || d->ldw < d->K || d->ldy < d->N) return LORA_ERR_SHAPE;
    if (d->ldx % ce || d->ldw % ce || d->ldy % ce) return LORA_ERR_ALIGNMENT;
    // the tiled kernels address X with 32-bit byte offsets from its start, W0 from a tile's first row
    const int64_t es = d->dtype == LORA_DTYPE_BF16 ? 2 : 4;
    if (plan->T * d->ldx * es >= (1ll << 32) || 256 * d->ldw * es >= (1ll << 32)) return LORA_ERR_SHAPE;
    if (plan->T > 0) {
        if (!d->X || !d->W0 || !d->Y) return LORA_ERR_INVALID_ARG;
        if (((uintptr_t)d->X | (uintptr_t)d->W0 | (uintptr_t)d->Y) & 15u) return LORA_ERR_ALIGNMENT;
        // Y must not overlap X, W0 or the workspace (extents from the leading dimensions)
        const uintptr_t y0 = (uintptr_t)d->Y, y1 = y0 + (uintptr_t)(((plan->T - 1) * d->ldy + d->N) * es);
        const uintptr_t x0 = (uintptr_t)d->X, x1 = x0 + (uintptr_t)(((plan->T - 1) * d->ldx + d->K) * es);
        const uintptr_t w0 = (uintptr_t)d->W0, w1 = w0 + (uintptr_t)(((int64_t)(d->N - 1) * d->ldw + d->K) * es);
        if ((y0 < x1 && x0 < y1) || (y0 < w1 && w0 < y1)) return LORA_ERR_INVALID_ARG;
        if (check_ws && d->workspace) {
            const uintptr_t s0 = (uintptr_t)d->workspace, s1 = s0 + d->workspace_bytes;
            if ((s0 < y1 && y0 < s1) || (s0 < x1 && x0 < s1) || (s0 < w1 && w0 < s1)) return LORA_ERR_INVALID_ARG;
        }
    }
    if (d->tbl) {
        if (d->tbl->n_adapters < plan->n_adapters) return LORA_ERR_INVALID_ARG;
        if (plan->n_adapters > 0 && (!d->tbl->A || !d->tbl->B || !d->tbl->scale)) return LORA_ERR_INVALID_ARG;
    }
    const WorkspaceLayout w = workspace_layout(plan->T, d->K, d->N, plan->r_max, d->dtype);
    if (plan->T > 0 && check_ws) {
        if (!d->workspace) return LORA_ERR_INVALID_ARG;
        if ((uintptr_t)d->workspace & 255u) return LORA_ERR_ALIGNMENT;
        if (d->workspace_bytes < w.total) return LORA_ERR_WORKSPACE_TOO_SMALL;
    }
    if (need_ctx && !ctx) return LORA_ERR_INVALID_ARG;  // last, so that the checks above run on a GPU-less host too
    return LORA_OK;
}

PlanView view_of(const lora_plan_t *plan) {
    PlanView v;
    v.perm = plan->perm;
    v.row_seg = plan->row_seg;
    v.row_adapter = plan->row_adapter;
    v.row_ext = plan->row_ext;
    v.seg_adapter = plan->seg_adapter;
    v.seg_indptr = plan->seg_indptr;
    v.seg_rank = plan->seg_rank;
    v.seg_ext = plan->seg_ext;
    v.seg_unit = plan->seg_unit;
    v.unit_rec = plan->unit_rec;
    v.ext_rec = plan->ext_rec;
    v.scalars = plan->scalars;
    return v;
}

bool has_adapters(const lora_plan_t *plan, const lora_linear_desc *d) {
    return d->tbl != nullptr && plan->n_adapters > 0 && plan->r_max > 0;
}

// Decode path, one projection: when the reduction's own expand -- every row gathers its adapter's B_a for the
// workgroup's 16 columns, and every workgroup re-reduces V -- would move more than ~24 MB through 16-byte gathers
// (T x r_max x N x 2 bytes: 8 MB at 64 rows of rank 16 and 4096 columns), V is reduced once by a launch of its own
// and the expand kernel streams each used B_a once, segment by segment.  Measured per layer, 64 rows on 64 adapters
// of rank 128: 4096 -> 4096 95 -> 59 us, 5120 -> 13824 306 -> 130 us.  Needs the workspace of the preferred size.
bool decode_adapters_heavy(const lora_ctx *ctx, const lora_plan_t *plan, const lora_linear_desc *d) {
    if (!has_adapters(plan, d)) return false;
    if (ctx->opt_expand_split == 0) return false;
    if (ctx->opt_expand_split == 1) return true;
    return 2.0e-6 * (double)plan->T * (double)plan->r_max * (double)d->N > 24.0;
}

// The two launches of the decode path share one argument block.  n > 1: several projections of the same X, their
// blocks of weight rows side by side in the first launch's grid and their column blocks in the second's.
DecodeArgs decode_args(const lora_ctx *ctx, const lora_plan_t *plan, const lora_linear_desc *const *descs, int n, const GemmChoice &c) {
    const lora_linear_desc *d = descs[0];
    bool any_ad = false;
    for (int i = 0; i < n; ++i) any_ad = any_ad || has_adapters(plan, descs[i]);
    // ranks the batch can use at most: one adapter per request, per slot, per row
    const int64_t segs = std::min<int64_t>(std::min<int64_t>(plan->n_req, plan->n_adapters), plan->T);
    DecodeArgs a;
    a.plan = view_of(plan);
    a.X = d->X;
    a.ldx = d->ldx;
    a.T = (int32_t)plan->T;
    a.K = d->K;
    a.r_max = plan->r_max;
    a.n_sets = n > 1 ? n : 0;
    long nblk = 0;
    for (int i = 0; i < n; ++i) {
        const lora_linear_desc *di = descs[i];
        const WorkspaceLayout w = workspace_layout(plan->T, di->K, di->N, plan->r_max, di->dtype);
        const DecodeGeom g = decode_geom(plan->T, di->K, di->N, any_ad ? segs * plan->r_max : 0);
        const bool ad = has_adapters(plan, di);
        DecodeSet &st = a.set[i];
        st.W = di->W0;
        st.ldw = di->ldw;
        st.A = ad ? di->tbl->A : nullptr;
        st.B = ad ? di->tbl->B : nullptr;
        st.scale = ad ? di->tbl->scale : nullptr;
        st.Y = di->Y;
        st.ldy = di->ldy;
        st.P = reinterpret_cast<float *>(static_cast<unsigned char *>(di->workspace) + w.p_off);
        st.N = di->N;
        st.nbw = g.nbw;
        st.n_adapters = ad ? di->tbl->n_adapters : 0;
        st.blk0 = st.cb0 = st.pad_ = 0;
        a.nbe_cap = g.nbe_cap;
        a.ks = g.ks;
        nblk += (long)g.nbe_cap + g.nbw;
    }
    const DecodeSet &s0 = a.set[0];  // (one projection: the launch's own fields)
    a.W = s0.W;
    a.ldw = s0.ldw;
    a.A = s0.A;
    a.B = s0.B;
    a.scale = s0.scale;
    a.Y = s0.Y;
    a.ldy = s0.ldy;
    a.P = s0.P;
    a.N = s0.N;
    a.nbw = s0.nbw;
    a.n_adapters = s0.n_adapters;
    // waves per workgroup: whole rounds of one workgroup per CU, as little of the last round idle as possible
    const int maxw = kDecodeMaxWaves;
    long best = -1;
    a.waves = kDecodeMinWaves;
    for (int w = maxw; w >= kDecodeMinWaves; --w) {
        const long wgs = ((nblk + w - 1) / w) * a.ks;
        const long cost = ((wgs + ctx->num_cu - 1) / ctx->num_cu) * w;
        if (best < 0 || cost < best) {
            best = cost;
            a.waves = w;
        }
    }
    if (ctx->opt_decode_waves >= kDecodeMinWaves && ctx->opt_decode_waves <= maxw) a.waves = ctx->opt_decode_waves;
    return a;
}

int do_decode(lora_ctx *ctx, const lora_plan_t *plan, const lora_linear_desc *const *descs, int n, const GemmChoice &c,
              hipStream_t stream) {
    const DecodeArgs a = decode_args(ctx, plan, descs, n, c);
    KernelTimer t1, t2;
    const bool timed1 = next_timer(ctx, kProfShrink, &t1);
    LORA_HIP(launch_decode_stream(a, c.tblk, stream, timed1 ? &t1 : nullptr));  // streams W0 and the used A_a against X
    const bool timed2 = next_timer(ctx, kProfGemm, &t2);
    LORA_HIP(launch_decode_reduce(a, c.tblk, stream, timed2 ? &t2 : nullptr));  // sums the slices, adds V B_a, stores Y
    return LORA_OK;
}

// (multi: several projections of the same X that go through one launch)
int do_shrink(lora_ctx *ctx, const lora_plan_t *plan, const lora_linear_desc *d, hipStream_t stream,
              const lora_linear_desc *const *multi = nullptr, int n_multi = 0) {
    if (n_multi == 0) {
        const GemmChoice c = choose_gemm(ctx, plan->T, d->K, d->N, d->dtype);
        if (c.variant == kGemmDecode) {  // decode-sized: the first launch streams W0 and the used A_a against X
            KernelTimer timer;
            const bool timed = next_timer(ctx, kProfShrink, &timer);
            LORA_HIP(launch_decode_stream(decode_args(ctx, plan, &d, 1, c), c.tblk, stream, timed ? &timer : nullptr));
            return LORA_OK;
        }
    }
    bool ad = has_adapters(plan, d);
    for (int i = 0; i < n_multi; ++i) ad = ad || has_adapters(plan, multi[i]);
    if (!ad) return LORA_OK;
    const WorkspaceLayout w = workspace_layout(plan->T, d->K, d->N, plan->r_max, d->dtype);
    unsigned char *ws = static_cast<unsigned char *>(d->workspace);
    ShrinkArgs a;
    a.plan = view_of(plan);
    a.X = d->X;
    a.ldx = d->ldx;
    a.K = d->K;
    a.T = (int32_t)plan->T;
    a.A = ad && n_multi == 0 ? d->tbl->A : nullptr;
    a.scale = ad && n_multi == 0 ? d->tbl->scale : nullptr;
    a.V = ws + w.v_off;
    a.r_max = plan->r_max;
    a.n_adapters = ad && n_multi == 0 ? d->tbl->n_adapters : 0;
    a.n_sets = n_multi;
    for (int i = 0; i < n_multi; ++i) {
        const lora_linear_desc *di = multi[i];
        const bool adi = has_adapters(plan, di);
        const WorkspaceLayout wi = workspace_layout(plan->T, di->K, di->N, plan->r_max, di->dtype);
        a.set[i].A = adi ? di->tbl->A : nullptr;
        a.set[i].scale = adi ? di->tbl->scale : nullptr;
        a.set[i].V = static_cast<unsigned char *>(di->workspace) + wi.v_off;
        a.set[i].n_adapters = adi ? di->tbl->n_adapters : 0;
        a.set[i].pad_ = 0;
    }
    // units <= sum over segments of ceil(rows / unit_rows) <= T / unit_rows + number of adapter segments
    const int64_t seg_bound = plan->n_adapters < plan->n_req ? plan->n_adapters : plan->n_req;
    const int64_t seg_bound2 = seg_bound < plan->T ? seg_bound : plan->T;
    a.max_units = ad ? (int32_t)(plan->T / plan->unit_rows + seg_bound2) : 0;
    // With few units (decode-sized batches) a unit's ranks are dealt to several workgroups: every A_a
    // is streamed once either way, and it takes most of the chip to stream them at HBM speed.
    const int64_t wide_groups = (plan->r_max + kShrinkRanks - 1) / kShrinkRanks;
    const int64_t mid_groups = (plan->r_max + 15) / 16;
    // (every rank block of a unit reads the unit's rows of X again: only worth it while X is small)
    const bool small_x = plan->T <= 256;
    int rank_block = !ad                                                  ? kShrinkRanks
                     : !small_x ? (a.max_units * wide_groups < (int64_t)ctx->num_cu && plan->r_max > 32 ? 32 : kShrinkRanks)
                     : a.max_units * mid_groups < 2 * (int64_t)ctx->num_cu  ? 8
                     : a.max_units * wide_groups < 2 * (int64_t)ctx->num_cu ? 16
                                                                            : kShrinkRanks;
    if (ctx->opt_shrink_rank_block > 0) rank_block = ctx->opt_shrink_rank_block;
    a.rank_block = rank_block;
    a.rank_groups = ad ? (plan->r_max + rank_block - 1) / rank_block : 1;
    a.xlds_bytes = ad && plan->T <= 256 ? 64 * 1024 : 0;  // small batches: units of a few rows, one workgroup per CU is plenty
    KernelTimer timer;
    const bool timed = next_timer(ctx, kProfShrink, &timer);
    LORA_HIP(launch_shrink(a, d->dtype, stream, timed ? &timer : nullptr));
    return LORA_OK;
}

// The adapter term of one projection: fused into the GEMM, or -- batches of many small segments, where an M tile
// of the fused kernel would hold dozens of adapters, a few rows each -- computed per segment by a weight-streaming
// kernel of its own into the workspace (fp32), which is launched here, and added by the GEMM to its accumulators;
// the second only if the caller's workspace has the room.  Describes the projection for the GEMM in *out.
// (collect: several projections in one launch -- the expand kernel's arguments are gathered there, not launched)
// (all_in_d: the whole adapter term through the expand kernel -- the caller has checked the workspace -- for a GEMM
// that adds nothing itself)
int prepare_set(lora_ctx *ctx, const lora_plan_t *plan, const lora_linear_desc *d, int variant, hipStream_t stream,
                const KernelTimer *expand_timer, GemmSet *out, bool *split_out, ExpandArgs *collect = nullptr,
                bool all_in_d = false) {
    const WorkspaceLayout w = workspace_layout(plan->T, d->K, d->N, plan->r_max, d->dtype);
    unsigned char *ws = static_cast<unsigned char *>(d->workspace);
    const bool ad = has_adapters(plan, d);
    GemmSet g{};
    g.W = d->W0;
    g.ldw = d->ldw;
    g.Y = d->Y;
    g.ldy = d->ldy;
    g.V = ad ? ws + w.v_off : nullptr;
    g.B = ad ? d->tbl->B : nullptr;
    g.N = d->N;
    bool split = false;
    if (ad && w.d_bytes > 0 && d->workspace_bytes >= w.total_preferred) {
        const int64_t segs = plan->n_adapters < plan->n_req ? plan->n_adapters : plan->n_req;  // upper bound
        split = segs > 0 && plan->T / segs < 64;
        if (ctx->opt_expand_split >= 0) split = ctx->opt_expand_split == 1;
        if (all_in_d) split = true;
    }
    if (split) {
        ExpandArgs e;
        e.plan = view_of(plan);
        e.V = ws + w.v_off;
        e.B = d->tbl->B;
        e.D = reinterpret_cast<float *>(ws + w.d_off);
        e.ldd = (int64_t)w.ldd;
        e.r_max = plan->r_max;
        e.N = d->N;
        const int64_t seg_bound = plan->n_adapters < plan->n_req ? plan->n_adapters : plan->n_req;
        const int64_t seg_bound2 = seg_bound < plan->T ? seg_bound : plan->T;
        e.max_units = (int32_t)(plan->T / plan->unit_rows + seg_bound2);  // as for the shrink grid
        e.unit_rows = plan->unit_rows;
        e.col_groups = 0;
        // The tiled GEMM keeps the long segments' term to itself (an extension stage per 64 ranks of each such segment
        // of an M tile, ~2 us each, against 8 bytes of D traffic per element and the units' reads of B_a saved: worth
        // it up to rank 64 -- C3 gate_proj 150 -> 140 us; at rank 128, C4, 428 -> 434 us) and takes the short
        // segments' from D; the other kernels take all of it from D.
        const bool tiled = plan->r_max <= 64 && !all_in_d;
        e.skip_long = tiled ? 1 : 0;
        if (collect != nullptr) {
            const int i = collect->n_sets;
            e.n_sets = 0;
            if (i == 0) *collect = e;
            collect->set[i] = ExpandSet{e.V, e.B, e.D, e.ldd, e.N, e.skip_long, 0, 0};
            collect->n_sets = i + 1;
        } else {
            KernelTimer et;
            const bool etimed = expand_timer != nullptr && next_timer(ctx, kProfExpand, &et);
            LORA_HIP(launch_expand(e, d->dtype, stream, etimed ? &et : nullptr));
        }
        if (tiled) {
            g.long_rows = kLongSegRows;
        } else {
            g.B = nullptr;
            g.V = nullptr;
        }
        g.D = e.D;
        g.ldd = e.ldd;
    }
    *out = g;
    *split_out = split;
    return LORA_OK;
}

int do_gemm(lora_ctx *ctx, const lora_plan_t *plan, const lora_linear_desc *d, hipStream_t stream) {
    GemmChoice c = choose_gemm(ctx, plan->T, d->K, d->N, d->dtype);
    KernelTimer timer, etimer;
    const bool timed = next_timer(ctx, kProfGemm, &timer);
    const WorkspaceLayout w = workspace_layout(plan->T, d->K, d->N, plan->r_max, d->dtype);
    if (c.variant == kGemmDecode) {  // decode-sized: the second launch sums the slices, adds V B_a, stores Y
        DecodeArgs a = decode_args(ctx, plan, &d, 1, c);
        if (d->workspace_bytes >= w.total_preferred && w.d_bytes > 0 && decode_adapters_heavy(ctx, plan, d)) {
            // much adapter work: V once, the expand kernel for the term, the reduction only adds it
            unsigned char *ws = static_cast<unsigned char *>(d->workspace);
            a.V = ws + w.v_off;
            KernelTimer vt;
            const bool vtimed = timed && next_timer(ctx, kProfShrink, &vt);
            LORA_HIP(launch_decode_v(a, c.tblk, stream, vtimed ? &vt : nullptr));
            ExpandArgs e;
            e.plan = a.plan;
            e.V = a.V;
            e.B = d->tbl->B;
            e.D = reinterpret_cast<float *>(ws + w.d_off);
            e.ldd = (int64_t)w.ldd;
            e.r_max = plan->r_max;
            e.N = d->N;
            const int64_t seg_bound = std::min<int64_t>(std::min<int64_t>(plan->n_adapters, plan->n_req), plan->T);
            e.max_units = (int32_t)(plan->T / plan->unit_rows + seg_bound);
            e.unit_rows = plan->unit_rows;
            e.col_groups = 0;
            e.skip_long = 0;
            const bool etimed = timed && next_timer(ctx, kProfExpand, &etimer);
            LORA_HIP(launch_expand(e, d->dtype, stream, etimed ? &etimer : nullptr));
            a.B = nullptr;
            a.D = e.D;
            a.ldd = e.ldd;
        }
        LORA_HIP(launch_decode_reduce(a, c.tblk, stream, timed ? &timer : nullptr));
        return LORA_OK;
    }
    SplitK sk = choose_split_k(plan->T, d->K, d->N, d->dtype);
    if (ctx->opt_gemm_split_k == 0 || (ctx->opt_gemm_variant >= 0 && ctx->opt_gemm_variant != sk.variant) ||
        d->workspace_bytes < w.total_preferred || (has_adapters(plan, d) && w.d_bytes == 0))
        sk = SplitK{1, 0, kGemmTile128x128};
    if (sk.s > 1) c.variant = sk.variant;
    GemmSet g;
    bool split = false;
    const int rc = prepare_set(ctx, plan, d, c.variant, stream, timed ? &etimer : nullptr, &g, &split, nullptr, sk.s > 1);
    if (rc != LORA_OK) return rc;
    if (sk.s > 1) {  // partial products per stretch of K, then one launch that sums them, adds the adapter term and rounds
        GemmArgs a;
        a.plan = view_of(plan);
        a.X = d->X;
        a.ldx = d->ldx;
        a.W = g.W;
        a.ldw = g.ldw;
        a.Y = g.Y;
        a.ldy = g.ldy;
        a.V = nullptr;
        a.B = nullptr;
        a.D = nullptr;
        a.ldd = 0;
        a.r_max = plan->r_max;
        a.T = (int32_t)plan->T;
        a.K = d->K;
        a.N = d->N;
        a.split_k = sk.s;
        a.k_chunk = sk.k_chunk;
        a.P = reinterpret_cast<float *>(static_cast<unsigned char *>(d->workspace) + w.sk_off);
        a.ldp = (int64_t)w.ldd;
        LORA_HIP(launch_gemm_tile(a, d->dtype, c.variant, stream, timed ? &timer : nullptr));
        SplitReduceArgs r;
        r.plan = a.plan;
        r.P = a.P;
        r.ldp = a.ldp;
        r.split_k = sk.s;
        r.D = g.D;  // (null when the call has no adapters)
        r.ldd = g.ldd;
        r.Y = d->Y;
        r.ldy = d->ldy;
        r.T = a.T;
        r.N = d->N;
        KernelTimer rtimer;
        const bool rtimed = timed && next_timer(ctx, kProfGemm, &rtimer);
        LORA_HIP(launch_splitk_reduce(r, d->dtype, stream, rtimed ? &rtimer : nullptr));
        return LORA_OK;
    }
    GemmArgs a;
    a.plan = view_of(plan);
    a.X = d->X;
    a.ldx = d->ldx;
    a.W = g.W;
    a.ldw = g.ldw;
    a.Y = g.Y;
    a.ldy = g.ldy;
    a.V = g.V;
    a.B = g.B;
    a.D = g.D;
    a.ldd = g.ldd;
    a.long_rows = g.long_rows;
    a.r_max = plan->r_max;
    a.T = (int32_t)plan->T;
    a.K = d->K;
    a.N = d->N;
    const KernelTimer *tg = timed ? &timer : nullptr;
    LORA_HIP(launch_gemm_tile(a, d->dtype, c.variant, stream, tg));
    return LORA_OK;
}

// Several projections of the same X in one GEMM launch (their column tiles side by side in one grid: one ramp, one
// set of whole rounds of tiles for all of them).  0: this batch / these options take the projections one by one;
// 1: the tiled kernel (one launch of each kernel for all of them); 2: the decode path's two launches for all of them.
int multi_kind(const lora_ctx *ctx, const lora_plan_t *plan, const lora_linear_desc *const *descs, int n, GemmChoice *c) {
    int32_t ns[kMaxGemmSets];
    for (int i = 0; i < n; ++i) ns[i] = descs[i]->N;
    *c = choose_gemm(ctx, plan->T, descs[0]->K, descs[0]->N, descs[0]->dtype);
    if (c->variant == kGemmDecode) {
        // (much adapter work: each projection through its own launches and the expand kernel, see decode_adapters_heavy)
        for (int i = 0; i < n; ++i) {
            const WorkspaceLayout w = workspace_layout(plan->T, descs[i]->K, descs[i]->N, plan->r_max, descs[i]->dtype);
            if (descs[i]->workspace_bytes >= w.total_preferred && decode_adapters_heavy(ctx, plan, descs[i])) return 0;
            if (choose_gemm(ctx, plan->T, descs[i]->K, descs[i]->N, descs[i]->dtype).variant != kGemmDecode) return 0;
        }
        return 2;
    }
    *c = choose_gemm_sets(ctx, plan->T, descs[0]->K, ns, n, descs[0]->dtype);
    if (c->variant == kGemmDecode) return 0;
    return 1;
}

int do_gemm_multi(lora_ctx *ctx, const lora_plan_t *plan, const lora_linear_desc *const *descs, int n, const GemmChoice &c,
                  hipStream_t stream) {
    GemmArgs a;
    a.plan = view_of(plan);
    a.X = descs[0]->X;
    a.ldx = descs[0]->ldx;
    a.W = nullptr;
    a.ldw = 0;
    a.Y = nullptr;
    a.ldy = 0;
    a.V = nullptr;
    a.B = nullptr;
    a.D = nullptr;
    a.ldd = 0;
    a.r_max = plan->r_max;
    a.T = (int32_t)plan->T;
    a.K = descs[0]->K;
    a.N = 0;
    a.n_sets = n;
    KernelTimer timer;
    const bool timed = next_timer(ctx, kProfGemm, &timer);
    ExpandArgs e;
    e.n_sets = 0;
    for (int i = 0; i < n; ++i) {
        bool split = false;
        const int rc = prepare_set(ctx, plan, descs[i], c.variant, stream, nullptr, &a.set[i], &split, &e);
        if (rc != LORA_OK) return rc;
    }
    if (e.n_sets > 0) {  // one launch for every projection that takes it
        KernelTimer et;
        const bool etimed = timed && next_timer(ctx, kProfExpand, &et);
        LORA_HIP(launch_expand(e, descs[0]->dtype, stream, etimed ? &et : nullptr));
    }
    LORA_HIP(launch_gemm_tile(a, descs[0]->dtype, c.variant, stream, timed ? &timer : nullptr));
    return LORA_OK;
}

}  // namespace

// =========================================================================================================
extern "C" {

int lora_ctx_create(lora_ctx **out, int device_ordinal) {
    if (!out) return LORA_ERR_INVALID_ARG;
    *out = nullptr;
    if (device_ordinal < 0) return LORA_ERR_INVALID_ARG;
    int count = 0;
    LORA_HIP(hipGetDeviceCount(&count));
    if (device_ordinal >= count) return LORA_ERR_INVALID_ARG;
    lora_ctx *ctx = new (std::nothrow) lora_ctx();
    if (!ctx) return LORA_ERR_INVALID_ARG;
    ctx->device = device_ordinal;
    DeviceGuard guard(device_ordinal);
    hipError_t e = guard.err;
    hipDeviceProp_t prop;
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, device_ordinal);
    if (e == hipSuccess) {
        ctx->num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
        e = hipHostMalloc(reinterpret_cast<void **>(&ctx->ring), kRingSlots * kRingSlotInts * sizeof(int32_t), hipHostMallocDefault);
    }
    for (int i = 0; i < kRingSlots && e == hipSuccess; ++i) e = hipEventCreateWithFlags(&ctx->ring_event[i], hipEventDisableTiming);
    // per-device set-up of the kernels: dynamic-LDS grants of every instantiation (so that no launch has to make one,
    // under stream capture or from two threads at once), and this device's address of the static scratch array
    if (e == hipSuccess) e = init_gemm_tile_kernels();
    if (e == hipSuccess) e = init_decode_kernels();
    if (e == hipSuccess) e = init_shrink_kernels();
    if (e == hipSuccess) e = init_expand_kernels();
    if (e == hipSuccess) e = hipGetSymbolAddress(reinterpret_cast<void **>(&ctx->static_scratch), HIP_SYMBOL(scratch));
    if (e != hipSuccess) {
        for (int i = 0; i < kRingSlots; ++i)
            if (ctx->ring_event[i]) (void)hipEventDestroy(ctx->ring_event[i]);
        if (ctx->ring) (void)hipHostFree(ctx->ring);
        delete ctx;
        return hip_fail(e);
    }
    *out = ctx;
    return LORA_OK;
}

int lora_ctx_destroy(lora_ctx *ctx) {
    if (!ctx) return LORA_ERR_INVALID_ARG;
    DeviceGuard guard(ctx->device);
    for (int i = 0; i < kRingSlots; ++i) {
        if (ctx->ring_event[i]) {
            if (ctx->ring_used[i]) (void)hipEventSynchronize(ctx->ring_event[i]);
            (void)hipEventDestroy(ctx->ring_event[i]);
        }
    }
    if (ctx->ring) (void)hipHostFree(ctx->ring);
    free_profiler(ctx);
    delete ctx;
    return LORA_OK;
}

int lora_ctx_set_option(lora_ctx *ctx, const char *name, int value) {
    if (!ctx || !name) return LORA_ERR_INVALID_ARG;
    if (!strcmp(name, "gemm_variant")) {
        if (value >= kGemmVariantCount || value == 2 || (value >= 6 && value <= 8)) return LORA_ERR_INVALID_ARG;
        ctx->opt_gemm_variant = value;
    } else if (!strcmp(name, "decode_waves")) {
        if (value >= 0 && (value < kDecodeMinWaves || value > kDecodeMaxWaves)) return LORA_ERR_INVALID_ARG;
        ctx->opt_decode_waves = value;
    } else if (!strcmp(name, "decode_max_rows")) {
        ctx->opt_decode_max_rows = value;
    } else if (!strcmp(name, "plan_fused_rows")) {
        ctx->opt_plan_fused_rows = value;
    } else if (!strcmp(name, "gemm_split_k")) {
        if (value > 1) return LORA_ERR_INVALID_ARG;
        ctx->opt_gemm_split_k = value;
    } else if (!strcmp(name, "expand_split")) {
        if (value > 1) return LORA_ERR_INVALID_ARG;
        ctx->opt_expand_split = value;
    } else if (!strcmp(name, "plan_variant")) {
        if (value > 1) return LORA_ERR_INVALID_ARG;
        ctx->opt_plan_variant = value;
    } else if (!strcmp(name, "shrink_rank_block")) {
        if (value > 0 && value != 8 && value != 16 && value != 32 && value != 64) return LORA_ERR_INVALID_ARG;
        ctx->opt_shrink_rank_block = value;
    } else {
        return LORA_ERR_INVALID_ARG;
    }
    return LORA_OK;
}

int lora_plan_validate(const int32_t *req_adapter, const int32_t *req_ntok, int32_t n_req, const int32_t *adapter_rank,
                       int32_t n_adapters, int32_t r_max, int64_t T_expected, int32_t *n_seg_out, int64_t *ext_total_out) {
    return validate_batch(req_adapter, req_ntok, n_req, adapter_rank, n_adapters, r_max, T_expected, n_seg_out, ext_total_out);
}

size_t lora_plan_bytes(int32_t n_req, int64_t T, int32_t n_adapters, int32_t r_max) {
    if (!plan_sizes_ok(n_req, T, n_adapters, r_max)) return 0;
    return plan_layout(n_req, T, n_adapters, r_max).total_bytes;
}

int lora_plan(lora_ctx *ctx, const int32_t *req_adapter, const int32_t *req_ntok, int32_t n_req, const int32_t *adapter_rank,
              int32_t n_adapters, int32_t r_max, int64_t T_expected, void *plan_buf, size_t plan_buf_bytes,
              lora_stream_t stream_, lora_plan_t *out) {
    int rc = validate_batch(req_adapter, req_ntok, n_req, adapter_rank, n_adapters, r_max, T_expected, nullptr, nullptr);
    if (rc != LORA_OK) return rc;
    const PlanLayout L = plan_layout(n_req, T_expected, n_adapters, r_max);
    rc = check_plan_buf(plan_buf, plan_buf_bytes, L, out);
    if (rc != LORA_OK) return rc;
    if (!ctx) return LORA_ERR_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    DeviceGuard guard(ctx->device);
    if (guard.err != hipSuccess) return hip_fail(guard.err);
    int32_t *base = static_cast<int32_t *>(plan_buf);
    int32_t *staged = base + L.staged;
    const size_t n_ints = 2 * (size_t)n_req + (size_t)n_adapters;
    if (n_ints > 0) {
        std::lock_guard<std::mutex> lock(ctx->ring_mutex);
        const int slot = ctx->ring_next;
        ctx->ring_next = (slot + 1) % kRingSlots;
        if (ctx->ring_used[slot]) LORA_HIP(hipEventSynchronize(ctx->ring_event[slot]));
        int32_t *host = ctx->ring + (size_t)slot * kRingSlotInts;
        if (n_req > 0) {
            memcpy(host, req_adapter, sizeof(int32_t) * (size_t)n_req);
            memcpy(host + n_req, req_ntok, sizeof(int32_t) * (size_t)n_req);
        }
        if (n_adapters > 0) memcpy(host + 2 * (size_t)n_req, adapter_rank, sizeof(int32_t) * (size_t)n_adapters);
        LORA_HIP(hipMemcpyAsync(staged, host, n_ints * sizeof(int32_t), hipMemcpyHostToDevice, stream));
        LORA_HIP(hipEventRecord(ctx->ring_event[slot], stream));
        ctx->ring_used[slot] = true;
    }
    return build_plan(ctx, staged, staged + n_req, staged + 2 * (size_t)n_req, n_req, n_adapters, r_max, T_expected, L, base,
                      stream, out);
}

int lora_plan_device(lora_ctx *ctx, const int32_t *req_adapter, const int32_t *req_ntok, int32_t n_req,
                     const int32_t *adapter_rank, int32_t n_adapters, int32_t r_max, int64_t T_expected, void *plan_buf,
                     size_t plan_buf_bytes, lora_stream_t stream_, lora_plan_t *out) {
    if (!plan_sizes_ok(n_req, T_expected, n_adapters, r_max)) return LORA_ERR_INVALID_ARG;
    if (n_req > 0 && (!req_adapter || !req_ntok)) return LORA_ERR_INVALID_ARG;
    if (n_adapters > 0 && !adapter_rank) return LORA_ERR_INVALID_ARG;
    const PlanLayout L = plan_layout(n_req, T_expected, n_adapters, r_max);
    int rc = check_plan_buf(plan_buf, plan_buf_bytes, L, out);
    if (rc != LORA_OK) return rc;
    if (!ctx) return LORA_ERR_INVALID_ARG;
    DeviceGuard guard(ctx->device);
    if (guard.err != hipSuccess) return hip_fail(guard.err);
    return build_plan(ctx, req_adapter, req_ntok, adapter_rank, n_req, n_adapters, r_max, T_expected, L,
                      static_cast<int32_t *>(plan_buf), static_cast<hipStream_t>(stream_), out);
}

int lora_plan_status(lora_ctx *ctx, const lora_plan_t *plan, lora_stream_t stream_, int32_t *n_seg_out) {
    if (!ctx || !plan) return LORA_ERR_INVALID_ARG;
    if (plan->magic != kPlanMagic || !plan->scalars) return LORA_ERR_PLAN;
    DeviceGuard guard(ctx->device);
    if (guard.err != hipSuccess) return hip_fail(guard.err);
    LORA_HIP(hipStreamSynchronize(static_cast<hipStream_t>(stream_)));
    int32_t sc[8];
    LORA_HIP(hipMemcpy(sc, plan->scalars, sizeof sc, hipMemcpyDeviceToHost));
    if (n_seg_out) *n_seg_out = sc[kScNSeg];
    return sc[kScStatus] != 0 ? sc[kScStatus] : sc[kScEvicted];
}

size_t lora_linear_workspace_bytes(int64_t T, int32_t K, int32_t N, int32_t r_max, int32_t dtype) {
    if (T < 0 || K <= 0 || N <= 0 || r_max < 0 || (dtype != LORA_DTYPE_BF16 && dtype != LORA_DTYPE_F32)) return 0;
    return workspace_layout(T, K, N, r_max, dtype).total;
}

size_t lora_linear_workspace_bytes_preferred(int64_t T, int32_t K, int32_t N, int32_t r_max, int32_t dtype) {
    if (T < 0 || K <= 0 || N <= 0 || r_max < 0 || (dtype != LORA_DTYPE_BF16 && dtype != LORA_DTYPE_F32)) return 0;
    return workspace_layout(T, K, N, r_max, dtype).total_preferred;
}

int lora_shrink(lora_ctx *ctx, const lora_plan_t *plan, const lora_linear_desc *desc, lora_stream_t stream) {
    int rc = check_linear(ctx, plan, desc);
    if (rc != LORA_OK) return rc;
    if (plan->T == 0) return LORA_OK;
    DeviceGuard guard(ctx->device);
    if (guard.err != hipSuccess) return hip_fail(guard.err);
    return do_shrink(ctx, plan, desc, static_cast<hipStream_t>(stream));
}

int lora_gemm_expand(lora_ctx *ctx, const lora_plan_t *plan, const lora_linear_desc *desc, lora_stream_t stream) {
    int rc = check_linear(ctx, plan, desc);
    if (rc != LORA_OK) return rc;
    if (plan->T == 0) return LORA_OK;
    DeviceGuard guard(ctx->device);
    if (guard.err != hipSuccess) return hip_fail(guard.err);
    hipStream_t s = static_cast<hipStream_t>(stream);
    return do_gemm(ctx, plan, desc, s);
}

int lora_linear(lora_ctx *ctx, const lora_plan_t *plan, const lora_linear_desc *desc, lora_stream_t stream) {
    int rc = check_linear(ctx, plan, desc);
    if (rc != LORA_OK) return rc;
    if (plan->T == 0) return LORA_OK;
    DeviceGuard guard(ctx->device);
    if (guard.err != hipSuccess) return hip_fail(guard.err);
    hipStream_t s = static_cast<hipStream_t>(stream);
    rc = do_shrink(ctx, plan, desc, s);
    if (rc != LORA_OK) return rc;
    return do_gemm(ctx, plan, desc, s);
}

int lora_linear_static(lora_ctx *ctx, const lora_plan_t *plan, const lora_linear_desc *desc, lora_stream_t stream) {
    if (!desc) return LORA_ERR_INVALID_ARG;
    if (desc->workspace != nullptr || desc->workspace_bytes != 0) return LORA_ERR_INVALID_ARG;
    if (!plan) return LORA_ERR_INVALID_ARG;
    // (sizes first, so that an oversized problem is reported as such whatever else is wrong with it)
    if (plan->T >= 0 && desc->K > 0 && desc->N > 0 && plan->r_max >= 0 &&
        (desc->dtype == LORA_DTYPE_BF16 || desc->dtype == LORA_DTYPE_F32) &&
        workspace_layout(plan->T, desc->K, desc->N, plan->r_max, desc->dtype).total > (size_t)LORA_STATIC_SCRATCH_BYTES)
        return LORA_ERR_WORKSPACE_TOO_SMALL;
    int rc = check_linear(ctx, plan, desc, true, false);
    if (rc != LORA_OK) return rc;
    lora_linear_desc d = *desc;
    d.workspace = ctx->static_scratch;
    d.workspace_bytes = LORA_STATIC_SCRATCH_BYTES;
    if (plan->T == 0) return LORA_OK;
    DeviceGuard guard(ctx->device);
    if (guard.err != hipSuccess) return hip_fail(guard.err);
    hipStream_t s = static_cast<hipStream_t>(stream);
    rc = do_shrink(ctx, plan, &d, s);
    if (rc != LORA_OK) return rc;
    return do_gemm(ctx, plan, &d, s);
}

int lora_linear_multi(lora_ctx *ctx, const lora_plan_t *plan, const lora_linear_desc *const *descs, int32_t n,
                      lora_stream_t stream) {
    if (!descs || n < 1 || n > LORA_MAX_MULTI) return LORA_ERR_INVALID_ARG;
    for (int i = 0; i < n; ++i) {
        if (!descs[i]) return LORA_ERR_INVALID_ARG;
        const int rc = check_linear(ctx, plan, descs[i], false);
        if (rc != LORA_OK) return rc;
        if (descs[i]->X != descs[0]->X || descs[i]->ldx != descs[0]->ldx || descs[i]->K != descs[0]->K ||
            descs[i]->dtype != descs[0]->dtype)
            return LORA_ERR_INVALID_ARG;
        for (int j = 0; j < i; ++j)
            if (plan->T > 0 && (descs[i]->Y == descs[j]->Y || descs[i]->workspace == descs[j]->workspace)) return LORA_ERR_INVALID_ARG;
    }
    if (!ctx) return LORA_ERR_INVALID_ARG;  // (last: the checks above run on a GPU-less host too)
    if (plan->T == 0) return LORA_OK;
    DeviceGuard guard(ctx->device);
    if (guard.err != hipSuccess) return hip_fail(guard.err);
    hipStream_t s = static_cast<hipStream_t>(stream);
    GemmChoice c;
    const int kind = n == 1 ? 0 : multi_kind(ctx, plan, descs, n, &c);
    if (kind == 0) {  // one after the other
        for (int i = 0; i < n; ++i) {
            int rc = do_shrink(ctx, plan, descs[i], s);
            if (rc == LORA_OK) rc = do_gemm(ctx, plan, descs[i], s);
            if (rc != LORA_OK) return rc;
        }
        return LORA_OK;
    }
    if (kind == 2) return do_decode(ctx, plan, descs, n, c, s);
    const int rc = do_shrink(ctx, plan, descs[0], s, descs, n);  // one launch: the single projection's grid once per projection
    if (rc != LORA_OK) return rc;
    return do_gemm_multi(ctx, plan, descs, n, c, s);
}

int lora_profile_begin(lora_ctx *ctx, int max_launches) {
    if (!ctx || max_launches <= 0 || max_launches > (1 << 20)) return LORA_ERR_INVALID_ARG;
    DeviceGuard guard(ctx->device);
    if (guard.err != hipSuccess) return hip_fail(guard.err);
    if (max_launches > ctx->prof_cap) {
        free_profiler(ctx);
        for (int k = 0; k < kProfKinds; ++k) {
            ctx->prof_start[k] = new (std::nothrow) hipEvent_t[max_launches]();
            ctx->prof_stop[k] = new (std::nothrow) hipEvent_t[max_launches]();
            if (!ctx->prof_start[k] || !ctx->prof_stop[k]) return LORA_ERR_INVALID_ARG;
        }
        ctx->prof_cap = max_launches;
        for (int k = 0; k < kProfKinds; ++k)
            for (int i = 0; i < max_launches; ++i) {
                LORA_HIP(hipEventCreate(&ctx->prof_start[k][i]));
                LORA_HIP(hipEventCreate(&ctx->prof_stop[k][i]));
            }
    }
    for (int k = 0; k < kProfKinds; ++k) ctx->prof_used[k] = 0;
    ctx->prof_on = true;
    return LORA_OK;
}

int lora_profile_end(lora_ctx *ctx, lora_stream_t stream, double *avg_us, int32_t *counts) {
    if (!ctx || !avg_us || !counts) return LORA_ERR_INVALID_ARG;
    if (!ctx->prof_on) return LORA_ERR_INVALID_ARG;
    ctx->prof_on = false;
    DeviceGuard guard(ctx->device);
    if (guard.err != hipSuccess) return hip_fail(guard.err);
    LORA_HIP(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
    for (int k = 0; k < kProfKinds; ++k) {
        double sum = 0.0;
        for (int i = 0; i < ctx->prof_used[k]; ++i) {
            float ms = 0.f;
            LORA_HIP(hipEventElapsedTime(&ms, ctx->prof_start[k][i], ctx->prof_stop[k][i]));
            sum += (double)ms * 1000.0;
        }
        counts[k] = ctx->prof_used[k];
        avg_us[k] = ctx->prof_used[k] > 0 ? sum / ctx->prof_used[k] : 0.0;
        ctx->prof_used[k] = 0;
    }
    return LORA_OK;
}

static_assert(sizeof(hipIpcMemHandle_t) == LORA_IPC_HANDLE_BYTES, "IPC handle size out of sync");

int lora_backbone_alloc(int device_ordinal, size_t bytes, void **dev_ptr_out) {
    if (!dev_ptr_out || bytes == 0 || device_ordinal < 0) return LORA_ERR_INVALID_ARG;
    *dev_ptr_out = nullptr;
    DeviceGuard guard(device_ordinal);
    if (guard.err != hipSuccess) return hip_fail(guard.err);
    LORA_HIP(hipMalloc(dev_ptr_out, bytes));
    return LORA_OK;
}

int lora_backbone_free(int device_ordinal, void *dev_ptr) {
    if (!dev_ptr || device_ordinal < 0) return LORA_ERR_INVALID_ARG;
    DeviceGuard guard(device_ordinal);
    if (guard.err != hipSuccess) return hip_fail(guard.err);
    LORA_HIP(hipFree(dev_ptr));
    return LORA_OK;
}

int lora_backbone_export(int device_ordinal, const void *dev_ptr, unsigned char handle_out[LORA_IPC_HANDLE_BYTES]) {
    if (!dev_ptr || !handle_out || device_ordinal < 0) return LORA_ERR_INVALID_ARG;
    DeviceGuard guard(device_ordinal);
    if (guard.err != hipSuccess) return hip_fail(guard.err);
    hipIpcMemHandle_t h;
    LORA_HIP(hipIpcGetMemHandle(&h, const_cast<void *>(dev_ptr)));
    memcpy(handle_out, &h, sizeof h);
    return LORA_OK;
}

int lora_backbone_open(int device_ordinal, const unsigned char handle[LORA_IPC_HANDLE_BYTES], void **dev_ptr_out) {
    if (!handle || !dev_ptr_out || device_ordinal < 0) return LORA_ERR_INVALID_ARG;
    *dev_ptr_out = nullptr;
    DeviceGuard guard(device_ordinal);
    if (guard.err != hipSuccess) return hip_fail(guard.err);
    hipIpcMemHandle_t h;
    memcpy(&h, handle, sizeof h);
    LORA_HIP(hipIpcOpenMemHandle(dev_ptr_out, h, hipIpcMemLazyEnablePeerAccess));
    return LORA_OK;
}

int lora_backbone_close(int device_ordinal, void *dev_ptr) {
    if (!dev_ptr || device_ordinal < 0) return LORA_ERR_INVALID_ARG;
    DeviceGuard guard(device_ordinal);
    if (guard.err != hipSuccess) return hip_fail(guard.err);
    LORA_HIP(hipIpcCloseMemHandle(dev_ptr));
    return LORA_OK;
}

const char *lora_gemm_kernel_name(lora_ctx *ctx, int64_t T, int32_t K, int32_t N, int32_t dtype) {
    static thread_local char buf[64];
    const GemmChoice c = choose_gemm(ctx, T, K, N, dtype);
    // (with a workspace of the preferred size and an adapter table, or none)
    const SplitK sk = choose_split_k(T, K, N, dtype);
    if (c.variant != kGemmDecode && sk.s > 1 && !(ctx && ctx->opt_gemm_split_k == 0) &&
        !(ctx && ctx->opt_gemm_variant >= 0 && ctx->opt_gemm_variant != sk.variant)) {
        snprintf(buf, sizeof buf, sk.variant == kGemmTile128x128 ? "tile_128x128_splitk%d" : "tile_256x256_splitk%d", sk.s);
        return buf;
    }
    switch (c.variant) {
        case kGemmDecode:
            snprintf(buf, sizeof buf, "decode_tb%d", c.tblk);
            break;
        case kGemmTile64x64:
            snprintf(buf, sizeof buf, "tile_64x64");
            break;
        case kGemmTile128x128:
            snprintf(buf, sizeof buf, "tile_128x128");
            break;
        case kGemmTile256x128:
            snprintf(buf, sizeof buf, "tile_256x128");
            break;
        case kGemmTile256x256w4:
            snprintf(buf, sizeof buf, "tile_256x256w4");
            break;
        case kGemmTile128x192:
            snprintf(buf, sizeof buf, "tile_128x192");
            break;
        case kGemmTile256x192:
            snprintf(buf, sizeof buf, "tile_256x192");
            break;
        case kGemmTile256x224:
            snprintf(buf, sizeof buf, "tile_256x224");
            break;
        default:
            snprintf(buf, sizeof buf, "unknown");
    }
    return buf;
}

const char *lora_strerror(int status) {
    switch (status) {
        case LORA_OK:
            return "ok";
        case LORA_ERR_INVALID_ARG:
            return "invalid argument";
        case LORA_ERR_BAD_ADAPTER_ID:
            return "adapter id outside [-1, n_adapters)";
        case LORA_ERR_LENGTH_MISMATCH:
            return "negative token count or token counts do not add up to T";
        case LORA_ERR_ADAPTER_NOT_RESIDENT:
            return "a used adapter is not resident (rank 0 or null weights)";
        case LORA_ERR_RANK_TOO_LARGE:
            return "a used adapter's rank exceeds r_max";
        case LORA_ERR_WORKSPACE_TOO_SMALL:
            return "plan buffer or workspace too small";
        case LORA_ERR_ALIGNMENT:
            return "pointer or row stride not aligned";
        case LORA_ERR_SHAPE:
            return "unsupported shape (K, N, leading dimension or rank)";
        case LORA_ERR_HIP:
            return "HIP runtime error";
        case LORA_ERR_PLAN:
            return "not a valid plan";
        default:
            return "unknown status";
    }
}

int lora_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
