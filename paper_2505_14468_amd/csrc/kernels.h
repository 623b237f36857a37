// Host-side launch interface between lora_api.hip and the kernel translation units.
#pragma once
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "common.hiph"

namespace lora {

struct PlanBuildArgs {
    const int32_t *req_adapter;  // device [n_req]
    const int32_t *req_ntok;     // device [n_req]
    const int32_t *rank;         // device [n_adapters]
    int32_t n_req, n_adapters, r_max;
    int32_t T;
    int32_t seg_cap, ext_cap;
    int32_t unit_rows, unit_shift;  // rows per work unit (kShrinkRows or kShrinkRowsSmall) and its log2
    // outputs / scratch, all device int32 arrays inside plan_buf
    int32_t *tok_off;      // [n_req+1]
    int32_t *req_dst;      // [n_req]  first slot of each request's rows
    int32_t *hist;         // [n_adapters+1] rows per key (key n_adapters = no adapter)
    int32_t *cursor;       // [n_adapters+1] running slot per key
    int32_t *key_seg;      // [n_adapters+1] segment of key or -1
    int32_t *perm;         // [T]
    int32_t *row_seg;      // [T]
    int32_t *row_adapter;  // [T]  adapter of every row, original order
    int32_t *row_ext;      // [T]  pack_row_ext(first extension column of the row's adapter, its rank), original order
    int32_t *seg_adapter;  // [seg_cap]
    int32_t *seg_indptr;   // [seg_cap+1]
    int32_t *seg_rank;     // [seg_cap]
    int32_t *seg_ext;      // [seg_cap+1]
    int32_t *seg_unit;     // [seg_cap+1]
    int32_t *unit_rec;     // [unit_cap*4] shrink work list: adapter, rank, first slot, rows
    int32_t *ext_rec;      // [ext_cap*4]
    int32_t *scalars;      // [8]
    long long *trace = nullptr;  // phase stamps (trace builds only)
};

// Optional pair of events recorded tightly around one kernel (profiling mode): the elapsed time
// between them is the kernel's own execution time, as a profiler reports it.
struct KernelTimer {
    hipEvent_t start, stop;
};

#ifdef LORA_TRACE
}  // namespace lora
#include "trace_build.h"  // phase stamps: trace builds only
namespace lora {
#else
#define LORA_TS(buf, i) \
    do {                \
    } while (0)
#define LORA_TS_WAVE(buf, i, w) \
    do {                        \
    } while (0)
#endif

// Launch with or without a timer.
template <typename F, typename... Args>
inline hipError_t launch_kernel(F kernel, dim3 grid, dim3 block, size_t smem, hipStream_t stream, const KernelTimer *timer,
                                Args... args) {
    if (timer != nullptr)
        hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)smem, stream, timer->start, timer->stop, 0, args...);
    else
        hipLaunchKernelGGL(kernel, grid, block, smem, stream, args...);
    return hipGetLastError();
}

// Enqueues the segment builder (one or two kernels).  `fuse_fill`: the single
// workgroup of the first kernel also fills the T-sized arrays.  `variant`: 0 = pick by size, 1 = never the
// decode-sized (one lane per request) kernel.  timers: [0] segments, [1] fill.
hipError_t launch_plan_build(const PlanBuildArgs &a, bool fuse_fill, int variant, hipStream_t stream, const KernelTimer *timers);

constexpr int kMaxGemmSets = 4;
// One projection of a launch that covers several projections of the same X (fused QKV, gate + up): the grid of the
// single-projection launch, once per projection.
struct ShrinkSet {
    const void *const *A;
    const float *scale;
    void *V;
    int32_t n_adapters;
    int32_t pad_;
};

struct ShrinkArgs {
    PlanView plan;
    const void *X;
    int64_t ldx;
    int32_t K;
    int32_t T;
    const void *const *A;  // device table
    const float *scale;    // device table
    void *V;               // [T, r_max] of E
    int32_t r_max;
    int32_t n_adapters;    // entries of the A / scale tables
    int32_t rank_block;    // ranks per workgroup: 8 or 16 (few units: spread them over the chip) or kShrinkRanks
    int32_t rank_groups;   // ceil(r_max / rank_block)
    int32_t max_units;     // upper bound of work units (shrink grid = max_units * rank_groups)
    int32_t xlds_bytes;    // LDS for staging the X rows of small units: 0 or 64 KiB (decode-sized batches)
    long long *trace = nullptr;  // phase stamps (trace builds only)
    int32_t n_sets = 0;    // > 0: the projections of the launch (A, scale, V, n_adapters above are then unused)
    ShrinkSet set[kMaxGemmSets];
};
hipError_t launch_shrink(const ShrinkArgs &a, int dtype, hipStream_t stream, const KernelTimer *timer);

// One projection of a tiled GEMM launch that covers several projections of the same X: its
// own weights, output, adapters and adapter term; the column tiles of the projections follow each other in the grid.
struct GemmSet {
    const void *W;
    int64_t ldw;
    void *Y;
    int64_t ldy;
    const void *V;
    const void *const *B;
    const float *D;
    int64_t ldd;
    int32_t long_rows;
    int32_t N;
    int32_t tile0;  // first column tile of this projection (set by the launcher)
    int32_t pad_;
};

struct GemmArgs {
    PlanView plan;
    const void *X;
    int64_t ldx;
    const void *W;
    int64_t ldw;
    void *Y;
    int64_t ldy;
    const void *V;         // [T, r_max] of E, original row order (null when no adapters)
    const void *const *B;  // device table (null when no adapters, or when all of the adapter term comes in D)
    const float *D;        // adapter term in fp32, [T, ldd], original row order, rows with an adapter only (null = none)
    int64_t ldd;
    int32_t long_rows = 0;  // > 0 (with B and D both set): D holds the term of segments shorter than this only,
                            // the tiled GEMM computes the others' as extension stages
    int32_t r_max;
    int32_t T, K, N;
    // split along K (mid-sized batches whose tiles would not fill the chip; one projection, no adapter term here):
    // workgroup (tile, s) multiplies columns [s * k_chunk, (s + 1) * k_chunk) of the contraction axis and stores its
    // fp32 partial tile to P[s][row][n] (row = original row index, rows ldp floats long); launch_splitk_reduce
    // sums the partials in order, adds the adapter term and stores Y.
    int32_t split_k = 0;   // > 1: number of splits
    int32_t k_chunk = 0;   // columns per split, a multiple of one stage (64 bf16 / 32 fp32 elements)
    float *P = nullptr;
    int64_t ldp = 0;
    // tiled kernel only: the projections of the launch (n_sets == 0: one, described by the fields above)
    int32_t n_sets = 0;
    GemmSet set[kMaxGemmSets];
    long long *trace = nullptr;  // phase stamps (trace builds only)
};

struct ExpandSet {
    const void *V;
    const void *const *B;
    float *D;
    int64_t ldd;
    int32_t N;
    int32_t skip_long;
    int32_t block0;  // first workgroup of this projection (set by the launcher)
    int32_t pad_;
};

// Separate expand kernel (many small segments): D[row, :] = V[row, :] B_a^T per shrink work unit, in fp32.
struct ExpandArgs {
    PlanView plan;
    const void *V;         // [T, r_max] of E, original row order
    const void *const *B;  // device table
    float *D;              // [T, ldd] fp32, original row order; rows without an adapter are not written
    int64_t ldd;
    int32_t r_max;
    int32_t N;
    int32_t max_units;     // upper bound of work units (grid = max_units * col_groups)
    int32_t col_groups;    // set by the launcher: ceil(N / columns per workgroup)
    int32_t unit_rows;     // most rows of a work unit in this plan (16 or 64)
    int32_t skip_long;     // 1: units of long segments (kUnitLongFlag) are left to the GEMM
    long long *trace = nullptr;  // phase stamps (trace builds only)
    int32_t n_sets = 0;    // > 0: the projections of the launch (V, B, D, ldd, N, skip_long above are then unused)
    ExpandSet set[kMaxGemmSets];
};
hipError_t launch_expand(const ExpandArgs &a, int dtype, hipStream_t stream, const KernelTimer *timer);

enum GemmVariant {
    kGemmTile128x128 = 0,
    kGemmTile256x128 = 1,
    // (2: not in use)
    kGemmTile64x64 = 3,
    kGemmDecode = 4,         // not a tile shape: the decode-sized path (decode_kernels.hip)
    kGemmTile256x256w4 = 5,  // 256x256 tile on 4 waves (128x128 per wave)
    // (6, 7, 8: not in use)
    kGemmTile128x192 = 9,    // 128 rows x 192 columns on 4 waves (fills the chip where 256x128 leaves CUs idle)
    kGemmTile256x192 = 10,   // 256 x 192 on 4 waves (a tile count just below a whole number of rounds where 256x256 is just above)
    kGemmTile256x224 = 11,   // 256 x 224 on 4 waves of 64 x 224 (likewise)
    kGemmVariantCount
};

hipError_t launch_gemm_tile(const GemmArgs &a, int dtype, int variant, hipStream_t stream, const KernelTimer *timer);

// Y[row, :] = sum over s (in order) of P[s][row, :]  +  D[row, :] for rows with an adapter (D null: none), rounded once.
struct SplitReduceArgs {
    PlanView plan;
    const float *P;
    int64_t ldp;
    int32_t split_k;
    const float *D;
    int64_t ldd;
    void *Y;
    int64_t ldy;
    int32_t T, N;
};
hipError_t launch_splitk_reduce(const SplitReduceArgs &a, int dtype, hipStream_t stream, const KernelTimer *timer);

// One projection of a decode launch that covers several projections of the same X (fused QKV, gate + up): its blocks of
// weight rows follow the previous projection's in the streaming kernel's grid, its column blocks in the reduction's.
struct DecodeSet {
    const void *W;
    int64_t ldw;
    const void *const *A;
    const void *const *B;
    const float *scale;
    void *Y;
    int64_t ldy;
    float *P;
    int32_t N;
    int32_t nbw;
    int32_t n_adapters;
    int32_t blk0;  // first block of weight rows (set by the launcher)
    int32_t cb0;   // first column block of the reduction's grid (set by the launcher)
    int32_t pad_;
};

// Decode-sized batches (bf16, at most kDecodeMaxRows rows): two launches, see decode_kernels.hip.
struct DecodeArgs {
    PlanView plan;
    const void *X;
    int64_t ldx;
    const void *W;
    int64_t ldw;
    const void *const *A;  // device tables (all three null when the call has no adapters)
    const void *const *B;
    const float *scale;
    void *Y;
    int64_t ldy;
    float *P;              // workspace: fp32 partial tiles, [nbe_cap + nbw][ks][tblk][64 lanes][4]
    int32_t T, K, N;
    int32_t r_max;         // the plan's largest rank
    int32_t n_adapters;    // entries of the A / B / scale tables
    int32_t nbw;           // blocks of 16 rows of W0: ceil(N / 16)
    int32_t nbe_cap;       // upper bound of the blocks of 16 extension rows (rows of the used A_a), which come first
    int32_t ks;            // slices of 512 along K
    int32_t waves;         // waves (= 16-row blocks) per workgroup of the streaming kernel
    long long *trace = nullptr;  // phase stamps (trace builds only)
    int32_t n_sets = 0;    // > 0: the projections of the launch (W .. P, N, nbw, n_adapters above are then unused)
    DecodeSet set[kMaxGemmSets];
    // Adapter term through the expand kernel (batches with much adapter work; one projection): launch_decode_v reduces
    // the extension rows' partial tiles to V ([T, r_max] of E, original row order, scaled), the expand kernel turns V
    // into the fp32 term D, and the reduction adds D instead of computing V B_a itself (B null).
    void *V = nullptr;
    const float *D = nullptr;
    int64_t ldd = 0;
};
constexpr int kDecodeMaxRows = 128;
constexpr int kDecodeMinWaves = 8, kDecodeMaxWaves = 12;
hipError_t init_decode_kernels();
hipError_t launch_decode_stream(const DecodeArgs &a, int tblk, hipStream_t stream, const KernelTimer *timer);
hipError_t launch_decode_reduce(const DecodeArgs &a, int tblk, hipStream_t stream, const KernelTimer *timer);
hipError_t launch_decode_v(const DecodeArgs &a, int tblk, hipStream_t stream, const KernelTimer *timer);

// Dynamic-LDS grants of every kernel instantiation, for the current device (context creation).
hipError_t init_gemm_tile_kernels();
hipError_t init_shrink_kernels();
hipError_t init_expand_kernels();


}  // namespace lora
