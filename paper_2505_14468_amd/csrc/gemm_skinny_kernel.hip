// Decode-sized batches (T <= 128 rows): the layer is a weight-streaming problem, bound by
// reading W0 (and the used B_a) from HBM once.  Same contraction as the tiled kernel --
//
//     Y[perm[slot], n] = sum_k X[perm[slot], k] W0[n, k]  +  sum_p V[slot, p] B_a(p)[n, p]
//
// (paper section 4.4: backbone and adapter results combined) -- but organised around the
// weight stream instead of around LDS tiles:
//   * a workgroup owns 64 output columns (16 per wave) and a contiguous share of the
//     contraction axis K' = K + (concatenated ranks of all adapters in the batch); K' is split
//     over `ksplit` workgroups so that >= 2 workgroups per CU are streaming at any time;
//   * W0 / B_a chunks go global -> VGPR -> MFMA A operand directly (every weight element is
//     used by exactly one wave, so LDS would only add a hop); loads for the next stage are in
//     flight while the current one feeds the matrix core;
//   * the X rows (all T of them) of the current K stage are staged once per workgroup in
//     LDS, double-buffered and XOR-swizzled, and read as the MFMA B operand by all 4 waves;
//   * MFMA 16x16x32: M = 16 output columns, N = 16 token rows, so T = 64 is 4 MFMAs per
//     weight chunk and the matrix core idles most of the time, as it should here;
//   * split-K partial tiles go to the workspace; the last workgroup to arrive for a column
//     tile (integer counter) adds them in split order -- a fixed order, so results are
//     reproducible -- and stores Y once.
#include <limits.h>

#include "kernels.h"

namespace lora {
namespace {

constexpr int kSkTab = 256;        // extension chunks described per batch
constexpr int kSkThreads = 256;
constexpr int kSkStageBytes = 32768;

struct SkTable {
    const void *ptr[kSkTab];
    int r[kSkTab];
    int j[kSkTab];
    int lo[kSkTab];
    int hi[kSkTab];
};

// chunk of the contraction axis that lane group lg feeds to MFMA step st: two consecutive
// steps cover 8 consecutive chunks, each lane group two adjacent ones (32 contiguous bytes).
__device__ __forceinline__ int chunk_of(int st, int lg) { return (st >> 1) * 8 + lg * 2 + (st & 1); }

template <int TBLK>
__global__ __launch_bounds__(kSkThreads) void gemm_skinny_kernel(GemmArgs p, int n_tiles) {
    typedef __bf16 E;
    constexpr int CE = 8;
    constexpr int ROWS = 16 * TBLK;
    constexpr int KS = 32 / TBLK;  // MFMA steps per X stage (stage = 32 KiB of X in LDS)
    constexpr int CPR = KS * 4;    // chunks per row per stage
    constexpr int XL = ROWS * CPR / kSkThreads;
    static_assert(ROWS * CPR * 16 == kSkStageBytes, "stage size");
    static_assert(CPR >= 16, "swizzle needs 16 chunk columns");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    chunk_t *sX = reinterpret_cast<chunk_t *>(smem);  // [2][ROWS*CPR]
    SkTable *tab = reinterpret_cast<SkTable *>(smem + 2 * kSkStageBytes);
    __shared__ int s_last;

    if (p.plan.scalars[kScStatus] != 0) return;

    const int ksplit = p.ksplit;
    const int n_tile = (blockIdx.x & 7) + 8 * (blockIdx.x / (8 * ksplit));
    const int split = (blockIdx.x >> 3) % ksplit;
    if (n_tile >= n_tiles) return;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 15, lg = lane >> 4;
    const int n0 = n_tile * kSkinnyBN;
    const int nrow = n0 + wave * 16 + li;  // weight row this lane streams
    const bool nvalid = nrow < p.N;

    const E *X = static_cast<const E *>(p.X);
    const E *V = static_cast<const E *>(p.V);
    const E *wrow = static_cast<const E *>(p.W) + (int64_t)(nvalid ? nrow : 0) * p.ldw;

    // ---- this workgroup's share of the MFMA steps (in pairs of steps = 64 elements) ---------
    const int kchunks = p.K / CE;
    const int base_pairs = (kchunks + 7) >> 3;
    const int ext_total = p.B != nullptr ? p.plan.scalars[kScExtTotal] : 0;
    const int ext_chunks = ext_total / CE;
    const int ext_pairs = (ext_chunks + 7) >> 3;
    const int tot_pairs = base_pairs + ext_pairs;
    const int pr0 = (int)((int64_t)tot_pairs * split / ksplit), pr1 = (int)((int64_t)tot_pairs * (split + 1) / ksplit);
    const int b0 = min(pr0, base_pairs) * 2, b1 = min(pr1, base_pairs) * 2;                       // base steps
    const int e0 = (max(pr0, base_pairs) - base_pairs) * 2, e1 = (max(pr1, base_pairs) - base_pairs) * 2;  // ext steps

    // ---- extension table (first batch) early, so its two dependent loads overlap the base loop --
    auto build_table = [&](int step0) {
        for (int idx = tid; idx < kSkTab; idx += kSkThreads) {
            const int st = step0 + (idx >> 2);
            const int ch = chunk_of(st, idx & 3);
            const void *ptr = nullptr;
            int r = 0, j = 0, lo = INT_MAX, hi = INT_MIN;
            if (st < e1 && ch < ext_chunks) {
                const int4 rec = reinterpret_cast<const int4 *>(p.plan.ext_rec)[ch];
                const E *b = rec.x >= 0 ? static_cast<const E *>(p.B[rec.x]) : nullptr;
                if (b != nullptr) {
                    r = rec.y >> 16;
                    j = rec.y & 0xffff;
                    lo = rec.z;
                    hi = rec.w;
                    ptr = b + j;
                } else {
                    atomicMin(&p.plan.scalars[kScStatus], kErrNotResident);
                }
            }
            tab->ptr[idx] = ptr;
            tab->r[idx] = r;
            tab->j[idx] = j;
            tab->lo[idx] = lo;
            tab->hi[idx] = hi;
        }
    };
    if (e1 > e0) build_table(e0);

    f32x4_t acc[TBLK];
#pragma unroll
    for (int tb = 0; tb < TBLK; ++tb) acc[tb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // ---- base product -------------------------------------------------------------------------
    // X stage loads: thread -> (row, chunk column) of the stage, coalesced along the row
    const E *xsrc[XL];
    int xcol[XL], xdst[XL];
#pragma unroll
    for (int i = 0; i < XL; ++i) {
        const int idx = tid + i * kSkThreads;
        const int row = idx / CPR, c = idx % CPR;
        xsrc[i] = row < p.T ? X + (int64_t)p.plan.perm[row] * p.ldx : nullptr;
        xcol[i] = c;
        xdst[i] = row * CPR + (c ^ (row & 15));
    }
    chunk_t xr[XL], wcur[KS], wnext[KS];

    auto load_stage = [&](int st0) {  // st0 = first MFMA step of the stage (even, multiple of KS from b0)
        const int c0 = (st0 >> 1) * 8;  // first chunk of the stage along K
#pragma unroll
        for (int i = 0; i < XL; ++i) {
            const int ch = c0 + xcol[i];
            xr[i] = (xsrc[i] != nullptr && ch < kchunks && (st0 + (xcol[i] >> 2)) < b1) ? load_chunk(xsrc[i] + ch * CE)
                                                                                       : zero_chunk();
        }
#pragma unroll
        for (int j = 0; j < KS; ++j) {
            const int st = st0 + j;
            const int ch = chunk_of(st, lg);
            wnext[j] = (nvalid && st < b1 && ch < kchunks) ? load_chunk(wrow + ch * CE) : zero_chunk();
        }
    };
    auto store_x = [&](int buf) {
#pragma unroll
        for (int i = 0; i < XL; ++i) sX[buf * ROWS * CPR + xdst[i]] = xr[i];
    };

    if (b1 > b0) {
        const int nstage = (b1 - b0 + KS - 1) / KS;
        load_stage(b0);
        store_x(0);
        __syncthreads();
        for (int s = 0; s < nstage; ++s) {
#pragma unroll
            for (int j = 0; j < KS; ++j) wcur[j] = wnext[j];
            const bool more = s + 1 < nstage;
            if (more) load_stage(b0 + (s + 1) * KS);
            const chunk_t *bx = sX + (s & 1) * ROWS * CPR;
#pragma unroll
            for (int j = 0; j < KS; ++j) {
                // chunk column inside the stage of (step j, lane group lg)
                const int c = chunk_of(j, lg);
#pragma unroll
                for (int tb = 0; tb < TBLK; ++tb) {
                    const int row = tb * 16 + li;
                    const chunk_t xf = bx[row * CPR + (c ^ (row & 15))];
                    Elem<E>::mma16(acc[tb], wcur[j], xf);
                }
            }
            if (more) store_x((s + 1) & 1);
            __syncthreads();
        }
    }

    // ---- extension: V (masked per adapter) against the B_a rows, straight from global ------------
    for (int step0 = e0; step0 < e1; step0 += kSkTab / 4) {
        if (step0 > e0) build_table(step0);
        __syncthreads();
        const int nst = min(e1 - step0, kSkTab / 4);
        for (int s = 0; s < nst; ++s) {
            const int idx = s * 4 + lg;
            const E *bp = static_cast<const E *>(tab->ptr[idx]);
            const int r = tab->r[idx], j = tab->j[idx], lo = tab->lo[idx], hi = tab->hi[idx];
            const chunk_t wf = (bp != nullptr && nvalid) ? load_chunk(bp + (int64_t)nrow * r) : zero_chunk();
#pragma unroll
            for (int tb = 0; tb < TBLK; ++tb) {
                const int t = tb * 16 + li;
                const chunk_t xf = (t >= lo && t < hi) ? load_chunk(V + (int64_t)t * p.r_max + j) : zero_chunk();
                Elem<E>::mma16(acc[tb], wf, xf);
            }
        }
        __syncthreads();
    }

    // ---- split-K: park the partial tile, the last arrival sums in split order ------------------------
    if (ksplit > 1) {
        float4 *part = reinterpret_cast<float4 *>(p.partials) + ((int64_t)n_tile * ksplit + split) * (TBLK * kSkThreads);
#pragma unroll
        for (int tb = 0; tb < TBLK; ++tb)
            part[tb * kSkThreads + tid] = make_float4(acc[tb][0], acc[tb][1], acc[tb][2], acc[tb][3]);
        __threadfence();
        __syncthreads();
        if (tid == 0) {
            const int old = atomicAdd(&p.counters[n_tile], 1);
            s_last = (old == ksplit - 1) ? 1 : 0;
        }
        __syncthreads();
        if (!s_last) return;
        __threadfence();
        const float4 *all = reinterpret_cast<const float4 *>(p.partials) + (int64_t)n_tile * ksplit * (TBLK * kSkThreads);
#pragma unroll
        for (int tb = 0; tb < TBLK; ++tb) acc[tb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        for (int sp = 0; sp < ksplit; ++sp) {
#pragma unroll
            for (int tb = 0; tb < TBLK; ++tb) {
                const float4 v = all[(int64_t)sp * (TBLK * kSkThreads) + tb * kSkThreads + tid];
                acc[tb][0] += v.x;
                acc[tb][1] += v.y;
                acc[tb][2] += v.z;
                acc[tb][3] += v.w;
            }
        }
        if (tid == 0) p.counters[n_tile] = 0;  // ready for the next call
    }

    // ---- store Y: acc[tb][e] = D[n = n0 + wave*16 + lg*4 + e][t = tb*16 + li] --------------------------
    E *Y = static_cast<E *>(p.Y);
    const int n = n0 + wave * 16 + lg * 4;
#pragma unroll
    for (int tb = 0; tb < TBLK; ++tb) {
        const int t = tb * 16 + li;
        if (t >= p.T) continue;
        E *yrow = Y + (int64_t)p.plan.perm[t] * p.ldy;
        if (n + 3 < p.N) {
            store4(yrow + n, acc[tb][0], acc[tb][1], acc[tb][2], acc[tb][3]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (n + e < p.N) store1(yrow + n + e, acc[tb][e]);
        }
    }
}

template <int TBLK>
hipError_t launch_sk(const GemmArgs &a, hipStream_t stream, const KernelTimer *timer) {
    const int n_tiles = (a.N + kSkinnyBN - 1) / kSkinnyBN;
    const size_t smem = 2 * kSkStageBytes + sizeof(SkTable);
    auto kern = gemm_skinny_kernel<TBLK>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const long grid = (long)((n_tiles + 7) / 8) * 8 * a.ksplit;
    return launch_kernel(kern, dim3((unsigned)grid), dim3(kSkThreads), smem, stream, timer, a, n_tiles);
}

}  // namespace

hipError_t launch_gemm_skinny(const GemmArgs &a, int tblk, hipStream_t stream, const KernelTimer *timer) {
    if (a.T <= 0 || a.N <= 0) return hipSuccess;
    switch (tblk) {
        case 1:
            return launch_sk<1>(a, stream, timer);
        case 2:
            return launch_sk<2>(a, stream, timer);
        case 4:
            return launch_sk<4>(a, stream, timer);
        case 8:
            return launch_sk<8>(a, stream, timer);
        default:
            return hipErrorInvalidValue;
    }
}

}  // namespace lora
