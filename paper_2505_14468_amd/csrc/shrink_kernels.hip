// Segmented LoRA shrink: V[row, j] = s_a * sum_k X[row, k] * A_a[k, j] for the rows of every
// adapter segment (first half of the adapter product of paper section 4.4).
//
// One workgroup = one work unit = (segment, block of <= 64 of its rows, group of <= 64 ranks).
// The unit list is part of the plan; the grid is an upper bound and surplus workgroups
// leave at once.  Inside a unit the NW waves split the contraction axis K between
// them; each wave runs 16x16 MFMA tiles with the adapter rows (ranks) as the MFMA M dimension
// and the token rows as the N dimension, both operands loaded straight from global memory as
// 16-byte chunks (A_a is [r, K] and X is [T, K]: both are contiguous along K, which is what
// the MFMA operand layout wants).  Loads are issued in batches of several MFMA steps with two
// batches in flight, because for decode-sized segments (a handful of rows, MFMA tile mostly
// empty) the kernel is bound by the latency and bandwidth of streaming A_a once.  The unit's
// shape picks the instantiation (1 or 4 token blocks, 1 / 2 / 4 rank blocks) so that small
// units spend their registers on loads in flight rather than on empty tiles.
// The per-wave partial tiles are summed through LDS in wave order, so the result is
// deterministic, scaled by s_a in fp32 and stored once (bf16 or fp32), in original row order.
#include "kernels.h"

namespace lora {
namespace {

constexpr int kShWaves = 8;
constexpr int kRS = kShrinkRanks + 1;             // padded row stride of the serial reduction buffer
constexpr int kRedBytes = kShrinkRows * kRS * 4;  // serial reduction buffer (large units)
constexpr int kPartBytes = kShWaves * 4 * 1024;   // per-wave partial tiles (units of at most 4 MFMA tiles)
constexpr int kXldsBytes = 64 * 1024;             // rows of X staged in LDS (units of a few rows)
constexpr int kXldsPad = 4;                       // chunks of padding per staged row: rows fall into different banks
constexpr int kXldsRows = 4;                      // at most this many rows are staged ...
constexpr int kXldsChunks = 2;                    // ... of at most this many chunks per thread (K <= 8192 in bf16)

// Dynamic LDS of the kernel: [reduction area][X staging area (only when launched with it)].
constexpr int kShSmemBase = kRedBytes > kPartBytes ? kRedBytes : kPartBytes;

template <typename E, int TB, int JB>
__device__ __forceinline__ void shrink_unit(const ShrinkArgs &p, const E *Aa, float scale, int slot0, int nrows, int j0,
                                            int nj, const int (&prow)[4], unsigned char *smem) {
    constexpr int CE = Elem<E>::CE;
    constexpr int LPS = TB + JB;
    constexpr int SB = (TB * JB >= 8 ? 12 : 16) / LPS;  // MFMA steps per load batch (2 batches in flight)
    // The wave index as a scalar: the K ranges, step counters and step offsets below then live in scalar
    // registers and cost the vector pipeline nothing.  (Units of a few rows are short serial instruction
    // streams; every dependent vector instruction is ~10 cycles of their run time.)
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, lg = lane >> 4;
    const int kchunks = p.K / CE;

    // A unit of a few rows (decode) keeps its rows of X in LDS: as MFMA operand, a row is wanted by
    // every lane group, and a global load costs the address unit the same whether its lanes read 16
    // distinct rows or the same one 16 times -- it would spend as long on X as on A_a.
    const bool xlds = TB == 1 && p.xlds_bytes > 0 && nrows <= kXldsRows && kchunks <= kXldsChunks * kShWaves * 64 &&
                      (int64_t)nrows * (kchunks + kXldsPad) * 16 <= p.xlds_bytes;
    chunk_t *xs = reinterpret_cast<chunk_t *>(smem + kShSmemBase);
    const int xstride = kchunks + kXldsPad;
    // Per-lane byte offsets into A_a / X: row (ranks and rows past the end of the unit are clamped to the
    // last one) and this lane group's first chunk of a 128-byte piece; what changes per step is a scalar.
    const char *Ab = reinterpret_cast<const char *>(Aa);
    unsigned aoff[JB];
#pragma unroll
    for (int jb = 0; jb < JB; ++jb)
        aoff[jb] = (unsigned)(((int64_t)(j0 + min(jb * 16 + li, nj - 1)) * p.K + 2 * lg * CE) * (int64_t)sizeof(E));
    const char *xrow[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
        xrow[tb] = reinterpret_cast<const char *>(p.X) + ((int64_t)prow[tb] * p.ldx + 2 * lg * CE) * (int64_t)sizeof(E);
    const chunk_t *xsrow = xs + min(li, nrows - 1) * xstride + 2 * lg;

    f32x4_t acc[TB][JB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int jb = 0; jb < JB; ++jb) acc[tb][jb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // This wave's share of the MFMA steps along K (one step = 4 chunks).  Steps come in pairs that
    // share one 128-byte piece of every row: step 2m takes its even chunks, step 2m+1 the odd ones
    // (lane group g: chunks 2g and 2g+1), so that both loads of a lane fall into the same line;
    // the order of the k terms inside a pair is free as long as A_a and X use the same one.
    // Whole pairs are dealt to the waves; a last partial pair (K not a multiple of 64) goes to the
    // last wave, masked.
    const int pairs = kchunks >> 3;
    const int st0 = 2 * (int)((int64_t)pairs * wave / kShWaves), st1 = 2 * (int)((int64_t)pairs * (wave + 1) / kShWaves);
    auto step_chunk = [&](int st) { return (st >> 1) * 8 + (st & 1); };  // without the lane group's 2g

    // Steps past the wave's range are skipped (a uniform branch), not loaded and dropped: the address
    // unit's time is what this kernel runs out of.
    chunk_t xa[SB][TB], aa[SB][JB], xb[SB][TB], ab[SB][JB];
    auto load_batch = [&](int s0, chunk_t (&xf)[SB][TB], chunk_t (&af)[SB][JB]) {
#pragma unroll
        for (int s = 0; s < SB; ++s) {
            const int st = s0 + s;
            if (st < st1) {
                const unsigned sb = (unsigned)step_chunk(st) * 16u;  // scalar byte offset of the step
                if (!xlds) {
#pragma unroll
                    for (int tb = 0; tb < TB; ++tb) xf[s][tb] = load_chunk(xrow[tb] + sb);
                }
#pragma unroll
                for (int jb = 0; jb < JB; ++jb) af[s][jb] = load_chunk(Ab + sb + aoff[jb]);
            }
        }
    };
    auto mma_batch = [&](int s0, const chunk_t (&xf)[SB][TB], const chunk_t (&af)[SB][JB]) {
#pragma unroll
        for (int s = 0; s < SB; ++s) {
            const int st = s0 + s;
            if (st < st1) {
                if (xlds) {
                    const chunk_t x = xsrow[step_chunk(st)];
#pragma unroll
                    for (int jb = 0; jb < JB; ++jb) Elem<E>::mma16(acc[0][jb], af[s][jb], x);
                } else {
#pragma unroll
                    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
                        for (int jb = 0; jb < JB; ++jb) Elem<E>::mma16(acc[tb][jb], af[s][jb], xf[s][tb]);
                }
            }
        }
    };
    LORA_TS(p.trace, 2);  // row map, adapter pointer, scale read
    // Everything that can be requested now is requested now, oldest first in the order it is needed
    // (loads return in order): the unit's rows of X (a few KB, from L2), then both batches of A_a --
    // at K = 4096 that is a wave's whole share.
    chunk_t xr[kXldsRows][kXldsChunks];
    if (xlds) {
#pragma unroll
        for (int t = 0; t < kXldsRows; ++t)
            if (t < nrows) {
                // lane t of the first lane group holds the row map entry of row t
                const int row = __builtin_amdgcn_readlane(prow[0], t);
                const E *src = static_cast<const E *>(p.X) + (int64_t)row * p.ldx;
#pragma unroll
                for (int u = 0; u < kXldsChunks; ++u) {
                    const int c = tid + u * (kShWaves * 64);
                    if (c < kchunks) xr[t][u] = load_chunk(src + (int64_t)c * CE);
                }
            }
    }
    load_batch(st0, xa, aa);
    load_batch(st0 + SB, xb, ab);
    LORA_TS(p.trace, 3);  // loads issued
    if (xlds) {
#pragma unroll
        for (int t = 0; t < kXldsRows; ++t)
            if (t < nrows) {
#pragma unroll
                for (int u = 0; u < kXldsChunks; ++u) {
                    const int c = tid + u * (kShWaves * 64);
                    if (c < kchunks) xs[t * xstride + c] = xr[t][u];
                }
            }
        __syncthreads();  // the staged rows are complete (uniform over the workgroup)
    }
    LORA_TS(p.trace, 4);  // rows staged
    for (int s0 = st0; s0 < st1; s0 += 2 * SB) {
        mma_batch(s0, xa, aa);
        load_batch(s0 + 2 * SB, xa, aa);
        mma_batch(s0 + SB, xb, ab);
        load_batch(s0 + 3 * SB, xb, ab);
    }
    if ((kchunks & 7) != 0 && wave == kShWaves - 1) {  // the partial pair: chunks past K are zeros
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int kc = pairs * 8 + 2 * lg + h;
            const bool ok = kc < kchunks;
            const int sb = ok ? (pairs * 8 + h) * 16 : -(2 * lg * 16);  // dropped loads read the start of the row
            chunk_t x[TB], a[JB];
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) x[tb] = keep_if(ok, load_chunk(xrow[tb] + sb));
#pragma unroll
            for (int jb = 0; jb < JB; ++jb) a[jb] = keep_if(ok, load_chunk(Ab + ((int64_t)aoff[jb] + sb)));
#pragma unroll
            for (int tb = 0; tb < TB; ++tb)
#pragma unroll
                for (int jb = 0; jb < JB; ++jb) Elem<E>::mma16(acc[tb][jb], a[jb], x[tb]);
        }
    }

    LORA_TS(p.trace, 5);  // K loop issued
    // Sum the per-wave partial tiles in wave order (fixed order -> deterministic), scale, store.
    // acc[tb][jb][e] holds D[j = jb*16 + lg*4 + e][t = tb*16 + li].
    E *V = static_cast<E *>(p.V);
    const int jchunks = nj / CE;  // ranks are multiples of 8
    if constexpr (TB * JB <= 4) {
        // small tiles: every wave parks its partial tile, then each thread sums one output over the waves
        float *part = reinterpret_cast<float *>(smem);
        constexpr int TILE = TB * JB * 256;  // floats per wave; element (t, j) at t * (JB*16) + j
#pragma unroll
        for (int tb = 0; tb < TB; ++tb)
#pragma unroll
            for (int jb = 0; jb < JB; ++jb)
#pragma unroll
                for (int e = 0; e < 4; ++e) part[wave * TILE + (tb * 16 + li) * (JB * 16) + jb * 16 + lg * 4 + e] = acc[tb][jb][e];
        __syncthreads();
        for (int e = tid; e < nrows * jchunks; e += kShWaves * 64) {
            const int t = e / jchunks, jc = e - t * jchunks;
            float sum[CE];
#pragma unroll
            for (int q = 0; q < CE; ++q) sum[q] = 0.f;
#pragma unroll
            for (int w = 0; w < kShWaves; ++w) {
                const float *src = &part[w * TILE + t * (JB * 16) + jc * CE];
#pragma unroll
                for (int q = 0; q < CE; ++q) sum[q] += src[q];
            }
            E *dst = V + (int64_t)p.plan.perm[slot0 + t] * p.r_max + j0 + jc * CE;
            store4(dst, scale * sum[0], scale * sum[1], scale * sum[2], scale * sum[3]);
            if constexpr (CE == 8) store4(dst + 4, scale * sum[4], scale * sum[5], scale * sum[6], scale * sum[7]);
        }
    } else {
        // large tiles (long K loops behind them): one wave after the other adds into one buffer
        float *red = reinterpret_cast<float *>(smem);
        for (int w = 0; w < kShWaves; ++w) {
            if (wave == w) {
#pragma unroll
                for (int tb = 0; tb < TB; ++tb)
#pragma unroll
                    for (int jb = 0; jb < JB; ++jb)
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            float *dst = &red[(tb * 16 + li) * kRS + jb * 16 + lg * 4 + e];
                            *dst = (w == 0) ? acc[tb][jb][e] : (*dst + acc[tb][jb][e]);
                        }
            }
            __syncthreads();
        }
        for (int e = tid; e < nrows * jchunks; e += kShWaves * 64) {
            const int t = e / jchunks, jc = e - t * jchunks;
            const float *src = &red[t * kRS + jc * CE];
            E *dst = V + (int64_t)p.plan.perm[slot0 + t] * p.r_max + j0 + jc * CE;
            store4(dst, scale * src[0], scale * src[1], scale * src[2], scale * src[3]);
            if constexpr (CE == 8) store4(dst + 4, scale * src[4], scale * src[5], scale * src[6], scale * src[7]);
        }
    }
}

// Fragment-major copy of X for the decode-sized GEMM: output-ordered, so the writes are contiguous.
template <typename E>
__device__ __forceinline__ void pack_x(const ShrinkArgs &p, int wg) {
    constexpr int CE = Elem<E>::CE;
    const int kchunks = p.K / CE;
    const int steps = ((kchunks + 7) >> 3) * 2;  // whole 64-k stages
    const int64_t total = (int64_t)steps * p.pack_tblk * 64;
    chunk_t *dst = static_cast<chunk_t *>(p.xpack);
    for (int64_t idx = (int64_t)wg * (kShWaves * 64) + threadIdx.x; idx < total; idx += (int64_t)p.pack_wgs * (kShWaves * 64)) {
        const int lane = (int)(idx & 63);
        const int64_t blk = idx >> 6;
        const int tb = (int)(blk % p.pack_tblk), s = (int)(blk / p.pack_tblk);
        const int t = tb * 16 + (lane & 15), kc = s * 4 + (lane >> 4);
        dst[idx] = (t < p.T && kc < kchunks) ? load_chunk(static_cast<const E *>(p.X) + (int64_t)t * p.ldx + kc * CE) : zero_chunk();
    }
}

template <typename E>
__global__ __launch_bounds__(kShWaves * 64) void shrink_kernel(ShrinkArgs p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x;
    LORA_TS(p.trace, 0);

    if ((int)blockIdx.x < p.pack_wgs) {
        if (p.plan.scalars[kScStatus] != 0) return;
        pack_x<E>(p, blockIdx.x);
        return;
    }
    // A unit is a chain of dependent loads (work list -> row map and adapter table -> operands), each a
    // round trip to memory in a kernel that lasts a few of them: loads that do not depend on each other
    // are issued together.  The grid is an upper bound of the unit count and the work list is that
    // long, so the record can be read before the unit is known to exist.
    const int bid = blockIdx.x - p.pack_wgs;
    const int jg = bid % p.rank_groups;
    const int unit = bid / p.rank_groups;
    const int4 rec = reinterpret_cast<const int4 *>(p.plan.unit_rec)[unit];
    const int status = p.plan.scalars[kScStatus], n_units = p.plan.scalars[kScNUnits];
    if (status != 0 || unit >= n_units) return;
    LORA_TS(p.trace, 1);  // work-list record read

    // the plan's work list names the unit: adapter, rank, first slot, rows (one load, no search)
    const int a = rec.x, r = rec.y, slot0 = rec.z, nrows = rec.w;
    const int j0 = jg * p.rank_block;
    if (a < 0 || j0 >= r || nrows <= 0) return;
    const int nj = min(p.rank_block, r - j0);
    // Rows past the end of the unit are clamped to its last one: they only feed accumulator
    // entries that are never stored.
    int prow[4];
    {
        const int li = tid & 15;
        prow[0] = p.plan.perm[slot0 + min(li, nrows - 1)];
#pragma unroll
        for (int tb = 1; tb < 4; ++tb) prow[tb] = nrows > 16 ? p.plan.perm[slot0 + min(tb * 16 + li, nrows - 1)] : prow[0];
    }
    const E *Aa = static_cast<const E *>(p.A[a]);
    const float scale = p.scale[a];

    if (Aa == nullptr) {  // slot emptied after the plan was built: flag it, contribute nothing
        E *V = static_cast<E *>(p.V);
        if (tid == 0) atomicMin(&p.plan.scalars[kScStatus], kErrNotResident);
        for (int e = tid; e < nrows * nj; e += kShWaves * 64) {
            const int t = e / nj, j = e - t * nj;
            V[(int64_t)p.plan.perm[slot0 + t] * p.r_max + j0 + j] = Elem<E>::from_f32(0.f);
        }
        return;
    }

    // unit shape -> instantiation (all branches are uniform over the workgroup)
    if (nrows <= 16) {
        if (nj <= 16)
            shrink_unit<E, 1, 1>(p, Aa, scale, slot0, nrows, j0, nj, prow, smem);
        else if (nj <= 32)
            shrink_unit<E, 1, 2>(p, Aa, scale, slot0, nrows, j0, nj, prow, smem);
        else
            shrink_unit<E, 1, 4>(p, Aa, scale, slot0, nrows, j0, nj, prow, smem);
    } else {
        if (nj <= 16)
            shrink_unit<E, 4, 1>(p, Aa, scale, slot0, nrows, j0, nj, prow, smem);
        else if (nj <= 32)
            shrink_unit<E, 4, 2>(p, Aa, scale, slot0, nrows, j0, nj, prow, smem);
        else
            shrink_unit<E, 4, 4>(p, Aa, scale, slot0, nrows, j0, nj, prow, smem);
    }
    LORA_TS(p.trace, 6);
}

}  // namespace

hipError_t launch_shrink(const ShrinkArgs &a, int dtype, hipStream_t stream, const KernelTimer *timer) {
    const long grid = (long)a.max_units * a.rank_groups + a.pack_wgs;
    if (grid <= 0) return hipSuccess;
    if (a.xlds_bytes != 0 && a.xlds_bytes != kXldsBytes) return hipErrorInvalidValue;
    const size_t smem = (size_t)kShSmemBase + (size_t)a.xlds_bytes;
    static bool attr_set = false;  // more than the default 64 KB of dynamic LDS
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(shrink_kernel<__bf16>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kShSmemBase + kXldsBytes);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(shrink_kernel<float>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    kShSmemBase + kXldsBytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
#ifdef LORA_TRACE
    return trace_launch("shrink", grid, [&](long long *buf) {
        ShrinkArgs b = a;
        b.trace = buf;
        if (dtype == 1) return launch_kernel(shrink_kernel<__bf16>, dim3((unsigned)grid), dim3(kShWaves * 64), smem, stream, timer, b);
        return launch_kernel(shrink_kernel<float>, dim3((unsigned)grid), dim3(kShWaves * 64), smem, stream, timer, b);
    });
#else
    if (dtype == 1) return launch_kernel(shrink_kernel<__bf16>, dim3((unsigned)grid), dim3(kShWaves * 64), smem, stream, timer, a);
    return launch_kernel(shrink_kernel<float>, dim3((unsigned)grid), dim3(kShWaves * 64), smem, stream, timer, a);
#endif
}

}  // namespace lora
