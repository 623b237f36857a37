// Segmented LoRA shrink: V[slot, j] = s_a * sum_k X[perm[slot], k] * A_a[k, j] for the rows of
// every adapter segment (first half of the adapter product of paper section 4.4).
//
// One workgroup = one work unit = (segment, block of <= 64 of its rows, group of <= 64 ranks).
// The unit list is the plan's seg_unit prefix sum; the grid is an upper bound and surplus
// workgroups leave at once.  Inside a unit the NW waves split the contraction axis K between
// them; each wave runs 16x16 MFMA tiles with the adapter rows (ranks) as the MFMA M dimension
// and the token rows as the N dimension, both operands loaded straight from global memory as
// 16-byte chunks (A_a is [r, K] and X is [T, K]: both are contiguous along K, which is what
// the MFMA operand layout wants).  Decode-sized segments (a handful of rows) simply leave
// most token columns of the tile empty: the kernel is bound by streaming A_a once, not by MFMA.
// The per-wave partial tiles are summed through LDS in wave order, so the result is
// deterministic, scaled by s_a in fp32 and stored once (bf16 or fp32).
#include "kernels.h"

namespace lora {
namespace {

template <typename E, int NW>
__global__ __launch_bounds__(NW * 64) void shrink_kernel(ShrinkArgs p) {
    constexpr int CE = Elem<E>::CE;
    constexpr int TB = kShrinkRows / 16;   // token blocks of 16
    constexpr int JB = kShrinkRanks / 16;  // rank blocks of 16
    constexpr int RS = kShrinkRanks + 1;   // padded row stride of the reduction buffer
    __shared__ float red[kShrinkRows * RS];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;

    if (p.plan.scalars[kScStatus] != 0) return;

    const int jg = blockIdx.x % p.rank_groups;
    const int unit = blockIdx.x / p.rank_groups;
    if (unit >= p.plan.scalars[kScNUnits]) return;

    // segment of this unit: last s with seg_unit[s] <= unit
    int lo = 0, hi = p.plan.scalars[kScNSeg];
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (p.plan.seg_unit[mid + 1] > unit)
            hi = mid;
        else
            lo = mid + 1;
    }
    const int s = lo;
    const int a = p.plan.seg_adapter[s];
    const int r = p.plan.seg_rank[s];
    const int j0 = jg * kShrinkRanks;
    if (a < 0 || j0 >= r) return;
    const int nj = min(kShrinkRanks, r - j0);
    const int slot0 = p.plan.seg_indptr[s] + (unit - p.plan.seg_unit[s]) * kShrinkRows;
    const int nrows = min(kShrinkRows, p.plan.seg_indptr[s + 1] - slot0);
    if (nrows <= 0) return;
    const E *Aa = static_cast<const E *>(p.A[a]);
    E *V = static_cast<E *>(p.V);

    if (Aa == nullptr) {  // slot emptied after the plan was built: flag it, contribute nothing
        if (tid == 0) atomicMin(&p.plan.scalars[kScStatus], kErrNotResident);
        for (int e = tid; e < nrows * nj; e += NW * 64) {
            const int t = e / nj, j = e - t * nj;
            V[(int64_t)(slot0 + t) * p.r_max + j0 + j] = Elem<E>::from_f32(0.f);
        }
        return;
    }
    const float scale = p.scale[a];

    // lane (i, g): row i of a 16-block, k-group g (one 16-byte chunk per MFMA step)
    const int li = lane & 15, lg = lane >> 4;
    const E *xrow[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        const int t = tb * 16 + li;
        xrow[tb] = t < nrows ? static_cast<const E *>(p.X) + (int64_t)p.plan.perm[slot0 + t] * p.ldx : nullptr;
    }
    const E *arow[JB];
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) {
        const int j = jb * 16 + li;
        arow[jb] = j < nj ? Aa + (int64_t)(j0 + j) * p.K : nullptr;
    }
    const int ntb = (nrows + 15) >> 4, njb = (nj + 15) >> 4;

    f32x4_t acc[TB][JB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int jb = 0; jb < JB; ++jb) acc[tb][jb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // this wave's share of the MFMA steps along K (one step = 4 chunks)
    const int kchunks = p.K / CE;
    const int steps = (kchunks + 3) >> 2;
    const int st0 = (int)((int64_t)steps * wave / NW), st1 = (int)((int64_t)steps * (wave + 1) / NW);
#pragma unroll 2
    for (int st = st0; st < st1; ++st) {
        const int kc = st * 4 + lg;
        const bool kvalid = kc < kchunks;
        const int koff = kc * CE;
        chunk_t xf[TB], af[JB];
#pragma unroll
        for (int tb = 0; tb < TB; ++tb)
            xf[tb] = (kvalid && xrow[tb] != nullptr && tb < ntb) ? load_chunk(xrow[tb] + koff) : zero_chunk();
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
            af[jb] = (kvalid && arow[jb] != nullptr && jb < njb) ? load_chunk(arow[jb] + koff) : zero_chunk();
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
            if (tb < ntb) {
#pragma unroll
                for (int jb = 0; jb < JB; ++jb)
                    if (jb < njb) Elem<E>::mma16(acc[tb][jb], af[jb], xf[tb]);
            }
        }
    }

    // sum the per-wave partial tiles in wave order (fixed order -> deterministic).
    // acc[tb][jb][e] holds D[j = jb*16 + lg*4 + e][t = tb*16 + li].
    for (int w = 0; w < NW; ++w) {
        if (wave == w) {
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) {
                if (tb < ntb) {
#pragma unroll
                    for (int jb = 0; jb < JB; ++jb) {
                        if (jb < njb) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                float *dst = &red[(tb * 16 + li) * RS + jb * 16 + lg * 4 + e];
                                *dst = (w == 0) ? acc[tb][jb][e] : (*dst + acc[tb][jb][e]);
                            }
                        }
                    }
                }
            }
        }
        __syncthreads();
    }

    // scale and store: one 16-byte chunk of V per thread
    const int jchunks = nj / CE;  // ranks are multiples of 8
    for (int e = tid; e < nrows * jchunks; e += NW * 64) {
        const int t = e / jchunks, jc = e - t * jchunks;
        const float *src = &red[t * RS + jc * CE];
        E *dst = V + (int64_t)(slot0 + t) * p.r_max + j0 + jc * CE;
        if constexpr (CE == 8) {
            store4(dst, scale * src[0], scale * src[1], scale * src[2], scale * src[3]);
            store4(dst + 4, scale * src[4], scale * src[5], scale * src[6], scale * src[7]);
        } else {
            store4(dst, scale * src[0], scale * src[1], scale * src[2], scale * src[3]);
        }
    }
}

}  // namespace

hipError_t launch_shrink(const ShrinkArgs &a, int dtype, hipStream_t stream, const KernelTimer *timer) {
    constexpr int NW = 8;
    const long grid = (long)a.max_units * a.rank_groups;
    if (grid <= 0) return hipSuccess;
    if (dtype == 1)
        return launch_kernel(shrink_kernel<__bf16, NW>, dim3((unsigned)grid), dim3(NW * 64), 0, stream, timer, a);
    return launch_kernel(shrink_kernel<float, NW>, dim3((unsigned)grid), dim3(NW * 64), 0, stream, timer, a);
}

}  // namespace lora
