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
constexpr int kRS = kShrinkRanks + 1;  // padded row stride of the reduction buffer

template <typename E, int TB, int JB>
__device__ __forceinline__ void shrink_unit(const ShrinkArgs &p, const E *Aa, float scale, int slot0, int nrows, int j0,
                                            int nj, float *red) {
    constexpr int CE = Elem<E>::CE;
    constexpr int LPS = TB + JB;
    constexpr int SB = (TB * JB >= 8 ? 12 : 20) / LPS;  // MFMA steps per load batch (2 batches in flight)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 15, lg = lane >> 4;

    // Rows / ranks past the end of the unit are clamped to its last one: they only feed
    // accumulator entries that are never stored.
    const E *xrow[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
        xrow[tb] = static_cast<const E *>(p.X) + (int64_t)p.plan.perm[slot0 + min(tb * 16 + li, nrows - 1)] * p.ldx;
    const E *arow[JB];
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) arow[jb] = Aa + (int64_t)(j0 + min(jb * 16 + li, nj - 1)) * p.K;

    f32x4_t acc[TB][JB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int jb = 0; jb < JB; ++jb) acc[tb][jb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // this wave's share of the MFMA steps along K (one step = 4 chunks)
    const int kchunks = p.K / CE;
    const int steps = (kchunks + 3) >> 2;
    const int st0 = (int)((int64_t)steps * wave / kShWaves), st1 = (int)((int64_t)steps * (wave + 1) / kShWaves);

    chunk_t xa[SB][TB], aa[SB][JB], xb[SB][TB], ab[SB][JB];
    auto load_batch = [&](int s0, chunk_t (&xf)[SB][TB], chunk_t (&af)[SB][JB]) {
#pragma unroll
        for (int s = 0; s < SB; ++s) {
            const int kc = (s0 + s) * 4 + lg;
            const bool ok = (s0 + s) < st1 && kc < kchunks;  // beyond the range: load chunk 0, drop it
            const int koff = ok ? kc * CE : 0;
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) xf[s][tb] = keep_if(ok, load_chunk(xrow[tb] + koff));
#pragma unroll
            for (int jb = 0; jb < JB; ++jb) af[s][jb] = keep_if(ok, load_chunk(arow[jb] + koff));
        }
    };
    auto mma_batch = [&](const chunk_t (&xf)[SB][TB], const chunk_t (&af)[SB][JB]) {
#pragma unroll
        for (int s = 0; s < SB; ++s)
#pragma unroll
            for (int tb = 0; tb < TB; ++tb)
#pragma unroll
                for (int jb = 0; jb < JB; ++jb) Elem<E>::mma16(acc[tb][jb], af[s][jb], xf[s][tb]);
    };
    load_batch(st0, xa, aa);
    for (int s0 = st0; s0 < st1; s0 += 2 * SB) {
        load_batch(s0 + SB, xb, ab);
        mma_batch(xa, aa);
        load_batch(s0 + 2 * SB, xa, aa);
        mma_batch(xb, ab);
    }

    // sum the per-wave partial tiles in wave order (fixed order -> deterministic).
    // acc[tb][jb][e] holds D[j = jb*16 + lg*4 + e][t = tb*16 + li].
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

    // scale and store: one 16-byte chunk of V per thread
    E *V = static_cast<E *>(p.V);
    const int jchunks = nj / CE;  // ranks are multiples of 8
    for (int e = tid; e < nrows * jchunks; e += kShWaves * 64) {
        const int t = e / jchunks, jc = e - t * jchunks;
        const float *src = &red[t * kRS + jc * CE];
        E *dst = V + (int64_t)p.plan.perm[slot0 + t] * p.r_max + j0 + jc * CE;
        if constexpr (CE == 8) {
            store4(dst, scale * src[0], scale * src[1], scale * src[2], scale * src[3]);
            store4(dst + 4, scale * src[4], scale * src[5], scale * src[6], scale * src[7]);
        } else {
            store4(dst, scale * src[0], scale * src[1], scale * src[2], scale * src[3]);
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
    __shared__ float red[kShrinkRows * kRS];
    const int tid = threadIdx.x;

    if (p.plan.scalars[kScStatus] != 0) return;
    if ((int)blockIdx.x < p.pack_wgs) {
        pack_x<E>(p, blockIdx.x);
        return;
    }
    const int bid = blockIdx.x - p.pack_wgs;
    const int jg = bid % p.rank_groups;
    const int unit = bid / p.rank_groups;
    if (unit >= p.plan.scalars[kScNUnits]) return;

    // the plan's work list names the unit: adapter, rank, first slot, rows (one load, no search)
    const int4 rec = reinterpret_cast<const int4 *>(p.plan.unit_rec)[unit];
    const int a = rec.x, r = rec.y, slot0 = rec.z, nrows = rec.w;
    const int j0 = jg * kShrinkRanks;
    if (a < 0 || j0 >= r || nrows <= 0) return;
    const int nj = min(kShrinkRanks, r - j0);
    const E *Aa = static_cast<const E *>(p.A[a]);

    if (Aa == nullptr) {  // slot emptied after the plan was built: flag it, contribute nothing
        E *V = static_cast<E *>(p.V);
        if (tid == 0) atomicMin(&p.plan.scalars[kScStatus], kErrNotResident);
        for (int e = tid; e < nrows * nj; e += kShWaves * 64) {
            const int t = e / nj, j = e - t * nj;
            V[(int64_t)p.plan.perm[slot0 + t] * p.r_max + j0 + j] = Elem<E>::from_f32(0.f);
        }
        return;
    }
    const float scale = p.scale[a];

    // unit shape -> instantiation (all branches are uniform over the workgroup)
    if (nrows <= 16) {
        if (nj <= 16)
            shrink_unit<E, 1, 1>(p, Aa, scale, slot0, nrows, j0, nj, red);
        else if (nj <= 32)
            shrink_unit<E, 1, 2>(p, Aa, scale, slot0, nrows, j0, nj, red);
        else
            shrink_unit<E, 1, 4>(p, Aa, scale, slot0, nrows, j0, nj, red);
    } else {
        if (nj <= 16)
            shrink_unit<E, 4, 1>(p, Aa, scale, slot0, nrows, j0, nj, red);
        else if (nj <= 32)
            shrink_unit<E, 4, 2>(p, Aa, scale, slot0, nrows, j0, nj, red);
        else
            shrink_unit<E, 4, 4>(p, Aa, scale, slot0, nrows, j0, nj, red);
    }
}

}  // namespace

hipError_t launch_shrink(const ShrinkArgs &a, int dtype, hipStream_t stream, const KernelTimer *timer) {
    const long grid = (long)a.max_units * a.rank_groups + a.pack_wgs;
    if (grid <= 0) return hipSuccess;
    if (dtype == 1) return launch_kernel(shrink_kernel<__bf16>, dim3((unsigned)grid), dim3(kShWaves * 64), 0, stream, timer, a);
    return launch_kernel(shrink_kernel<float>, dim3((unsigned)grid), dim3(kShWaves * 64), 0, stream, timer, a);
}

}  // namespace lora
