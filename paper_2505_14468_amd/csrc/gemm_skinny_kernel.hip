// Decode-sized batches (T <= 128 rows): the layer is a weight-streaming problem, bound by
// reading W0 (and the used B_a) from HBM once.  Same contraction as the tiled kernel --
//
//     Y[t, n] = sum_k X[t, k] W0[n, k]  +  sum_p V[t, p] B_a(p)[n, p]
//
// (paper section 4.4: backbone and adapter results combined) -- but organised around the
// weight stream, memory latency and the vector cache's line rate instead of around LDS tiles:
//   * the whole batch is one M tile, so rows stay in their original order: no gather;
//   * a workgroup owns 16*NB output columns and the whole contraction axis; its 8 waves
//     split that axis between them and no workgroup depends on another (no split-K through
//     memory, no fences, nothing to reduce across CUs);
//   * every CU needs all of X for its few columns, so X is the larger stream into a CU (from
//     L2).  An MFMA operand wants "row i, 16 bytes of k" per lane, which read straight from a
//     row-major matrix touches 16 cache lines per quarter-wave; the vector cache then runs at
//     a quarter of its rate and becomes the bound.  So X is read from the fragment-major copy
//     the shrink launch leaves in the workspace (one contiguous 1 KiB block per MFMA step
//     and 16-row block), and W0 -- which must stay in its owner's layout -- is loaded with
//     rows contiguous across lanes (8 rows x 128 bytes per instruction) and turned into MFMA
//     layout through a small wave-private, XOR-swizzled LDS buffer (no barrier needed);
//   * loads are issued in batches of several MFMA steps, two batches in flight per wave, so
//     that a CU keeps >100 KB outstanding: a kernel this short is otherwise a handful of
//     serial round trips to HBM;
//   * MFMA 16x16x32: M = 16 output columns, N = 16 token rows; the matrix core idles most of
//     the time, as it should in a bandwidth-bound kernel;
//   * the extension (V against B_a, rows of other adapters masked to zero) is dealt
//     round-robin to the waves as extra MFMA steps;
//   * the 8 per-wave partial tiles are summed through LDS in wave order (fixed order, so the
//     result is reproducible) and Y is stored once.
#include <limits.h>

#include "kernels.h"

namespace lora {
namespace {

constexpr int kSkWaves = 8;
constexpr int kSkThreads = kSkWaves * 64;
constexpr int kSkTab = 512;  // extension chunks described per batch (128 MFMA steps)

struct SkTable {
    const void *ptr[kSkTab];  // B_a + j
    int r[kSkTab];            // row stride of B_a
    int j[kSkTab];            // column inside V / B_a
    int a[kSkTab];            // adapter id (-2 = unused column)
};

template <int TBLK, int NB>
__global__ __launch_bounds__(kSkThreads) void gemm_skinny_kernel(GemmArgs p) {
    typedef __bf16 E;
    constexpr int CE = 8;
    constexpr int LPG = 2 * NB + 2 * TBLK;             // 16-byte loads per lane per stage (2 MFMA steps = 64 k)
    constexpr int SGB = (20 / LPG) > 0 ? 20 / LPG : 1;  // stages per load batch; two batches in flight
    constexpr int TILE = NB * TBLK * 256;              // floats of one wave's partial tile
    constexpr int WBUF = NB * 16 * 8;                  // chunks of one W staging buffer (16*NB rows x 128 B)

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float *red = reinterpret_cast<float *>(smem);  // [kSkWaves][TILE]
    chunk_t *wstage = reinterpret_cast<chunk_t *>(smem + (size_t)kSkWaves * TILE * sizeof(float));  // [kSkWaves][WBUF]
    SkTable *tab = reinterpret_cast<SkTable *>(wstage + kSkWaves * WBUF);

    // the wave index as a scalar: K ranges, stage counters and stage offsets then live in scalar registers
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, lg = lane >> 4;
    const int n0 = blockIdx.x * (16 * NB);

    const E *V = static_cast<const E *>(p.V);
    const E *W = static_cast<const E *>(p.W);
    const chunk_t *Xp = static_cast<const chunk_t *>(p.Xpack);

    // W loads: lane -> (row lane/8 + 8*i of the 16-row block, chunk lane%8 of the 128-byte stage).
    // Rows past N are clamped to the last row: they only feed accumulator entries never stored.
    const int wr = lane >> 3, wc = lane & 7;
    const E *wrow[NB][2];  // row start + this lane's chunk of a stage; what changes per stage is a scalar
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int i = 0; i < 2; ++i) wrow[nb][i] = W + (int64_t)min(n0 + nb * 16 + wr + 8 * i, p.N - 1) * p.ldw + wc * CE;
    // swizzled positions inside the wave's staging buffer
    int wdst[NB][2];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int row = wr + 8 * i;
            wdst[nb][i] = (nb * 16 + row) * 8 + (wc ^ ((row >> 1) & 7));
        }
    chunk_t *buf = wstage + wave * WBUF;  // one buffer is enough: a wave's LDS operations execute in order
    const chunk_t *xlane = Xp + lane;

    f32x4_t acc[NB][TBLK];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int tb = 0; tb < TBLK; ++tb) acc[nb][tb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // ---- base product: this wave's share of the stages (64 k each) along K ---------------------------
    // Whole stages are dealt to the waves and run without masks; a last partial stage (K not a
    // multiple of 64) goes to the last wave.  Stages past a wave's range are skipped (a uniform
    // branch), not loaded and dropped.
    const int kchunks = p.K / CE;
    const int full = kchunks >> 3;
    const int sg0 = (int)((int64_t)full * wave / kSkWaves), sg1 = (int)((int64_t)full * (wave + 1) / kSkWaves);

    chunk_t wa[SGB][NB][2], xa[SGB][2][TBLK], wb[SGB][NB][2], xb[SGB][2][TBLK];
    auto load_batch = [&](int g0, chunk_t (&wf)[SGB][NB][2], chunk_t (&xf)[SGB][2][TBLK]) {
#pragma unroll
        for (int g = 0; g < SGB; ++g) {
            const int sg = g0 + g;
            if (sg < sg1) {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int i = 0; i < 2; ++i) wf[g][nb][i] = load_chunk(wrow[nb][i] + sg * (8 * CE));
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int tb = 0; tb < TBLK; ++tb) xf[g][h][tb] = xlane[((sg * 2 + h) * TBLK + tb) * 64];
            }
        }
    };
    auto mma_stage = [&](const chunk_t (&wf)[NB][2], const chunk_t (&xf)[2][TBLK]) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int i = 0; i < 2; ++i) buf[wdst[nb][i]] = wf[nb][i];
        // lanes exchange data through the wave's own buffer: LDS operations of one wave execute in
        // order, the fences only keep the compiler from reordering across the exchange
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const chunk_t w = buf[(nb * 16 + li) * 8 + ((h * 4 + lg) ^ ((li >> 1) & 7))];
#pragma unroll
                for (int tb = 0; tb < TBLK; ++tb) Elem<E>::mma16(acc[nb][tb], w, xf[h][tb]);
            }
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    };
    auto mma_batch = [&](int g0, const chunk_t (&wf)[SGB][NB][2], const chunk_t (&xf)[SGB][2][TBLK]) {
#pragma unroll
        for (int g = 0; g < SGB; ++g)
            if (g0 + g < sg1) mma_stage(wf[g], xf[g]);
    };

    load_batch(sg0, wa, xa);
    // (the first loads do not depend on the plan: its status is looked at while they are in flight)
    if (p.plan.scalars[kScStatus] != 0) return;

    // ---- extension table: one entry per 8 ranks of the batch's concatenated rank space ----------------
    const int ext_chunks = p.B != nullptr ? p.plan.scalars[kScExtTotal] / CE : 0;
    auto build_table = [&](int chunk0) {
        for (int idx = tid; idx < kSkTab; idx += kSkThreads) {
            const int ch = chunk0 + idx;
            const void *ptr = nullptr;
            int r = 0, j = 0, a = -2;
            if (ch < ext_chunks) {
                const int4 rec = reinterpret_cast<const int4 *>(p.plan.ext_rec)[ch];
                const E *b = rec.x >= 0 ? static_cast<const E *>(p.B[rec.x]) : nullptr;
                if (b != nullptr) {
                    r = rec.y >> 16;
                    j = rec.y & 0xffff;
                    a = rec.x;
                    ptr = b + j;
                } else {
                    atomicMin(&p.plan.scalars[kScStatus], kErrNotResident);
                }
            }
            tab->ptr[idx] = ptr;
            tab->r[idx] = r;
            tab->j[idx] = j;
            tab->a[idx] = a;
        }
    };
    int row_ad[TBLK];
#pragma unroll
    for (int tb = 0; tb < TBLK; ++tb) row_ad[tb] = -1;
    if (ext_chunks > 0) {
#pragma unroll
        for (int tb = 0; tb < TBLK; ++tb) {
            const int t = tb * 16 + li;
            row_ad[tb] = t < p.T ? p.plan.row_adapter[t] : -1;
        }
        build_table(0);
    }

    for (int g0 = sg0; g0 < sg1; g0 += 2 * SGB) {
        load_batch(g0 + SGB, wb, xb);
        mma_batch(g0, wa, xa);
        load_batch(g0 + 2 * SGB, wa, xa);
        mma_batch(g0 + SGB, wb, xb);
    }
    if ((kchunks & 7) != 0 && wave == kSkWaves - 1) {  // the partial stage: chunks past K are zeros (X's copy holds zeros there)
        const bool ok = full * 8 + wc < kchunks;
        chunk_t wf[NB][2], xf[2][TBLK];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int i = 0; i < 2; ++i) wf[nb][i] = keep_if(ok, load_chunk(ok ? wrow[nb][i] + full * (8 * CE) : wrow[nb][i] - wc * CE));
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int tb = 0; tb < TBLK; ++tb) xf[h][tb] = xlane[((full * 2 + h) * TBLK + tb) * 64];
        mma_stage(wf, xf);
    }

    // ---- extension steps, dealt round-robin to the waves --------------------------------------------------
    for (int chunk0 = 0; chunk0 < ext_chunks; chunk0 += kSkTab) {
        if (chunk0 > 0) {
            __syncthreads();
            build_table(chunk0);
        }
        __syncthreads();
        const int nst = (min(ext_chunks - chunk0, kSkTab) + 3) >> 2;
        for (int s = wave; s < nst; s += 2 * kSkWaves) {  // two steps per trip: their loads overlap
            chunk_t wf[2][NB], xf[2][TBLK];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int idx = min(s + u * kSkWaves, kSkTab / 4 - 1) * 4 + lg;
                const bool live = s + u * kSkWaves < nst;
                const E *bp = static_cast<const E *>(tab->ptr[idx]);
                const int r = tab->r[idx], j = tab->j[idx], a = tab->a[idx];
                const bool wok = live && bp != nullptr;
                const E *bsrc = wok ? bp : W;  // W: some in-bounds address for the dropped loads
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const int n = min(n0 + nb * 16 + li, p.N - 1);
                    wf[u][nb] = keep_if(wok, load_chunk(bsrc + (wok ? (int64_t)n * r : 0)));
                }
#pragma unroll
                for (int tb = 0; tb < TBLK; ++tb) {
                    const int t = min(tb * 16 + li, p.T - 1);
                    const bool xok = live && row_ad[tb] == a;  // rows of other adapters contribute nothing
                    xf[u][tb] = keep_if(xok, load_chunk(V + (xok ? (int64_t)t * p.r_max + j : 0)));
                }
            }
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int tb = 0; tb < TBLK; ++tb) Elem<E>::mma16(acc[nb][tb], wf[u][nb], xf[u][tb]);
        }
    }

    // ---- sum the 8 partial tiles in wave order, store Y once ------------------------------------------------
    // acc[nb][tb][e] = D[n = n0 + nb*16 + lg*4 + e][t = tb*16 + li]
    float4 *mine = reinterpret_cast<float4 *>(red + (size_t)wave * TILE);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int tb = 0; tb < TBLK; ++tb)
            mine[(nb * TBLK + tb) * 64 + lane] = make_float4(acc[nb][tb][0], acc[nb][tb][1], acc[nb][tb][2], acc[nb][tb][3]);
    __syncthreads();
    E *Y = static_cast<E *>(p.Y);
    for (int idx = tid; idx < NB * TBLK * 64; idx += kSkThreads) {
        float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int w = 0; w < kSkWaves; ++w) {
            const float4 v = reinterpret_cast<const float4 *>(red + (size_t)w * TILE)[idx];
            s.x += v.x;
            s.y += v.y;
            s.z += v.z;
            s.w += v.w;
        }
        const int blk = idx >> 6, l = idx & 63;
        const int nb = blk / TBLK, tb = blk - nb * TBLK;
        const int t = tb * 16 + (l & 15);
        const int n = n0 + nb * 16 + (l >> 4) * 4;
        if (t >= p.T) continue;
        E *yrow = Y + (int64_t)t * p.ldy;
        if (n + 3 < p.N) {
            store4(yrow + n, s.x, s.y, s.z, s.w);
        } else {
            const float v[4] = {s.x, s.y, s.z, s.w};
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (n + e < p.N) store1(yrow + n + e, v[e]);
        }
    }
}

template <int TBLK, int NB>
hipError_t launch_sk(const GemmArgs &a, hipStream_t stream, const KernelTimer *timer) {
    const int n_tiles = (a.N + 16 * NB - 1) / (16 * NB);
    const size_t smem = (size_t)kSkWaves * NB * TBLK * 256 * sizeof(float) + (size_t)kSkWaves * NB * 16 * 8 * sizeof(chunk_t) +
                        sizeof(SkTable);
    auto kern = gemm_skinny_kernel<TBLK, NB>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    return launch_kernel(kern, dim3((unsigned)n_tiles), dim3(kSkThreads), smem, stream, timer, a);
}

}  // namespace

// tblk: 16-row blocks (1, 2, 4, 8); nb: 16-column blocks per workgroup (1, 2, 4; nb * tblk <= 8).
hipError_t launch_gemm_skinny(const GemmArgs &a, int tblk, int nb, hipStream_t stream, const KernelTimer *timer) {
    if (a.T <= 0 || a.N <= 0) return hipSuccess;
    if (a.Xpack == nullptr) return hipErrorInvalidValue;
#define LORA_SK_CASE(TB_, NB_) \
    if (tblk == TB_ && nb == NB_) return launch_sk<TB_, NB_>(a, stream, timer)
    LORA_SK_CASE(1, 1);
    LORA_SK_CASE(1, 2);
    LORA_SK_CASE(1, 4);
    LORA_SK_CASE(2, 1);
    LORA_SK_CASE(2, 2);
    LORA_SK_CASE(2, 4);
    LORA_SK_CASE(4, 1);
    LORA_SK_CASE(4, 2);
    LORA_SK_CASE(8, 1);
#undef LORA_SK_CASE
    return hipErrorInvalidValue;
}

}  // namespace lora
