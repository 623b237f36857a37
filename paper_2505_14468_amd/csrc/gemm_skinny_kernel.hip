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

template <int TBLK, int NB>
__global__ __launch_bounds__(kSkThreads) void gemm_skinny_kernel(GemmArgs p0) {
    typedef __bf16 E;
    constexpr int CE = 8;
    constexpr int WS = 8 / NB;  // stages of W0 requested ahead (a stage = 2 MFMA steps = 64 k; 2 * NB loads per lane)
    constexpr int XB0 = 4 / TBLK < WS / 2 ? 4 / TBLK : WS / 2;
    constexpr int XB = XB0 > 0 ? XB0 : 1;  // stages per batch of X loads (2 * TBLK loads per lane each); two batches in flight
    static_assert(WS % (2 * XB) == 0, "a W0 window is a whole number of X batch pairs");
    constexpr int TILE = NB * TBLK * 256;              // floats of one wave's partial tile
    constexpr int WBUF = NB * 16 * 8;                  // chunks of one W staging buffer (16*NB rows x 128 B)

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float *red = reinterpret_cast<float *>(smem);  // [kSkWaves][TILE]
    chunk_t *wstage = reinterpret_cast<chunk_t *>(smem + (size_t)kSkWaves * TILE * sizeof(float));  // [kSkWaves][WBUF]

    // the wave index as a scalar: K ranges, stage counters and stage offsets then live in scalar registers
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, lg = lane >> 4;
    // several projections of the same X: their column blocks follow each other in the grid
    GemmArgs p = p0;
    int blk = blockIdx.x;
    if (p0.n_sets > 0) {
        int si = 0;
        while (si + 1 < p0.n_sets && blk >= p0.set[si + 1].tile0) ++si;
        blk -= p0.set[si].tile0;
        p.W = p0.set[si].W;
        p.ldw = p0.set[si].ldw;
        p.Y = p0.set[si].Y;
        p.ldy = p0.set[si].ldy;
        p.V = p0.set[si].V;
        p.B = p0.set[si].B;
        p.N = p0.set[si].N;
    }
    const int n0 = blk * (16 * NB);
    LORA_TS(p.trace, 0);

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

    // W0 comes from HBM, X from L2, and loads return in order: a wait for X would also wait for every W0
    // load issued before it.  So the two streams are decoupled: the W0 loads of a whole window of stages
    // (all of a wave's share at K = 4096) go out first and have the X traffic to hide behind, then X
    // flows in small batches.
    chunk_t wq[WS][NB][2], xa[XB][2][TBLK], xb[XB][2][TBLK];
    auto load_w = [&](int S) {
#pragma unroll
        for (int q = 0; q < WS; ++q)
            if (S + q < sg1) {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int i = 0; i < 2; ++i) wq[q][nb][i] = load_chunk(wrow[nb][i] + (S + q) * (8 * CE));
            }
    };
    auto load_x = [&](int g0, chunk_t (&xf)[XB][2][TBLK]) {
#pragma unroll
        for (int g = 0; g < XB; ++g) {
            const int sg = g0 + g;
            if (sg < sg1) {
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
    // ---- extension: MFMA steps over the batch's concatenated rank space, dealt round-robin to the waves ----
    // A step is 4 chunks of 8 ranks; lane group g works on chunk 4 s + g, described by one record of the plan
    // (adapter, its rank, the chunk's offset inside it).  Every lane fetches the record and then the
    // adapter's B pointer for its own chunk -- two dependent loads, no table in LDS, no barrier.  Loads return
    // in order, so each of the two is issued just BEFORE a batch of the base product's loads: waiting for it
    // then waits for nothing younger, and the round trips hide behind the batches.  A trip is two steps.
    const int ext_chunks = p.B != nullptr ? p.plan.scalars[kScExtTotal] / CE : 0;
    const int status = p.plan.scalars[kScStatus];
    const int nst = (ext_chunks + 3) >> 2;
    int row_ad[TBLK];  // adapter of this lane's token rows (set below)
    auto fetch_rec = [&](int s, int4 (&rec)[2]) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int ch = (s + u * kSkWaves) * 4 + lg;
            rec[u] = make_int4(-2, 0, 0, 0);  // unused chunk
            if (ch < ext_chunks) rec[u] = reinterpret_cast<const int4 *>(p.plan.ext_rec)[ch];
        }
    };
    auto fetch_ptr = [&](const int4 (&rec)[2], const void *(&bp)[2]) {
#pragma unroll
        for (int u = 0; u < 2; ++u) bp[u] = rec[u].x >= 0 ? p.B[rec[u].x] : nullptr;
    };
    auto ext_load = [&](const int4 (&rec)[2], const void *(&bp)[2], chunk_t (&wf)[2][NB], chunk_t (&xf)[2][TBLK]) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int a = rec[u].x, r = rec[u].y >> 16, j = rec[u].y & 0xffff;
            const bool wok = bp[u] != nullptr;
            if (a >= 0 && !wok) atomicMin(&p.plan.scalars[kScEvicted], kErrNotResident);  // slot emptied after the plan
            const E *bsrc = wok ? static_cast<const E *>(bp[u]) + j : W;  // W: some in-bounds address for the dropped loads
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const int n = min(n0 + nb * 16 + li, p.N - 1);
                wf[u][nb] = keep_if(wok, load_chunk(bsrc + (wok ? (int64_t)n * r : 0)));
            }
#pragma unroll
            for (int tb = 0; tb < TBLK; ++tb) {
                const int t = min(tb * 16 + li, p.T - 1);
                const bool xok = wok && row_ad[tb] == a;  // rows of other adapters contribute nothing
                xf[u][tb] = keep_if(xok, load_chunk(V + (xok ? (int64_t)t * p.r_max + j : 0)));
            }
        }
    };
    auto ext_mma = [&](const chunk_t (&wf)[2][NB], const chunk_t (&xf)[2][TBLK]) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int tb = 0; tb < TBLK; ++tb) Elem<E>::mma16(acc[nb][tb], wf[u][nb], xf[u][tb]);
    };

    const bool ext_first = wave < nst;  // this wave has a first trip (steps wave and wave + 8)
    constexpr bool kEarly = TBLK * NB <= 4;  // registers to spare for the early fetch (else: after the K loop)
    int4 rec0[2];
    const void *bptr0[2];
    if (kEarly) fetch_rec(wave, rec0);
    load_w(sg0);
    load_x(sg0, xa);
    if (status != 0) return;
    if (kEarly) fetch_ptr(rec0, bptr0);
#pragma unroll
    for (int tb = 0; tb < TBLK; ++tb) {
        const int t = tb * 16 + li;
        row_ad[tb] = (ext_chunks > 0 && t < p.T) ? p.plan.row_adapter[t] : -1;
    }
    load_x(sg0 + XB, xb);
    LORA_TS(p.trace, 1);  // first window of W0 and two batches of X issued
    chunk_t ewf[2][NB], exf[2][TBLK];

    // ---- the K loop; the operands of the wave's first extension trip are fetched under its last pass ----
    bool ext_loaded = false;
    for (int S = sg0; S < sg1; S += WS) {
        if (kEarly && ext_first && S + WS >= sg1) {  // the last window hides the first extension trip's loads
            ext_load(rec0, bptr0, ewf, exf);
            ext_loaded = true;
        }
#pragma unroll
        for (int q = 0; q < WS; q += 2 * XB) {
#pragma unroll
            for (int g = 0; g < XB; ++g)
                if (S + q + g < sg1) mma_stage(wq[q + g], xa[g]);
            load_x(S + q + 2 * XB, xa);
#pragma unroll
            for (int g = 0; g < XB; ++g)
                if (S + q + XB + g < sg1) mma_stage(wq[q + XB + g], xb[g]);
            load_x(S + q + 3 * XB, xb);
        }
        load_w(S + WS);  // K beyond one window: its latency shows once per window
    }
    LORA_TS(p.trace, 3);  // K loop issued (MFMAs may still run)
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
    if (ext_first) {
        if (!kEarly) {
            fetch_rec(wave, rec0);
            fetch_ptr(rec0, bptr0);
        }
        if (!ext_loaded) ext_load(rec0, bptr0, ewf, exf);  // a wave without a share of K, or no registers to spare
        ext_mma(ewf, exf);
        for (int s = wave + 2 * kSkWaves; s < nst; s += 2 * kSkWaves) {  // more than 64 chunks of ranks in the batch
            int4 rec[2];
            const void *bp[2];
            fetch_rec(s, rec);
            fetch_ptr(rec, bp);
            ext_load(rec, bp, ewf, exf);
            ext_mma(ewf, exf);
        }
    }
    LORA_TS(p.trace, 4);  // extension issued
    // ---- sum the 8 partial tiles in wave order, store Y once ------------------------------------------------
    // acc[nb][tb][e] = D[n = n0 + nb*16 + lg*4 + e][t = tb*16 + li]
    float4 *mine = reinterpret_cast<float4 *>(red + (size_t)wave * TILE);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int tb = 0; tb < TBLK; ++tb)
            mine[(nb * TBLK + tb) * 64 + lane] = make_float4(acc[nb][tb][0], acc[nb][tb][1], acc[nb][tb][2], acc[nb][tb][3]);
    __syncthreads();
    LORA_TS(p.trace, 5);  // partial tiles parked
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
    LORA_TS(p.trace, 6);
}

template <int TBLK, int NB>
hipError_t launch_sk(const GemmArgs &a0, hipStream_t stream, const KernelTimer *timer) {
    GemmArgs a = a0;
    int n_tiles = (a.N + 16 * NB - 1) / (16 * NB);
    if (a.n_sets > 0) {
        n_tiles = 0;
        for (int i = 0; i < a.n_sets; ++i) {
            a.set[i].tile0 = n_tiles;
            n_tiles += (a.set[i].N + 16 * NB - 1) / (16 * NB);
        }
    }
    if (n_tiles <= 0) return hipSuccess;
    const size_t smem = (size_t)kSkWaves * NB * TBLK * 256 * sizeof(float) + (size_t)kSkWaves * NB * 16 * 8 * sizeof(chunk_t);
    auto kern = gemm_skinny_kernel<TBLK, NB>;
#ifdef LORA_TRACE
    return trace_launch("gemm_skinny", n_tiles, [&](long long *buf) {
        GemmArgs b = a;
        b.trace = buf;
        return launch_kernel(kern, dim3((unsigned)n_tiles), dim3(kSkThreads), smem, stream, timer, b);
    });
#else
    return launch_kernel(kern, dim3((unsigned)n_tiles), dim3(kSkThreads), smem, stream, timer, a);
#endif
}

template <int TBLK, int NB>
hipError_t init_sk() {
    const size_t smem = (size_t)kSkWaves * NB * TBLK * 256 * sizeof(float) + (size_t)kSkWaves * NB * 16 * 8 * sizeof(chunk_t);
    return hipFuncSetAttribute(reinterpret_cast<const void *>(gemm_skinny_kernel<TBLK, NB>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
}

}  // namespace

hipError_t init_gemm_skinny_kernels() {
    hipError_t e = init_sk<1, 1>();
    if (e == hipSuccess) e = init_sk<1, 2>();
    if (e == hipSuccess) e = init_sk<1, 4>();
    if (e == hipSuccess) e = init_sk<2, 1>();
    if (e == hipSuccess) e = init_sk<2, 2>();
    if (e == hipSuccess) e = init_sk<2, 4>();
    if (e == hipSuccess) e = init_sk<4, 1>();
    if (e == hipSuccess) e = init_sk<4, 2>();
    if (e == hipSuccess) e = init_sk<6, 1>();
    if (e == hipSuccess) e = init_sk<8, 1>();
    return e;
}

// tblk: 16-row blocks (1, 2, 4, 6, 8); nb: 16-column blocks per workgroup (1, 2, 4; nb * tblk <= 8).
hipError_t launch_gemm_skinny(const GemmArgs &a, int tblk, int nb, hipStream_t stream, const KernelTimer *timer) {
    if (a.T <= 0 || (a.n_sets == 0 && a.N <= 0)) return hipSuccess;
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
    LORA_SK_CASE(6, 1);
    LORA_SK_CASE(8, 1);
#undef LORA_SK_CASE
    return hipErrorInvalidValue;
}

}  // namespace lora
