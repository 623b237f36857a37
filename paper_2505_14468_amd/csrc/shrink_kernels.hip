// Segmented LoRA shrink: V[row, j] = s_a * sum_k X[row, k] * A_a[k, j] for the rows of every
// adapter segment (first half of the adapter product of paper section 4.4).
//
// One workgroup = one work unit = (segment, block of <= 64 of its rows, group of <= 64 ranks).
// The unit list is part of the plan; the grid is an upper bound and surplus workgroups
// leave at once.  Inside a unit the 8 waves split the contraction axis K between
// them; each wave runs 16x16 MFMA tiles with the adapter rows (ranks) as the MFMA M dimension
// and the token rows as the N dimension.  A_a is [r, K] and X is [T, K], both contiguous along
// K: a wave loads a stage (128 bytes of every row, two MFMA steps) of a 16-row block as two
// instructions of 8 rows x 128 bytes -- whole cache lines -- and turns it into MFMA operand
// layout through a 2 KB wave-private LDS buffer.  A ring of stages is kept in registers and a
// block is requested again for the stage one ring later as soon as it has been consumed, because
// for decode-sized segments (a handful of rows, MFMA tile mostly empty) the kernel is bound by
// the latency and bandwidth of streaming A_a once.  The unit's shape picks the instantiation
// (1 or 4 token blocks, 1 / 2 / 4 rank blocks) so that small units spend their registers on
// loads in flight rather than on empty tiles.
// The per-wave partial tiles are summed through LDS in wave order, so the result is
// deterministic, scaled by s_a in fp32 and stored once (bf16 or fp32), in original row order.
#include <type_traits>

#include "kernels.h"

namespace lora {
namespace {

constexpr int kShWaves = 8;
constexpr int kRedBytes = 16 * 64 * 16;           // serial reduction buffer (large units): [16 tiles][64 lanes] float4
constexpr int kPartBytes = kShWaves * 4 * 1024;   // per-wave partial tiles (units of at most 4 MFMA tiles)
constexpr int kStageBytes = kShWaves * 2048;       // per-wave buffers that turn loaded lines into MFMA operands
constexpr int kXldsBytes = 64 * 1024;             // rows of X staged in LDS (units of a few rows)
constexpr int kXldsPad = 4;                       // chunks of padding per staged row: rows fall into different banks
constexpr int kXldsRows = 4;                      // at most this many rows are staged ...
constexpr int kXldsChunks = 2;                    // ... of at most this many chunks per thread (K <= 8192 in bf16)

// Dynamic LDS of the kernel: [reduction area][operand buffers][X staging area (only when launched with it)].
constexpr int kShSmemBase = kRedBytes > kPartBytes ? kRedBytes : kPartBytes;

// (AH: the unit's block of ranks has at most 8 of them -- one load instruction per stage of A_a covers it; the
// upper half of the MFMA tile then multiplies stale LDS contents into accumulator rows that are never stored)
template <typename E, int TB, int JB, bool AH = false>
__device__ __forceinline__ void shrink_unit(const ShrinkArgs &p, const E *Aa, float scale, int slot0, int nrows, int j0,
                                            int nj, const int (&prow)[4][2], unsigned char *smem) {
    static_assert(!AH || JB == 1, "half blocks of ranks: one block only");
    constexpr int AI = AH ? 1 : 2;  // load instructions per stage and 16-rank block of A_a
    constexpr int CE = Elem<E>::CE;
    constexpr int LPS = TB + JB;
    // Stages (128 bytes of every row: two MFMA steps) of operand loads in flight per wave, held in a ring of
    // registers; a 16-row block is requested again for the stage RS later as soon as it has been consumed.
    constexpr int RS = LPS >= 8 ? 1 : 16 / LPS;
    // The wave index as a scalar: the K ranges, stage counters and stage offsets below then live in scalar
    // registers and cost the vector pipeline nothing.  (Units of a few rows are short serial instruction
    // streams; every dependent vector instruction is ~10 cycles of their run time.)
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, lg = lane >> 4;
    const int kchunks = p.K / CE;

    // A unit of a few rows (decode) keeps its rows of X in LDS, shared by the waves: as MFMA operand a row
    // is wanted by every lane group of every wave.
    const bool xlds = TB == 1 && p.xlds_bytes > 0 && nrows <= kXldsRows && kchunks <= kXldsChunks * kShWaves * 64 &&
                      (int64_t)nrows * (kchunks + kXldsPad) * 16 <= p.xlds_bytes;
    chunk_t *xs = reinterpret_cast<chunk_t *>(smem + kShSmemBase + kStageBytes);
    const int xstride = kchunks + kXldsPad;

    // Operand loads.  An MFMA operand wants "row lane % 16, 16 bytes of k" per lane; read like that from a
    // row-major matrix an instruction touches 16 cache lines for 64 bytes each, and the vector cache then
    // delivers a third of what it does for whole lines (measured per CU: ~30 against ~80 GB/s).  So a stage
    // (128 bytes of every row: two MFMA steps) of a 16-row block is loaded as two instructions of 8 rows x
    // 128 bytes -- lane -> (row lane / 8 + 8 i, chunk lane % 8) -- and turned into operand layout through
    // a 2 KB wave-private, XOR-swizzled LDS buffer (no barrier: LDS operations of one wave execute in
    // order).  Step h of a stage takes chunks 4 h .. 4 h + 3, lane group g chunk 4 h + g, for both operands.
    // Ranks and rows past the end of the unit are clamped to the last one.
    const int wr = lane >> 3, wc = lane & 7;
    const char *Ab = reinterpret_cast<const char *>(Aa);
    unsigned aoff[JB][2];
    const char *xrow[TB][2];
    int wdst[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int row = wr + 8 * i;
        wdst[i] = row * 8 + (wc ^ ((row >> 1) & 7));
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
            aoff[jb][i] = (unsigned)(((int64_t)(j0 + min(jb * 16 + row, nj - 1)) * p.K + wc * CE) * (int64_t)sizeof(E));
#pragma unroll
        for (int tb = 0; tb < TB; ++tb)
            xrow[tb][i] = reinterpret_cast<const char *>(p.X) + ((int64_t)prow[tb][i] * p.ldx + wc * CE) * (int64_t)sizeof(E);
    }
    chunk_t *buf = reinterpret_cast<chunk_t *>(smem + kShSmemBase) + wave * 128;
    const int rsrc = li * 8, rswz = (li >> 1) & 7;
    const chunk_t *xsrow = xs + min(li, nrows - 1) * xstride + lg;

    f32x4_t acc[TB][JB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int jb = 0; jb < JB; ++jb) acc[tb][jb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // This wave's share of the stages along K.  Whole stages are dealt to the waves; a last partial one
    // (K not a multiple of the 128-byte piece) goes to the last wave, masked.
    const int full = kchunks >> 3;
    const int sg0 = (int)((int64_t)full * wave / kShWaves), sg1 = (int)((int64_t)full * (wave + 1) / kShWaves);

    // Stages past the wave's range are skipped (a uniform branch), not loaded and dropped: the address
    // unit's time is what this kernel runs out of.
    struct StageRegs {
        chunk_t x[TB][2], a[JB][2];
    };
    StageRegs ring[RS];
    // (the caller guarantees sg < sg1, or skips the call under a uniform branch)
    auto load_x = [&](int sg, int tb, StageRegs &f) {
        if (!xlds) {
#pragma unroll
            for (int i = 0; i < 2; ++i) f.x[tb][i] = load_chunk(xrow[tb][i] + (unsigned)sg * 128u);  // scalar stage offset
        }
    };
    auto load_a = [&](int sg, int jb, StageRegs &f) {
#pragma unroll
        for (int i = 0; i < AI; ++i) f.a[jb][i] = load_chunk(Ab + (unsigned)sg * 128u + aoff[jb][i]);
    };
    // one 16-row block of one stage: through the wave's buffer into the two steps' operands
    auto to_operands = [&](const chunk_t (&in)[2], chunk_t (&out)[2], bool both = true) {
        buf[wdst[0]] = in[0];
        if (both) buf[wdst[1]] = in[1];
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");  // keeps the compiler from reordering across the exchange
        out[0] = buf[rsrc + (lg ^ rswz)];
        out[1] = buf[rsrc + ((4 + lg) ^ rswz)];
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    };
    // One stage: X blocks to operands, then rank block by rank block.  REFILL: every consumed block is
    // requested again for stage `next`, unconditionally -- loads behind a branch would make the compiler wait
    // for ALL loads in flight at every use, because it can no longer count the younger ones.
    auto mma_stage = [&](int sg, StageRegs &f, int next, auto refill, bool partial) {
        constexpr int REFILL = decltype(refill)::value;  // 0 never, 1 always, 2 if next < sg1
        const bool again = REFILL == 1 || (REFILL == 2 && next < sg1);
        chunk_t x[TB][2];
        if (xlds) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int kc = sg * 8 + h * 4;  // + lg is in xsrow
                x[0][h] = xsrow[kc];
                if (partial) x[0][h] = keep_if(kc + lg < kchunks, x[0][h]);  // the staged rows end at K
            }
        } else {
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) {
                to_operands(f.x[tb], x[tb]);
                if (again) load_x(next, tb, f);
            }
        }
#pragma unroll
        for (int jb = 0; jb < JB; ++jb) {
            chunk_t a[2];
            to_operands(f.a[jb], a, !AH);
            if (again) load_a(next, jb, f);
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int tb = 0; tb < TB; ++tb) Elem<E>::mma16(acc[tb][jb], a[h], x[tb][h]);
        }
    };
    LORA_TS(p.trace, 2);  // row map, adapter pointer, scale read
    // Everything that can be requested now is requested now, oldest first in the order it is needed
    // (loads return in order): the unit's rows of X (a few KB, from L2), then the ring of operand
    // stages -- for a unit of one block each at K = 4096 that is a wave's whole share.
    chunk_t xr[kXldsRows][kXldsChunks];
    if (xlds) {
#pragma unroll
        for (int t = 0; t < kXldsRows; ++t)
            if (t < nrows) {
                // lane 8 t holds the row map entry of row t
                const int row = __builtin_amdgcn_readlane(prow[0][0], 8 * t);
                const E *src = static_cast<const E *>(p.X) + (int64_t)row * p.ldx;
#pragma unroll
                for (int u = 0; u < kXldsChunks; ++u) {
                    const int c = tid + u * (kShWaves * 64);
                    if (c < kchunks) xr[t][u] = load_chunk(src + (int64_t)c * CE);
                }
            }
    }
    if (sg0 < sg1) {  // (a wave with fewer than RS stages requests its last one more than once)
#pragma unroll
        for (int q = 0; q < RS; ++q) {
            const int sg = min(sg0 + q, sg1 - 1);
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) load_x(sg, tb, ring[q]);
#pragma unroll
            for (int jb = 0; jb < JB; ++jb) load_a(sg, jb, ring[q]);
        }
    }
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
    int g0 = sg0;
    for (; g0 + 2 * RS <= sg1; g0 += RS) {  // every stage here has its refill stage inside the wave's range
#pragma unroll
        for (int q = 0; q < RS; ++q) mma_stage(g0 + q, ring[q], g0 + q + RS, std::integral_constant<int, 1>{}, false);
    }
    if (g0 + RS < sg1) {  // the last ring-ful with refills: some of them
#pragma unroll
        for (int q = 0; q < RS; ++q) mma_stage(g0 + q, ring[q], g0 + q + RS, std::integral_constant<int, 2>{}, false);
        g0 += RS;
    }
#pragma unroll
    for (int q = 0; q < RS; ++q)
        if (g0 + q < sg1) mma_stage(g0 + q, ring[q], 0, std::integral_constant<int, 0>{}, false);
    if ((kchunks & 7) != 0 && wave == kShWaves - 1) {  // the partial stage: chunks past K are zeros
        const bool ok = full * 8 + wc < kchunks;
        const int sb = ok ? full * 128 : -(wc * 16);  // dropped loads read the start of the row
        StageRegs f;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            if (!xlds) {
#pragma unroll
                for (int tb = 0; tb < TB; ++tb) f.x[tb][i] = keep_if(ok, load_chunk(xrow[tb][i] + sb));
            }
#pragma unroll
            for (int jb = 0; jb < JB; ++jb) f.a[jb][i] = keep_if(ok, load_chunk(Ab + ((int64_t)aoff[jb][i] + sb)));
        }
        mma_stage(full, f, 0, std::integral_constant<int, 0>{}, true);
    }

    LORA_TS(p.trace, 5);  // K loop done (first wave)
    LORA_TS_WAVE(p.trace, 7, kShWaves - 1);  // (last wave)
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
        // large tiles (long K loops behind them): one wave after the other adds into one buffer, every lane into
        // its own 16-byte slot of every tile -- [tile][lane] float4: one conflict-free LDS read and write per tile
        float4 *red = reinterpret_cast<float4 *>(smem);
        for (int w = 0; w < kShWaves; ++w) {
            if (wave == w) {
#pragma unroll
                for (int tb = 0; tb < TB; ++tb)
#pragma unroll
                    for (int jb = 0; jb < JB; ++jb) {
                        float4 *dst = &red[(tb * JB + jb) * 64 + lane];
                        float4 v = make_float4(acc[tb][jb][0], acc[tb][jb][1], acc[tb][jb][2], acc[tb][jb][3]);
                        if (w != 0) {
                            const float4 o = *dst;
                            v.x += o.x;
                            v.y += o.y;
                            v.z += o.z;
                            v.w += o.w;
                        }
                        *dst = v;
                    }
            }
            __syncthreads();
        }
        // element (t, j) of the unit sits in tile (t / 16, j / 16), lane t % 16 + 16 * (j % 16 / 4), component j % 4
        for (int e = tid; e < nrows * jchunks; e += kShWaves * 64) {
            const int t = e / jchunks, jc = e - t * jchunks;
            float src[CE];
#pragma unroll
            for (int q = 0; q < CE / 4; ++q) {
                const int j = jc * CE + q * 4;
                const float4 v = red[((t >> 4) * JB + (j >> 4)) * 64 + (t & 15) + 16 * ((j & 15) >> 2)];
                src[q * 4 + 0] = v.x;
                src[q * 4 + 1] = v.y;
                src[q * 4 + 2] = v.z;
                src[q * 4 + 3] = v.w;
            }
            E *dst = V + (int64_t)p.plan.perm[slot0 + t] * p.r_max + j0 + jc * CE;
            store4(dst, scale * src[0], scale * src[1], scale * src[2], scale * src[3]);
            if constexpr (CE == 8) store4(dst + 4, scale * src[4], scale * src[5], scale * src[6], scale * src[7]);
        }
    }
}

template <typename E>
__global__ __launch_bounds__(kShWaves * 64) void shrink_kernel(ShrinkArgs p0) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x;
    LORA_TS(p0.trace, 0);

    // several projections of the same X: the single-projection grid with the projections innermost, eight
    // workgroups at a time -- workgroup ids go round-robin to the eight XCDs, so the workgroups that read the same
    // rows of X (one unit, one rank block, every projection) get ids that differ by 8: the same XCD, one after the
    // other, and a row of X comes from memory once and from that XCD's L2 for the others
    ShrinkArgs p = p0;
    int bid = blockIdx.x;
    if (p0.n_sets > 0) {
        const int q = bid >> 3;
        const int si = q % p0.n_sets;
        bid = (q / p0.n_sets) * 8 + (bid & 7);
        p.A = p0.set[si].A;
        p.scale = p0.set[si].scale;
        p.V = p0.set[si].V;
        p.n_adapters = p0.set[si].n_adapters;
        if (p.A == nullptr) return;  // a projection without adapters
    }
    // A unit is a chain of dependent loads (work list -> row map and adapter table -> operands), each a
    // round trip to memory in a kernel that lasts a few of them: loads that do not depend on each other
    // are issued together.  The grid is an upper bound of the unit count and the work list is that
    // long, so the record can be read before the unit is known to exist.
    // Grid order, chosen from the plan's totals (read in the same round trip as the work-list records of both
    // orders).  Adapters mostly of full rank (sum of the used ranks >= 3/4 of segments x r_max): the rank blocks of
    // a unit next to each other -- they read the same rows of X, and run at the same time.  Otherwise the unit index
    // fastest: the rank blocks past a small adapter's rank have nothing to do and exit at once, and with them
    // interleaved (period = rank_groups, a divisor of the eight XCDs the workgroups go to in turn) every unit with
    // work sits on the same XCDs and in the grid's second round.
    // (full ranks: the rank blocks of a unit get ids 8 apart -- the same XCD, whose L2 then serves the unit's rows of X
    // to all of them)
    const int mu8 = (p.max_units + 7) / 8 * 8;
    const int unit_a = bid % mu8, unit_b = ((bid >> 3) / p.rank_groups) * 8 + (bid & 7);
    const int4 rec_a = reinterpret_cast<const int4 *>(p.plan.unit_rec)[unit_a];
    const int4 rec_b = p.rank_groups > 1 ? reinterpret_cast<const int4 *>(p.plan.unit_rec)[unit_b] : rec_a;
    // Guessed ahead, in the same round trip as the record: lane i reads entry i of the adapter tables and of the
    // row map.  A decode batch (at most 64 rows, a pool of at most 64 adapters) finds everything it needs there
    // and skips the second round trip.
    const int lane = tid & 63;
    const void *a_guess = lane < p.n_adapters ? p.A[lane] : nullptr;
    const float s_guess = lane < p.n_adapters ? p.scale[lane] : 0.f;
    const int perm_guess = lane < p.T ? p.plan.perm[lane] : 0;
    const int status = p.plan.scalars[kScStatus], n_units = p.plan.scalars[kScNUnits];
    const int n_seg = p.plan.scalars[kScNSeg], ext_total = p.plan.scalars[kScExtTotal];
    const bool full_ranks = p.rank_groups > 1 && (long long)ext_total * 4 >= 3ll * p.r_max * n_seg;
    const int unit = full_ranks ? unit_b : unit_a;
    const int jg = full_ranks ? (bid >> 3) % p.rank_groups : bid / mu8;
    const int4 rec = full_ranks ? rec_b : rec_a;
    if (status != 0 || unit >= n_units) return;  // (n_units <= max_units: the grid's padding to eight units ends here too)
    LORA_TS(p.trace, 1);  // work-list record read

    // the plan's work list names the unit: adapter, rank, first slot, rows (one load, no search)
    const int a = rec.x, r = rec.y & 0xffff, slot0 = rec.z;
    const int nrows = rec.w;
    const int j0 = jg * p.rank_block;
    if (a < 0 || j0 >= r || nrows <= 0) return;
    const int nj = min(p.rank_block, r - j0);
    // Rows past the end of the unit are clamped to its last one: they only feed accumulator
    // entries that are never stored.
    int prow[4][2];  // lane -> row lane / 8 + 8 i of each 16-row block (the operand loads' mapping)
    const bool rows_guessed = slot0 + nrows <= 64;  // (uniform)
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int row = (lane >> 3) + 8 * i;
        if (rows_guessed) {
            prow[0][i] = __shfl(perm_guess, slot0 + min(row, nrows - 1));
#pragma unroll
            for (int tb = 1; tb < 4; ++tb) prow[tb][i] = nrows > 16 ? __shfl(perm_guess, slot0 + min(tb * 16 + row, nrows - 1)) : prow[0][i];
        } else {
            prow[0][i] = p.plan.perm[slot0 + min(row, nrows - 1)];
#pragma unroll
            for (int tb = 1; tb < 4; ++tb) prow[tb][i] = nrows > 16 ? p.plan.perm[slot0 + min(tb * 16 + row, nrows - 1)] : prow[0][i];
        }
    }
    const E *Aa;
    float scale;
    if (a < 64) {  // (uniform: the record is the same for every lane)
        const int as = __builtin_amdgcn_readfirstlane(a);
        const unsigned long long bits = (unsigned long long)a_guess;
        const unsigned lo = __builtin_amdgcn_readlane((unsigned)bits, as), hi = __builtin_amdgcn_readlane((unsigned)(bits >> 32), as);
        Aa = reinterpret_cast<const E *>(((unsigned long long)hi << 32) | lo);
        scale = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(s_guess), as));
    } else {
        Aa = static_cast<const E *>(p.A[a]);
        scale = p.scale[a];
    }

    if (Aa == nullptr) {  // slot emptied after the plan was built: flag it, contribute nothing
        E *V = static_cast<E *>(p.V);
        if (tid == 0) atomicMin(&p.plan.scalars[kScEvicted], kErrNotResident);
        for (int e = tid; e < nrows * nj; e += kShWaves * 64) {
            const int t = e / nj, j = e - t * nj;
            V[(int64_t)p.plan.perm[slot0 + t] * p.r_max + j0 + j] = Elem<E>::from_f32(0.f);
        }
        return;
    }

    // unit shape -> instantiation (all branches are uniform over the workgroup)
    if (nrows <= 16) {
        if (nj <= 8)
            shrink_unit<E, 1, 1, true>(p, Aa, scale, slot0, nrows, j0, nj, prow, smem);
        else if (nj <= 16)
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

// (more than the default 64 KB of dynamic LDS: granted per kernel and device before the first launch)
hipError_t init_shrink_kernels() {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(shrink_kernel<__bf16>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kShSmemBase + kStageBytes + kXldsBytes);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(shrink_kernel<float>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                kShSmemBase + kStageBytes + kXldsBytes);
    return e;
}

hipError_t launch_shrink(const ShrinkArgs &a, int dtype, hipStream_t stream, const KernelTimer *timer) {
    const long grid = (long)((a.max_units + 7) / 8 * 8) * a.rank_groups * (a.n_sets > 0 ? a.n_sets : 1);
    if (grid <= 0) return hipSuccess;
    if (a.xlds_bytes != 0 && a.xlds_bytes != kXldsBytes) return hipErrorInvalidValue;
    const size_t smem = (size_t)kShSmemBase + kStageBytes + (size_t)a.xlds_bytes;
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
