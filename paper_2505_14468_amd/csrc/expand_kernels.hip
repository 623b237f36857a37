// Segmented LoRA expand as a kernel of its own, for batches of many small segments:
//
//     D[row, n] = sum_j V[row, j] * B_a[n, j]        for the rows of every adapter segment, in fp32
//
// (second half of the adapter product of paper section 4.4; the base GEMM that runs next adds D to
// its fp32 accumulators before it rounds and stores Y, once).  When an M tile of the fused GEMM holds dozens of adapters, every
// extension stage there serves a handful of rows, and the adapters' B matrices -- together larger
// than W0 in such a batch -- arrive through a two-deep, latency-bound pipeline.  Here the same work
// is a weight-streaming problem laid out like the shrink:
//
//   * a workgroup = one work unit of the plan's list (<= 64 rows of one segment, <= 16 in small plans) x 1024 output columns
//     (long enough a stream of B_a to pay for the unit's set-up: work list, row map, V);
//   * the unit's rows of V (<= 64 x r, a few KB) are staged in LDS once; as MFMA operand they are
//     read from there, so global loads carry B_a only;
//   * each of the 8 waves walks 16-column blocks; MFMA 16x16x32 with the 16 output columns as M
//     (operand rows = rows of B_a, contiguous along the rank) and 16 token rows as N; four groups
//     of loads (16 KB per wave) are in flight while one is multiplied, across block boundaries;
//   * steps come in pairs that share one 128-byte piece of every B_a row (step 2m takes the even
//     16-byte chunks, step 2m+1 the odd ones), so a load instruction covers whole cache lines;
//   * every (row, column) with an adapter belongs to exactly one unit, so D is stored, not accumulated;
//     rows without an adapter are never written and never read.  D costs 8 bytes of traffic per output
//     element with an adapter, against the B_a bytes streamed at HBM speed instead of through a
//     latency-bound pipeline; the host picks this path for batches of many small segments only;
//   * units of long segments (flagged in the work list) are skipped when the GEMM computes those itself;
//   * one launch can cover several projections of the same batch (ExpandSet), grid after grid.
#include "kernels.h"

namespace lora {
namespace {

constexpr int kExWaves = 8;
constexpr int kExBlocksPerWave = 8;                               // 16-column blocks per wave
constexpr int kExCols = kExWaves * kExBlocksPerWave * 16;         // output columns per workgroup
constexpr int kExGroup = 4;                                       // MFMA steps per load group
constexpr int kExRing = 4;                                        // load groups in flight per wave
constexpr int kExPad = 1;                                         // chunks of padding per staged row of V

template <typename E, int TB>
__device__ __forceinline__ void expand_unit(const ExpandArgs &p, const E *Ba, int r, int slot0, int nrows, int nwg0,
                                            unsigned char *smem) {
    constexpr int CE = Elem<E>::CE;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, lg = lane >> 4;
    const int rchunks = r / CE;
    const int vstride = rchunks + kExPad;
    chunk_t *vs = reinterpret_cast<chunk_t *>(smem);
    const E *V = static_cast<const E *>(p.V);

    // rows of D this lane stores (rows past the unit: never stored)
    int64_t drow[TB];
    bool rok[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        const int t = tb * 16 + li;
        rok[tb] = t < nrows;
        drow[tb] = (int64_t)p.plan.perm[slot0 + min(t, nrows - 1)] * p.ldd;
    }
    const chunk_t *vrow[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) vrow[tb] = vs + min(tb * 16 + li, nrows - 1) * vstride;

    // MFMA steps over the rank: pairs of steps, lane group g takes chunks 2g (even step) and 2g+1 (odd step)
    // of each 8-chunk piece; chunks past the rank contribute zeros (the V operand is zeroed).
    const int steps = 2 * ((rchunks + 7) >> 3);
    const int groups = (steps + kExGroup - 1) / kExGroup;
    auto chunk_of = [&](int st) { return (st >> 1) * 8 + 2 * lg + (st & 1); };

    // this wave's column blocks, b = 0 .. kExBlocksPerWave-1 (those below N): pairs of adjacent blocks (32 columns:
    // a row's two stores fall into one 128-byte line), pair p of wave w at column 32 * (w + 8 p)
    auto block_n0 = [&](int b) { return nwg0 + (2 * wave + (b & 1) + 2 * kExWaves * (b >> 1)) * 16; };
    int nblk = 0;
#pragma unroll
    for (int b = 0; b < kExBlocksPerWave; ++b) nblk += block_n0(b) < p.N ? 1 : 0;
    const int total = nblk * groups;  // (block, group) pairs, walked in order

    auto load_group = [&](int q, chunk_t (&wf)[kExGroup]) {
        if (q < total) {
            const int b = q / groups, g = q - b * groups;
            const E *brow = Ba + (int64_t)min(block_n0(b) + li, p.N - 1) * r;  // columns past N: clamped, never stored
#pragma unroll
            for (int s = 0; s < kExGroup; ++s) {
                const int st = g * kExGroup + s;
                const int kc = chunk_of(st);
                wf[s] = load_chunk(brow + (int64_t)((st < steps && kc < rchunks) ? kc : 0) * CE);
            }
        }
    };
    f32x4_t acc[TB];
    auto mma_group = [&](int q, const chunk_t (&wf)[kExGroup]) {
        const int g = q % groups;
#pragma unroll
        for (int s = 0; s < kExGroup; ++s) {
            const int st = g * kExGroup + s;
            if (st < steps) {
                const int kc = chunk_of(st);
                const bool ok = kc < rchunks;
#pragma unroll
                for (int tb = 0; tb < TB; ++tb) {
                    const chunk_t v = keep_if(ok, vrow[tb][ok ? kc : 0]);
                    Elem<E>::mma16(acc[tb], wf[s], v);
                }
            }
        }
    };
    // acc[tb][e] = D[n = n0 + lg*4 + e][t = tb*16 + li]: a lane stores 4 consecutive columns of one row
    auto flush_block = [&](int b) {
        const int n = block_n0(b) + lg * 4;
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
            if (!rok[tb]) continue;
            float *dst = p.D + drow[tb] + n;
            if (n + 3 < p.N) {
                store4(dst, acc[tb][0], acc[tb][1], acc[tb][2], acc[tb][3]);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (n + e < p.N) dst[e] = acc[tb][e];
            }
        }
    };

    // ---- stage the unit's rows of V (original row order in memory: gather through the row map) ----
    // V first: it comes from L2 and loads return in order -- behind B_a's loads from HBM it would arrive last.
    LORA_TS(p.trace, 2);  // row map read
    for (int e = tid; e < nrows * rchunks; e += kExWaves * 64) {
        const int t = e / rchunks, c = e - t * rchunks;
        vs[t * vstride + c] = load_chunk(V + (int64_t)p.plan.perm[slot0 + t] * p.r_max + (int64_t)c * CE);
    }
    // ---- a ring of kExRing groups of B_a loads in flight per wave ----
    chunk_t ring[kExRing][kExGroup];
#pragma unroll
    for (int i = 0; i < kExRing; ++i) load_group(i, ring[i]);
    __syncthreads();
    LORA_TS(p.trace, 3);  // V staged
    for (int q0 = 0; q0 < total; q0 += kExRing) {
#pragma unroll
        for (int i = 0; i < kExRing; ++i) {
            const int q = q0 + i;
            if (q < total) {
                if (q % groups == 0) {
#pragma unroll
                    for (int tb = 0; tb < TB; ++tb) acc[tb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                }
                mma_group(q, ring[i]);
                if ((q + 1) % groups == 0) flush_block(q / groups);
                load_group(q + kExRing, ring[i]);
            }
        }
    }
}

// The common shapes -- a whole group of 1024 columns, rank <= 128 (bf16) -- with every index a compile-time constant:
// S MFMA steps per 16-column block (2: at most 8 chunks of rank, 4: at most 16), the B_a loads of RING blocks in flight
// per wave (all 8: everything is requested before the first MFMA), the results of all 8 blocks kept in
// registers and stored after the last load has been consumed.  Loads and stores are counted by one in-order
// counter, so a store issued between loads makes the next wait for a load wait for the store's acknowledgement
// from memory as well; and no load sits behind a branch, so that the compiler can count the loads in flight.
template <typename E, int TB, int S, int RING>
__device__ __forceinline__ void expand_unit_whole(const ExpandArgs &p, const E *Ba, int r, int slot0, int nrows, int nwg0,
                                                  unsigned char *smem) {
    constexpr int CE = Elem<E>::CE;
    constexpr int NBLK = kExBlocksPerWave;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, lg = lane >> 4;
    const int rchunks = r / CE;
    const int vstride = rchunks + kExPad;
    chunk_t *vs = reinterpret_cast<chunk_t *>(smem);
    const E *V = static_cast<const E *>(p.V);

    // ---- the unit's rows of V: two chunks per thread at most (64 rows x 16 chunks), requested first ----
    chunk_t vreg[2];
    int vdst[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int e = tid + u * (kExWaves * 64);
        const bool ok = e < nrows * rchunks;
        const int t = ok ? e / rchunks : 0, c = ok ? e - t * rchunks : 0;
        vdst[u] = ok ? t * vstride + c : -1;
        vreg[u] = load_chunk(V + (int64_t)p.plan.perm[slot0 + t] * p.r_max + (int64_t)c * CE);
    }
    // ---- B_a: lane -> (column block_n0 + li, chunk of the step); chunks past the rank are read from chunk 0
    //      and meet a zeroed V operand ----
    auto block_n0 = [&](int b) { return nwg0 + (2 * wave + (b & 1) + 2 * kExWaves * (b >> 1)) * 16; };
    int kc[S];
    bool kok[S];
#pragma unroll
    for (int st = 0; st < S; ++st) {
        const int c = (st >> 1) * 8 + 2 * lg + (st & 1);
        kok[st] = c < rchunks;
        kc[st] = kok[st] ? c : 0;
    }
    auto load_block = [&](int b, chunk_t (&wf)[S]) {
        const E *brow = Ba + (int64_t)(block_n0(b) + li) * r;
#pragma unroll
        for (int st = 0; st < S; ++st) wf[st] = load_chunk(brow + kc[st] * CE);
    };
    chunk_t ring[RING][S];
#pragma unroll
    for (int i = 0; i < RING; ++i) load_block(i, ring[i]);
    LORA_TS(p.trace, 2);
#pragma unroll
    for (int u = 0; u < 2; ++u)
        if (vdst[u] >= 0) vs[vdst[u]] = vreg[u];
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");  // LDS only: the B_a loads stay in flight
    LORA_TS(p.trace, 3);  // V staged

    // V operands of this lane: row tb * 16 + li (clamped), the step's chunk; the same for every block
    chunk_t vop[TB][S];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int st = 0; st < S; ++st) vop[tb][st] = keep_if(kok[st], vs[min(tb * 16 + li, nrows - 1) * vstride + kc[st]]);

    f32x4_t acc[NBLK][TB];
#pragma unroll
    for (int b = 0; b < NBLK; ++b) {
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) acc[b][tb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int st = 0; st < S; ++st)
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) Elem<E>::mma16(acc[b][tb], ring[b % RING][st], vop[tb][st]);
        if (b + RING < NBLK) load_block(b + RING, ring[b % RING]);
    }
    LORA_TS(p.trace, 4);
    // acc[b][tb][e] = D[n = block_n0(b) + lg*4 + e][t = tb*16 + li]: a lane stores 4 consecutive columns of one row
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        const int t = tb * 16 + li;
        if (t >= nrows) continue;
        float *drow = p.D + (int64_t)p.plan.perm[slot0 + t] * p.ldd;
#pragma unroll
        for (int b = 0; b < NBLK; ++b) store4(drow + block_n0(b) + lg * 4, acc[b][tb][0], acc[b][tb][1], acc[b][tb][2], acc[b][tb][3]);
    }
}

// SMALL: every unit of the plan has at most 16 rows.  That instantiation keeps a quarter of the accumulators and
// half the loads in flight, fits 128 registers (4 waves per SIMD), and two workgroups share a CU: a unit of a few
// rows is a chain of dependent round trips (work list, row map and adapter table, operands) more than it is a
// stream, and one workgroup's chain overlaps the other's loads.
template <typename E, bool SMALL>
__global__ __launch_bounds__(kExWaves * 64, SMALL ? 4 : 2) void expand_kernel(ExpandArgs p0) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    LORA_TS(p0.trace, 0);
    // several projections of the same batch: the single-projection grids one after the other
    ExpandArgs p = p0;
    int bid = blockIdx.x;
    if (p0.n_sets > 0) {
        int si = 0;
        while (si + 1 < p0.n_sets && bid >= p0.set[si + 1].block0) ++si;
        bid -= p0.set[si].block0;
        p.V = p0.set[si].V;
        p.B = p0.set[si].B;
        p.D = p0.set[si].D;
        p.ldd = p0.set[si].ldd;
        p.N = p0.set[si].N;
        p.skip_long = p0.set[si].skip_long;
        p.col_groups = (p.N + kExCols - 1) / kExCols;
    }
    const int unit = bid / p.col_groups;
    const int cg = bid - unit * p.col_groups;
    // the grid is an upper bound of the unit count and the work list is that long
    const int4 rec = reinterpret_cast<const int4 *>(p.plan.unit_rec)[unit];
    const int status = p.plan.scalars[kScStatus], n_units = p.plan.scalars[kScNUnits];
    if (status != 0 || unit >= n_units) return;
    const int a = rec.x, r = rec.y & 0xffff, slot0 = rec.z, nrows = rec.w;
    if (a < 0 || r <= 0 || nrows <= 0) return;
    if (p.skip_long && (rec.y & kUnitLongFlag)) return;  // the GEMM computes this segment's term itself
    const E *Ba = static_cast<const E *>(p.B[a]);
    LORA_TS(p.trace, 1);  // work-list record read
    if (Ba == nullptr) {  // slot emptied after the plan was built: flag it, contribute nothing
        if (threadIdx.x == 0) atomicMin(&p.plan.scalars[kScEvicted], kErrNotResident);
        const int n_lo = cg * kExCols, n_hi = min(n_lo + kExCols, p.N);
        for (int e = threadIdx.x; e < nrows * (n_hi - n_lo); e += kExWaves * 64) {
            const int t = e / (n_hi - n_lo), n = n_lo + e - t * (n_hi - n_lo);
            p.D[(int64_t)p.plan.perm[slot0 + t] * p.ldd + n] = 0.f;
        }
        return;
    }
    const int rchunks = r / Elem<E>::CE;
    if ((cg + 1) * kExCols <= p.N && rchunks <= 16) {  // a whole column group, at most 4 MFMA steps along the rank
        if constexpr (SMALL) {
            if (rchunks <= 8)
                expand_unit_whole<E, 1, 2, 8>(p, Ba, r, slot0, nrows, cg * kExCols, smem);
            else
                expand_unit_whole<E, 1, 4, 4>(p, Ba, r, slot0, nrows, cg * kExCols, smem);
        } else if (nrows <= 16) {
            if (rchunks <= 8)
                expand_unit_whole<E, 1, 2, 8>(p, Ba, r, slot0, nrows, cg * kExCols, smem);
            else
                expand_unit_whole<E, 1, 4, 8>(p, Ba, r, slot0, nrows, cg * kExCols, smem);
        } else {
            if (rchunks <= 8)
                expand_unit_whole<E, 4, 2, 8>(p, Ba, r, slot0, nrows, cg * kExCols, smem);
            else
                expand_unit_whole<E, 4, 4, 4>(p, Ba, r, slot0, nrows, cg * kExCols, smem);
        }
    } else if (SMALL || nrows <= 16) {
        expand_unit<E, 1>(p, Ba, r, slot0, nrows, cg * kExCols, smem);
    } else {
        expand_unit<E, 4>(p, Ba, r, slot0, nrows, cg * kExCols, smem);
    }
    LORA_TS(p.trace, 5);
}

}  // namespace

size_t expand_smem_bytes(int r_max, int dtype) {
    const int ce = dtype == 1 ? 8 : 4;
    return (size_t)kShrinkRows * (size_t)(r_max / ce + kExPad) * 16;
}

// (ranks above ~480 need more than the default 64 KB of dynamic LDS: granted per kernel and device before the first launch)
hipError_t init_expand_kernels() {
    const void *fns[4] = {reinterpret_cast<const void *>(expand_kernel<__bf16, true>), reinterpret_cast<const void *>(expand_kernel<__bf16, false>),
                          reinterpret_cast<const void *>(expand_kernel<float, true>), reinterpret_cast<const void *>(expand_kernel<float, false>)};
    for (int i = 0; i < 4; ++i) {
        const size_t smem = expand_smem_bytes(kMaxRank, i < 2 ? 1 : 0);
        hipError_t e = hipFuncSetAttribute(fns[i], hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_expand(const ExpandArgs &a0, int dtype, hipStream_t stream, const KernelTimer *timer) {
    if (a0.max_units <= 0 || (a0.n_sets == 0 && a0.N <= 0)) return hipSuccess;
    ExpandArgs a = a0;
    long grid;
    if (a.n_sets > 0) {
        grid = 0;
        for (int i = 0; i < a.n_sets; ++i) {
            a.set[i].block0 = (int32_t)grid;
            grid += (long)a.max_units * ((a.set[i].N + kExCols - 1) / kExCols);
        }
    } else {
        a.col_groups = (a.N + kExCols - 1) / kExCols;
        grid = (long)a.max_units * a.col_groups;
    }
    if (grid <= 0) return hipSuccess;
    const size_t smem = expand_smem_bytes(a.r_max, dtype);
    const bool small = a.unit_rows <= kShrinkRowsSmall;
    auto launch = [&](const ExpandArgs &b) {
        const dim3 g((unsigned)grid), t(kExWaves * 64);
        if (dtype == 1)
            return small ? launch_kernel(expand_kernel<__bf16, true>, g, t, smem, stream, timer, b)
                         : launch_kernel(expand_kernel<__bf16, false>, g, t, smem, stream, timer, b);
        return small ? launch_kernel(expand_kernel<float, true>, g, t, smem, stream, timer, b)
                     : launch_kernel(expand_kernel<float, false>, g, t, smem, stream, timer, b);
    };
#ifdef LORA_TRACE
    return trace_launch("expand", grid, [&](long long *buf) {
        ExpandArgs b = a;
        b.trace = buf;
        return launch(b);
    });
#else
    return launch(a);
#endif
}

}  // namespace lora
