// LDS-tiled MFMA GEMM with the LoRA expand fused as extra K-steps:
//
//     Y[row, n] = sum_k X[row, k] W0[n, k]  +  sum_{p in ext(row)} V[row, p] B_a[n, p],   row = perm[slot]
//
// (paper section 4.4: backbone result and adapter result are combined; here they are combined
// in the fp32 accumulators, before Y is rounded and stored, once.)
//
// Rows are processed in the plan's slot order (sorted by adapter), so the rows of one adapter
// are contiguous.  For an M-tile the adapters of its rows form a contiguous range of segments,
// and the concatenation of their ranks is one more stretch of the contraction axis: the "X
// operand" there is V (zero for rows that belong to another adapter), the "W operand" is the
// matching B_a slice.  B_a is stored [N, r] (r contiguous) and W0 [N, K] (K contiguous), so both
// feed the same MFMA operand path unchanged.  MFMA work in the extension is skipped for 32-row
// blocks that hold no row of the adapter at hand.
//
// Tile: BM token rows x BN output columns, BK = 8 chunks (128 bytes) of the contraction axis
// per stage, double-buffered in LDS, global -> registers -> LDS.  The base product is a
// hand-written software pipeline: MFMA operands are read from LDS one use ahead, the last
// k-step of a stage is split around the stage's barrier, and two register sets of
// staged operands keep the loads of the stage after next in flight while the next one is
// written to LDS, a third in each of a stage's first three k-steps (4 waves per workgroup, one per SIMD, for
// every tile shape); the issue order inside a k-step is fixed with scheduling groups: MFMA, other, MFMA, other.  MFMA orientation: M = output column n (W rows),
// N = token row t (X rows), so that every lane ends up with 4 consecutive n of one row.
// LDS rows are 8 chunks long and XOR-swizzled by (row >> 1) & 7 so that both the 16-byte
// stores (8 lanes per row) and the MFMA operand reads (32 rows, one chunk column) spread
// over all banks.
//
// The extension columns of a tile are described by a table in LDS, packed to the columns in use; its first
// stage is requested in front of the last base stage.  When the adapter term of the short segments comes
// from the expand kernel (GemmSet::D, long_rows > 0), only segments of long_rows rows and more are
// extension columns here, and only the rows of the shorter ones add D in the epilogue.  One launch can
// cover several projections of the same X (GemmSet): their column tiles follow each other in the grid.
//
// Workgroup -> tile mapping is XCD-aware: consecutive workgroup ids go round-robin to the 8
// XCDs, so id % 8 picks the XCD and each XCD walks a contiguous, M-grouped range of tiles
// that share W0 / X panels in its own L2.
#include <limits.h>

#include <type_traits>

#include "kernels.h"

namespace lora {
namespace {

constexpr int kTabCap = 512;  // extension chunk columns described per batch (64 stages)

__device__ __forceinline__ int swz(int row, int c) { return row * 8 + (c ^ ((row >> 1) & 7)); }

struct ExtTable {
    const void *ptr[kTabCap];  // B_a + j (null = column unused)
    int r[kTabCap];            // row stride of B_a (its rank)
    int j[kTabCap];            // column offset inside V / B_a
    int lo[kTabCap];           // tile-relative rows [lo, hi) that belong to the adapter
    int hi[kTabCap];
    int cnt[kTabCap / 64];     // columns in use per wave-sized piece of a batch (while the table is built)
    unsigned char use_d[256];  // tile row takes its adapter term from D (the expand kernel's result)
};

// SPLIT: the launch is split along K (grid y = split index); partial tiles go to GemmArgs::P in fp32.
template <typename E, int BM, int BN, int WM, int WN, bool SPLIT>
__global__ __launch_bounds__(WM *WN * 64) void gemm_tile_kernel(GemmArgs p, int tiles_m, int tiles_n, int group_m) {
    constexpr int CE = Elem<E>::CE;
    constexpr int NT = WM * WN * 64;
    constexpr int WTM = BM / WM, WTN = BN / WN;  // wave tile: rows t, columns n
    constexpr int NBT = WTM / 32, NBN = WTN / 32;
    constexpr int XL = BM * 8 / NT, WL = BN * 8 / NT;  // 16-byte loads per thread per stage
    constexpr int RPP = NT / 8;                        // rows covered per load pass
    static_assert(XL >= 1 && WL >= 1 && NBT >= 1 && NBN >= 1, "tile too small for the workgroup");
    static_assert(kTabCap % NT == 0 && BM <= 256, "extension table layout");
    // Every tile shape runs on 4 waves (up to 512 registers each): the base product keeps two register sets of
    // staged operands (see the loop below).
    static_assert(XL + WL >= 4 && WM * WN == 4, "the two-set pipeline deals a stage's loads to four k-steps of one wave per SIMD");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    chunk_t *sW = reinterpret_cast<chunk_t *>(smem);                 // [2][BN*8]
    chunk_t *sX = sW + 2 * BN * 8;                                   // [2][BM*8]
    ExtTable *tab = reinterpret_cast<ExtTable *>(sX + 2 * BM * 8);

    if (p.plan.scalars[kScStatus] != 0) return;

    // ---- workgroup -> tile (XCD-aware, M-grouped) --------------------------------------
    const int total = tiles_m * tiles_n;
    const int per_xcd = (total + 7) >> 3;
    const int lin = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (lin >= total) return;
    const int width = group_m * tiles_n;
    const int grp = lin / width;
    const int first_m = grp * group_m;
    const int gsz = min(tiles_m - first_m, group_m);
    const int pm = first_m + (lin % width) % gsz;
    const int pn = (lin % width) / gsz;
    // the projection this column tile belongs to (one, or several that share X and the plan)
    int si = 0;
    while (si + 1 < p.n_sets && pn >= p.set[si + 1].tile0) ++si;
    const GemmSet g = p.set[si];
    const int m0 = pm * BM, n0 = (pn - g.tile0) * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wn0 = (wave % WN) * WTN, wm0 = (wave / WN) * WTM;
    const int l31 = lane & 31, lh = lane >> 5;

    // this workgroup's stretch of the contraction axis
    int k0 = 0, Kloc = p.K;
    if constexpr (SPLIT) {
        k0 = (int)blockIdx.y * p.k_chunk;
        Kloc = min(p.K - k0, p.k_chunk);
    }
    const E *W = static_cast<const E *>(g.W) + k0;
    const E *V = static_cast<const E *>(g.V);

    // ---- per-thread load slots ------------------------------------------------------------
    const int lrow = tid >> 3, lc = tid & 7;
    // 32-bit byte offsets (row start + this thread's chunk of a stage) against a scalar base that moves along K:
    // a load then needs no vector address arithmetic at all, and one register of address.  X is
    // addressed from its start (the host checks that it is smaller than 4 GiB), W0 from the tile's first row.
    const BufferDesc Xd = make_buffer_desc(static_cast<const E *>(p.X) + k0);
    const BufferDesc Wd = make_buffer_desc(W + (int64_t)n0 * g.ldw);
    unsigned xoff[XL], woff[WL];
    int xrowi[XL];  // original row index of each load slot (V is stored in original row order)
#pragma unroll
    for (int i = 0; i < XL; ++i) {  // rows past T / N are clamped: they only feed outputs that are never stored
        xrowi[i] = p.plan.perm[min(m0 + lrow + i * RPP, p.T - 1)];
        xoff[i] = (unsigned)(((int64_t)xrowi[i] * p.ldx + lc * CE) * (int64_t)sizeof(E));
    }
#pragma unroll
    for (int i = 0; i < WL; ++i)
        woff[i] = (unsigned)(((int64_t)(min(n0 + lrow + i * RPP, g.N - 1) - n0) * g.ldw + lc * CE) * (int64_t)sizeof(E));

    // ---- extension range of this M-tile -----------------------------------------------------
    int pbeg = 0, pend = 0;
    if (g.B != nullptr) {
        const int s_first = p.plan.row_seg[m0];
        const int s_last = p.plan.row_seg[min(m0 + BM, p.T) - 1];
        pbeg = p.plan.seg_ext[s_first];
        pend = p.plan.seg_ext[s_last + 1];
    }
    const int ext_chunks = (pend - pbeg) / CE;
    // Which rows take their adapter term from D: those with an adapter -- of a short segment only, when the long
    // segments' term is computed here (long_rows > 0).  Read in the epilogue.
    if (g.D != nullptr) {
        for (int r = tid; r < BM; r += NT) {
            const int s = p.plan.row_seg[min(m0 + r, p.T - 1)];
            const bool lng = g.long_rows > 0 && p.plan.seg_indptr[s + 1] - p.plan.seg_indptr[s] >= g.long_rows;
            tab->use_d[r] = p.plan.seg_adapter[s] >= 0 && !lng;
        }
    }

    // One batch of the table: the chunk columns [chunk0, chunk0 + kTabCap) of the tile's extension axis, those in
    // use (a resident adapter; a long segment, when the short ones' term comes in D) packed to the front in axis
    // order -- a stage then holds 8 columns in use whatever the ranks in between add up to.  Returns their number.
    // Two phases around a barrier: count per wave, then place.
    auto build_table = [&](int chunk0) -> int {
        constexpr int IT = kTabCap / NT, WV = NT / 64;
        const void *e_ptr[IT];
        int e_r[IT], e_j[IT], e_lo[IT], e_hi[IT];
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            const int idx = it * NT + tid;
            const int pe = pbeg + (chunk0 + idx) * CE;
            e_ptr[it] = nullptr;
            e_r[it] = 0, e_j[it] = 0, e_lo[it] = INT_MAX, e_hi[it] = INT_MIN;
            bool wanted = pe < pend;
            int4 rec = make_int4(-1, 0, 0, 0);
            if (wanted) {
                rec = reinterpret_cast<const int4 *>(p.plan.ext_rec)[pe >> 3];
                wanted = rec.w - rec.z >= g.long_rows;  // (short segments' term comes in D when long_rows > 0)
            }
            if (wanted) {
                const E *b = rec.x >= 0 ? static_cast<const E *>(g.B[rec.x]) : nullptr;
                if (b != nullptr) {
                    e_r[it] = rec.y >> 16;
                    e_j[it] = (rec.y & 0xffff) + (pe & 7);
                    e_lo[it] = max(rec.z - m0, 0);
                    e_hi[it] = min(rec.w - m0, BM);
                    e_ptr[it] = b + e_j[it];
                } else {
                    atomicMin(&p.plan.scalars[kScEvicted], kErrNotResident);
                }
            }
            const unsigned long long used = __builtin_amdgcn_ballot_w64(e_ptr[it] != nullptr);
            if (lane == 0) tab->cnt[it * WV + wave] = __builtin_popcountll(used);
        }
        __syncthreads();
        int total = 0;
#pragma unroll
        for (int k = 0; k < IT * WV; ++k) total += tab->cnt[k];
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            int pos = 0;
#pragma unroll
            for (int k = 0; k < IT * WV; ++k) pos += k < it * WV + wave ? tab->cnt[k] : 0;
            const unsigned long long used = __builtin_amdgcn_ballot_w64(e_ptr[it] != nullptr);
            pos += __builtin_popcountll(used & ((1ull << lane) - 1ull));
            if (e_ptr[it] != nullptr) {
                tab->ptr[pos] = e_ptr[it];
                tab->r[pos] = e_r[it];
                tab->j[pos] = e_j[it];
                tab->lo[pos] = e_lo[it];
                tab->hi[pos] = e_hi[it];
            }
        }
        if (tid < 8 && total + tid < ((total + 7) & ~7)) {  // the unused columns of the last stage
            tab->ptr[total + tid] = nullptr;
            tab->r[total + tid] = 0;
            tab->j[total + tid] = 0;
            tab->lo[total + tid] = INT_MAX;
            tab->hi[total + tid] = INT_MIN;
        }
        return total;
    };
    int ext_used = 0;  // columns in use in the current batch of the table
    if (ext_chunks > 0) ext_used = build_table(0);  // visible after the first barrier of the base loop

    f32x16_t acc[NBN][NBT];
#pragma unroll
    for (int nb = 0; nb < NBN; ++nb)
#pragma unroll
        for (int tb = 0; tb < NBT; ++tb)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[nb][tb][e] = 0.f;

    chunk_t xr[XL], wr[WL];

    // Loads are branch-free so that all of a stage's loads are in flight together.  Full stages need
    // no mask at all; the last, partial stage of K loads chunk 0 instead and drops it.
    auto load_base = [&](int kt, bool partial) {
        if (!partial) {
#pragma unroll
            for (int i = 0; i < XL; ++i) xr[i] = buffer_load_chunk(Xd, xoff[i], kt * 128);
#pragma unroll
            for (int i = 0; i < WL; ++i) wr[i] = buffer_load_chunk(Wd, woff[i], kt * 128);
        } else {
            const bool kv = (kt * 8 + lc) * CE < Kloc;
            // dropped loads read the start of the row (all of it in the per-lane offset: the scalar one must be uniform)
            const unsigned adj = kv ? (unsigned)kt * 128u : 0u - (unsigned)lc * 16u;
#pragma unroll
            for (int i = 0; i < XL; ++i) xr[i] = keep_if(kv, buffer_load_chunk(Xd, xoff[i] + adj, 0));
#pragma unroll
            for (int i = 0; i < WL; ++i) wr[i] = keep_if(kv, buffer_load_chunk(Wd, woff[i] + adj, 0));
        }
    };
    // Extension loads are requested unmasked (from a clamped address where a row or chunk column does not
    // take part); the mask is applied when the stage is written to LDS.  Masking the loaded value at once would
    // make every load wait for its own data right behind its issue: no two loads in flight.
    auto load_ext = [&](int se) {  // se = stage inside the current table batch
        const int idx = se * 8 + lc;
        const E *bp = static_cast<const E *>(tab->ptr[idx]);
        const int r = tab->r[idx], j = tab->j[idx], lo = tab->lo[idx], hi = tab->hi[idx];
#pragma unroll
        for (int i = 0; i < XL; ++i) {
            const int row = lrow + i * RPP;
            const bool ok = row >= lo && row < hi;  // rows of other adapters contribute nothing
            xr[i] = load_chunk(V + (ok ? (int64_t)xrowi[i] * p.r_max + j : 0));
        }
        const bool wok = bp != nullptr;
        const E *bsrc = wok ? bp : W;  // W: some in-bounds address for the dropped loads
#pragma unroll
        for (int i = 0; i < WL; ++i) {
            const int n = min(n0 + lrow + i * RPP, g.N - 1);
            wr[i] = load_chunk(bsrc + (wok ? (int64_t)n * r : 0));
        }
    };
    auto store_stage_ext = [&](int buf, int se) {
        const int idx = se * 8 + lc;
        const bool wok = tab->ptr[idx] != nullptr;
        const int lo = tab->lo[idx], hi = tab->hi[idx];
#pragma unroll
        for (int i = 0; i < XL; ++i) {
            const int row = lrow + i * RPP;
            sX[buf * BM * 8 + swz(row, lc)] = keep_if(row >= lo && row < hi, xr[i]);
        }
#pragma unroll
        for (int i = 0; i < WL; ++i) sW[buf * BN * 8 + swz(lrow + i * RPP, lc)] = keep_if(wok, wr[i]);
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < XL; ++i) sX[buf * BM * 8 + swz(lrow + i * RPP, lc)] = xr[i];
#pragma unroll
        for (int i = 0; i < WL; ++i) sW[buf * BN * 8 + swz(lrow + i * RPP, lc)] = wr[i];
    };
    auto compute = [&](int buf, int se) {  // se < 0: base stage (no skipping)
        const chunk_t *bw = sW + buf * BN * 8;
        const chunk_t *bx = sX + buf * BM * 8;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            int lo = 0, hi = BM;
            if (se >= 0) {
                const int i0 = se * 8 + 2 * kk;
                lo = min(tab->lo[i0], tab->lo[i0 + 1]);
                hi = max(tab->hi[i0], tab->hi[i0 + 1]);
                if (hi <= lo) continue;
            }
            const int cc = 2 * kk + lh;
            chunk_t wf[NBN], xf[NBT];
#pragma unroll
            for (int nb = 0; nb < NBN; ++nb) wf[nb] = bw[swz(wn0 + nb * 32 + l31, cc)];
#pragma unroll
            for (int tb = 0; tb < NBT; ++tb) {
                const int t0 = wm0 + tb * 32;
                if (se < 0 || (lo < t0 + 32 && hi > t0)) {
                    xf[tb] = bx[swz(t0 + l31, cc)];
#pragma unroll
                    for (int nb = 0; nb < NBN; ++nb) Elem<E>::mma32(acc[nb][tb], wf[nb], xf[tb]);
                }
            }
        }
    };

    // ---- base product: sum over K ---------------------------------------------------------------
    // One barrier per stage, and the matrix cores have work queued on both sides of it: operands are
    // read from LDS one use ahead, in place -- a W operand is requested for the next k-step as soon
    // as its two MFMAs of this one are issued, the two X operands alternate between two register
    // sets.  The last k-step of a stage is split: half of its MFMAs go out before the stage's stores
    // and barrier, the other half after the barrier, behind the first operand reads of the next
    // stage, whose latency they cover.
    const int KT = (Kloc + 8 * CE - 1) / (8 * CE);
    const int KT_full = Kloc / (8 * CE);  // stages that lie entirely inside K
    auto read_w = [&](int buf, int kk, int nb) { return sW[buf * BN * 8 + swz(wn0 + nb * 32 + l31, 2 * kk + lh)]; };
    auto read_x = [&](int buf, int kk, int tb) { return sX[buf * BM * 8 + swz(wm0 + tb * 32 + l31, 2 * kk + lh)]; };
    load_base(0, KT_full < 1);
    store_stage(0);
    if (KT > 1) load_base(1, 1 >= KT_full);
    __syncthreads();
    chunk_t wf[NBN], xf[2][NBT];
#pragma unroll
    for (int tb = 0; tb < NBT; ++tb) xf[0][tb] = read_x(0, 0, tb);
#pragma unroll
    for (int nb = 0; nb < NBN; ++nb) wf[nb] = read_w(0, 0, nb);
    bool ext_loaded = false;
    // (stage 1 was requested by every wave before the loop)
    int kt = 0;
    {
        // Two register sets of staged operands: while stage kt is multiplied, the loads of stage kt + 2 go out
        // into one set and the other set, which holds stage kt + 1, is written to the LDS buffer that stage
        // kt - 1 was read from -- a third of each in each of the first three k-steps, so neither the address unit
        // nor LDS sees a burst and a load has a whole stage to arrive (loads or stores bunched into one or two
        // k-steps, for more time between a load and its store, cost 4 to 17 %).  The barrier waits for LDS traffic
        // only, never for the loads in flight across it.
        chunk_t xr2[XL], wr2[WL];
        // the XL + WL load slots of a stage (X slots first), dealt to the first three k-steps as evenly as they divide: the
        // last LDS store of a stage then has the first half of the fourth k-step's MFMAs behind it, and the wait for
        // LDS in front of the stage's barrier finds it done
        constexpr int NS = XL + WL;
        constexpr auto gk = [](int s_) { return s_ * 3 / NS; };  // k-step in which slot s_ is loaded (stage kt + 2) ...
        constexpr auto wk = [](int s_) { return s_ * 3 / NS; };  // ... and stored to LDS (stage kt + 1): exactly one stage later
        auto gload_q = [&](chunk_t (&xs)[XL], chunk_t (&ws)[WL], int kq, int q, bool partial) {
            const bool kv = !partial || (kq * 8 + lc) * CE < Kloc;
            // (partial stage: all of the offset per lane -- the scalar one must be uniform; dropped loads read the row start)
            const unsigned adj = !partial ? 0u : (kv ? (unsigned)kq * 128u : 0u - (unsigned)lc * 16u);
            const int soff = partial ? 0 : kq * 128;
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                if (gk(s) != q) continue;
                if (s < XL) {
                    xs[s < XL ? s : 0] = buffer_load_chunk(Xd, xoff[s < XL ? s : 0] + adj, soff);
                    if (partial) xs[s < XL ? s : 0] = keep_if(kv, xs[s < XL ? s : 0]);
                } else {
                    ws[s >= XL ? s - XL : 0] = buffer_load_chunk(Wd, woff[s >= XL ? s - XL : 0] + adj, soff);
                    if (partial) ws[s >= XL ? s - XL : 0] = keep_if(kv, ws[s >= XL ? s - XL : 0]);
                }
            }
        };
        auto lstore_q = [&](const chunk_t (&xs)[XL], const chunk_t (&ws)[WL], int buf, int q) {
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                if (wk(s) != q) continue;
                if (s < XL)
                    sX[buf * BM * 8 + swz(lrow + s * RPP, lc)] = xs[s < XL ? s : 0];
                else
                    sW[buf * BN * 8 + swz(lrow + (s - XL) * RPP, lc)] = ws[s >= XL ? s - XL : 0];
            }
        };
        auto lds_barrier = [&]() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };
        // Issue order inside a scheduling region: a wave issues in order, and an MFMA occupies the matrix core for 32
        // cycles during which the wave can issue its other instructions for nothing -- but only if they sit BETWEEN the
        // MFMAs in program order.  Left to itself the compiler emits the region's LDS reads, loads and LDS stores in
        // runs of 4 to 12 in front of runs of MFMAs.  Here: every MFMA followed by its share of the region's nr LDS
        // reads, then of its ngw (load, LDS store) pairs.
        auto interleave = [](auto nm_c, auto nr_c, auto ng_c, auto nw_c) __attribute__((always_inline)) {
            constexpr int nm = decltype(nm_c)::value, nr = decltype(nr_c)::value, ng = decltype(ng_c)::value, nw = decltype(nw_c)::value;
            constexpr int others = nr + ng + nw, dm = nm > 0 ? nm : 1, pairs = ng < nw ? ng : nw;
#pragma unroll
            for (int i = 0; i < nm; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
#pragma unroll
                for (int j = i * others / dm; j < (i + 1) * others / dm; ++j) {
                    // the region's reads first, then (load, store) pairs, then whichever of the two kinds is left over
                    const int k = j - nr;
                    const bool is_read = j < nr;
                    const bool is_load = !is_read && (k < 2 * pairs ? (k & 1) == 0 : ng > nw);
                    if (is_read)
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // one LDS read
                    else if (is_load)
                        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // one global load
                    else
                        __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);  // one LDS store
                }
            }
        };
        constexpr auto count_k = [](auto f, int q) {
            int n = 0;
            for (int s_ = 0; s_ < NS; ++s_) n += f(s_) == q;
            return n;
        };
        using std::integral_constant;
        // stage kt: set (lx, lw) receives stage kt + 2, set (sx, sw) holds stage kt + 1
        auto stage_deep = [&](int kq, chunk_t (&lx)[XL], chunk_t (&lw)[WL], chunk_t (&sx)[XL], chunk_t (&sw)[WL], bool more,
                              bool load2, bool partial2) {
            const int buf = kq & 1;
#pragma unroll
            for (int kk = 0; kk < 3; ++kk) {
                const int cur = kk & 1;
#pragma unroll
                for (int tb = 0; tb < NBT; ++tb) xf[cur ^ 1][tb] = read_x(buf, kk + 1, tb);
#pragma unroll
                for (int nb = 0; nb < NBN; ++nb) {
#pragma unroll
                    for (int tb = 0; tb < NBT; ++tb) Elem<E>::mma32(acc[nb][tb], wf[nb], xf[cur][tb]);
                    wf[nb] = read_w(buf, kk + 1, nb);
                }
                if (load2) gload_q(lx, lw, kq + 2, kk, partial2);
                if (more) lstore_q(sx, sw, buf ^ 1, kk);
                if (kk == 0)
                    interleave(integral_constant<int, NBN * NBT>{}, integral_constant<int, NBN + NBT>{}, integral_constant<int, count_k(gk, 0)>{}, integral_constant<int, count_k(wk, 0)>{});
                else if (kk == 1)
                    interleave(integral_constant<int, NBN * NBT>{}, integral_constant<int, NBN + NBT>{}, integral_constant<int, count_k(gk, 1)>{}, integral_constant<int, count_k(wk, 1)>{});
                else
                    interleave(integral_constant<int, NBN * NBT>{}, integral_constant<int, NBN + NBT>{}, integral_constant<int, count_k(gk, 2)>{}, integral_constant<int, count_k(wk, 2)>{});
                __builtin_amdgcn_sched_barrier(0);  // nothing moves between k-steps: register lifetimes stay as written
            }
            constexpr int H = NBN > 1 ? NBN / 2 : 1;
#pragma unroll
            for (int nb = 0; nb < H; ++nb)
#pragma unroll
                for (int tb = 0; tb < NBT; ++tb) Elem<E>::mma32(acc[nb][tb], wf[nb], xf[1][tb]);
            __builtin_amdgcn_sched_barrier(0);
            lds_barrier();
            __builtin_amdgcn_sched_barrier(0);
            if (more) {
#pragma unroll
                for (int tb = 0; tb < NBT; ++tb) xf[0][tb] = read_x(buf ^ 1, 0, tb);
#pragma unroll
                for (int nb = 0; nb < H; ++nb) wf[nb] = read_w(buf ^ 1, 0, nb);
            }
#pragma unroll
            for (int nb = H; nb < NBN; ++nb) {
#pragma unroll
                for (int tb = 0; tb < NBT; ++tb) Elem<E>::mma32(acc[nb][tb], wf[nb], xf[1][tb]);
                if (more) wf[nb] = read_w(buf ^ 1, 0, nb);
            }
            interleave(integral_constant<int, (NBN - H) * NBT>{}, integral_constant<int, NBN + NBT>{}, integral_constant<int, 0>{}, integral_constant<int, 0>{});
            __builtin_amdgcn_sched_barrier(0);
        };
        for (; kt + 3 < KT_full; kt += 2) {  // the steady state, two stages per trip: the sets swap roles
            stage_deep(kt, xr2, wr2, xr, wr, true, true, false);  // (stage 1 came into the first set before the loop)
            stage_deep(kt + 1, xr, wr, xr2, wr2, true, true, false);
        }
        // The last stage loads and stores nothing, so both register sets are free: the first extension stage in
        // use is requested in front of it and arrives while it is multiplied.
        // (not beside a 256x256 tile on 4 waves: the registers that keeps alive through the last stage are spilled)
        constexpr bool PREFETCH_EXT = XL + WL < 16;
        auto prefetch_ext = [&]() __attribute__((always_inline)) {
            if constexpr (PREFETCH_EXT) {
                ext_loaded = ext_used > 0;
                if (ext_loaded) load_ext(0);
            }
        };
        for (; kt < KT; kt += 2) {
            if (kt + 1 == KT) prefetch_ext();
            stage_deep(kt, xr2, wr2, xr, wr, kt + 1 < KT, kt + 2 < KT, kt + 2 >= KT_full);
            if (kt + 1 < KT) {
                if (kt + 2 == KT) prefetch_ext();
                stage_deep(kt + 1, xr, wr, xr2, wr2, kt + 2 < KT, kt + 3 < KT, kt + 3 >= KT_full);
            }
        }
    }
    __syncthreads();  // (NBN == 1: the second half above is empty and reads of the last buffer end after its barrier)

    // ---- extension: sum over the concatenated ranks of this tile's adapters -----------------------
    for (int chunk0 = 0; chunk0 < ext_chunks; chunk0 += kTabCap) {
        if (chunk0 > 0) {
            ext_used = build_table(chunk0);
            __syncthreads();
        }
        const int nst = (ext_used + 7) >> 3;
        if (nst > 0) {
            if (!(chunk0 == 0 && ext_loaded)) load_ext(0);
            store_stage_ext(0, 0);
            __syncthreads();
        }
        for (int se = 0; se < nst; ++se) {
            const bool more = se + 1 < nst;
            if (more) load_ext(se + 1);
            compute(se & 1, se);
            if (more) store_stage_ext((se + 1) & 1, se + 1);
            __syncthreads();
        }
    }

    // ---- single store of Y: acc[nb][tb][g*4+e] = D[n = nb*32 + g*8 + lh*4 + e][t = tb*32 + l31] -------
    if constexpr (SPLIT) {  // the partial tile, in fp32, to this split's copy of the output
        float *P = p.P + (int64_t)blockIdx.y * p.T * p.ldp;
#pragma unroll
        for (int tb = 0; tb < NBT; ++tb) {
            const int t = m0 + wm0 + tb * 32 + l31;
            float *prow = P + (int64_t)p.plan.perm[min(t, p.T - 1)] * p.ldp;
#pragma unroll
            for (int nb = 0; nb < NBN; ++nb) store_acc_tile<float>(acc[nb][tb], prow, nullptr, n0 + wn0 + nb * 32, lh, g.N, t < p.T);
        }
        return;
    }
    E *Y = static_cast<E *>(g.Y);
    if (g.D == nullptr) {
#pragma unroll
        for (int tb = 0; tb < NBT; ++tb) {
            const int t = m0 + wm0 + tb * 32 + l31;
            E *yrow = Y + (int64_t)p.plan.perm[min(t, p.T - 1)] * g.ldy;
#pragma unroll
            for (int nb = 0; nb < NBN; ++nb) store_acc_tile<E>(acc[nb][tb], yrow, nullptr, n0 + wn0 + nb * 32, lh, g.N, t < p.T);
        }
    } else {
        // The adapter term, when a kernel of its own has computed it (rows with an adapter only), is read one
        // row block ahead of the stores it is added into: written inside the store loop, every piece of it
        // would be a round trip to memory of its own (the compiler does not move a load above a store).
        float term[2][NBN][16];
        auto row_of = [&](int tb) { return p.plan.perm[min(m0 + wm0 + tb * 32 + l31, p.T - 1)]; };
        auto fetch = [&](int tb, int row, float (&d)[NBN][16]) {
            const float *drow = tab->use_d[wm0 + tb * 32 + l31] ? g.D + (int64_t)row * g.ldd : nullptr;
#pragma unroll
            for (int nb = 0; nb < NBN; ++nb) load_term_tile(drow, g.D, n0 + wn0 + nb * 32, lh, (int)g.ldd, d[nb]);
        };
        int row = row_of(0);
        fetch(0, row, term[0]);
#pragma unroll
        for (int tb = 0; tb < NBT; ++tb) {
            const int t = m0 + wm0 + tb * 32 + l31;
            E *yrow = Y + (int64_t)row * g.ldy;
            if (tb + 1 < NBT) {
                row = row_of(tb + 1);
                fetch(tb + 1, row, term[(tb + 1) & 1]);
            }
#pragma unroll
            for (int nb = 0; nb < NBN; ++nb)
                store_acc_tile_with<E>(acc[nb][tb], term[tb & 1][nb], yrow, n0 + wn0 + nb * 32, lh, g.N, t < p.T);
        }
    }
}

template <typename E, int BM, int BN, int WM, int WN, bool CAN_SPLIT = false>
hipError_t launch_tile(const GemmArgs &a0, hipStream_t stream, const KernelTimer *timer) {
    GemmArgs a = a0;
    if (a.n_sets == 0) {  // a single projection, described by the plain fields
        a.n_sets = 1;
        a.set[0] = GemmSet{a.W, a.ldw, a.Y, a.ldy, a.V, a.B, a.D, a.ldd, a.long_rows, a.N, 0, 0};
    }
    const int tiles_m = (a.T + BM - 1) / BM;
    int tiles_n = 0;
    for (int i = 0; i < a.n_sets; ++i) {
        a.set[i].tile0 = tiles_n;
        tiles_n += (a.set[i].N + BN - 1) / BN;
    }
    const long total = (long)tiles_m * tiles_n;
    if (total <= 0) return hipSuccess;
    const size_t smem = (size_t)(BM + BN) * 8 * 16 * 2 + sizeof(ExtTable);
    const long grid = ((total + 7) / 8) * 8;
    const int group_m = 8;
    if (a.split_k > 1) {
        if constexpr (CAN_SPLIT) {
            constexpr int stage = 8 * Elem<E>::CE;
            if (a.n_sets != 1 || a.set[0].B != nullptr || a.set[0].D != nullptr || a.P == nullptr || a.k_chunk <= 0 ||
                a.k_chunk % stage != 0 || (long)a.k_chunk * (a.split_k - 1) >= a.K || (long)a.k_chunk * a.split_k < a.K ||
                a.ldp < a.set[0].N || (a.ldp & 7) != 0)
                return hipErrorInvalidValue;
            return launch_kernel(gemm_tile_kernel<E, BM, BN, WM, WN, true>, dim3((unsigned)grid, (unsigned)a.split_k), dim3(WM * WN * 64),
                                 smem, stream, timer, a, tiles_m, tiles_n, group_m);
        } else {
            return hipErrorInvalidValue;
        }
    }
    return launch_kernel(gemm_tile_kernel<E, BM, BN, WM, WN, false>, dim3((unsigned)grid), dim3(WM * WN * 64), smem, stream, timer, a,
                         tiles_m, tiles_n, group_m);
}

// Dynamic LDS above the default 64 KB has to be granted per kernel and device before the first launch.
template <typename E, int BM, int BN, int WM, int WN, bool CAN_SPLIT = false>
hipError_t init_tile() {
    const size_t smem = (size_t)(BM + BN) * 8 * 16 * 2 + sizeof(ExtTable);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(gemm_tile_kernel<E, BM, BN, WM, WN, false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if constexpr (CAN_SPLIT) {
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(gemm_tile_kernel<E, BM, BN, WM, WN, true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    }
    return e;
}
template <typename E>
hipError_t init_tiles() {
    hipError_t e = init_tile<E, 64, 64, 2, 2>();
    if (e == hipSuccess) e = init_tile<E, 128, 128, 2, 2, true>();
    if (e == hipSuccess) e = init_tile<E, 256, 128, 2, 2>();
    if (e == hipSuccess) e = init_tile<E, 256, 256, 2, 2, true>();
    if (e == hipSuccess) e = init_tile<E, 128, 192, 2, 2>();
    if (e == hipSuccess) e = init_tile<E, 256, 192, 2, 2>();
    if (e == hipSuccess) e = init_tile<E, 256, 224, 4, 1>();
    return e;
}

template <typename E>
hipError_t launch_variant(const GemmArgs &a, int variant, hipStream_t stream, const KernelTimer *timer) {
    switch (variant) {
        case kGemmTile64x64:
            return launch_tile<E, 64, 64, 2, 2>(a, stream, timer);
        case kGemmTile128x128:
            return launch_tile<E, 128, 128, 2, 2, true>(a, stream, timer);
        case kGemmTile256x128:
            return launch_tile<E, 256, 128, 2, 2>(a, stream, timer);
        case kGemmTile256x256w4:
            return launch_tile<E, 256, 256, 2, 2, true>(a, stream, timer);
        case kGemmTile128x192:
            return launch_tile<E, 128, 192, 2, 2>(a, stream, timer);
        case kGemmTile256x192:
            return launch_tile<E, 256, 192, 2, 2>(a, stream, timer);
        case kGemmTile256x224:
            return launch_tile<E, 256, 224, 4, 1>(a, stream, timer);
        default:
            return hipErrorInvalidValue;
    }
}

// The second launch of a GEMM split along K: one thread = 8 consecutive columns of one row; the splits' partials are
// requested together and summed in split order, the adapter term of rows with an adapter is added, Y is rounded once.
template <typename E>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(SplitReduceArgs p) {
    if (p.plan.scalars[kScStatus] != 0) return;
    const int n8 = (p.N + 7) >> 3;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long)p.T * n8) return;
    const int row = (int)(idx / n8), n = (int)(idx % n8) * 8;
    const bool has = p.D != nullptr && p.plan.row_adapter[row] >= 0 && row_ext_rank(p.plan.row_ext[row]) > 0;
    constexpr int kMaxSplit = 8;
    chunk_t q[kMaxSplit][2];
    const float *src = p.P + (int64_t)row * p.ldp + n;  // (rows are ldp >= N rounded up to 8 floats long: whole pieces are readable)
#pragma unroll
    for (int s = 0; s < kMaxSplit; ++s) {
        const float *ps = src + (int64_t)min(s, p.split_k - 1) * p.T * p.ldp;
        q[s][0] = load_chunk(ps);
        q[s][1] = load_chunk(ps + 4);
    }
    const float *dsrc = has ? p.D + (int64_t)row * p.ldd + n : src;
    const chunk_t d0 = load_chunk(dsrc), d1 = load_chunk(dsrc + 4);
    float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < kMaxSplit; ++s) {
        if (s < p.split_k) {
            v[0] += __uint_as_float(q[s][0].x);
            v[1] += __uint_as_float(q[s][0].y);
            v[2] += __uint_as_float(q[s][0].z);
            v[3] += __uint_as_float(q[s][0].w);
            v[4] += __uint_as_float(q[s][1].x);
            v[5] += __uint_as_float(q[s][1].y);
            v[6] += __uint_as_float(q[s][1].z);
            v[7] += __uint_as_float(q[s][1].w);
        }
    }
    if (has) {
        v[0] += __uint_as_float(d0.x);
        v[1] += __uint_as_float(d0.y);
        v[2] += __uint_as_float(d0.z);
        v[3] += __uint_as_float(d0.w);
        v[4] += __uint_as_float(d1.x);
        v[5] += __uint_as_float(d1.y);
        v[6] += __uint_as_float(d1.z);
        v[7] += __uint_as_float(d1.w);
    }
    E *y = static_cast<E *>(p.Y) + (int64_t)row * p.ldy + n;
    if (n + 7 < p.N) {
        store8(y, v);
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (n + e < p.N) store1(y + e, v[e]);
    }
}

}  // namespace

hipError_t init_gemm_tile_kernels() {
    hipError_t e = init_tiles<__bf16>();
    if (e == hipSuccess) e = init_tiles<float>();
    return e;
}

hipError_t launch_gemm_tile(const GemmArgs &a, int dtype, int variant, hipStream_t stream, const KernelTimer *timer) {
    return dtype == 1 ? launch_variant<__bf16>(a, variant, stream, timer) : launch_variant<float>(a, variant, stream, timer);
}

hipError_t launch_splitk_reduce(const SplitReduceArgs &a, int dtype, hipStream_t stream, const KernelTimer *timer) {
    if (a.T <= 0 || a.N <= 0) return hipSuccess;
    if (a.split_k < 1 || a.split_k > 8 || a.P == nullptr || a.Y == nullptr || a.ldp < a.N || (a.ldp & 7) != 0 ||
        (a.D != nullptr && (a.ldd < a.N || (a.ldd & 7) != 0)))
        return hipErrorInvalidValue;
    const long threads = (long)a.T * ((a.N + 7) / 8);
    const dim3 grid((unsigned)((threads + 255) / 256));
    if (dtype == 1) return launch_kernel(splitk_reduce_kernel<__bf16>, grid, dim3(256), 0, stream, timer, a);
    return launch_kernel(splitk_reduce_kernel<float>, grid, dim3(256), 0, stream, timer, a);
}

}  // namespace lora
