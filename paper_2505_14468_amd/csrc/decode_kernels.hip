// Decode-sized batches (T <= 128 rows, bf16): the layer is a weight-streaming problem, bound by reading W0 and
// the used A_a, B_a from HBM once.  Two launches, no workgroup waits for another:
//
//   1. decode_stream_kernel: the contraction axis is cut into slices of 512 and the rows of the "weight" matrix
//      -- W0's N rows followed by the rows of the used A_a (the plan's concatenated rank axis) -- into blocks of
//      16.  A wave multiplies one 16-row block by the whole batch over one slice; a workgroup holds 8..12 waves
//      on consecutive blocks of one slice and stages that slice of X in LDS once.  fp32 partial tiles go to the
//      workspace.  So a CU ingests ~150 KB of weights and 64 KB of X instead of all of X for 16 columns, and the
//      shrink (V = X A_a: paper section 4.4's adapter product, first half) costs no launch of its own: A_a's
//      rows are just more weight rows.
//   2. decode_reduce_kernel: one workgroup per 16 output columns sums the slices' partial tiles in slice order
//      (fixed order: reproducible), gathers every row's V from the partial tiles of its adapter's rank block,
//      scales it by s_a, adds V B_a in fp32 (V is never rounded here) and stores Y once.
//   With much adapter work (many high-rank adapters in the batch) two launches go in between: decode_v_kernel
//   reduces V once (rounded to bf16 like the shrink kernel's V), the expand kernel turns it into the fp32 adapter
//   term segment by segment, and decode_reduce_kernel only adds that term.
//
// Same contraction as the tiled path:  Y[t, n] = sum_k X[t, k] W0[n, k] + s_a sum_j (sum_k X[t, k] A_a[j, k]) B_a[n, j].
//
// Loads: weight rows are requested 8 rows x 128 bytes per instruction (whole cache lines) and turned into MFMA
// operand layout through a 2 KB wave-private, XOR-swizzled LDS buffer; a wave requests all 16 KB of its block
// before it consumes any, right behind its share of the X slice (X comes from L2 and returns first: loads
// return in order).  MFMA 16x16x32: M = 16 weight rows, N = 16 token rows.
#include "kernels.h"

namespace lora {
namespace {

constexpr int kDsSliceChunks = 64;  // 16-byte chunks of the contraction axis per slice (512 bf16)

// Entry `idx` (< 64) of a table of which lane i holds entry i: the tables of adapter pointers and scales are read one
// entry per lane in the same round trip as the index into them, which saves the dependent trip for pools of up to 64
// adapters (larger indices take it).
__device__ __forceinline__ const void *lane_entry(const void *mine, int idx) {
    const unsigned long long v = reinterpret_cast<unsigned long long>(mine);
    const unsigned lo = (unsigned)__builtin_amdgcn_ds_bpermute(idx << 2, (int)(unsigned)v);
    const unsigned hi = (unsigned)__builtin_amdgcn_ds_bpermute(idx << 2, (int)(unsigned)(v >> 32));
    return reinterpret_cast<const void *>(((unsigned long long)hi << 32) | lo);
}
__device__ __forceinline__ float lane_entry(float mine, int idx) {
    return __int_as_float(__builtin_amdgcn_ds_bpermute(idx << 2, __float_as_int(mine)));
}

__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// The projection a block of weight rows (streaming kernel) or a column block (reduction) belongs to, and the index
// inside it: the launch's fields are overwritten with that projection's.
__device__ __forceinline__ void select_set(DecodeArgs &p, const DecodeArgs &p0, int &idx, bool by_column) {
    if (p0.n_sets <= 0) return;
    int si = 0;
    while (si + 1 < p0.n_sets && idx >= (by_column ? p0.set[si + 1].cb0 : p0.set[si + 1].blk0)) ++si;
    idx -= by_column ? p0.set[si].cb0 : p0.set[si].blk0;
    p.W = p0.set[si].W;
    p.ldw = p0.set[si].ldw;
    p.A = p0.set[si].A;
    p.B = p0.set[si].B;
    p.scale = p0.set[si].scale;
    p.Y = p0.set[si].Y;
    p.ldy = p0.set[si].ldy;
    p.P = p0.set[si].P;
    p.N = p0.set[si].N;
    p.nbw = p0.set[si].nbw;
    p.n_adapters = p0.set[si].n_adapters;
}

template <int TBLK, int MAXW>
__global__ __launch_bounds__(MAXW * 64) void decode_stream_kernel(DecodeArgs p0) {
    typedef __bf16 E;
    constexpr int CE = 8;
    constexpr int XROWS = TBLK * 16;
    constexpr int XIT = TBLK * 2;  // chunk loads per thread that cover the X slice with at least 512 threads

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    chunk_t *xs = reinterpret_cast<chunk_t *>(smem);  // [XROWS][64], chunk c of row t at t * 64 + (c ^ (t & 15))
    chunk_t *wstage = xs + XROWS * kDsSliceChunks;     // [waves][128]

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nthreads = blockDim.x, nw = nthreads >> 6;
    const int li = lane & 15, lg = lane >> 4;
    const int slice = blockIdx.x % p0.ks, grp = blockIdx.x / p0.ks;
    int blk = grp * nw + wave;
    DecodeArgs p = p0;
    select_set(p, p0, blk, false);  // (a workgroup's waves may belong to two projections: the X slice is the same)
    // (the plan's status is wanted only before anything is stored: nothing requested until then depends on a valid
    // plan -- a failed build leaves an extension axis of length 0 -- so its round trip is not waited for here)
    const int status = p.plan.scalars[kScStatus];
    LORA_TS(p.trace, 0);

    const int kchunks = p.K / CE;
    const int kc0 = slice * kDsSliceChunks;
    const int nstages = (min(kDsSliceChunks, kchunks - kc0) + 7) >> 3;

    // ---- this wave's block of 16 weight rows: extension blocks (rows of the used A_a) first, then W0's ----
    const int nrec = p.A != nullptr ? p.plan.scalars[kScExtTotal] >> 3 : 0;  // records of 8 ranks
    const bool is_ext = blk < p.nbe_cap;
    const bool valid = is_ext ? blk * 2 < nrec : blk - p.nbe_cap < p.nbw;
    const int wr = lane >> 3, wc = lane & 7;  // load slot: row wr + 8 i of the block, chunk wc of a 128-byte stage
    int4 rec[2] = {make_int4(-1, 0, 0, 0), make_int4(-1, 0, 0, 0)};
    const void *a_guess = nullptr;  // entry `lane` of the table of A pointers, read in the records' round trip
    if (is_ext) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
            if (blk * 2 + i < nrec) rec[i] = reinterpret_cast<const int4 *>(p.plan.ext_rec)[blk * 2 + i];
        if (lane < p.n_adapters) a_guess = p.A[lane];
    }

    // ---- the X slice: requested first (L2), all threads, whole rows per wave instruction ----
    chunk_t xv[XIT];
#pragma unroll
    for (int it = 0; it < XIT; ++it) {
        const int idx = tid + it * nthreads;
        const int row = min(idx >> 6, p.T - 1), c = min(kc0 + (idx & 63), kchunks - 1);
        xv[it] = load_chunk(static_cast<const E *>(p.X) + (int64_t)row * p.ldx + c * CE);
    }

    // Every wave's share of X is requested before any wave's weights: a CU serves its requests in order, and an X
    // request queued behind other waves' HBM-bound weight requests would hold the whole workgroup at the barrier
    // below for their latency (measured: 4.5 us instead of ~1).
    __builtin_amdgcn_s_barrier();

    const char *rowp[2];
    bool rowok[2];
    if (is_ext) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int a = rec[i].x, j = rec[i].y & 0xffff;
            const void *ap = lane_entry(a_guess, a & 63);  // (every lane takes part in the exchange)
            if (a >= 64) ap = p.A[a];
            if (a < 0) ap = nullptr;
            if (a >= 0 && ap == nullptr) atomicMin(&p.plan.scalars[kScEvicted], kErrNotResident);  // slot emptied after the plan
            rowok[i] = ap != nullptr;
            rowp[i] = rowok[i] ? static_cast<const char *>(ap) + (int64_t)(j + wr) * p.K * (int64_t)sizeof(E)
                               : static_cast<const char *>(p.W);  // (some in-bounds address for the dropped loads)
        }
    } else {
#pragma unroll
        for (int i = 0; i < 2; ++i) {  // rows past N are clamped: they only feed partial sums that are never read
            const int n = min(max(blk - p.nbe_cap, 0) * 16 + wr + 8 * i, p.N - 1);
            rowok[i] = true;
            rowp[i] = static_cast<const char *>(p.W) + (int64_t)n * p.ldw * (int64_t)sizeof(E);
        }
    }
    // The block's 16 KB, eight stages of 2 KB (chunks past K are clamped: X holds zeros there).  A CU keeps a bounded
    // number of requests in flight, so requesting all eight at once only holds the wave at its load instructions
    // until most of the data is back; four go out ahead of the X slice's trip through LDS, one behind it, the rest one per stage consumed.
    chunk_t wq[8][2];
    auto load_w = [&](int s) {
        const unsigned coff = (unsigned)min(kc0 + s * 8 + wc, kchunks - 1) * 16u;
#pragma unroll
        for (int i = 0; i < 2; ++i) wq[s][i] = load_chunk(rowp[i] + coff);
    };
#pragma unroll
    for (int s = 0; s < 4; ++s) load_w(s);

    LORA_TS(p.trace, 1);  // X and the first half of the weights requested
    // ---- X slice to LDS (zeros past T and K) ----
#pragma unroll
    for (int it = 0; it < XIT; ++it) {
        const int idx = tid + it * nthreads;
        const int row = idx >> 6, c = idx & 63;
        if (idx < XROWS * kDsSliceChunks) xs[row * kDsSliceChunks + (c ^ (row & 15))] = keep_if(row < p.T && kc0 + c < kchunks, xv[it]);
    }
    lds_barrier();  // (LDS traffic only: the weight loads stay in flight across it)
    LORA_TS(p.trace, 2);  // X slice staged
    if (!valid || status != 0) return;
    load_w(4);

    f32x4_t acc[TBLK];
#pragma unroll
    for (int tb = 0; tb < TBLK; ++tb) acc[tb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    chunk_t *buf = wstage + wave * 128;
    int wdst[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int row = wr + 8 * i;
        wdst[i] = row * 8 + (wc ^ ((row >> 1) & 7));
    }
    const int rsrc = li * 8, rswz = (li >> 1) & 7;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        if (s + 5 < 8) load_w(s + 5);
        if (s < nstages) {
            // lanes exchange data through the wave's own buffer: LDS operations of one wave execute in order, the
            // fences only keep the compiler from reordering across the exchange
            buf[wdst[0]] = keep_if(rowok[0], wq[s][0]);
            buf[wdst[1]] = keep_if(rowok[1], wq[s][1]);
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const chunk_t w = buf[rsrc + ((h * 4 + lg) ^ rswz)];
#pragma unroll
                for (int tb = 0; tb < TBLK; ++tb) {
                    const chunk_t x = xs[(tb * 16 + li) * kDsSliceChunks + ((s * 8 + h * 4 + lg) ^ li)];
                    Elem<E>::mma16(acc[tb], w, x);
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        }
    }
    LORA_TS(p.trace, 3);  // stages consumed (MFMAs may still run)
    // acc[tb][e] = D[weight row blk * 16 + lg * 4 + e][token tb * 16 + li]: one contiguous KiB per 16-row token block
    float4 *P4 = reinterpret_cast<float4 *>(p.P) + ((int64_t)(blk * p.ks + slice) * TBLK) * 64 + lane;
#pragma unroll
    for (int tb = 0; tb < TBLK; ++tb) P4[tb * 64] = make_float4(acc[tb][0], acc[tb][1], acc[tb][2], acc[tb][3]);
    LORA_TS(p.trace, 4);
}

__device__ __forceinline__ float bf16_lo(unsigned v) { return __uint_as_float(v << 16); }
__device__ __forceinline__ float bf16_hi(unsigned v) { return __uint_as_float(v & 0xffff0000u); }

constexpr int kVsStride = 68;  // floats per row of the staged rank tile (64 + padding: rows fall into different banks)

// RQ: quads of ranks a lane gathers per 64-rank tile of V (1, 2 or 4: enough for the plan's largest rank, so that the
// gather needs no per-lane branch -- loads behind a branch would each be waited for on their own).
template <int TBLK, int RQ>
__global__ __launch_bounds__(TBLK * 64) void decode_reduce_kernel(DecodeArgs p0) {
    typedef __bf16 E;
    __shared__ __attribute__((aligned(16))) float vs[TBLK * 16 * kVsStride];
    const int tid = threadIdx.x, lane = tid & 63, tb = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, lg = lane >> 4;
    LORA_TS(p0.trace, 0);
    int cb = blockIdx.x;
    DecodeArgs p = p0;
    select_set(p, p0, cb, true);
    const int n = cb * 16 + lg * 4;
    const int t = tb * 16 + li;
    const bool tv = t < p.T;
    const bool has = tv && p.B != nullptr;
    // Loads return in order, so they are requested in the order their results are wanted, each dependent request as
    // soon as what it depends on is back: plan status and row -> adapter; the adapter's pointer and scale; only then
    // the partial tiles of the base product (a longer trip: another XCD wrote them), which the pointer would
    // otherwise queue behind; then B_a's rows and the row's V quads.
    const int status = p.plan.scalars[kScStatus];
    const int a0 = has ? p.plan.row_adapter[t] : -1;
    const int rx0 = has ? p.plan.row_ext[t] : 0;
    const bool hasd = tv && p.D != nullptr;
    const int a0d = hasd ? p.plan.row_adapter[t] : -1;
    const int rx0d = hasd ? p.plan.row_ext[t] : 0;
    const bool gl = p.B != nullptr && lane < p.n_adapters;  // entry `lane` of the two tables, in the same round trip
    const void *b_guess = gl ? p.B[lane] : nullptr;
    const float s_guess = gl ? p.scale[lane] : 0.f;
    if (status != 0) return;
    const int a = a0, rx = rx0;
    const int r = row_ext_rank(rx), e0 = row_ext_offset(rx);
    const E *Bp = static_cast<const E *>(lane_entry(b_guess, a & 63));  // (every lane takes part in the exchange)
    float sc = lane_entry(s_guess, a & 63);
    if (a >= 64) {
        Bp = static_cast<const E *>(p.B[a]);
        sc = p.scale[a];
    }
    if (a < 0 || r <= 0) Bp = nullptr;
    const float4 *P4 = reinterpret_cast<const float4 *>(p.P);
    const int64_t sstride = (int64_t)TBLK * 64;
    const float4 *pb = P4 + ((int64_t)(p.nbe_cap + cb) * p.ks * TBLK + tb) * 64 + lane;
    float4 pq[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) pq[s] = pb[min(s, p.ks - 1) * sstride];
    if (a >= 0 && r > 0 && Bp == nullptr) atomicMin(&p.plan.scalars[kScEvicted], kErrNotResident);  // slot emptied after the plan

    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    // ---- adapter term: V of this row from its adapter's rank blocks, then V B_a, 64 ranks at a time ----
    float *vrow = vs + (tb * 16 + li) * kVsStride;
    if (Bp != nullptr) {
        for (int j0 = 0; j0 < r; j0 += 64) {
            const int nc = min(64, r - j0) >> 3;  // chunks of 8 ranks in this tile
            // the first two chunks of B_a's four rows (HBM) are requested ahead of the V gather (L2): both are wanted
            // before the first product, and the longer trip starts first
            chunk_t bq[2][4];
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    bq[c][e] = load_chunk(Bp + (int64_t)min(n + e, p.N - 1) * r + j0 + min(c, nc - 1) * 8);
            // the four lanes of a row gather the tile's quads of ranks between them (quad lg, lg + 4, ...), slice by
            // slice, eight slices in flight; quads past the row's rank are read from a clamped address and dropped
            const float4 *pv[RQ];
            float4 q[RQ];
#pragma unroll
            for (int i = 0; i < RQ; ++i) {
                const int e = e0 + min(j0 + 4 * (lg + 4 * i), r - 4);
                pv[i] = P4 + ((int64_t)(e >> 4) * p.ks * TBLK + tb) * 64 + ((e & 15) >> 2) * 16 + li;
                q[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
            for (int s0 = 0; s0 < p.ks; s0 += 8) {
                float4 g[8][RQ];
#pragma unroll
                for (int s = 0; s < 8; ++s)
#pragma unroll
                    for (int i = 0; i < RQ; ++i) g[s][i] = pv[i][min(s0 + s, p.ks - 1) * sstride];
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    const float m = s0 + s < p.ks ? 1.f : 0.f;
#pragma unroll
                    for (int i = 0; i < RQ; ++i) {
                        q[i].x += m * g[s][i].x;
                        q[i].y += m * g[s][i].y;
                        q[i].z += m * g[s][i].z;
                        q[i].w += m * g[s][i].w;
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < RQ; ++i)
                if (4 * (lg + 4 * i) < 8 * nc)
                    *reinterpret_cast<float4 *>(vrow + 4 * (lg + 4 * i)) = make_float4(q[i].x * sc, q[i].y * sc, q[i].z * sc, q[i].w * sc);
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");  // (a row's four lanes are in one wave: LDS operations in order)
            auto fma8 = [&](int c, const chunk_t &b, float &out) {
                const float4 v0 = *reinterpret_cast<const float4 *>(vrow + c * 8);
                const float4 v1 = *reinterpret_cast<const float4 *>(vrow + c * 8 + 4);
                out += v0.x * bf16_lo(b.x) + v0.y * bf16_hi(b.x) + v0.z * bf16_lo(b.y) + v0.w * bf16_hi(b.y) +
                       v1.x * bf16_lo(b.z) + v1.y * bf16_hi(b.z) + v1.z * bf16_lo(b.w) + v1.w * bf16_hi(b.w);
            };
#pragma unroll
            for (int c = 0; c < 2; ++c)
                if (c < nc) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) fma8(c, bq[c][e], acc[e]);
                }
            for (int c = 2; c < nc; ++c) {
#pragma unroll
                for (int e = 0; e < 4; ++e) fma8(c, load_chunk(Bp + (int64_t)min(n + e, p.N - 1) * r + j0 + c * 8), acc[e]);
            }
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        }
    }
    LORA_TS(p.trace, 1);  // adapter term done
    // ---- base product: the slices' partial tiles in slice order ----
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        if (s < p.ks) {
            acc[0] += pq[s].x;
            acc[1] += pq[s].y;
            acc[2] += pq[s].z;
            acc[3] += pq[s].w;
        }
    }
    for (int s = 8; s < p.ks; ++s) {
        const float4 v = pb[s * sstride];
        acc[0] += v.x;
        acc[1] += v.y;
        acc[2] += v.z;
        acc[3] += v.w;
    }

    LORA_TS(p.trace, 2);  // base partial sums added
    if (!tv) return;
    if (p.D != nullptr && a0d >= 0 && row_ext_rank(rx0d) > 0) {  // the adapter term, computed by the expand kernel
        const float4 d = *reinterpret_cast<const float4 *>(p.D + (int64_t)t * p.ldd + min(n, (int)p.ldd - 4));
        acc[0] += d.x;
        acc[1] += d.y;
        acc[2] += d.z;
        acc[3] += d.w;
    }
    E *yrow = static_cast<E *>(p.Y) + (int64_t)t * p.ldy;
    if (n + 3 < p.N) {
        store4(yrow + n, acc[0], acc[1], acc[2], acc[3]);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (n + e < p.N) store1(yrow + n + e, acc[e]);
    }
    LORA_TS(p.trace, 3);
}

// V[t, j .. j + 3] = scale_a * sum over the K slices (in order) of the extension rows' partial tiles, rounded to E: one
// thread per row and quad of ranks.  For batches with much adapter work, whose term the expand kernel then computes from
// V segment by segment instead of every workgroup of the reduction gathering V B_a row by row.
template <int TBLK>
__global__ __launch_bounds__(256) void decode_v_kernel(DecodeArgs p) {
    typedef __bf16 E;
    if (p.plan.scalars[kScStatus] != 0) return;
    const int quads = p.r_max >> 2;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long)p.T * quads) return;
    const int t = (int)(idx / quads), j = (int)(idx % quads) * 4;
    const int a = p.plan.row_adapter[t];
    const int rx = p.plan.row_ext[t];
    if (a < 0 || j >= row_ext_rank(rx)) return;
    const float sc = p.scale[a];
    const int e = row_ext_offset(rx) + j;
    const float4 *src = reinterpret_cast<const float4 *>(p.P) + ((int64_t)(e >> 4) * p.ks * TBLK + (t >> 4)) * 64 + ((e & 15) >> 2) * 16 + (t & 15);
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s0 = 0; s0 < p.ks; s0 += 8) {
        float4 g[8];
#pragma unroll
        for (int s = 0; s < 8; ++s) g[s] = src[(int64_t)min(s0 + s, p.ks - 1) * TBLK * 64];
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const float m = s0 + s < p.ks ? 1.f : 0.f;
            v.x += m * g[s].x;
            v.y += m * g[s].y;
            v.z += m * g[s].z;
            v.w += m * g[s].w;
        }
    }
    store4(static_cast<E *>(p.V) + (int64_t)t * p.r_max + j, v.x * sc, v.y * sc, v.z * sc, v.w * sc);
}

template <int TBLK>
hipError_t launch_v_t(const DecodeArgs &a, hipStream_t stream, const KernelTimer *timer) {
    const long threads = (long)a.T * (a.r_max >> 2);
    if (threads <= 0) return hipSuccess;
    return launch_kernel(decode_v_kernel<TBLK>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream, timer, a);
}

template <int TBLK, int MAXW>
size_t stream_smem(int waves) {
    return (size_t)TBLK * 16 * kDsSliceChunks * 16 + (size_t)waves * 2048;
}

template <int TBLK, int MAXW>
hipError_t init_stream() {
    return hipFuncSetAttribute(reinterpret_cast<const void *>(decode_stream_kernel<TBLK, MAXW>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)stream_smem<TBLK, MAXW>(MAXW));
}

// Lays the projections of a launch out in the two grids; returns the totals.
void layout_sets(DecodeArgs &a, long *blocks_out, long *cols_out) {
    if (a.n_sets <= 0) {
        *blocks_out = (long)a.nbe_cap + a.nbw;
        *cols_out = a.nbw;
        return;
    }
    long blk = 0, cb = 0;
    for (int i = 0; i < a.n_sets; ++i) {
        a.set[i].blk0 = (int32_t)blk;
        a.set[i].cb0 = (int32_t)cb;
        blk += (long)a.nbe_cap + a.set[i].nbw;
        cb += a.set[i].nbw;
    }
    *blocks_out = blk;
    *cols_out = cb;
}

template <int TBLK, int MAXW>
hipError_t launch_stream_t(const DecodeArgs &a0, hipStream_t stream, const KernelTimer *timer) {
    if (a0.waves < kDecodeMinWaves || a0.waves > MAXW) return hipErrorInvalidValue;
    DecodeArgs a = a0;
    long blocks = 0, cols = 0;
    layout_sets(a, &blocks, &cols);
    const long groups = (blocks + a.waves - 1) / a.waves;
    const long grid = groups * a.ks;
    if (grid <= 0) return hipSuccess;
#ifdef LORA_TRACE
    return trace_launch("decode_stream", grid, [&](long long *buf) {
        DecodeArgs b = a;
        b.trace = buf;
        return launch_kernel(decode_stream_kernel<TBLK, MAXW>, dim3((unsigned)grid), dim3(a.waves * 64),
                             stream_smem<TBLK, MAXW>(a.waves), stream, timer, b);
    });
#else
    return launch_kernel(decode_stream_kernel<TBLK, MAXW>, dim3((unsigned)grid), dim3(a.waves * 64), stream_smem<TBLK, MAXW>(a.waves),
                         stream, timer, a);
#endif
}

template <int TBLK, int RQ>
hipError_t launch_reduce_q(const DecodeArgs &a0, hipStream_t stream, const KernelTimer *timer) {
    DecodeArgs a = a0;
    long blocks = 0, cols = 0;
    layout_sets(a, &blocks, &cols);
    if (cols <= 0) return hipSuccess;
#ifdef LORA_TRACE
    return trace_launch("decode_reduce", cols, [&](long long *buf) {
        DecodeArgs b = a;
        b.trace = buf;
        return launch_kernel(decode_reduce_kernel<TBLK, RQ>, dim3((unsigned)cols), dim3(TBLK * 64), 0, stream, timer, b);
    });
#else
    return launch_kernel(decode_reduce_kernel<TBLK, RQ>, dim3((unsigned)cols), dim3(TBLK * 64), 0, stream, timer, a);
#endif
}

template <int TBLK>
hipError_t launch_reduce_t(const DecodeArgs &a, hipStream_t stream, const KernelTimer *timer) {
    if (a.r_max <= 16) return launch_reduce_q<TBLK, 1>(a, stream, timer);
    if (a.r_max <= 32) return launch_reduce_q<TBLK, 2>(a, stream, timer);
    return launch_reduce_q<TBLK, 4>(a, stream, timer);
}

bool decode_args_ok(const DecodeArgs &a, int tblk) {
    if (!(a.T > 0 && a.T <= tblk * 16 && a.K > 0 && (a.K & 7) == 0 && a.nbe_cap >= 0 && a.X != nullptr &&
          a.ks == (a.K / 8 + kDsSliceChunks - 1) / kDsSliceChunks && a.n_sets >= 0 && a.n_sets <= kMaxGemmSets))
        return false;
    if (a.n_sets == 0) return a.N > 0 && a.nbw == (a.N + 15) / 16 && a.P != nullptr && a.W != nullptr && a.Y != nullptr;
    for (int i = 0; i < a.n_sets; ++i) {
        const DecodeSet &s = a.set[i];
        if (!(s.N > 0 && s.nbw == (s.N + 15) / 16 && s.P != nullptr && s.W != nullptr && s.Y != nullptr)) return false;
    }
    return true;
}

}  // namespace

hipError_t init_decode_kernels() {
    hipError_t e = init_stream<1, kDecodeMaxWaves>();
    if (e == hipSuccess) e = init_stream<2, kDecodeMaxWaves>();
    if (e == hipSuccess) e = init_stream<4, kDecodeMaxWaves>();
    if (e == hipSuccess) e = init_stream<6, kDecodeMaxWaves>();
    if (e == hipSuccess) e = init_stream<8, kDecodeMaxWaves>();
    return e;
}

// tblk: 16-row blocks of the batch (1, 2, 4, 6, 8).
hipError_t launch_decode_stream(const DecodeArgs &a, int tblk, hipStream_t stream, const KernelTimer *timer) {
    if (!decode_args_ok(a, tblk)) return hipErrorInvalidValue;
    switch (tblk) {
        case 1:
            return launch_stream_t<1, kDecodeMaxWaves>(a, stream, timer);
        case 2:
            return launch_stream_t<2, kDecodeMaxWaves>(a, stream, timer);
        case 4:
            return launch_stream_t<4, kDecodeMaxWaves>(a, stream, timer);
        case 6:
            return launch_stream_t<6, kDecodeMaxWaves>(a, stream, timer);
        case 8:
            return launch_stream_t<8, kDecodeMaxWaves>(a, stream, timer);
        default:
            return hipErrorInvalidValue;
    }
}

hipError_t launch_decode_reduce(const DecodeArgs &a, int tblk, hipStream_t stream, const KernelTimer *timer) {
    if (!decode_args_ok(a, tblk)) return hipErrorInvalidValue;
    switch (tblk) {
        case 1:
            return launch_reduce_t<1>(a, stream, timer);
        case 2:
            return launch_reduce_t<2>(a, stream, timer);
        case 4:
            return launch_reduce_t<4>(a, stream, timer);
        case 6:
            return launch_reduce_t<6>(a, stream, timer);
        case 8:
            return launch_reduce_t<8>(a, stream, timer);
        default:
            return hipErrorInvalidValue;
    }
}

hipError_t launch_decode_v(const DecodeArgs &a, int tblk, hipStream_t stream, const KernelTimer *timer) {
    if (!decode_args_ok(a, tblk) || a.n_sets != 0 || a.V == nullptr || a.scale == nullptr || (a.r_max & 7) != 0) return hipErrorInvalidValue;
    switch (tblk) {
        case 1:
            return launch_v_t<1>(a, stream, timer);
        case 2:
            return launch_v_t<2>(a, stream, timer);
        case 4:
            return launch_v_t<4>(a, stream, timer);
        case 6:
            return launch_v_t<6>(a, stream, timer);
        case 8:
            return launch_v_t<8>(a, stream, timer);
        default:
            return hipErrorInvalidValue;
    }
}

}  // namespace lora
