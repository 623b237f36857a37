// Pipelined LDS-tiled MFMA GEMM with the LoRA expand fused as extra K-steps (prefill-sized batches):
//
//     Y[row, n] = sum_k X[row, k] W0[n, k]  +  sum_{p in ext(row)} V[row, p] B_a[n, p],   row = perm[slot]
//
// (paper section 4.4: backbone result and adapter result are combined; here in the fp32
// accumulators, before Y is rounded and stored, once.)  Same tiling, MFMA orientation, row
// order and extension logic as gemm_tile_kernel.hip; what differs is how the base product is fed,
// so that the matrix core never waits at a stage boundary:
//
//   * global -> LDS directly (buffer_load_dwordx4 ... lds): no staging registers, no ds_write, and the
//     loads of two stages stay in flight while the matrix core works.  A wave-level load writes 64
//     consecutive 16-byte LDS slots, so the XOR swizzle that keeps the MFMA operand reads
//     conflict-free is applied on the global side: the lane that fills slot (row, pos) fetches
//     chunk pos ^ swz(row) of that row (still one contiguous row segment per row);
//   * a ring of four stage buffers (a stage = 4 chunks = 32 bf16 k per row); "my loads of stage
//     s+1 have landed" is an explicit vmcnt wait with the number of younger loads, followed by a
//     bare s_barrier;
//   * that one barrier per stage sits in the MIDDLE of the stage: it certifies stage s+1 (all
//     threads' loads landed) and frees the buffer of stage s-1 (all waves are past it), so the
//     operand reads are software-pipelined straight across stage boundaries: while the MFMAs of one
//     half-stage run, the LDS reads of the next half-stage (possibly of the next stage) are in
//     flight.  A micro-benchmark of exactly this loop shape sustains ~1.9 PFLOP/s of the 2.5 peak
//     with a barrier every 16 MFMAs, against ~1.0 when the reads start after the barrier;
//   * the operand reads of that loop are issued as ds_read_b128 with explicit lgkmcnt waits: written
//     as ordinary LDS array reads, the compiler cannot tell that a read of one buffer does not
//     depend on the loads in flight into another and drains them all before every read.
// A trailing partial K stage and the extension stages (masked V rows, B_a gathered through the
// table) go through registers (load, mask, ds_write) into the same buffers, with ordinary reads.
#include <limits.h>

#include <type_traits>
#include <utility>

#include "kernels.h"

namespace lora {
namespace {

#define LORA_LPTR(p) ((__attribute__((address_space(3))) void *)(p))

constexpr int kPipeTab = 256;  // extension chunk columns described per batch

struct PipeTable {
    const void *ptr[kPipeTab];  // B_a + j (null = column unused)
    int r[kPipeTab];            // row stride of B_a (its rank)
    int j[kPipeTab];            // column offset inside V / B_a
    int lo[kPipeTab];           // tile-relative rows [lo, hi) that belong to the adapter
    int hi[kPipeTab];
};

typedef unsigned raw4_t __attribute__((ext_vector_type(4)));  // a 16-byte chunk as the register quad an LDS read fills

// s_waitcnt with only vmcnt set (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] at [15:14])
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

template <int BKC>
__device__ __forceinline__ int swz(int row) {
    return BKC == 8 ? ((row >> 1) & 7) : ((row >> 2) & 3);
}

// Issue one 16-byte LDS read at addr + OFF.  The destination is valid only after lds_settle() has
// waited for it: until then nothing may touch the value.
template <int OFF>
__device__ __forceinline__ raw4_t lds_read_async(unsigned addr) {
    static_assert(OFF >= 0 && OFF < 65536, "ds_read immediate offset range");
    raw4_t v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
    return v;
}
template <int OFF, int STRIDE, int... I>
__device__ __forceinline__ void lds_read_async_seq(raw4_t *dst, unsigned addr, std::integer_sequence<int, I...>) {
    ((dst[I] = lds_read_async<OFF + I * STRIDE>(addr)), ...);
}
// Wait until at most YOUNGER LDS reads are outstanding (they return in order), and make every later
// use of the N values in v depend on that wait.
template <int YOUNGER, int N>
__device__ __forceinline__ void lds_settle(raw4_t (&v)[N]) {
    static_assert(YOUNGER >= 0 && YOUNGER < 16, "lgkmcnt range");
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(YOUNGER) : "memory");
#pragma unroll
    for (int i = 0; i < N; ++i) asm volatile("" : "+v"(v[i]));
}

template <typename E, int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(WM *WN * 64) void gemm_pipe_kernel(GemmArgs p, int tiles_m, int tiles_n, int group_m) {
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass only needs the launch stub (and has no buffer-resource type)
    constexpr int CE = Elem<E>::CE;
    constexpr int BKC = 4;  // chunks per row per stage
    constexpr int NT = WM * WN * 64;
    constexpr int WTM = BM / WM, WTN = BN / WN;  // wave tile: rows t, columns n
    constexpr int NBT = WTM / 32, NBN = WTN / 32;
    constexpr int ROWS = BN + BM;                 // W rows first, then X rows
    constexpr int SLOTS = ROWS * BKC;             // chunks per stage buffer
    constexpr int STAGE_BYTES = SLOTS * 16;
    constexpr int LPT = ROWS * BKC / NT;          // 16-byte loads per thread per stage
    constexpr int RPP = NT / BKC;                 // rows covered per load pass
    constexpr int SUB = BKC / 2;                  // MFMA substeps per stage
    constexpr int NR = NBN + NBT;                 // LDS reads per half-stage
    static_assert(ROWS * BKC % NT == 0 && NBT >= 1 && NBN >= 1, "tile / workgroup mismatch");

    __shared__ __attribute__((aligned(16))) chunk_t ring[4 * SLOTS];
    __shared__ PipeTable tab;
    chunk_t *const s0 = ring, *const s1 = ring + SLOTS;

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
    const int m0 = pm * BM, n0 = pn * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn0 = (wave % WN) * WTN, wm0 = (wave / WN) * WTM;
    const int l31 = lane & 31, lh = lane >> 5;

    const E *X = static_cast<const E *>(p.X);
    const E *W = static_cast<const E *>(p.W);
    const E *V = static_cast<const E *>(p.V);

    // ---- per-thread load slots: LDS slot (row, pos) of pass i is filled with chunk pos ^ swz(row) ----
    // Addressed as buffer loads: base in SGPRs, one 32-bit byte offset per lane, the stage's K offset
    // in an SGPR, so a stage costs no address arithmetic.
    static_assert(BN % RPP == 0, "a load pass must not straddle W rows and X rows");
    const int lpos = tid % BKC;
    const __amdgpu_buffer_rsrc_t rsW = __builtin_amdgcn_make_buffer_rsrc(const_cast<E *>(W), 0, 0x7fffffff, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsX = __builtin_amdgcn_make_buffer_rsrc(const_cast<E *>(X), 0, 0x7fffffff, 0x00020000);
    int voff[LPT];  // byte offset of (row, swizzled chunk) from the W0 / X base; the host checked that it fits 31 bits
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
        const int row = tid / BKC + i * RPP;
        const int c = lpos ^ swz<BKC>(row);
        if (row < BN)  // rows past N / T are clamped: they only feed outputs that are never stored
            voff[i] = (int)(((int64_t)min(n0 + row, p.N - 1) * p.ldw + c * CE) * (int64_t)sizeof(E));
        else
            voff[i] = (int)(((int64_t)p.plan.perm[min(m0 + row - BN, p.T - 1)] * p.ldx + c * CE) * (int64_t)sizeof(E));
    }

    // ---- extension range of this M-tile -----------------------------------------------------
    int pbeg = 0, pend = 0;
    if (p.B != nullptr) {
        const int s_first = p.plan.row_seg[m0];
        const int s_last = p.plan.row_seg[min(m0 + BM, p.T) - 1];
        pbeg = p.plan.seg_ext[s_first];
        pend = p.plan.seg_ext[s_last + 1];
    }
    const int ext_chunks = (pend - pbeg) / CE;

    f32x16_t acc[NBN][NBT];
#pragma unroll
    for (int nb = 0; nb < NBN; ++nb)
#pragma unroll
        for (int tb = 0; tb < NBT; ++tb)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[nb][tb][e] = 0.f;

    // MFMA operand positions of this lane inside a stage buffer
    int wpos[NBN], xpos[NBT];
#pragma unroll
    for (int nb = 0; nb < NBN; ++nb) wpos[nb] = (wn0 + nb * 32 + l31) * BKC;
#pragma unroll
    for (int tb = 0; tb < NBT; ++tb) xpos[tb] = (BN + wm0 + tb * 32 + l31) * BKC;
    const int lsw = swz<BKC>(l31);  // wave tiles start at multiples of 32 rows: the swizzle depends on the lane only

    // ---- base product over the stages that lie entirely inside K ----------------------------------
    // operand fragments of one half-stage (two chunk columns = 16 bf16 k per lane pair)
    struct Frag {
        raw4_t w[NBN], x[NBT];
    };
    // LDS byte addresses of this lane's operand chunk in row block 0 of buffer 0, per half (the other
    // half is the chunk position with bit 1 flipped); row blocks are immediate offsets, the buffer is added.
    unsigned aW[2], aX[2];
    {
        const unsigned base = (unsigned)(size_t)LORA_LPTR(ring);
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            aW[kk] = base + (unsigned)(wpos[0] + ((2 * kk + lh) ^ lsw)) * 16u;
            aX[kk] = base + (unsigned)(xpos[0] + ((2 * kk + lh) ^ lsw)) * 16u;
        }
    }
    auto read_half = [&](int buf, auto kk_, Frag &f) {
        constexpr int KK = decltype(kk_)::value;
        const unsigned off = (unsigned)buf * STAGE_BYTES;
        lds_read_async_seq<0, 32 * BKC * 16>(f.w, aW[KK] + off, std::make_integer_sequence<int, NBN>{});
        lds_read_async_seq<0, 32 * BKC * 16>(f.x, aX[KK] + off, std::make_integer_sequence<int, NBT>{});
    };
    auto settle = [&](auto younger_, Frag &f) {
        constexpr int Y = decltype(younger_)::value;
        lds_settle<Y>(f.w);
        lds_settle<Y>(f.x);
    };
    auto mma_half = [&](const Frag &f) {
#pragma unroll
        for (int tb = 0; tb < NBT; ++tb)
#pragma unroll
            for (int nb = 0; nb < NBN; ++nb)
                Elem<E>::mma32(acc[nb][tb], __builtin_bit_cast(chunk_t, f.w[nb]), __builtin_bit_cast(chunk_t, f.x[tb]));
    };
    // asynchronous fill of a stage buffer with stage kt of the base product
    auto dma = [&](int buf, int kt) {
        const int koff = kt * (BKC * CE * (int)sizeof(E));
        chunk_t *dst = ring + buf * SLOTS + wave * 64;
#pragma unroll
        for (int i = 0; i < LPT; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(i * RPP < BN ? rsW : rsX, LORA_LPTR(dst + i * NT), 16, voff[i], koff, 0, 0);
    };

    const int KT_full = p.K / (BKC * CE);
    if (KT_full > 0) {
        using I0 = std::integral_constant<int, 0>;
        using I1 = std::integral_constant<int, 1>;
        using INR = std::integral_constant<int, NR>;
        const int last = KT_full - 1;
        Frag fa, fb;  // fa: first half of the current stage, fb: second half
        dma(0, 0);
        dma(1, min(1, last));
        dma(2, min(2, last));
        wait_vmcnt<2 * LPT>();
        __builtin_amdgcn_s_barrier();
        read_half(0, I0(), fa);
        // One stage per trip (stage s in buffer s % 4): the reads of half 2 fly during the MFMAs of
        // half 1; then wait for my loads of stage s+1 (stage s+2 may stay in flight), barrier, refill
        // the buffer that held stage s-1, and the reads of stage s+1's half 1 fly during half 2.
        // Stages past the end are replaced by a reload of the last one, whose buffer is then never
        // consumed: every trip has the same shape, and the wait counts hold up to the last trip.
        // (the sched_barriers pin the order "issue the reads, then the MFMAs that hide them")
#pragma unroll 1
        for (int s = 0; s < KT_full; ++s) {
            read_half(s & 3, I1(), fb);
            settle(INR(), fa);
            __builtin_amdgcn_sched_barrier(0);
            mma_half(fa);
            __builtin_amdgcn_sched_barrier(0);
            wait_vmcnt<LPT>();
            __builtin_amdgcn_s_barrier();
            dma((s + 3) & 3, min(s + 3, last));
            read_half((s + 1) & 3, I0(), fa);
            settle(INR(), fb);
            __builtin_amdgcn_sched_barrier(0);
            mma_half(fb);
            __builtin_amdgcn_sched_barrier(0);
        }
        settle(I0(), fa);  // the last trip's look-ahead reads: nothing may reuse their registers before they land
        wait_vmcnt<0>();
    }
    __syncthreads();  // every load has landed and every wave is done with the ring

    // ---- staged tail: a partial last K stage, then the extension stages --------------------------------
    // (per-thread state of this phase is derived here, not kept alive across the pipelined loop)
    chunk_t regs[LPT];
    int srow[LPT];   // row inside the stage buffer
    int xrowi[LPT];  // original row index (X rows), -1 for W rows
    if (KT_full * BKC * CE < p.K || ext_chunks > 0) {
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            srow[i] = tid / BKC + i * RPP;
            xrowi[i] = srow[i] < BN ? -1 : p.plan.perm[min(m0 + srow[i] - BN, p.T - 1)];
        }
    }
    auto load_partial = [&]() {
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            const int c = lpos ^ swz<BKC>(srow[i]);
            const bool kv = (KT_full * BKC + c) * CE < p.K;
            const E *rowp = xrowi[i] < 0 ? W + (int64_t)min(n0 + srow[i], p.N - 1) * p.ldw : X + (int64_t)xrowi[i] * p.ldx;
            regs[i] = keep_if(kv, load_chunk(kv ? rowp + (int64_t)(KT_full * BKC + c) * CE : rowp));
        }
    };
    auto load_ext = [&](int se) {  // se = stage inside the current table batch
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            const int c = lpos ^ swz<BKC>(srow[i]);
            const int idx = se * BKC + c;
            const E *bp = static_cast<const E *>(tab.ptr[idx]);
            const int r = tab.r[idx], j = tab.j[idx], lo = tab.lo[idx], hi = tab.hi[idx];
            if (xrowi[i] < 0) {
                const bool ok = bp != nullptr;
                const int n = min(n0 + srow[i], p.N - 1);
                regs[i] = keep_if(ok, load_chunk(ok ? bp + (int64_t)n * r : W));
            } else {
                const int row = srow[i] - BN;
                const bool ok = row >= lo && row < hi;  // rows of other adapters contribute nothing
                regs[i] = keep_if(ok, load_chunk(ok ? V + (int64_t)xrowi[i] * p.r_max + j : V));
            }
        }
    };
    auto store_regs = [&](chunk_t *buf) {
#pragma unroll
        for (int i = 0; i < LPT; ++i) buf[i * NT + tid] = regs[i];
    };
    auto compute_ext = [&](const chunk_t *buf, int se) {  // skips 32-row blocks without a row of the adapters at hand
#pragma unroll
        for (int kk = 0; kk < SUB; ++kk) {
            const int i0 = se * BKC + 2 * kk;
            const int lo = min(tab.lo[i0], tab.lo[i0 + 1]);
            const int hi = max(tab.hi[i0], tab.hi[i0 + 1]);
            if (hi <= lo) continue;
            const int cc = 2 * kk + lh;
            chunk_t wf[NBN];
#pragma unroll
            for (int nb = 0; nb < NBN; ++nb) wf[nb] = buf[wpos[nb] + (cc ^ lsw)];
#pragma unroll
            for (int tb = 0; tb < NBT; ++tb) {
                const int t0 = wm0 + tb * 32;
                if (lo < t0 + 32 && hi > t0) {
                    const chunk_t xf = buf[xpos[tb] + (cc ^ lsw)];
#pragma unroll
                    for (int nb = 0; nb < NBN; ++nb) Elem<E>::mma32(acc[nb][tb], wf[nb], xf);
                }
            }
        }
    };
    auto build_table = [&](int chunk0) {
        for (int idx = tid; idx < kPipeTab; idx += NT) {
            const int pe = pbeg + (chunk0 + idx) * CE;
            const void *ptr = nullptr;
            int r = 0, j = 0, lo = INT_MAX, hi = INT_MIN;
            if (pe < pend) {
                const int4 rec = reinterpret_cast<const int4 *>(p.plan.ext_rec)[pe >> 3];
                const E *b = rec.x >= 0 ? static_cast<const E *>(p.B[rec.x]) : nullptr;
                if (b != nullptr) {
                    r = rec.y >> 16;
                    j = (rec.y & 0xffff) + (pe & 7);
                    lo = max(rec.z - m0, 0);
                    hi = min(rec.w - m0, BM);
                    ptr = b + j;
                } else {
                    atomicMin(&p.plan.scalars[kScStatus], kErrNotResident);
                }
            }
            tab.ptr[idx] = ptr;
            tab.r[idx] = r;
            tab.j[idx] = j;
            tab.lo[idx] = lo;
            tab.hi[idx] = hi;
        }
    };

    // full MFMA work of one stage, not pipelined (partial K stage)
    auto compute = [&](const chunk_t *buf) {
#pragma unroll
        for (int kk = 0; kk < SUB; ++kk) {
            const int cc = 2 * kk + lh;
            chunk_t wf[NBN], xf[NBT];
#pragma unroll
            for (int nb = 0; nb < NBN; ++nb) wf[nb] = buf[wpos[nb] + (cc ^ lsw)];
#pragma unroll
            for (int tb = 0; tb < NBT; ++tb) xf[tb] = buf[xpos[tb] + (cc ^ lsw)];
#pragma unroll
            for (int tb = 0; tb < NBT; ++tb)
#pragma unroll
                for (int nb = 0; nb < NBN; ++nb) Elem<E>::mma32(acc[nb][tb], wf[nb], xf[tb]);
        }
    };
    if (KT_full * BKC * CE < p.K) {
        load_partial();
        store_regs(s0);
        __syncthreads();
        compute(s0);
        __syncthreads();
    }
    for (int chunk0 = 0; chunk0 < ext_chunks; chunk0 += kPipeTab) {
        build_table(chunk0);
        __syncthreads();
        const int nst = (min(ext_chunks - chunk0, kPipeTab) + BKC - 1) / BKC;
        load_ext(0);
        store_regs(s0);
        __syncthreads();
        for (int se = 0; se < nst; ++se) {
            const bool more = se + 1 < nst;
            if (more) load_ext(se + 1);
            if (se & 1) {
                compute_ext(s1, se);
                if (more) store_regs(s0);
            } else {
                compute_ext(s0, se);
                if (more) store_regs(s1);
            }
            __syncthreads();
        }
    }

    // ---- single store of Y: acc[nb][tb][g*4+e] = D[n = nb*32 + g*8 + lh*4 + e][t = tb*32 + l31] -------
    E *Y = static_cast<E *>(p.Y);
#pragma unroll
    for (int tb = 0; tb < NBT; ++tb) {
        const int t = m0 + wm0 + tb * 32 + l31;
        const bool row_ok = t < p.T;
        const int row = p.plan.perm[min(t, p.T - 1)];
        E *yrow = Y + (int64_t)row * p.ldy;
        // the adapter term, when a kernel of its own has computed it (rows with an adapter only)
        const float *drow = (p.D != nullptr && p.plan.row_adapter[row] >= 0) ? p.D + (int64_t)row * p.ldd : nullptr;
#pragma unroll
        for (int nb = 0; nb < NBN; ++nb) store_acc_tile<E>(acc[nb][tb], yrow, drow, n0 + wn0 + nb * 32, lh, p.N, row_ok);
    }
#endif  // __HIP_DEVICE_COMPILE__
}

template <typename E, int BM, int BN, int WM, int WN>
hipError_t launch_pipe(const GemmArgs &a, hipStream_t stream, const KernelTimer *timer) {
    const int tiles_m = (a.T + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
    const long total = (long)tiles_m * tiles_n;
    if (total <= 0) return hipSuccess;
    auto kern = gemm_pipe_kernel<E, BM, BN, WM, WN>;
    const long grid = ((total + 7) / 8) * 8;
    const int group_m = 8;
    return launch_kernel(kern, dim3((unsigned)grid), dim3(WM * WN * 64), 0, stream, timer, a, tiles_m, tiles_n, group_m);
}

template <typename E>
hipError_t launch_pipe_variant(const GemmArgs &a, int variant, hipStream_t stream, const KernelTimer *timer) {
    switch (variant) {
        case kGemmPipe256x256w8:
            return launch_pipe<E, 256, 256, 4, 2>(a, stream, timer);
        case kGemmPipe256x256w4:
            return launch_pipe<E, 256, 256, 2, 2>(a, stream, timer);
        case kGemmPipe128x128w4:
            return launch_pipe<E, 128, 128, 2, 2>(a, stream, timer);
        default:
            return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_gemm_pipe(const GemmArgs &a, int dtype, int variant, hipStream_t stream, const KernelTimer *timer) {
    return dtype == 1 ? launch_pipe_variant<__bf16>(a, variant, stream, timer) : launch_pipe_variant<float>(a, variant, stream, timer);
}

}  // namespace lora
