// Pipelined LDS-tiled MFMA GEMM with the LoRA expand fused as extra K-steps (prefill-sized batches):
//
//     Y[row, n] = sum_k X[row, k] W0[n, k]  +  sum_{p in ext(row)} V[row, p] B_a[n, p],   row = perm[slot]
//
// (paper section 4.4: backbone result and adapter result are combined; here in the fp32
// accumulators, before Y is rounded and stored, once.)  Same tiling, MFMA orientation, row
// order and extension logic as gemm_tile_kernel.hip; what differs is how the base product is fed:
//
//   * global -> LDS directly (global_load_lds_dwordx4): no staging registers, no ds_write, and the
//     loads of several stages stay in flight while the matrix core works.  A wave-level load
//     writes 64 consecutive 16-byte LDS slots, so the XOR swizzle that keeps the MFMA operand
//     reads conflict-free is applied on the global side: the lane that fills slot (row, pos)
//     fetches chunk pos ^ swz(row) of that row (still one contiguous row segment per row);
//   * NBUF stage buffers in a ring, each its own LDS array, so that the compiler can tell that
//     reading one buffer does not depend on the loads in flight into another; the waits for
//     "my loads of stage kt have landed" are explicit vmcnt waits with the number of younger
//     loads, followed by a bare s_barrier (all threads' loads landed / all waves are done
//     with the buffer that is about to be refilled);
//   * one barrier per stage, nothing else synchronises.
// A trailing partial K stage and the extension stages (masked V rows, B_a gathered through the
// table) go through registers (load, mask, ds_write) into the same buffers.
#include <limits.h>

#include "kernels.h"

namespace lora {
namespace {

#define LORA_GPTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define LORA_LPTR(p) ((__attribute__((address_space(3))) void *)(p))

constexpr int kPipeTab = 256;  // extension chunk columns described per batch

struct PipeTable {
    const void *ptr[kPipeTab];  // B_a + j (null = column unused)
    int r[kPipeTab];            // row stride of B_a (its rank)
    int j[kPipeTab];            // column offset inside V / B_a
    int lo[kPipeTab];           // tile-relative rows [lo, hi) that belong to the adapter
    int hi[kPipeTab];
};

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

template <typename E, int BM, int BN, int WM, int WN, int BKC, int NBUF>
__global__ __launch_bounds__(WM *WN * 64) void gemm_pipe_kernel(GemmArgs p, int tiles_m, int tiles_n, int group_m) {
    constexpr int CE = Elem<E>::CE;
    constexpr int NT = WM * WN * 64;
    constexpr int WTM = BM / WM, WTN = BN / WN;  // wave tile: rows t, columns n
    constexpr int NBT = WTM / 32, NBN = WTN / 32;
    constexpr int ROWS = BN + BM;                 // W rows first, then X rows
    constexpr int LPT = ROWS * BKC / NT;          // 16-byte loads per thread per stage
    constexpr int RPP = NT / BKC;                 // rows covered per load pass
    constexpr int SUB = BKC / 2;                  // MFMA substeps per stage
    static_assert(NBUF == 2 || NBUF == 4, "ring of 2 or 4 stage buffers");
    static_assert(ROWS * BKC % NT == 0 && NBT >= 1 && NBN >= 1, "tile / workgroup mismatch");

    __shared__ __attribute__((aligned(16))) chunk_t s0[ROWS * BKC];
    __shared__ __attribute__((aligned(16))) chunk_t s1[ROWS * BKC];
    __shared__ __attribute__((aligned(16))) chunk_t s2[NBUF == 4 ? ROWS * BKC : 1];
    __shared__ __attribute__((aligned(16))) chunk_t s3[NBUF == 4 ? ROWS * BKC : 1];
    __shared__ PipeTable tab;

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
    const int lane = tid & 63, wave = tid >> 6;
    const int wn0 = (wave % WN) * WTN, wm0 = (wave / WN) * WTM;
    const int l31 = lane & 31, lh = lane >> 5;

    const E *X = static_cast<const E *>(p.X);
    const E *W = static_cast<const E *>(p.W);
    const E *V = static_cast<const E *>(p.V);

    // ---- per-thread load slots: LDS slot (row, pos) of pass i is filled with chunk pos ^ swz(row) ----
    const int lpos = tid % BKC;
    const E *src[LPT];   // row base in global memory (W0 row or gathered X row), plus the swizzled chunk offset
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
        const int row = tid / BKC + i * RPP;
        const int c = lpos ^ swz<BKC>(row);
        if (row < BN)  // rows past N / T are clamped: they only feed outputs that are never stored
            src[i] = W + (int64_t)min(n0 + row, p.N - 1) * p.ldw + c * CE;
        else
            src[i] = X + (int64_t)p.plan.perm[min(m0 + row - BN, p.T - 1)] * p.ldx + c * CE;
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
    int wsw[NBN], xsw[NBT];
#pragma unroll
    for (int nb = 0; nb < NBN; ++nb) wsw[nb] = swz<BKC>(wn0 + nb * 32 + l31);
#pragma unroll
    for (int tb = 0; tb < NBT; ++tb) xsw[tb] = swz<BKC>(BN + wm0 + tb * 32 + l31);

    // full MFMA work of one stage
    auto compute = [&](const chunk_t *buf) {
#pragma unroll
        for (int kk = 0; kk < SUB; ++kk) {
            const int cc = 2 * kk + lh;
            chunk_t wf[NBN], xf[NBT];
#pragma unroll
            for (int nb = 0; nb < NBN; ++nb) wf[nb] = buf[wpos[nb] + (cc ^ wsw[nb])];
#pragma unroll
            for (int tb = 0; tb < NBT; ++tb) xf[tb] = buf[xpos[tb] + (cc ^ xsw[tb])];
#pragma unroll
            for (int tb = 0; tb < NBT; ++tb)
#pragma unroll
                for (int nb = 0; nb < NBN; ++nb) Elem<E>::mma32(acc[nb][tb], wf[nb], xf[tb]);
        }
    };
    // asynchronous fill of a stage buffer with stage kt of the base product
    auto dma = [&](chunk_t *buf, int kt) {
#pragma unroll
        for (int i = 0; i < LPT; ++i)
            __builtin_amdgcn_global_load_lds(LORA_GPTR(src[i] + (int64_t)kt * (BKC * CE)), LORA_LPTR(buf + i * NT + wave * 64), 16, 0,
                                             0);
    };

    // ---- base product over the stages that lie entirely inside K ----------------------------------
    const int KT_full = p.K / (BKC * CE);
    // One pipeline step: wait for my loads of stage kt, let everybody arrive (all loads of the stage
    // landed, all waves done with the buffer read last step), refill that buffer, compute.
    // Steady state: every step has NBUF-1 younger stages and no branch.
#define LORA_PIPE_STEP(BUF, REFILL, KT_)          \
    do {                                          \
        wait_vmcnt<(NBUF - 2) * LPT>();           \
        __builtin_amdgcn_s_barrier();             \
        dma(REFILL, (KT_) + NBUF - 1);            \
        compute(BUF);                             \
    } while (0)
    // Drain: the last stages, where younger stages may be missing (then wait for everything).
#define LORA_PIPE_DRAIN(BUF, REFILL, KT_)                                   \
    do {                                                                     \
        const int kt_ = (KT_);                                               \
        if (kt_ < KT_full) {                                                 \
            if (kt_ + NBUF - 1 <= KT_full)                                   \
                wait_vmcnt<(NBUF - 2) * LPT>();                              \
            else                                                             \
                wait_vmcnt<0>();                                             \
            __builtin_amdgcn_s_barrier();                                    \
            if (kt_ + NBUF - 1 < KT_full) dma(REFILL, kt_ + NBUF - 1);       \
            compute(BUF);                                                    \
        }                                                                    \
    } while (0)

    int kt = 0;
    if (KT_full > 0) dma(s0, 0);
    if constexpr (NBUF == 4) {
        if (KT_full > 1) dma(s1, 1);
        if (KT_full > 2) dma(s2, 2);
        for (; kt + 2 * NBUF - 2 < KT_full; kt += 4) {
            LORA_PIPE_STEP(s0, s3, kt);
            LORA_PIPE_STEP(s1, s0, kt + 1);
            LORA_PIPE_STEP(s2, s1, kt + 2);
            LORA_PIPE_STEP(s3, s2, kt + 3);
        }
        for (; kt < KT_full; kt += 4) {
            LORA_PIPE_DRAIN(s0, s3, kt);
            LORA_PIPE_DRAIN(s1, s0, kt + 1);
            LORA_PIPE_DRAIN(s2, s1, kt + 2);
            LORA_PIPE_DRAIN(s3, s2, kt + 3);
        }
    } else {
        for (; kt + 2 * NBUF - 2 < KT_full; kt += 2) {
            LORA_PIPE_STEP(s0, s1, kt);
            LORA_PIPE_STEP(s1, s0, kt + 1);
        }
        for (; kt < KT_full; kt += 2) {
            LORA_PIPE_DRAIN(s0, s1, kt);
            LORA_PIPE_DRAIN(s1, s0, kt + 1);
        }
    }
#undef LORA_PIPE_DRAIN
#undef LORA_PIPE_STEP
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
            regs[i] = keep_if(kv, load_chunk(kv ? src[i] + (int64_t)KT_full * (BKC * CE) : src[i] - c * CE));
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
            for (int nb = 0; nb < NBN; ++nb) wf[nb] = buf[wpos[nb] + (cc ^ wsw[nb])];
#pragma unroll
            for (int tb = 0; tb < NBT; ++tb) {
                const int t0 = wm0 + tb * 32;
                if (lo < t0 + 32 && hi > t0) {
                    const chunk_t xf = buf[xpos[tb] + (cc ^ xsw[tb])];
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
        if (t >= p.T) continue;
        E *yrow = Y + (int64_t)p.plan.perm[t] * p.ldy;
#pragma unroll
        for (int nb = 0; nb < NBN; ++nb) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n0 + wn0 + nb * 32 + g * 8 + lh * 4;
                const f32x16_t &c = acc[nb][tb];
                if (n + 3 < p.N) {
                    store4(yrow + n, c[g * 4 + 0], c[g * 4 + 1], c[g * 4 + 2], c[g * 4 + 3]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (n + e < p.N) store1(yrow + n + e, c[g * 4 + e]);
                }
            }
        }
    }
}

template <typename E, int BM, int BN, int WM, int WN, int BKC, int NBUF>
hipError_t launch_pipe(const GemmArgs &a, hipStream_t stream, const KernelTimer *timer) {
    const int tiles_m = (a.T + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
    const long total = (long)tiles_m * tiles_n;
    if (total <= 0) return hipSuccess;
    auto kern = gemm_pipe_kernel<E, BM, BN, WM, WN, BKC, NBUF>;
    const long grid = ((total + 7) / 8) * 8;
    const int group_m = 8;
    return launch_kernel(kern, dim3((unsigned)grid), dim3(WM * WN * 64), 0, stream, timer, a, tiles_m, tiles_n, group_m);
}

template <typename E>
hipError_t launch_pipe_variant(const GemmArgs &a, int variant, hipStream_t stream, const KernelTimer *timer) {
    switch (variant) {
        case kGemmPipe256x256k32:
            return launch_pipe<E, 256, 256, 4, 2, 4, 4>(a, stream, timer);
        case kGemmPipe256x256k64:
            return launch_pipe<E, 256, 256, 4, 2, 8, 2>(a, stream, timer);
        case kGemmPipe128x128k64:
            return launch_pipe<E, 128, 128, 2, 2, 8, 4>(a, stream, timer);
        default:
            return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_gemm_pipe(const GemmArgs &a, int dtype, int variant, hipStream_t stream, const KernelTimer *timer) {
    return dtype == 1 ? launch_pipe_variant<__bf16>(a, variant, stream, timer) : launch_pipe_variant<float>(a, variant, stream, timer);
}

}  // namespace lora
