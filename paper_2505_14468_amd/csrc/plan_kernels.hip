// Device-side segment / indptr builder: groups the token rows of a batch by adapter.
//
// Input is one (adapter id, token count) pair per request, as a batching scheduler hands a
// batch over (paper section 4.2).  Output is a stable counting sort of the rows by adapter:
// histogram of rows per adapter -> exclusive scans -> per-request destination -> per-row
// scatter, plus the derived tables the compute kernels index (per-segment rank prefix, the
// shrink work list and one record per 8 ranks of the concatenated rank space).
//
// All arithmetic is integer, so integer atomics keep the result deterministic.
#include <limits.h>

#include "kernels.h"

namespace lora {
namespace {

constexpr int kPlanThreads = 1024;
constexpr int kPlanWaves = kPlanThreads / 64;

// Exclusive scan of one int per thread over the whole workgroup.  Every thread calls it.
__device__ int block_exscan(int v, int &total, int *wave_sums) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int o = __shfl_up(inc, d);
        if (lane >= d) inc += o;
    }
    __syncthreads();  // wave_sums may still be read from the previous call
    if (lane == 63) wave_sums[wave] = inc;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kPlanWaves; ++w) {
        int s = wave_sums[w];
        if (w < wave) base += s;
        tot += s;
    }
    total = tot;
    return base + inc - v;
}

// For the 64 requests of one wave: rows of earlier lanes with the same key (off), and whether
// this lane is the last one with its key.  Fully unrolled so that every cross-lane read is a
// v_readlane with a constant lane index (a handful of cycles; a shuffle through the LDS crossbar
// costs two orders of magnitude more latency and this loop is serial).
__device__ __forceinline__ void rank_among_equal_keys(int key, int L, int lane, int &off, bool &last) {
#pragma unroll
    for (int l2 = 0; l2 < 64; ++l2) {
        const int k2 = __builtin_amdgcn_readlane(key, l2);
        const int L2 = __builtin_amdgcn_readlane(L, l2);
        if (k2 == key) {
            if (l2 < lane)
                off += L2;
            else if (l2 > lane)
                last = false;
        }
    }
}

// Four exclusive scans at once (their cross-lane steps overlap instead of running back to back).
__device__ void block_exscan4(int4 v, int4 &ex, int4 &total, int *wave_sums /* [4][kPlanWaves] */) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int4 inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int ox = __shfl_up(inc.x, d), oy = __shfl_up(inc.y, d), oz = __shfl_up(inc.z, d), ow = __shfl_up(inc.w, d);
        if (lane >= d) {
            inc.x += ox;
            inc.y += oy;
            inc.z += oz;
            inc.w += ow;
        }
    }
    __syncthreads();  // wave_sums may still be read from the previous call
    if (lane == 63) {
        wave_sums[0 * kPlanWaves + wave] = inc.x;
        wave_sums[1 * kPlanWaves + wave] = inc.y;
        wave_sums[2 * kPlanWaves + wave] = inc.z;
        wave_sums[3 * kPlanWaves + wave] = inc.w;
    }
    __syncthreads();
    int4 base = make_int4(0, 0, 0, 0), tot = make_int4(0, 0, 0, 0);
#pragma unroll
    for (int w = 0; w < kPlanWaves; ++w) {
        const int a = wave_sums[0 * kPlanWaves + w], b = wave_sums[1 * kPlanWaves + w], c = wave_sums[2 * kPlanWaves + w],
                  d = wave_sums[3 * kPlanWaves + w];
        if (w < wave) {
            base.x += a;
            base.y += b;
            base.z += c;
            base.w += d;
        }
        tot.x += a;
        tot.y += b;
        tot.z += c;
        tot.w += d;
    }
    total = tot;
    ex = make_int4(base.x + inc.x - v.x, base.y + inc.y - v.y, base.z + inc.z - v.z, base.w + inc.w - v.w);
}

// perm / row_seg: one thread per original row.
__device__ void fill_rows(const PlanBuildArgs &p, int start, int stride) {
    const int T = p.T, R = p.n_req;
    for (int t = start; t < T; t += stride) {
        int lo = 0, hi = R;  // first request whose end offset exceeds t
        while (lo < hi) {
            int mid = (lo + hi) >> 1;
            if (p.tok_off[mid + 1] > t)
                hi = mid;
            else
                lo = mid + 1;
        }
        const int i = lo;
        const int a = p.req_adapter[i];
        const int key = a < 0 ? p.n_adapters : a;
        const int slot = p.req_dst[i] + (t - p.tok_off[i]);
        const int sg = p.key_seg[key];
        p.perm[slot] = t;
        p.row_seg[slot] = sg;
        p.row_adapter[t] = a;
        p.row_ext[t] = pack_row_ext(p.seg_ext[sg], p.seg_rank[sg]);
    }
}

// ext_rec: one record per 8 consecutive ranks of the concatenation of all segments' ranks.
__device__ void fill_ext(const PlanBuildArgs &p, int start, int stride) {
    const int n_rec = p.scalars[kScExtTotal] >> 3;
    const int n_seg = p.scalars[kScNSeg];
    for (int q = start; q < n_rec; q += stride) {
        const int pel = q << 3;
        int lo = 0, hi = n_seg;  // first segment whose rank range ends beyond pel
        while (lo < hi) {
            int mid = (lo + hi) >> 1;
            if (p.seg_ext[mid + 1] > pel)
                hi = mid;
            else
                lo = mid + 1;
        }
        const int s = lo;
        int4 rec;
        rec.x = p.seg_adapter[s];
        rec.y = (p.seg_rank[s] << 16) | (pel - p.seg_ext[s]);
        rec.z = p.seg_indptr[s];
        rec.w = p.seg_indptr[s + 1];
        reinterpret_cast<int4 *>(p.ext_rec)[q] = rec;
    }
}

// unit_rec: one record per shrink work unit (<= 64 rows of one adapter segment).
__device__ void fill_units(const PlanBuildArgs &p, int start, int stride) {
    const int n_units = p.scalars[kScNUnits];
    const int n_seg = p.scalars[kScNSeg];
    for (int u = start; u < n_units; u += stride) {
        int lo = 0, hi = n_seg;  // first segment whose unit range ends beyond u
        while (lo < hi) {
            int mid = (lo + hi) >> 1;
            if (p.seg_unit[mid + 1] > u)
                hi = mid;
            else
                lo = mid + 1;
        }
        const int s = lo;
        const int slot0 = p.seg_indptr[s] + (u - p.seg_unit[s]) * p.unit_rows;
        int4 rec;
        rec.x = p.seg_adapter[s];
        rec.y = p.seg_rank[s] | (p.seg_indptr[s + 1] - p.seg_indptr[s] >= kLongSegRows ? kUnitLongFlag : 0);
        rec.z = slot0;
        rec.w = min(p.unit_rows, p.seg_indptr[s + 1] - slot0);
        reinterpret_cast<int4 *>(p.unit_rec)[u] = rec;
    }
}

__device__ void write_failed(const PlanBuildArgs &p, int status) {
    p.scalars[kScNSeg] = 0;
    p.scalars[kScStatus] = status;
    p.scalars[kScEvicted] = 0;
    p.scalars[kScExtTotal] = 0;
    p.scalars[kScNUnits] = 0;
    p.scalars[kScT] = 0;
    p.seg_indptr[0] = 0;
    p.seg_ext[0] = 0;
    p.seg_unit[0] = 0;
}

__global__ __launch_bounds__(kPlanThreads) void plan_segments_kernel(PlanBuildArgs p, int fuse_fill) {
    __shared__ int wave_sums[4][kPlanWaves];
    __shared__ int s_status;
    __shared__ unsigned long long s_sum;
    const int tid = threadIdx.x;
    const int R = p.n_req, n_ad = p.n_adapters;

    if (tid == 0) {
        s_status = 0;
        s_sum = 0ull;
    }
    for (int k = tid; k <= n_ad; k += kPlanThreads) p.hist[k] = 0;
    __syncthreads();

    // 1. validate the requests, histogram of rows per key (key n_ad = "no adapter")
    {
        unsigned long long local = 0ull;
        int st = 0;
        for (int i = tid; i < R; i += kPlanThreads) {
            const int a = p.req_adapter[i], L = p.req_ntok[i];
            if (a < -1 || a >= n_ad) {
                st = min(st, kErrBadAdapterId);
            } else if (L < 0) {
                st = min(st, kErrLengthMismatch);
            } else if (L > 0) {
                local += (unsigned long long)L;
                atomicAdd(&p.hist[a < 0 ? n_ad : a], L);
            }
        }
        if (st != 0) atomicMin(&s_status, st);
        if (local != 0ull) atomicAdd(&s_sum, local);
    }
    __syncthreads();
    if (tid == 0 && s_status == 0 && s_sum != (unsigned long long)(unsigned)p.T) s_status = kErrLengthMismatch;
    __syncthreads();
    if (s_status != 0) {
        if (tid == 0) write_failed(p, s_status);
        return;
    }

    // 2. first row of every request
    {
        int carry = 0;
        for (int base = 0; base < R; base += kPlanThreads) {
            const int i = base + tid;
            const int v = i < R ? p.req_ntok[i] : 0;
            int tot;
            const int ex = block_exscan(v, tot, wave_sums[0]);
            if (i < R) p.tok_off[i] = carry + ex;
            carry += tot;
        }
        if (tid == 0) p.tok_off[R] = carry;
    }

    // 3. segments = keys with rows, in ascending key order; four prefix sums at once
    int c_seg = 0, c_row = 0, c_ext = 0, c_unit = 0;
    {
        int st = 0;
        for (int base = 0; base <= n_ad; base += kPlanThreads) {
            const int k = base + tid;
            const int h = k <= n_ad ? p.hist[k] : 0;
            const int flag = h > 0 ? 1 : 0;
            int rk = 0, units = 0;
            if (flag && k < n_ad) {
                rk = p.rank[k];
                if (rk <= 0) {
                    st = min(st, kErrNotResident);
                    rk = 0;
                } else if (rk & 7) {
                    st = min(st, kErrShape);
                    rk = 0;
                } else if (rk > p.r_max) {
                    st = min(st, kErrRankTooLarge);
                    rk = 0;
                }
                units = (h + p.unit_rows - 1) >> p.unit_shift;
            }
            int4 ex4, tot4;
            block_exscan4(make_int4(flag, h, rk, units), ex4, tot4, &wave_sums[0][0]);
            const int e_seg = ex4.x, e_row = ex4.y, e_ext = ex4.z, e_unit = ex4.w;
            const int t_seg = tot4.x, t_row = tot4.y, t_ext = tot4.z, t_unit = tot4.w;
            if (flag) {
                const int s = c_seg + e_seg;
                p.seg_adapter[s] = k < n_ad ? k : -1;
                p.seg_indptr[s] = c_row + e_row;
                p.seg_rank[s] = rk;
                p.seg_ext[s] = c_ext + e_ext;
                p.seg_unit[s] = c_unit + e_unit;
                p.cursor[k] = c_row + e_row;
                p.key_seg[k] = s;
            } else if (k <= n_ad) {
                p.key_seg[k] = -1;
            }
            c_seg += t_seg;
            c_row += t_row;
            c_ext += t_ext;
            c_unit += t_unit;
        }
        if (st != 0) atomicMin(&s_status, st);
    }
    __syncthreads();
    if (s_status != 0) {
        if (tid == 0) write_failed(p, s_status);
        return;
    }
    if (tid == 0) {
        p.seg_indptr[c_seg] = c_row;
        p.seg_ext[c_seg] = c_ext;
        p.seg_unit[c_seg] = c_unit;
        p.scalars[kScNSeg] = c_seg;
        p.scalars[kScStatus] = 0;
        p.scalars[kScEvicted] = 0;
        p.scalars[kScExtTotal] = c_ext;
        p.scalars[kScNUnits] = c_unit;
        p.scalars[kScT] = c_row;
    }
    __syncthreads();

    // 4. first slot of every request: requests of one key keep their order (stable).
    //    One wave walks the requests 64 at a time; lanes with the same key are ranked
    //    against each other with cross-lane reads, then the running slot of each key moves on.
    if (tid < 64) {
        volatile int32_t *cur = p.cursor;
        const int lane = tid;
        for (int base = 0; base < R; base += 64) {
            const int i = base + lane;
            const bool valid = i < R;
            const int a = valid ? p.req_adapter[i] : 0;
            const int L = valid ? p.req_ntok[i] : 0;
            const int key = valid ? (a < 0 ? n_ad : a) : -2;
            int off = 0;
            bool last = true;
            rank_among_equal_keys(key, L, lane, off, last);
            int b = 0;
            if (valid) {
                b = cur[key];
                p.req_dst[i] = b + off;
            }
            __threadfence();  // every lane has read its key's running slot before any lane moves one
            if (valid && last) cur[key] = b + off + L;
            __threadfence();
        }
    }
    __syncthreads();

    if (fuse_fill) {
        fill_rows(p, tid, kPlanThreads);
        fill_ext(p, tid, kPlanThreads);
        fill_units(p, tid, kPlanThreads);
    }
}

// Small batches (the common case in serving: at most 2048 requests, 2047 adapter slots, 8192 rows):
// the same algorithm with every intermediate array in LDS, so that the only global round trips
// are the initial read of the request arrays and the final writes.  Latency, not bytes, is what
// this kernel costs.
constexpr int kSmallReq = 2048;
constexpr int kSmallKeys = 2048;
constexpr int kSmallRows = 8192;

__global__ __launch_bounds__(kPlanThreads) void plan_small_kernel(PlanBuildArgs p) {
    __shared__ int s_a[kSmallReq], s_L[kSmallReq + 64], s_key[kSmallReq + 64], s_tok[kSmallReq + 1], s_dst[kSmallReq];
    __shared__ int s_hist[kSmallKeys], s_cur[kSmallKeys], s_kseg[kSmallKeys], s_ofl[kSmallReq];
    __shared__ int s_sad[kSmallKeys + 1], s_sip[kSmallKeys + 1], s_srk[kSmallKeys + 1], s_sex[kSmallKeys + 1], s_sun[kSmallKeys + 1];
    __shared__ int wave_sums[4][kPlanWaves];
    __shared__ int s_status;
    __shared__ unsigned long long s_sum;
    const int tid = threadIdx.x;
    const int R = p.n_req, n_ad = p.n_adapters;
    LORA_TS(p.trace, 0);

    for (int i = tid; i < R + 64; i += kPlanThreads) {
        const int a = i < R ? p.req_adapter[i] : -3;
        if (i < R) s_a[i] = a;
        s_L[i] = i < R ? p.req_ntok[i] : 0;
        s_key[i] = a < -1 ? -3 : (a < 0 ? n_ad : a);  // key n_ad = "no adapter"; the tail matches nothing
    }
    for (int k = tid; k <= n_ad; k += kPlanThreads) s_hist[k] = 0;
    if (tid == 0) {
        s_status = 0;
        s_sum = 0ull;
    }
    __syncthreads();

    // 1. validate, histogram of rows per key
    {
        unsigned long long local = 0ull;
        int st = 0;
        for (int i = tid; i < R; i += kPlanThreads) {
            const int a = s_a[i], L = s_L[i];
            if (a < -1 || a >= n_ad) {
                st = min(st, kErrBadAdapterId);
            } else if (L < 0) {
                st = min(st, kErrLengthMismatch);
            } else if (L > 0) {
                local += (unsigned long long)L;
                atomicAdd(&s_hist[a < 0 ? n_ad : a], L);
            }
        }
        if (st != 0) atomicMin(&s_status, st);
        if (local != 0ull) atomicAdd(&s_sum, local);
    }
    __syncthreads();
    if (tid == 0 && s_status == 0 && s_sum != (unsigned long long)(unsigned)p.T) s_status = kErrLengthMismatch;
    __syncthreads();
    if (s_status != 0) {
        if (tid == 0) write_failed(p, s_status);
        return;
    }

    LORA_TS(p.trace, 1);  // requests read, validated, histogram
    // 2. first row of every request
    {
        int carry = 0;
        for (int base = 0; base < R; base += kPlanThreads) {
            const int i = base + tid;
            const int v = i < R ? s_L[i] : 0;
            int tot;
            const int ex = block_exscan(v, tot, wave_sums[0]);
            if (i < R) {
                s_tok[i] = carry + ex;
                p.tok_off[i] = carry + ex;
            }
            carry += tot;
        }
        if (tid == 0) {
            s_tok[R] = carry;
            p.tok_off[R] = carry;
        }
    }

    LORA_TS(p.trace, 2);  // token offsets
    // 3. segments
    int c_seg = 0, c_row = 0, c_ext = 0, c_unit = 0;
    {
        int st = 0;
        for (int base = 0; base <= n_ad; base += kPlanThreads) {
            const int k = base + tid;
            const int h = k <= n_ad ? s_hist[k] : 0;
            const int flag = h > 0 ? 1 : 0;
            int rk = 0, units = 0;
            if (flag && k < n_ad) {
                rk = p.rank[k];
                if (rk <= 0) {
                    st = min(st, kErrNotResident);
                    rk = 0;
                } else if (rk & 7) {
                    st = min(st, kErrShape);
                    rk = 0;
                } else if (rk > p.r_max) {
                    st = min(st, kErrRankTooLarge);
                    rk = 0;
                }
                units = (h + p.unit_rows - 1) >> p.unit_shift;
            }
            int4 ex4, tot4;
            block_exscan4(make_int4(flag, h, rk, units), ex4, tot4, &wave_sums[0][0]);
            const int e_seg = ex4.x, e_row = ex4.y, e_ext = ex4.z, e_unit = ex4.w;
            const int t_seg = tot4.x, t_row = tot4.y, t_ext = tot4.z, t_unit = tot4.w;
            if (flag) {
                const int s = c_seg + e_seg;
                s_sad[s] = k < n_ad ? k : -1;
                s_sip[s] = c_row + e_row;
                s_srk[s] = rk;
                s_sex[s] = c_ext + e_ext;
                s_sun[s] = c_unit + e_unit;
                s_cur[k] = c_row + e_row;
                s_kseg[k] = s;
            } else if (k <= n_ad) {
                s_kseg[k] = -1;
            }
            c_seg += t_seg;
            c_row += t_row;
            c_ext += t_ext;
            c_unit += t_unit;
        }
        if (st != 0) atomicMin(&s_status, st);
    }
    __syncthreads();
    if (s_status != 0) {
        if (tid == 0) write_failed(p, s_status);
        return;
    }
    if (tid == 0) {
        s_sip[c_seg] = c_row;
        s_sex[c_seg] = c_ext;
        s_sun[c_seg] = c_unit;
        p.scalars[kScNSeg] = c_seg;
        p.scalars[kScStatus] = 0;
        p.scalars[kScEvicted] = 0;
        p.scalars[kScExtTotal] = c_ext;
        p.scalars[kScNUnits] = c_unit;
        p.scalars[kScT] = c_row;
    }
    __syncthreads();
    for (int s = tid; s <= c_seg; s += kPlanThreads) {  // publish the segment arrays
        if (s < c_seg) {
            p.seg_adapter[s] = s_sad[s];
            p.seg_rank[s] = s_srk[s];
        }
        p.seg_indptr[s] = s_sip[s];
        p.seg_ext[s] = s_sex[s];
        p.seg_unit[s] = s_sun[s];
    }

    LORA_TS(p.trace, 3);  // segments
    // 4. stable destination of every request, 64 requests (one wave) at a time.
    //    4a, all waves, a chunk of 64 requests each: rows of earlier requests of the chunk with the same key,
    //        and whether a later request of the chunk has the key -- the other requests' (key, rows) are
    //        broadcast one by one from scalar registers.
    //    4b, one wave, chunk after chunk (the only serial part: two LDS accesses per chunk): running slot of
    //        the key + offset inside the chunk; the last request of a key in the chunk advances the slot.
    {
        const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        for (int base = wave * 64; base < R; base += kPlanThreads) {
            const int i = base + lane;
            const bool valid = i < R;
            const int key = valid ? s_key[i] : -2;
            const int L = valid ? s_L[i] : 0;
            int off = 0, later = 0;
#pragma unroll 16
            for (int l2 = 0; l2 < 64; ++l2) {
                const int k2 = __builtin_amdgcn_readlane(key, l2);
                const int L2 = __builtin_amdgcn_readlane(L, l2);
                const bool same = k2 == key;
                off += (same && l2 < lane) ? L2 : 0;
                later |= (same && l2 > lane) ? 1 : 0;
            }
            if (valid) s_ofl[i] = (off << 1) | (later ? 0 : 1);
        }
    }
    __syncthreads();
    LORA_TS(p.trace, 4);  // ranking inside chunks
    if (tid < 64) {
        volatile int *cur = s_cur;
        const int lane = tid;
        for (int base = 0; base < R; base += 64) {
            const int i = base + lane;
            const bool valid = i < R;
            int b = 0, off = 0, last = 0, key = 0;
            if (valid) {
                key = s_key[i];
                const int ofl = s_ofl[i];
                off = ofl >> 1;
                last = ofl & 1;
                b = cur[key];
                s_dst[i] = b + off;
            }
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");  // all lanes have read before any lane writes
            if (valid && last) cur[key] = b + off + s_L[i];
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        }
    }
    __syncthreads();

    LORA_TS(p.trace, 5);  // chunk walk
    // 5. per-row scatter
    for (int t = tid; t < c_row; t += kPlanThreads) {
        int lo = 0, hi = R;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (s_tok[mid + 1] > t)
                hi = mid;
            else
                lo = mid + 1;
        }
        const int a = s_a[lo];
        const int slot = s_dst[lo] + (t - s_tok[lo]);
        const int sg = s_kseg[a < 0 ? n_ad : a];
        p.perm[slot] = t;
        p.row_seg[slot] = sg;
        p.row_adapter[t] = a;
        p.row_ext[t] = pack_row_ext(s_sex[sg], s_srk[sg]);
    }
    LORA_TS(p.trace, 6);  // row scatter
    // 6. one record per 8 ranks of the extension axis, one per shrink work unit
    for (int q = tid; q < (c_ext >> 3); q += kPlanThreads) {
        const int pel = q << 3;
        int lo = 0, hi = c_seg;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (s_sex[mid + 1] > pel)
                hi = mid;
            else
                lo = mid + 1;
        }
        int4 rec;
        rec.x = s_sad[lo];
        rec.y = (s_srk[lo] << 16) | (pel - s_sex[lo]);
        rec.z = s_sip[lo];
        rec.w = s_sip[lo + 1];
        reinterpret_cast<int4 *>(p.ext_rec)[q] = rec;
    }
    for (int u = tid; u < c_unit; u += kPlanThreads) {
        int lo = 0, hi = c_seg;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (s_sun[mid + 1] > u)
                hi = mid;
            else
                lo = mid + 1;
        }
        const int slot0 = s_sip[lo] + (u - s_sun[lo]) * p.unit_rows;
        int4 rec;
        rec.x = s_sad[lo];
        rec.y = s_srk[lo] | (s_sip[lo + 1] - s_sip[lo] >= kLongSegRows ? kUnitLongFlag : 0);
        rec.z = slot0;
        rec.w = min(p.unit_rows, s_sip[lo + 1] - slot0);
        reinterpret_cast<int4 *>(p.unit_rec)[u] = rec;
    }
    LORA_TS(p.trace, 7);
}

// Decode-sized batches (at most 64 requests, any number of adapter slots): one lane per request.
// Every request-level quantity is a sum over the other requests -- rows of requests with a smaller
// key (first slot of the segment), rows of earlier requests with the same key (stable order inside
// it), rows of the key (its shrink units), whether an earlier request has the key (first of its
// segment) -- so it is accumulated lane-parallel while the other requests' (key, rows) are
// broadcast one at a time from a scalar register (v_readlane: no LDS round trip, no scan, no
// histogram over the adapter slots).  Four waves take a quarter of the broadcasts each; a second
// pass over the first requests of the segments yields segment index and rank / unit prefixes.
constexpr int kTinyReq = 64;
constexpr int kTinyWaves = 4;

__global__ __launch_bounds__(kPlanThreads) void plan_tiny_kernel(PlanBuildArgs p) {
    __shared__ int s_p1[kTinyWaves][5][64];  // pass 1 partials: less, equal-before, rows of key, rows before, earlier-same flag
    __shared__ int s_p2[kTinyWaves][3][64];  // pass 2 partials: segments, ranks, units of smaller keys
    __shared__ unsigned long long s_rows[kTinyWaves];
    __shared__ int s_tot[kTinyWaves][2];     // ranks, units of all segments (per wave's share)
    __shared__ int s_tok[kTinyReq + 1], s_dst[kTinyReq], s_rseg[kTinyReq], s_a[kTinyReq];
    __shared__ int s_sad[kTinyReq + 1], s_sip[kTinyReq + 1], s_srk[kTinyReq + 1], s_sex[kTinyReq + 1], s_sun[kTinyReq + 1];
    __shared__ int s_hdr[4];  // status, segments, total ranks, total units
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int R = p.n_req, n_ad = p.n_adapters;

    // request state, kept by each of the four working waves
    int a = -1, L = 0, key = INT_MAX, rows = 0, rk = 0;
    bool bad = false, neg = false, active = false;
    if (wave < kTinyWaves) {
        const bool valid = lane < R;
        a = valid ? p.req_adapter[lane] : -1;
        L = valid ? p.req_ntok[lane] : 0;
        bad = valid && (a < -1 || a >= n_ad);
        neg = valid && !bad && L < 0;
        active = valid && !bad && !neg && L > 0;
        key = active ? (a < 0 ? n_ad : a) : INT_MAX;  // key n_ad = "no adapter"; idle lanes match nothing that counts
        rows = active ? L : 0;
        rk = (active && a >= 0) ? p.rank[a] : 0;  // wanted in pass 2 only: in flight during pass 1

        // ---- pass 1: this wave's quarter of the requests, broadcast one by one ----
        int less = 0, eqb = 0, h = 0, before = 0, earlier = 0;
        unsigned long long total = 0ull;
#pragma unroll
        for (int jj = 0; jj < 64 / kTinyWaves; ++jj) {
            const int j = wave * (64 / kTinyWaves) + jj;
            if (j < R) {
                const int kj = __builtin_amdgcn_readlane(key, j);
                const int Lj = __builtin_amdgcn_readlane(rows, j);
                const bool same = kj == key, prior = j < lane;
                less += kj < key ? Lj : 0;
                h += same ? Lj : 0;
                eqb += (same && prior) ? Lj : 0;
                before += prior ? Lj : 0;
                earlier |= (same && prior) ? 1 : 0;
                total += (unsigned long long)(unsigned)Lj;
            }
        }
        s_p1[wave][0][lane] = less;
        s_p1[wave][1][lane] = eqb;
        s_p1[wave][2][lane] = h;
        s_p1[wave][3][lane] = before;
        s_p1[wave][4][lane] = earlier;
        if (lane == 0) s_rows[wave] = total;
    }
    __syncthreads();

    int less = 0, eqb = 0, h = 0, before = 0, rkf = 0, units = 0, st = 0;
    bool first = false;
    if (wave < kTinyWaves) {
        int earlier = 0;
#pragma unroll
        for (int w = 0; w < kTinyWaves; ++w) {
            less += s_p1[w][0][lane];
            eqb += s_p1[w][1][lane];
            h += s_p1[w][2][lane];
            before += s_p1[w][3][lane];
            earlier |= s_p1[w][4][lane];
        }
        first = active && earlier == 0;
        // status, in the order and with the precedence of the general kernel (the smallest code wins)
        if (__builtin_amdgcn_ballot_w64(bad) != 0ull) st = min(st, kErrBadAdapterId);
        if (__builtin_amdgcn_ballot_w64(neg) != 0ull) st = min(st, kErrLengthMismatch);
        if (st == 0) {
            unsigned long long total = 0ull;
#pragma unroll
            for (int w = 0; w < kTinyWaves; ++w) total += s_rows[w];
            if (total != (unsigned long long)(unsigned)p.T) st = kErrLengthMismatch;
        }
        if (st == 0) {
            const bool seg_ad = first && a >= 0;
            const bool not_res = seg_ad && rk <= 0;
            const bool shape = seg_ad && rk > 0 && (rk & 7) != 0;
            const bool large = seg_ad && rk > 0 && (rk & 7) == 0 && rk > p.r_max;
            if (__builtin_amdgcn_ballot_w64(not_res) != 0ull) st = min(st, kErrNotResident);
            if (__builtin_amdgcn_ballot_w64(large) != 0ull) st = min(st, kErrRankTooLarge);
            if (__builtin_amdgcn_ballot_w64(shape) != 0ull) st = min(st, kErrShape);
            rkf = (seg_ad && !not_res && !shape && !large) ? rk : 0;
            units = seg_ad ? (h + p.unit_rows - 1) >> p.unit_shift : 0;
        }

        // ---- pass 2: the first requests of the segments (this wave's quarter), broadcast one by one ----
        const unsigned long long fmask = __builtin_amdgcn_ballot_w64(first);
        int seg = 0, ext = 0, un = 0, tot_ext = 0, tot_un = 0;
        if (st == 0) {
#pragma unroll
            for (int jj = 0; jj < 64 / kTinyWaves; ++jj) {
                const int j = wave * (64 / kTinyWaves) + jj;
                if ((fmask >> j) & 1ull) {
                    const int kj = __builtin_amdgcn_readlane(key, j);
                    const int rj = __builtin_amdgcn_readlane(rkf, j);
                    const int uj = __builtin_amdgcn_readlane(units, j);
                    const bool lt = kj < key;
                    seg += lt ? 1 : 0;
                    ext += lt ? rj : 0;
                    un += lt ? uj : 0;
                    tot_ext += rj;
                    tot_un += uj;
                }
            }
        }
        s_p2[wave][0][lane] = seg;
        s_p2[wave][1][lane] = ext;
        s_p2[wave][2][lane] = un;
        if (lane == 0) {
            s_tot[wave][0] = tot_ext;
            s_tot[wave][1] = tot_un;
        }
        if (wave == 0 && lane == 0) s_hdr[0] = st;  // every working wave computed the same status
    }
    __syncthreads();
    if (s_hdr[0] != 0) {
        if (tid == 0) write_failed(p, s_hdr[0]);
        return;
    }

    if (wave == 0) {  // publish: request arrays and segment arrays, to LDS for the fill below and to the plan
        int seg = 0, ext = 0, un = 0, c_ext = 0, c_unit = 0;
#pragma unroll
        for (int w = 0; w < kTinyWaves; ++w) {
            seg += s_p2[w][0][lane];
            ext += s_p2[w][1][lane];
            un += s_p2[w][2][lane];
            c_ext += s_tot[w][0];
            c_unit += s_tot[w][1];
        }
        const unsigned long long fmask = __builtin_amdgcn_ballot_w64(first);
        const int c_seg = __builtin_popcountll(fmask);
        if (lane < R) {
            s_tok[lane] = before;
            s_dst[lane] = less + eqb;
            s_rseg[lane] = seg;
            s_a[lane] = a;
            p.tok_off[lane] = before;
        }
        if (first) {
            s_sad[seg] = a >= 0 ? a : -1;
            s_sip[seg] = less;
            s_srk[seg] = rkf;
            s_sex[seg] = ext;
            s_sun[seg] = un;
            p.seg_adapter[seg] = a >= 0 ? a : -1;
            p.seg_indptr[seg] = less;
            p.seg_rank[seg] = rkf;
            p.seg_ext[seg] = ext;
            p.seg_unit[seg] = un;
        }
        if (lane == 0) {
            s_tok[R] = p.T;
            p.tok_off[R] = p.T;
            s_sip[c_seg] = p.T;
            s_sex[c_seg] = c_ext;
            s_sun[c_seg] = c_unit;
            p.seg_indptr[c_seg] = p.T;
            p.seg_ext[c_seg] = c_ext;
            p.seg_unit[c_seg] = c_unit;
            p.scalars[kScNSeg] = c_seg;
            p.scalars[kScStatus] = 0;
            p.scalars[kScEvicted] = 0;
            p.scalars[kScExtTotal] = c_ext;
            p.scalars[kScNUnits] = c_unit;
            p.scalars[kScT] = p.T;
            s_hdr[1] = c_seg;
            s_hdr[2] = c_ext;
            s_hdr[3] = c_unit;
        }
    }
    __syncthreads();
    const int c_seg = s_hdr[1], c_ext = s_hdr[2], c_unit = s_hdr[3];

    // per-row scatter, extension records, shrink work list: as in the small-batch kernel
    for (int t = tid; t < p.T; t += kPlanThreads) {
        int lo = 0, hi = R;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (s_tok[mid + 1] > t)
                hi = mid;
            else
                lo = mid + 1;
        }
        const int slot = s_dst[lo] + (t - s_tok[lo]);
        p.perm[slot] = t;
        p.row_seg[slot] = s_rseg[lo];
        p.row_adapter[t] = s_a[lo];
        p.row_ext[t] = pack_row_ext(s_sex[s_rseg[lo]], s_srk[s_rseg[lo]]);
    }
    for (int q = tid; q < (c_ext >> 3); q += kPlanThreads) {
        const int pel = q << 3;
        int lo = 0, hi = c_seg;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (s_sex[mid + 1] > pel)
                hi = mid;
            else
                lo = mid + 1;
        }
        int4 rec;
        rec.x = s_sad[lo];
        rec.y = (s_srk[lo] << 16) | (pel - s_sex[lo]);
        rec.z = s_sip[lo];
        rec.w = s_sip[lo + 1];
        reinterpret_cast<int4 *>(p.ext_rec)[q] = rec;
    }
    for (int u = tid; u < c_unit; u += kPlanThreads) {
        int lo = 0, hi = c_seg;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (s_sun[mid + 1] > u)
                hi = mid;
            else
                lo = mid + 1;
        }
        const int slot0 = s_sip[lo] + (u - s_sun[lo]) * p.unit_rows;
        int4 rec;
        rec.x = s_sad[lo];
        rec.y = s_srk[lo] | (s_sip[lo + 1] - s_sip[lo] >= kLongSegRows ? kUnitLongFlag : 0);
        rec.z = slot0;
        rec.w = min(p.unit_rows, s_sip[lo + 1] - slot0);
        reinterpret_cast<int4 *>(p.unit_rec)[u] = rec;
    }
}

// Up to 128 requests: the same one-lane-per-request scheme on more waves.  Wave (g, q), g < 2, keeps the requests
// 64 g .. 64 g + 63 (one per lane) and takes quarter q of the broadcasts: 16 lanes of each 64-request group of
// sources, read with v_readlane out of registers that hold (key, rows) of that group; the four waves of a
// group add their partial sums through LDS.  The second pass (first requests of the segments: segment index,
// rank and unit prefixes) needs flags of all groups, which go through LDS once.
constexpr int kMidReq = 128;  // (the work grows with the square of the request count: beyond this the scans of the general kernel win)
constexpr int kMidGroups = kMidReq / 64;
constexpr int kMidParts = kPlanWaves / kMidGroups;  // waves per group of 64 requests
constexpr int kMidLanes = 64 / kMidParts;            // source lanes of a group that one wave broadcasts

__global__ __launch_bounds__(kPlanThreads) void plan_mid_kernel(PlanBuildArgs p) {
    __shared__ int s_p1[kPlanWaves][5][64];  // pass 1 partials: less, equal-before, rows of key, rows before, earlier-same flag
    __shared__ int s_p2[kPlanWaves][3][64];  // pass 2 partials: segments, ranks, units of smaller keys
    __shared__ unsigned long long s_rows[kPlanWaves];
    __shared__ int s_tot[kPlanWaves][2];  // ranks, units of all segments (per wave's share)
    __shared__ int s_flag[kMidGroups][5];  // per group: any bad id, negative length, not resident, rank too large, bad rank
    __shared__ int s_first[kMidReq], s_rkf[kMidReq], s_units[kMidReq];
    __shared__ int s_tok[kMidReq + 1], s_dst[kMidReq], s_rseg[kMidReq], s_a[kMidReq];
    __shared__ int s_sad[kMidReq + 1], s_sip[kMidReq + 1], s_srk[kMidReq + 1], s_sex[kMidReq + 1], s_sun[kMidReq + 1];
    __shared__ int s_hdr[4];  // status, segments, total ranks, total units
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = wave / kMidParts, q = wave % kMidParts;
    const int R = p.n_req, n_ad = p.n_adapters;
    const int G = (R + 63) >> 6;  // groups in use

    // (key, rows) of a request; key n_ad = "no adapter", idle or invalid requests match nothing that counts
    auto classify = [&](int j, int &a, int &L, bool &bad, bool &neg, bool &active, int &key, int &rows) {
        const bool valid = j < R;
        a = valid ? p.req_adapter[j] : -1;
        L = valid ? p.req_ntok[j] : 0;
        bad = valid && (a < -1 || a >= n_ad);
        neg = valid && !bad && L < 0;
        active = valid && !bad && !neg && L > 0;
        key = active ? (a < 0 ? n_ad : a) : INT_MAX;
        rows = active ? L : 0;
    };
    // this lane's own request, and the sources of every group
    const int i = 64 * g + lane;
    int a, L, key, rows;
    bool bad, neg, active;
    classify(i, a, L, bad, neg, active, key, rows);
    const int rk = (active && a >= 0) ? p.rank[a] : 0;  // wanted after pass 1 only: in flight during it
    int skey[kMidGroups], srow[kMidGroups];
#pragma unroll
    for (int sg = 0; sg < kMidGroups; ++sg) {
        int a2, L2;
        bool b2, n2, act2;
        classify(64 * sg + lane, a2, L2, b2, n2, act2, skey[sg], srow[sg]);
    }

    // ---- pass 1: this wave's quarter of every group of sources, broadcast one by one ----
    {
        int less = 0, eqb = 0, h = 0, before = 0, earlier = 0;
        unsigned long long total = 0ull;
#pragma unroll
        for (int sg = 0; sg < kMidGroups; ++sg) {
            if (sg < G) {
#pragma unroll
                for (int jj = 0; jj < kMidLanes; ++jj) {
                    const int l2 = q * kMidLanes + jj, j = 64 * sg + l2;
                    if (j < R) {
                        const int kj = __builtin_amdgcn_readlane(skey[sg], l2);
                        const int Lj = __builtin_amdgcn_readlane(srow[sg], l2);
                        const bool same = kj == key, prior = j < i;
                        less += kj < key ? Lj : 0;
                        h += same ? Lj : 0;
                        eqb += (same && prior) ? Lj : 0;
                        before += prior ? Lj : 0;
                        earlier |= (same && prior) ? 1 : 0;
                        total += (unsigned long long)(unsigned)Lj;
                    }
                }
            }
        }
        s_p1[wave][0][lane] = less;
        s_p1[wave][1][lane] = eqb;
        s_p1[wave][2][lane] = h;
        s_p1[wave][3][lane] = before;
        s_p1[wave][4][lane] = earlier;
        if (lane == 0) s_rows[wave] = total;
    }
    __syncthreads();

    int less = 0, eqb = 0, h = 0, before = 0, earlier = 0;
#pragma unroll
    for (int w = 0; w < kMidParts; ++w) {
        less += s_p1[g * kMidParts + w][0][lane];
        eqb += s_p1[g * kMidParts + w][1][lane];
        h += s_p1[g * kMidParts + w][2][lane];
        before += s_p1[g * kMidParts + w][3][lane];
        earlier |= s_p1[g * kMidParts + w][4][lane];
    }
    const bool first = active && earlier == 0;
    const bool seg_ad = first && a >= 0;
    const bool not_res = seg_ad && rk <= 0;
    const bool shape = seg_ad && rk > 0 && (rk & 7) != 0;
    const bool large = seg_ad && rk > 0 && (rk & 7) == 0 && rk > p.r_max;
    const int rkf = (seg_ad && !not_res && !shape && !large) ? rk : 0;
    const int units = seg_ad ? (h + p.unit_rows - 1) >> p.unit_shift : 0;
    if (q == 0) {  // one wave per group passes the group's flags and per-request values on
        const int f0 = __builtin_amdgcn_ballot_w64(bad) != 0ull, f1 = __builtin_amdgcn_ballot_w64(neg) != 0ull;
        const int f2 = __builtin_amdgcn_ballot_w64(not_res) != 0ull, f3 = __builtin_amdgcn_ballot_w64(large) != 0ull;
        const int f4 = __builtin_amdgcn_ballot_w64(shape) != 0ull;
        if (lane == 0) {
            s_flag[g][0] = f0;
            s_flag[g][1] = f1;
            s_flag[g][2] = f2;
            s_flag[g][3] = f3;
            s_flag[g][4] = f4;
        }
        s_first[i] = first ? 1 : 0;
        s_rkf[i] = rkf;
        s_units[i] = units;
    }
    __syncthreads();

    // status, in the order and with the precedence of the general kernel (the smallest code wins)
    int st = 0;
    {
        int any[5] = {0, 0, 0, 0, 0};
#pragma unroll
        for (int sg = 0; sg < kMidGroups; ++sg)
#pragma unroll
            for (int f = 0; f < 5; ++f) any[f] |= s_flag[sg][f];
        if (any[0]) st = min(st, kErrBadAdapterId);
        if (any[1]) st = min(st, kErrLengthMismatch);
        if (st == 0) {
            unsigned long long total = 0ull;
#pragma unroll
            for (int w = 0; w < kMidParts; ++w) total += s_rows[w];  // the waves of a group cover every source once
            if (total != (unsigned long long)(unsigned)p.T) st = kErrLengthMismatch;
        }
        if (st == 0) {
            if (any[2]) st = min(st, kErrNotResident);
            if (any[3]) st = min(st, kErrRankTooLarge);
            if (any[4]) st = min(st, kErrShape);
        }
    }
    if (st != 0) {  // (uniform over the workgroup)
        if (tid == 0) write_failed(p, st);
        return;
    }

    // ---- pass 2: the first requests of the segments, this wave's quarter of every group, broadcast one by one ----
    unsigned long long fmask[kMidGroups];
    int c_seg = 0;
    {
        int srk[kMidGroups], sun[kMidGroups];
#pragma unroll
        for (int sg = 0; sg < kMidGroups; ++sg) {
            fmask[sg] = __builtin_amdgcn_ballot_w64(s_first[64 * sg + lane] != 0);
            srk[sg] = s_rkf[64 * sg + lane];
            sun[sg] = s_units[64 * sg + lane];
            c_seg += __builtin_popcountll(fmask[sg]);
        }
        int seg = 0, ext = 0, un = 0, tot_ext = 0, tot_un = 0;
#pragma unroll
        for (int sg = 0; sg < kMidGroups; ++sg) {
            if (sg < G) {
#pragma unroll
                for (int jj = 0; jj < kMidLanes; ++jj) {
                    const int l2 = q * kMidLanes + jj;
                    if ((fmask[sg] >> l2) & 1ull) {
                        const int kj = __builtin_amdgcn_readlane(skey[sg], l2);
                        const int rj = __builtin_amdgcn_readlane(srk[sg], l2);
                        const int uj = __builtin_amdgcn_readlane(sun[sg], l2);
                        const bool lt = kj < key;
                        seg += lt ? 1 : 0;
                        ext += lt ? rj : 0;
                        un += lt ? uj : 0;
                        tot_ext += rj;
                        tot_un += uj;
                    }
                }
            }
        }
        s_p2[wave][0][lane] = seg;
        s_p2[wave][1][lane] = ext;
        s_p2[wave][2][lane] = un;
        if (lane == 0) {
            s_tot[wave][0] = tot_ext;
            s_tot[wave][1] = tot_un;
        }
    }
    __syncthreads();

    if (q == 0) {  // publish: request arrays and segment arrays, to LDS for the fill below and to the plan
        int seg = 0, ext = 0, un = 0, c_ext = 0, c_unit = 0;
#pragma unroll
        for (int w = 0; w < kMidParts; ++w) {
            seg += s_p2[g * kMidParts + w][0][lane];
            ext += s_p2[g * kMidParts + w][1][lane];
            un += s_p2[g * kMidParts + w][2][lane];
            c_ext += s_tot[w][0];  // (the waves of a group cover every source once)
            c_unit += s_tot[w][1];
        }
        if (i < R) {
            s_tok[i] = before;
            s_dst[i] = less + eqb;
            s_rseg[i] = seg;
            s_a[i] = a;
            p.tok_off[i] = before;
        }
        if (first) {
            s_sad[seg] = a >= 0 ? a : -1;
            s_sip[seg] = less;
            s_srk[seg] = rkf;
            s_sex[seg] = ext;
            s_sun[seg] = un;
            p.seg_adapter[seg] = a >= 0 ? a : -1;
            p.seg_indptr[seg] = less;
            p.seg_rank[seg] = rkf;
            p.seg_ext[seg] = ext;
            p.seg_unit[seg] = un;
        }
        if (wave == 0 && lane == 0) {
            s_tok[R] = p.T;
            p.tok_off[R] = p.T;
            s_sip[c_seg] = p.T;
            s_sex[c_seg] = c_ext;
            s_sun[c_seg] = c_unit;
            p.seg_indptr[c_seg] = p.T;
            p.seg_ext[c_seg] = c_ext;
            p.seg_unit[c_seg] = c_unit;
            p.scalars[kScNSeg] = c_seg;
            p.scalars[kScStatus] = 0;
            p.scalars[kScEvicted] = 0;
            p.scalars[kScExtTotal] = c_ext;
            p.scalars[kScNUnits] = c_unit;
            p.scalars[kScT] = p.T;
            s_hdr[1] = c_seg;
            s_hdr[2] = c_ext;
            s_hdr[3] = c_unit;
        }
    }
    __syncthreads();
    const int c_ext = s_hdr[2], c_unit = s_hdr[3];

    // per-row scatter, extension records, shrink work list: as in the small-batch kernel
    for (int t = tid; t < p.T; t += kPlanThreads) {
        int lo = 0, hi = R;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (s_tok[mid + 1] > t)
                hi = mid;
            else
                lo = mid + 1;
        }
        const int slot = s_dst[lo] + (t - s_tok[lo]);
        p.perm[slot] = t;
        p.row_seg[slot] = s_rseg[lo];
        p.row_adapter[t] = s_a[lo];
        p.row_ext[t] = pack_row_ext(s_sex[s_rseg[lo]], s_srk[s_rseg[lo]]);
    }
    for (int u = tid; u < (c_ext >> 3); u += kPlanThreads) {
        const int pel = u << 3;
        int lo = 0, hi = c_seg;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (s_sex[mid + 1] > pel)
                hi = mid;
            else
                lo = mid + 1;
        }
        int4 rec;
        rec.x = s_sad[lo];
        rec.y = (s_srk[lo] << 16) | (pel - s_sex[lo]);
        rec.z = s_sip[lo];
        rec.w = s_sip[lo + 1];
        reinterpret_cast<int4 *>(p.ext_rec)[u] = rec;
    }
    for (int u = tid; u < c_unit; u += kPlanThreads) {
        int lo = 0, hi = c_seg;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (s_sun[mid + 1] > u)
                hi = mid;
            else
                lo = mid + 1;
        }
        const int slot0 = s_sip[lo] + (u - s_sun[lo]) * p.unit_rows;
        int4 rec;
        rec.x = s_sad[lo];
        rec.y = s_srk[lo] | (s_sip[lo + 1] - s_sip[lo] >= kLongSegRows ? kUnitLongFlag : 0);
        rec.z = slot0;
        rec.w = min(p.unit_rows, s_sip[lo + 1] - slot0);
        reinterpret_cast<int4 *>(p.unit_rec)[u] = rec;
    }
}

__global__ __launch_bounds__(256) void plan_fill_kernel(PlanBuildArgs p) {
    if (p.scalars[kScStatus] != 0) return;
    const int start = blockIdx.x * 256 + threadIdx.x;
    const int stride = gridDim.x * 256;
    fill_rows(p, start, stride);
    fill_ext(p, start, stride);
    fill_units(p, start, stride);
}

}  // namespace

hipError_t launch_plan_build(const PlanBuildArgs &a, bool fuse_fill, int variant, hipStream_t stream, const KernelTimer *timers) {
    if (fuse_fill && variant != 1 && a.n_req <= kTinyReq && a.T <= kSmallRows)
        return launch_kernel(plan_tiny_kernel, dim3(1), dim3(kPlanThreads), 0, stream, timers ? &timers[0] : nullptr, a);
    if (fuse_fill && variant != 1 && a.n_req <= kMidReq && a.T <= kSmallRows)
        return launch_kernel(plan_mid_kernel, dim3(1), dim3(kPlanThreads), 0, stream, timers ? &timers[0] : nullptr, a);
    if (fuse_fill && a.n_req <= kSmallReq && a.n_adapters + 1 <= kSmallKeys && a.T <= kSmallRows) {
#ifdef LORA_TRACE
        return trace_launch("plan_small", 1, [&](long long *buf) {
            PlanBuildArgs b = a;
            b.trace = buf;
            return launch_kernel(plan_small_kernel, dim3(1), dim3(kPlanThreads), 0, stream, timers ? &timers[0] : nullptr, b);
        });
#else
        return launch_kernel(plan_small_kernel, dim3(1), dim3(kPlanThreads), 0, stream, timers ? &timers[0] : nullptr, a);
#endif
    }
    hipError_t e = launch_kernel(plan_segments_kernel, dim3(1), dim3(kPlanThreads), 0, stream, timers ? &timers[0] : nullptr, a,
                                 fuse_fill ? 1 : 0);
    if (e != hipSuccess) return e;
    if (!fuse_fill) {
        long work = a.T > (long)a.ext_cap ? (long)a.T : (long)a.ext_cap;
        int grid = (int)((work + 255) / 256);
        if (grid < 1) grid = 1;
        if (grid > 2048) grid = 2048;
        e = launch_kernel(plan_fill_kernel, dim3(grid), dim3(256), 0, stream, timers ? &timers[1] : nullptr, a);
    }
    return e;
}

}  // namespace lora
