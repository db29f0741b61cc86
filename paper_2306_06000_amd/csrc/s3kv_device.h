// Device-side helpers shared by the attention kernels of libs3kv (gfx950): kernel arguments, bounds
// checks of the device arrays, lane reductions, 16-bit dot / accumulate steps, output stores, the
// LDS batch view (work list) and the chunk-partial merge.  Included by the .hip files only.
#pragma once
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "s3kv_internal.h"

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

#define S3_MAX_BATCH 4095

struct AttnArgs {
    char *kplane;
    char *vplane;
    const char *q;
    const int64_t *slot_off;
    const int32_t *cur_len;  // rows to attend minus len_add
    void *out;
    float *part_acc;   // [n][max_chunks][H][D]
    float2 *part_ml;   // [n][max_chunks][H]  (running max in log2 units, sum)
    int64_t n_tokens;  // arena capacity N
    int32_t n, H, chunk, max_chunks, out_dtype, max_len;  // H: heads of a K/V row
    int32_t Hq;            // query heads (= H unless grouped-query / multi-query attention)
    int32_t ncls;          // length classes of the work order (1..8)
    int32_t len_add;    // 0: cur_len is the context length; 1 (fused step): cur_len is the append position
    float scale_log2e;  // scale * log2(e): scores are kept in log2 units so that exp is v_exp_f32
    // fused step only
    const char *k_new;
    const char *v_new;
    int32_t *len_out;        // may be null
    unsigned int *arrivals;  // [n][n_hgb] chunk-arrival counters, zero between launches
    int32_t merge_sync;      // how chunks that meet inside one launch are ordered: see chunk_arrived()
    int32_t merge_in_kernel; // matrix-core kernel for shared heads: chunks meet inside the launch (no merge launch follows)
    unsigned int *queue;     // [2] kernels with a dynamic work list: positions claimed, workgroups gone; zero between launches
    int32_t stream_k;        // matrix-core kernel for shared heads: K rows with the streaming hint (1), plain (0), by launch size (< 0)
    int32_t dyn_list;        // matrix-core kernel for shared heads: per cent of the list dealt by stride before waves claim positions from `queue` (0: all by stride)
};

__device__ __forceinline__ int checked_len(const AttnArgs &a, int b) {
    const int64_t off = a.slot_off[b];
    const int32_t raw = a.cur_len[b];
    const int64_t len = (int64_t)raw + a.len_add;
    const bool ok = off >= 0 && raw >= 0 && len <= a.max_len && off + len <= a.n_tokens;
    return ok ? (int)len : 0;
}

template <int CTRL>
__device__ __forceinline__ float dpp_sum_step(float v) {
    const int bits = __builtin_bit_cast(int, v);
    const int moved = __builtin_amdgcn_update_dpp(0, bits, CTRL, 0xF, 0xF, true);
    return v + __builtin_bit_cast(float, moved);
}

// Sum over groups of LANES adjacent lanes (4, 8, 16 or 32); every lane of a group gets the sum.
template <int LANES>
__device__ __forceinline__ float group_sum(float v) {
    v = dpp_sum_step<0xB1>(v);   // quad_perm [1,0,3,2]: lane ^ 1
    v = dpp_sum_step<0x4E>(v);   // quad_perm [2,3,0,1]: lane ^ 2
    if (LANES >= 8) v = dpp_sum_step<0x141>(v);  // row_half_mirror: the other quad of each 8
    if (LANES >= 16) v = dpp_sum_step<0x140>(v);  // row_mirror: the other 8 of each 16
    if (LANES >= 32) {
        const int bits = __builtin_bit_cast(int, v);
        const int other = __builtin_amdgcn_ds_swizzle(bits, 0x401F);  // lane ^ 16
        v += __builtin_bit_cast(float, other);
    }
    return v;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Note: __builtin_bit_cast applied directly to a vector-element expression (v[i]) reads element 0
// with this compiler, so elements are always copied into a scalar first.
template <int DT>
__device__ __forceinline__ float dot8(const u32x4 a, const u32x4 b) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const unsigned ai = a[i], bi = b[i];
        if (DT == S3_F16)
            s = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, ai), __builtin_bit_cast(f16x2, bi), s, false);
        else
            s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, ai), __builtin_bit_cast(bf16x2, bi), s, false);
    }
    return s;
}

template <int DT>
__device__ __forceinline__ void axpy8(float (&acc)[8], const float p, const u32x4 v) {
#pragma unroll
    for (int i = 0; i < 4; i++) {
        float lo, hi;
        const unsigned vi = v[i];
        if (DT == S3_F16) {
            const f16x2 h = __builtin_bit_cast(f16x2, vi);
            lo = (float)h[0];
            hi = (float)h[1];
        } else {
            const unsigned lo_bits = vi << 16, hi_bits = vi & 0xFFFF0000u;
            lo = __builtin_bit_cast(float, lo_bits);
            hi = __builtin_bit_cast(float, hi_bits);
        }
        acc[2 * i] = fmaf(p, lo, acc[2 * i]);
        acc[2 * i + 1] = fmaf(p, hi, acc[2 * i + 1]);
    }
}

__device__ __forceinline__ unsigned f32_to_bf16_rne(float f) {
    unsigned u = __builtin_bit_cast(unsigned, f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;  // NaN stays NaN
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// Store 8 consecutive output elements starting at element index e of `out`.
__device__ __forceinline__ void store_out8(void *out, int out_dtype, int64_t e, const float (&v)[8]) {
    if (out_dtype == S3_F32) {
        f32x4 *p = (f32x4 *)((float *)out + e);
        p[0] = (f32x4){v[0], v[1], v[2], v[3]};
        p[1] = (f32x4){v[4], v[5], v[6], v[7]};
    } else {
        u32x4 w;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            if (out_dtype == S3_F16) {
                const f16x2 h = {(_Float16)v[2 * i], (_Float16)v[2 * i + 1]};
                const unsigned packed = __builtin_bit_cast(unsigned, h);
                w[i] = packed;
            } else {
                w[i] = f32_to_bf16_rne(v[2 * i]) | (f32_to_bf16_rne(v[2 * i + 1]) << 16);
            }
        }
        *(u32x4 *)((uint16_t *)out + e) = w;
    }
}

template <bool NT>
__device__ __forceinline__ u32x4 load16(const char *p) {
    return NT ? __builtin_nontemporal_load((const u32x4 *)p) : *(const u32x4 *)p;
}

// Work order of a launch: longest contexts first.  Contexts are put into `ncls` length classes
// relative to the longest context of the batch; the work list holds the chunks of class 0 (the longest)
// in batch order, then class 1, and so on.  Long items therefore start first and the short ones fill
// the end of the kernel (a ragged batch in random order ran 10 % slower), and the cross-workgroup
// merges of multi-chunk contexts overlap with the streaming of the rest.  The whole workgroup builds
// one exclusive prefix sum of chunk counts per class in LDS: pre[c][0..n] at cum[c * (n + 1)].
#define S3_MAX_CLASSES 8
#define S3_MAX_WAVES 16

__device__ __forceinline__ int chunks_of(const AttnArgs &a, int b, int chunk) {
    return (checked_len(a, b) + chunk - 1) / chunk;
}

__device__ __forceinline__ int class_of(int len, int max_len_seen, int ncls) {
    return ncls - 1 - min(ncls - 1, len * ncls / (max_len_seen + 1));  // len * ncls < 2^31: len <= max_len <= 2^20
}

// Inclusive prefix sum over the 64 lanes of a wave with DPP row operations (no LDS round trips):
// shifts by 1, 2, 4, 8 inside each row of 16 lanes, then the row totals are carried into the
// following rows (row_bcast:15 into rows 1 and 3, row_bcast:31 into rows 2 and 3).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_scan_step(int v) {
    return v + __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xF, false);
}
__device__ __forceinline__ int wave_inclusive_scan(int v) {
    v = dpp_scan_step<0x111, 0xF>(v);  // row_shr:1
    v = dpp_scan_step<0x112, 0xF>(v);  // row_shr:2
    v = dpp_scan_step<0x114, 0xF>(v);  // row_shr:4
    v = dpp_scan_step<0x118, 0xF>(v);  // row_shr:8
    v = dpp_scan_step<0x142, 0xA>(v);  // row_bcast:15 -> rows 1, 3
    v = dpp_scan_step<0x143, 0xC>(v);  // row_bcast:31 -> rows 2, 3
    return v;
}

// Maximum of a non-negative value over the 64 lanes, same DPP ladder (lanes shifted in from outside a
// row read as 0, the identity here); every lane gets the result.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_max_step(int v) {
    return max(v, __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xF, false));
}
__device__ __forceinline__ int wave_max_nonneg(int v) {
    v = dpp_max_step<0x111, 0xF>(v);
    v = dpp_max_step<0x112, 0xF>(v);
    v = dpp_max_step<0x114, 0xF>(v);
    v = dpp_max_step<0x118, 0xF>(v);
    v = dpp_max_step<0x142, 0xA>(v);
    v = dpp_max_step<0x143, 0xC>(v);
    return __builtin_amdgcn_readlane(v, 63);
}

// LDS picture of the batch built by every workgroup at kernel start (dynamic shared memory):
//   off[n] (int64), len[n] (int32, 0 for refused entries), pre[ncls][n + 1] (int32)
struct BatchView {
    const int64_t *off;
    const int *len;
    const int *pre;
    int n, ncls, total;
};

__device__ __forceinline__ size_t batch_view_bytes(int n, int ncls) {
    return (size_t)n * 8 + (size_t)((n + 1) & ~1) * 4 + (size_t)ncls * (n + 1) * 4;
}

// The one-wave build of the view: lane l owns entries l*E .. l*E+E-1 (n <= 64*E).
template <int E>
__device__ __forceinline__ void one_wave_view(const AttnArgs &a, int64_t *off_s, int *len_s, int *pre) {
    const int lane = threadIdx.x & 63;
    const int ncls = a.ncls, chunk = a.chunk, n = a.n;
    int len[E], cls[E], cnt[E];
    int mx = 0;
#pragma unroll
    for (int e = 0; e < E; e++) {
        const int b = lane * E + e;
        len[e] = 0;
        if (b < n) {
            len[e] = checked_len(a, b);
            len_s[b] = len[e];
            off_s[b] = a.slot_off[b];
        }
        mx = max(mx, len[e]);
    }
    mx = wave_max_nonneg(mx);
#pragma unroll
    for (int e = 0; e < E; e++) {
        cls[e] = class_of(len[e], mx, ncls);
        cnt[e] = (len[e] + chunk - 1) / chunk;
    }
    for (int c = 0; c < ncls; c++) {
        int loc[E], lsum = 0;
#pragma unroll
        for (int e = 0; e < E; e++) {
            loc[e] = lsum;
            if (cls[e] == c) lsum += cnt[e];
        }
        const int incl = wave_inclusive_scan(lsum);
#pragma unroll
        for (int e = 0; e < E; e++) {
            const int b = lane * E + e;
            if (b < n) pre[c * (n + 1) + b] = incl - lsum + loc[e];
        }
        if (lane == 63) pre[c * (n + 1) + n] = incl;
    }
}

// One pass over the device arrays (each entry is read from global memory once and checked once),
// then class-wise exclusive prefix sums of the chunk counts.
__device__ __forceinline__ BatchView build_batch_view(const AttnArgs &a, char *dyn, int *wave_sums) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nthreads = blockDim.x, nwaves = nthreads >> 6;
    const int ncls = a.ncls, chunk = a.chunk, n = a.n;
    int64_t *off_s = (int64_t *)dyn;
    int *len_s = (int *)(dyn + (size_t)n * 8);
    int *pre = len_s + ((n + 1) & ~1);
    if (n <= 64 * 8) {
        // Batches of up to 512 sequences: wave 0 builds the whole view by itself (lane l takes entries
        // l*E .. l*E+E-1; a serial prefix inside the lane, one DPP scan across lanes per class) and the
        // workgroup meets at ONE barrier.  The general path below needs four barriers and LDS round trips
        // between them, which cost every workgroup of a small launch about 1.5 us before its first load.
        // E is a compile-time constant per batch size class: the per-entry work (two integer divisions) is
        // not spent on entries a small batch does not have.
        if (wave == 0) {
            if (n <= 64) one_wave_view<1>(a, off_s, len_s, pre);
            else if (n <= 128) one_wave_view<2>(a, off_s, len_s, pre);
            else if (n <= 256) one_wave_view<4>(a, off_s, len_s, pre);
            else one_wave_view<8>(a, off_s, len_s, pre);
        }
        __syncthreads();
        BatchView v;
        v.off = off_s;
        v.len = len_s;
        v.pre = pre;
        v.n = n;
        v.ncls = ncls;
        v.total = 0;
        for (int c = 0; c < ncls; c++) v.total += pre[c * (n + 1) + n];
        return v;
    }
    const int per = (n + nthreads - 1) / nthreads;
    const int b0 = min(n, tid * per), b1 = min(n, b0 + per);
    int mx = 0;
    for (int b = b0; b < b1; b++) {
        const int len = checked_len(a, b);
        len_s[b] = len;
        off_s[b] = a.slot_off[b];
        mx = max(mx, len);
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) mx = max(mx, __shfl_xor(mx, d));
    if (lane == 0) wave_sums[wave] = mx;
    __syncthreads();
    for (int i = 0; i < nwaves; i++) mx = max(mx, wave_sums[i]);
    __syncthreads();  // wave_sums is reused below
    int cnt[S3_MAX_CLASSES], incl[S3_MAX_CLASSES];
#pragma unroll
    for (int c = 0; c < S3_MAX_CLASSES; c++) cnt[c] = 0;
    for (int b = b0; b < b1; b++) {
        const int len = len_s[b];
        const int k = (len + chunk - 1) / chunk;
        const int cl = class_of(len, mx, ncls);
#pragma unroll
        for (int c = 0; c < S3_MAX_CLASSES; c++) cnt[c] += (c == cl) ? k : 0;
    }
#pragma unroll
    for (int c = 0; c < S3_MAX_CLASSES; c++) {
        if (c < ncls) {  // uniform
            const int v = wave_inclusive_scan(cnt[c]);
            incl[c] = v;
            if (lane == 63) wave_sums[c * S3_MAX_WAVES + wave] = v;
        }
    }
    __syncthreads();
    int run[S3_MAX_CLASSES];
#pragma unroll
    for (int c = 0; c < S3_MAX_CLASSES; c++) {
        run[c] = 0;
        if (c < ncls) {
            int base = 0;
            for (int i = 0; i < wave; i++) base += wave_sums[c * S3_MAX_WAVES + i];
            run[c] = base + incl[c] - cnt[c];
        }
    }
    for (int b = b0; b < b1; b++) {
        const int len = len_s[b];
        const int k = (len + chunk - 1) / chunk;
        const int cl = class_of(len, mx, ncls);
#pragma unroll
        for (int c = 0; c < S3_MAX_CLASSES; c++) {
            if (c < ncls) pre[c * (n + 1) + b] = run[c];
            run[c] += (c == cl) ? k : 0;
        }
    }
    if (tid == nthreads - 1) {
#pragma unroll
        for (int c = 0; c < S3_MAX_CLASSES; c++)
            if (c < ncls) pre[c * (n + 1) + n] = run[c];
    }
    __syncthreads();
    BatchView v;
    v.off = off_s;
    v.len = len_s;
    v.pre = pre;
    v.n = n;
    v.ncls = ncls;
    v.total = 0;
    for (int c = 0; c < ncls; c++) v.total += pre[c * (n + 1) + n];
    return v;
}

// Partials that cross workgroups inside ONE launch (fused step) must not sit in a cache that
// another XCD cannot see: they are written and read with volatile 64- and 128-bit vector accesses,
// which on gfx950 are plain stores / loads marked to go through to memory-side coherence.  No cache
// write-back or invalidate is needed then (those cost far more than the partials themselves).
typedef float f32x2 __attribute__((ext_vector_type(2)));
template <bool COHERENT>
__device__ __forceinline__ void put_partial4(float *p, const f32x4 v) {
    if (COHERENT) *(volatile f32x4 *)p = v;
    else *(f32x4 *)p = v;
}
template <bool COHERENT>
__device__ __forceinline__ void put_partial2(float *p, const f32x2 v) {
    if (COHERENT) *(volatile f32x2 *)p = v;
    else *(f32x2 *)p = v;
}
template <bool COHERENT>
__device__ __forceinline__ f32x4 get_partial4(const float *p) {
    if (COHERENT) return *(const volatile f32x4 *)p;
    return *(const f32x4 *)p;
}
template <bool COHERENT>
__device__ __forceinline__ f32x2 get_partial2(const float *p) {
    if (COHERENT) return *(const volatile f32x2 *)p;
    return *(const f32x2 *)p;
}

// A wave has written its chunk's partial: count the chunk on the context's arrival counter.  Returns true
// (to every lane) in the wave that delivered the LAST chunk of the context; that wave then merges the chunks,
// and the counter is back at zero for the next launch.  Called by whole waves in uniform control flow.
// Two orderings of "my partial is visible before my count, the others' partials are visible after theirs":
//   merge_sync 0  the partials are written and read with the write-through / cache-bypassing accesses above,
//                 so they are at the memory side once this wave's vector-memory counter has drained
//                 (s_waitcnt 0); the counter is a relaxed device-scope atomic.  This rests on `volatile`
//                 vector accesses being emitted with the sc0 sc1 cache bits on gfx950 (a host-side test
//                 compiles these helpers and checks the bits in the emitted code).
//   merge_sync 1  the same accesses, ordered by the memory model instead: a device-scope release fence
//                 before the count and an acquire fence in the wave that merges (L2 write-back and
//                 invalidate on this device, which cost far more than the partials themselves).
__device__ __forceinline__ bool chunk_arrived(const AttnArgs &a, unsigned int *cnt, int nchunks) {
    const int lane = threadIdx.x & 63;
    if (a.merge_sync) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    else __builtin_amdgcn_s_waitcnt(0);  // this wave's partial stores have completed
    unsigned int old = 0;
    if (lane == 0) old = atomicAdd(cnt, 1u);
    old = __builtin_amdgcn_readfirstlane(old);
    if (old != (unsigned int)(nchunks - 1)) return false;
    if (lane == 0) atomicExch(cnt, 0u);  // leave the counter clean for the next launch
    if (a.merge_sync) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    return true;
}

// Merge the chunk partials of (sequence b, head h) for this lane's 8-element slice and store the
// final output row slice; H is the head count of the partial and output arrays.  nchunks >= 2.  Four chunks are loaded per round so that the (cache
// bypassing) loads of a round are in flight together.
template <int D, bool COHERENT>
__device__ __forceinline__ void merge_chunks(const AttnArgs &a, int H, int b, int h, int dl, int nchunks) {
    const int64_t p0 = ((int64_t)b * a.max_chunks) * H + h;
    const float *ml = (const float *)a.part_ml;
    float mm = -INFINITY, l = 0.f;
    float o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int c0 = 0; c0 < nchunks; c0 += 4) {
        float mv[4], lv[4], av[4][8];
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const int64_t pi = p0 + (int64_t)min(c0 + u, nchunks - 1) * H;
            const f32x2 mlv = get_partial2<COHERENT>(ml + 2 * pi);
            mv[u] = mlv[0];
            lv[u] = mlv[1];
            const float *pa = a.part_acc + pi * D + dl * 8;
            const f32x4 lo = get_partial4<COHERENT>(pa), hi = get_partial4<COHERENT>(pa + 4);
#pragma unroll
            for (int i = 0; i < 4; i++) {
                av[u][i] = lo[i];
                av[u][4 + i] = hi[i];
            }
        }
        float mn = mm;
#pragma unroll
        for (int u = 0; u < 4; u++) mn = fmaxf(mn, mv[u]);  // repeats of the last chunk do not change the max
        const float alpha = fast_exp2(mm - mn);
        l *= alpha;
#pragma unroll
        for (int i = 0; i < 8; i++) o[i] *= alpha;
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const float wgt = (c0 + u < nchunks) ? fast_exp2(mv[u] - mn) : 0.f;
            l += wgt * lv[u];
#pragma unroll
            for (int i = 0; i < 8; i++) o[i] += wgt * av[u][i];
        }
        mm = mn;
    }
    const float inv = 1.f / l;
#pragma unroll
    for (int i = 0; i < 8; i++) o[i] *= inv;
    store_out8(a.out, a.out_dtype, ((int64_t)b * H + h) * D + dl * 8, o);
}

// What a workgroup item is: chunk c of sequence b for head block hgb.
struct Item {
    int b, c, nchunks, len, hgb;
    int clen;  // rows per chunk of this context: the context is cut into nchunks near-equal pieces
    int64_t off;
};

// Rows per chunk when a context of len rows is cut into nchunks pieces: near-equal pieces; falls
// back to `chunk` if rounding would leave the last piece empty.
__device__ __forceinline__ int balanced_chunk_len(int len, int nchunks, int chunk) {
    if (nchunks <= 1) return chunk;
    const int clen = (len + nchunks - 1) / nchunks;
    return (nchunks - 1) * clen < len ? clen : chunk;
}

// Rows [j0, j1) of item `it` that token split ts of TS takes: the item's rows are divided evenly
// (split 0 is never empty; trailing splits may be).
__device__ __forceinline__ void split_rows(const Item &it, int ts, int TS, int &j0, int &j1) {
    const int start = it.c * it.clen;
    const int end = min(it.len, start + it.clen);
    const int per = (end - start + TS - 1) / TS;
    j0 = min(end, start + ts * per);
    j1 = min(end, j0 + per);
}

// Work-list position -> item.  Called by whole waves (every lane with the same `item`): the class
// totals are read by the first lanes at once and the sequence is found by counting, lanes in parallel,
// the entries whose inclusive prefix does not exceed the position (the prefix sums are non-decreasing,
// so that count is the first sequence whose range holds it): three dependent LDS round trips
// instead of a serial class walk plus a binary search.
__device__ __forceinline__ Item decode_item(const AttnArgs &a, const BatchView &v, int64_t item, int n_hgb) {
    Item it;
    const int lane = threadIdx.x & 63;
    int w = (int)(item / n_hgb);
    it.hgb = (int)(item - (int64_t)w * n_hgb);
    const int tot = lane < v.ncls ? v.pre[lane * (v.n + 1) + v.n] : 0;
    int cls = v.ncls - 1;
    for (int c = 0; c < v.ncls - 1; c++) {  // which class the item falls into
        const int t = __builtin_amdgcn_readlane(tot, c);
        if (w < t) {
            cls = c;
            break;
        }
        w -= t;
    }
    const int *pre = v.pre + cls * (v.n + 1);
    int lo = 0;
    for (int base = 0; base < v.n; base += 64) {
        const int b = base + lane;
        const bool below = b < v.n && pre[b + 1] <= w;
        lo += __builtin_popcountll(__builtin_amdgcn_ballot_w64(below));
    }
    lo = min(lo, v.n - 1);  // a consistent view never needs this
    it.b = lo;
    it.c = w - pre[lo];
    it.nchunks = pre[lo + 1] - pre[lo];
    it.len = v.len[lo];
    it.off = v.off[lo];
    if (it.c < 0 || it.c >= it.nchunks) {  // cannot happen with a consistent view; never index rows from it
        it.c = 0;
        it.nchunks = 1;
        it.len = 0;
    }
    it.clen = balanced_chunk_len(it.len, it.nchunks, a.chunk);
    return it;
}

// A wave-uniform value as the compiler should see it: in scalar registers, so that addresses and branches
// derived from it are scalar too.
__device__ __forceinline__ int64_t uniform64(int64_t v) {
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

__device__ __forceinline__ Item uniform_item(const Item &i) {
    Item o;
    o.b = __builtin_amdgcn_readfirstlane(i.b);
    o.c = __builtin_amdgcn_readfirstlane(i.c);
    o.nchunks = __builtin_amdgcn_readfirstlane(i.nchunks);
    o.len = __builtin_amdgcn_readfirstlane(i.len);
    o.hgb = __builtin_amdgcn_readfirstlane(i.hgb);
    o.clen = __builtin_amdgcn_readfirstlane(i.clen);
    o.off = uniform64(i.off);
    return o;
}

typedef void (*attn_fn)(const AttnArgs);

// Kernel for shared key/value heads (defined in s3kv_gqa.hip): gq query heads per K/V head and
// lane (1, 2, 4 or 8), shape = index into its (waves, rows per load batch) table, < 0 for the
// default of that gq.  Returns the kernel and its workgroup size, or null.
attn_fn s3i_pick_gqa(int dt, int d, int gq, int shape, int *threads);
// Kernels for 8-bit (e4m3) cache rows (defined in s3kv_fp8.hip): the attention kernel for activation
// type act (S3_F16 / S3_BF16) and its workgroup size, and the append that quantises a new row.
attn_fn s3i_pick_fp8(int act, int d, int shape, int *threads);
typedef void (*append_fp8_fn)(char *, char *, const int64_t *, const int32_t *, const char *, const char *, int32_t,
                              int64_t, int32_t);
append_fp8_fn s3i_pick_append_fp8(int act);
// Matrix-core kernel for shared key/value heads (defined in s3kv_gqa_mfma.hip); 256 threads per
// workgroup, one work item per wave.
attn_fn s3i_pick_gqa_mfma(int dt, int d);
attn_fn s3i_pick_gqa_mfma8(int act, int d);  // the same over 8-bit (e4m3) rows, q of type act
