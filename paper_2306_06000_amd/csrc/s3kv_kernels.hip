// HIP kernels of libs3kv for gfx950 (MI355X): append, ragged decode-step attention
// (split over the sequence axis + merge), plane copies (grow / fill / read-back).
//
// Arena layout.  Plane p = 2*layer + (0: K, 1: V) holds N token rows of H*D elements,
// token-major: element (token t, head h, d) of a plane sits at ((t*H + h)*D + d).  A slot is the
// row range [off, off+cap) in EVERY plane, so one sequence's rows of one plane are one
// contiguous run and the attention kernel streams them with 128-bit loads.
//
// Attention work decomposition.  The method is bound by HBM bandwidth (about one flop per byte),
// so the unit of parallelism is bytes, not sequences: every context is cut into chunks of
// `chunk` tokens and the (chunk, head-group) pairs of the whole ragged batch form one flat work
// list that a fixed grid walks with a stride.  A wavefront covers GH = 512/D adjacent heads of
// one token per 128-bit load (64 lanes x 16 B = 1 KiB of contiguous memory); the D/8 lanes of a
// head reduce their dot product with DPP row operations, keep a running maximum and sum in
// fp32, and accumulate their 8-element slice of the output.  The TS waves of a workgroup that
// share a head group split the chunk's tokens and merge through LDS; chunks of one context
// merge in a second kernel.  Score s_j = q.K_j * scale as in the section 2.1 equation of the
// S3 paper; softmax is max-subtracted; everything after the 16-bit loads is fp32.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "s3kv_internal.h"

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

#define S3_MAX_BATCH 4095

static int hip_fail(const char *what, hipError_t e) {
    s3i_set_hip_error(what, (int)e, hipGetErrorString(e));
    return S3_ERR_HIP;
}
#define HIP_TRY(call)                                     \
    do {                                                  \
        hipError_t e_ = (call);                           \
        if (e_ != hipSuccess) return hip_fail(#call, e_); \
    } while (0)

int s3i_device_cus(int32_t *cus) {
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    int n = 0;
    HIP_TRY(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev));
    *cus = n;
    return S3_OK;
}

// ------------------------------------------------------------------------------------------
// plane copies
// ------------------------------------------------------------------------------------------
// blockIdx.y = plane; each thread moves 16-byte pieces; nbytes is a multiple of 16.
__global__ void __launch_bounds__(256) copy_planes_kernel(const char *src, char *dst, size_t n16,
                                                          size_t src_plane_stride, size_t dst_plane_stride) {
    const u32x4 *s = (const u32x4 *)(src + (size_t)blockIdx.y * src_plane_stride);
    u32x4 *d = (u32x4 *)(dst + (size_t)blockIdx.y * dst_plane_stride);
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) d[i] = s[i];
}

int s3i_launch_copy_planes(const char *src, char *dst, size_t nbytes, size_t src_plane_stride,
                           size_t dst_plane_stride, int planes, void *stream) {
    if (nbytes == 0 || planes <= 0) return S3_OK;
    if ((nbytes & 15) || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return S3_ERR_INVALID;
    const size_t n16 = nbytes / 16;
    size_t blocks = (n16 + 1023) / 1024;  // four pieces per thread
    if (blocks > 4096) blocks = 4096;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(copy_planes_kernel, dim3((unsigned)blocks, (unsigned)planes), dim3(256), 0,
                       (hipStream_t)stream, src, dst, n16, src_plane_stride, dst_plane_stride);
    HIP_TRY(hipGetLastError());
    return S3_OK;
}

// ------------------------------------------------------------------------------------------
// append
// ------------------------------------------------------------------------------------------
// grid (n, 2): block (b, which) copies one row of H*D elements into row off+pos of the plane.
__global__ void __launch_bounds__(256) append_kernel(char *kplane, char *vplane, const int64_t *slot_off,
                                                     const int32_t *pos, const char *k_new, const char *v_new,
                                                     int64_t row_bytes, int64_t n_tokens, int32_t max_len) {
    const int b = blockIdx.x;
    const int64_t off = slot_off[b];
    const int64_t p = pos[b];
    if (off < 0 || p < 0 || p >= max_len || off + p >= n_tokens) return;  // never leave the arena
    const u32x4 *s = (const u32x4 *)((blockIdx.y ? v_new : k_new) + (int64_t)b * row_bytes);
    u32x4 *d = (u32x4 *)((blockIdx.y ? vplane : kplane) + (off + p) * row_bytes);
    const int n16 = (int)(row_bytes >> 4);
    for (int i = threadIdx.x; i < n16; i += 256) d[i] = s[i];
}

// ------------------------------------------------------------------------------------------
// attention
// ------------------------------------------------------------------------------------------
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
    int32_t n, H, chunk, max_chunks, out_dtype, max_len;
    int32_t len_add;    // 0: cur_len is the context length; 1 (fused step): cur_len is the append position
    float scale_log2e;  // scale * log2(e): scores are kept in log2 units so that exp is v_exp_f32
    // fused step only
    const char *k_new;
    const char *v_new;
    int32_t *len_out;        // may be null
    unsigned int *arrivals;  // [n][n_hgb] chunk-arrival counters, zero between launches
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

// Sum over groups of LANES adjacent lanes (8, 16 or 32); every lane of a group gets the sum.
template <int LANES>
__device__ __forceinline__ float group_sum(float v) {
    v = dpp_sum_step<0xB1>(v);   // quad_perm [1,0,3,2]: lane ^ 1
    v = dpp_sum_step<0x4E>(v);   // quad_perm [2,3,0,1]: lane ^ 2
    v = dpp_sum_step<0x141>(v);  // row_half_mirror: the other quad of each 8
    if (LANES >= 16) v = dpp_sum_step<0x140>(v);  // row_mirror: the other 8 of each 16
    if (LANES >= 32)
    {
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

// Exclusive prefix sum of per-sequence chunk counts into cum[0..n] (LDS), by the whole workgroup.
__device__ __forceinline__ void scan_chunks(const AttnArgs &a, int *cum, int *wave_sums) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nthreads = blockDim.x;
    const int per = (a.n + nthreads - 1) / nthreads;
    const int b0 = min(a.n, tid * per), b1 = min(a.n, b0 + per);
    int sum = 0;
    for (int b = b0; b < b1; b++) sum += (checked_len(a, b) + a.chunk - 1) / a.chunk;
    int incl = sum;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int t = __shfl_up(incl, d);
        if (lane >= d) incl += t;
    }
    if (lane == 63) wave_sums[wave] = incl;
    __syncthreads();
    int base = 0;
    for (int i = 0; i < wave; i++) base += wave_sums[i];
    int run = base + incl - sum;
    for (int b = b0; b < b1; b++) {
        cum[b] = run;
        run += (checked_len(a, b) + a.chunk - 1) / a.chunk;
    }
    if (tid == nthreads - 1) cum[a.n] = run;
    __syncthreads();
}

// Merge the chunk partials of (sequence b, head h) for this lane's 8-element slice and store the
// final output row slice.  nchunks >= 2.
template <int D>
__device__ __forceinline__ void merge_chunks(const AttnArgs &a, int b, int h, int dl, int nchunks) {
    const int64_t p0 = ((int64_t)b * a.max_chunks) * a.H + h;
    float mm = -INFINITY;
    for (int c = 0; c < nchunks; c++) mm = fmaxf(mm, a.part_ml[p0 + (int64_t)c * a.H].x);
    float l = 0.f;
    float o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int c = 0; c < nchunks; c++) {
        const int64_t pi = p0 + (int64_t)c * a.H;
        const float2 ml = a.part_ml[pi];
        const float wgt = fast_exp2(ml.x - mm);
        l += wgt * ml.y;
        const f32x4 *pa = (const f32x4 *)(a.part_acc + pi * D + dl * 8);
        const f32x4 x = pa[0], y = pa[1];
#pragma unroll
        for (int i = 0; i < 4; i++) {
            o[i] += wgt * x[i];
            o[4 + i] += wgt * y[i];
        }
    }
    const float inv = 1.f / l;
#pragma unroll
    for (int i = 0; i < 8; i++) o[i] *= inv;
    store_out8(a.out, a.out_dtype, ((int64_t)b * a.H + h) * D + dl * 8, o);
}

// DT: element type of q/K/V.  D: head_dim.  TS: waves splitting a chunk's tokens.  HS: head groups
// per workgroup.  U: tokens per load batch.  NT: non-temporal loads of K/V.
// FUSED: one launch does the whole layer-step: the token at row cur_len[b] (the append position) is
// taken from k_new/v_new instead of the arena and written into the arena by the wave that owns it,
// attention runs over cur_len[b]+1 rows, the workgroup that delivers the last chunk of a (sequence,
// head block) merges the chunks (arrival counter), empty contexts get their zero row, and
// len_out[b] = cur_len[b]+1 is published for the next step.
template <int DT, int D, int TS, int HS, int U, bool NT, bool FUSED>
__global__ void __launch_bounds__(TS *HS * 64) attn_partial_kernel(const AttnArgs a) {
    constexpr int LPH = D / 8;    // lanes per head
    constexpr int GH = 64 / LPH;  // heads per wave
    constexpr int NW = TS * HS;
    extern __shared__ int cum[];  // [n + 1]
    __shared__ int wave_sums[NW];
    __shared__ int last_flag;
    __shared__ float comb[TS > 1 ? NW : 1][10][64];

    scan_chunks(a, cum, wave_sums);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ts = wave % TS, hs = wave / TS;
    const int g = lane / LPH, dl = lane % LPH;
    const int n_hg = (a.H + GH - 1) / GH;
    const int n_hgb = (n_hg + HS - 1) / HS;
    const int64_t total = (int64_t)cum[a.n] * n_hgb;
    const int64_t rstride = (int64_t)a.H * D * 2;
    const int tok_per_wave = a.chunk / TS;

    if (FUSED && blockIdx.x == 0) {
        for (int b = threadIdx.x; b < a.n; b += NW * 64) {
            if (a.len_out) a.len_out[b] = a.cur_len[b] + 1;
            if (cum[b + 1] == cum[b]) {  // empty or refused context: zero output row
                for (int e = 0; e < a.H * D; e += 8) {
                    const float z[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                    store_out8(a.out, a.out_dtype, (int64_t)b * a.H * D + e, z);
                }
            }
        }
    }

    for (int64_t item = blockIdx.x; item < total; item += gridDim.x) {
        const int w = (int)(item / n_hgb);
        const int hgb = (int)(item - (int64_t)w * n_hgb);
        int lo = 0, hi = a.n - 1;
        while (lo < hi) {  // first b with cum[b+1] > w
            const int mid = (lo + hi) >> 1;
            if (cum[mid + 1] > w) hi = mid; else lo = mid + 1;
        }
        const int b = lo;
        const int c = w - cum[b];
        const int nchunks = cum[b + 1] - cum[b];
        const int len = checked_len(a, b);
        const int64_t off = a.slot_off[b];
        const int h = (hgb * HS + hs) * GH + g;
        const bool h_ok = h < a.H;
        const int hc = h_ok ? h : a.H - 1;

        const int j0 = c * a.chunk + ts * tok_per_wave;
        const int j1 = min(len, j0 + tok_per_wave);
        const int64_t lane_byte = ((int64_t)hc * D + dl * 8) * 2;
        const char *kp = a.kplane + off * rstride + lane_byte;
        const char *vp = a.vplane + off * rstride + lane_byte;
        const int64_t in_byte = ((int64_t)b * a.H * D) * 2 + lane_byte;  // this lane's slice of row b of q/k_new/v_new
        const u32x4 qv = *(const u32x4 *)(a.q + in_byte);
        const int jnew = FUSED ? len - 1 : -1;  // the row that is still only in k_new / v_new

        float m = -INFINITY, l = 0.f;
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int j = j0; j < j1; j += U) {
            u32x4 kk[U], vv[U];
#pragma unroll
            for (int u = 0; u < U; u++) {
                const int jj = min(j + u, j1 - 1);
                const char *src = kp + (int64_t)jj * rstride;
                if (FUSED) src = (jj == jnew) ? a.k_new + in_byte : src;
                kk[u] = load16<NT>(src);
            }
#pragma unroll
            for (int u = 0; u < U; u++) {
                const int jj = min(j + u, j1 - 1);
                const char *src = vp + (int64_t)jj * rstride;
                if (FUSED) src = (jj == jnew) ? a.v_new + in_byte : src;
                vv[u] = load16<NT>(src);
            }
            float s[U];
#pragma unroll
            for (int u = 0; u < U; u++) s[u] = dot8<DT>(qv, kk[u]);
#pragma unroll
            for (int u = 0; u < U; u++) s[u] = group_sum<LPH>(s[u]);
            float mb = -INFINITY;
#pragma unroll
            for (int u = 0; u < U; u++) {
                s[u] = (j + u < j1) ? s[u] * a.scale_log2e : -INFINITY;
                mb = fmaxf(mb, s[u]);
            }
            const float mn = fmaxf(m, mb);  // finite: the batch holds at least one real token
            const float alpha = fast_exp2(m - mn);
            l *= alpha;
#pragma unroll
            for (int i = 0; i < 8; i++) acc[i] *= alpha;
#pragma unroll
            for (int u = 0; u < U; u++) {
                const float p = fast_exp2(s[u] - mn);
                l += p;
                axpy8<DT>(acc, p, vv[u]);
            }
            m = mn;
        }
        if (FUSED && h_ok && j0 <= jnew && jnew < j1) {  // the append: this wave owns the new row's slice
            *(u32x4 *)(a.kplane + (off + jnew) * rstride + lane_byte) = *(const u32x4 *)(a.k_new + in_byte);
            *(u32x4 *)(a.vplane + (off + jnew) * rstride + lane_byte) = *(const u32x4 *)(a.v_new + in_byte);
        }

        if (TS > 1) {  // merge the TS token splits of this head group through LDS
            comb[wave][0][lane] = m;
            comb[wave][1][lane] = l;
#pragma unroll
            for (int i = 0; i < 8; i++) comb[wave][2 + i][lane] = acc[i];
            __syncthreads();
            if (ts == 0) {
                float mm = m;
                for (int t = 1; t < TS; t++) mm = fmaxf(mm, comb[wave + t][0][lane]);
                const float w0 = fast_exp2(m - mm);  // split 0 is never empty, so mm is finite
                l *= w0;
#pragma unroll
                for (int i = 0; i < 8; i++) acc[i] *= w0;
                for (int t = 1; t < TS; t++) {
                    const float wt = fast_exp2(comb[wave + t][0][lane] - mm);
                    l += wt * comb[wave + t][1][lane];
#pragma unroll
                    for (int i = 0; i < 8; i++) acc[i] += wt * comb[wave + t][2 + i][lane];
                }
                m = mm;
            }
        }
        if (ts == 0 && h_ok) {
            if (nchunks == 1) {
                const float inv = 1.f / l;
                float o[8];
#pragma unroll
                for (int i = 0; i < 8; i++) o[i] = acc[i] * inv;
                store_out8(a.out, a.out_dtype, ((int64_t)b * a.H + h) * D + dl * 8, o);
            } else {
                const int64_t pi = ((int64_t)b * a.max_chunks + c) * a.H + h;
                if (dl == 0) a.part_ml[pi] = make_float2(m, l);
                f32x4 *pa = (f32x4 *)(a.part_acc + pi * D + dl * 8);
                pa[0] = (f32x4){acc[0], acc[1], acc[2], acc[3]};
                pa[1] = (f32x4){acc[4], acc[5], acc[6], acc[7]};
            }
        }
        if (FUSED && nchunks > 1) {  // uniform over the workgroup: b is
            __threadfence();         // this wave's partials are visible device-wide ...
            __syncthreads();         // ... before thread 0 announces the chunk
            if (threadIdx.x == 0) {
                unsigned int *cnt = a.arrivals + (int64_t)b * n_hgb + hgb;
                const unsigned int old = atomicAdd(cnt, 1u);
                const int last = old == (unsigned int)(nchunks - 1);
                if (last) atomicExch(cnt, 0u);  // every chunk has arrived: leave the counter clean
                last_flag = last;
            }
            __syncthreads();
            if (last_flag) {
                __threadfence();  // see the other workgroups' partials
                if (ts == 0 && h_ok) merge_chunks<D>(a, b, h, dl, nchunks);
            }
        }
        if (TS > 1 || FUSED) __syncthreads();  // comb / last_flag are reused by the next item
    }
}

// One wave per (sequence, head group): merge the chunk partials of contexts longer than one
// chunk; write zeros for empty contexts; leave single-chunk contexts (already final) alone.
template <int D>
__global__ void __launch_bounds__(256) attn_merge_kernel(const AttnArgs a) {
    constexpr int LPH = D / 8;
    constexpr int GH = 64 / LPH;
    const int lane = threadIdx.x & 63;
    const int n_hg = (a.H + GH - 1) / GH;
    const int64_t wid = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (wid >= (int64_t)a.n * n_hg) return;
    const int b = (int)(wid / n_hg), hg = (int)(wid % n_hg);
    const int h = hg * GH + lane / LPH, dl = lane % LPH;
    if (h >= a.H) return;
    const int nchunks = (checked_len(a, b) + a.chunk - 1) / a.chunk;
    if (nchunks == 1) return;
    if (nchunks > 1) {
        merge_chunks<D>(a, b, h, dl, nchunks);
        return;
    }
    const float z[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    store_out8(a.out, a.out_dtype, ((int64_t)b * a.H + h) * D + dl * 8, z);
}

// ------------------------------------------------------------------------------------------
// variant table and launchers
// ------------------------------------------------------------------------------------------
struct Variant {
    int ts, hs, u, nt;
};
static const Variant kVariants[] = {
    {4, 1, 4, 1},   // 0
    {8, 1, 4, 1},   // 1
    {4, 2, 4, 1},   // 2
    {1, 4, 4, 1},   // 3
    {8, 1, 8, 1},   // 4
    {16, 1, 4, 1},  // 5
    {2, 8, 4, 1},   // 6
    {4, 1, 2, 1},   // 7
    {4, 1, 4, 0},   // 8
    {8, 1, 4, 0},   // 9
    {4, 1, 8, 1},   // 10
    {2, 2, 4, 1},   // 11
};
int s3i_num_variants() { return (int)(sizeof(kVariants) / sizeof(kVariants[0])); }

typedef void (*attn_fn)(const AttnArgs);

template <int DT, int D, bool FUSED>
static attn_fn pick_variant(int v) {
    switch (v) {
        case 0: return attn_partial_kernel<DT, D, 4, 1, 4, true, FUSED>;
        case 1: return attn_partial_kernel<DT, D, 8, 1, 4, true, FUSED>;
        case 2: return attn_partial_kernel<DT, D, 4, 2, 4, true, FUSED>;
        case 3: return attn_partial_kernel<DT, D, 1, 4, 4, true, FUSED>;
        case 4: return attn_partial_kernel<DT, D, 8, 1, 8, true, FUSED>;
        case 5: return attn_partial_kernel<DT, D, 16, 1, 4, true, FUSED>;
        case 6: return attn_partial_kernel<DT, D, 2, 8, 4, true, FUSED>;
        case 7: return attn_partial_kernel<DT, D, 4, 1, 2, true, FUSED>;
        case 8: return attn_partial_kernel<DT, D, 4, 1, 4, false, FUSED>;
        case 9: return attn_partial_kernel<DT, D, 8, 1, 4, false, FUSED>;
        case 10: return attn_partial_kernel<DT, D, 4, 1, 8, true, FUSED>;
        case 11: return attn_partial_kernel<DT, D, 2, 2, 4, true, FUSED>;
        default: return nullptr;
    }
}

template <bool FUSED>
static attn_fn pick_kernel(int dt, int d, int v) {
    if (dt == S3_F16) {
        if (d == 64) return pick_variant<S3_F16, 64, FUSED>(v);
        if (d == 128) return pick_variant<S3_F16, 128, FUSED>(v);
        if (d == 256) return pick_variant<S3_F16, 256, FUSED>(v);
    } else if (dt == S3_BF16) {
        if (d == 64) return pick_variant<S3_BF16, 64, FUSED>(v);
        if (d == 128) return pick_variant<S3_BF16, 128, FUSED>(v);
        if (d == 256) return pick_variant<S3_BF16, 256, FUSED>(v);
    }
    return nullptr;
}

static int ensure_scratch(s3_arena *a, size_t need) {
    if (need <= a->scratch_bytes) return S3_OK;
    if (a->scratch) {
        HIP_TRY(hipDeviceSynchronize());
        HIP_TRY(hipFree(a->scratch));
        a->scratch = nullptr;
        a->scratch_bytes = 0;
    }
    HIP_TRY(hipMalloc(&a->scratch, need));
    a->scratch_bytes = need;
    HIP_TRY(hipMemset(a->scratch, 0, need));  // the arrival counters at its head must start at zero
    return S3_OK;
}

// ---- optional event timing of the attention kernels -------------------------------------
static int prof_next_event(s3_arena *a, hipEvent_t *ev) {
    if (a->prof_used == a->prof_events.size()) {
        hipEvent_t e;
        HIP_TRY(hipEventCreate(&e));
        a->prof_events.push_back((void *)e);
    }
    *ev = (hipEvent_t)a->prof_events[a->prof_used++];
    return S3_OK;
}

int s3i_profile_collect(s3_arena *a) {
    for (size_t i = 0; i + 2 < a->prof_used; i += 3) {
        hipEvent_t e0 = (hipEvent_t)a->prof_events[i], e1 = (hipEvent_t)a->prof_events[i + 1],
                   e2 = (hipEvent_t)a->prof_events[i + 2];
        HIP_TRY(hipEventSynchronize(e2));
        float p = 0.f, m = 0.f;
        HIP_TRY(hipEventElapsedTime(&p, e0, e1));
        HIP_TRY(hipEventElapsedTime(&m, e1, e2));
        a->prof_partial_ms += p;
        a->prof_merge_ms += m;
        a->prof_launches++;
    }
    a->prof_used = 0;
    return S3_OK;
}

void s3i_profile_reset(s3_arena *a) {
    (void)s3i_profile_collect(a);
    a->prof_partial_ms = a->prof_merge_ms = 0.0;
    a->prof_launches = 0;
}

extern "C" void s3_kv_arena_destroy(s3_arena *a) {
    if (!a) return;
    if (!a->prof_events.empty()) {
        (void)hipDeviceSynchronize();
        for (void *e : a->prof_events) (void)hipEventDestroy((hipEvent_t)e);
    }
    if (a->scratch) {
        (void)hipDeviceSynchronize();
        (void)hipFree(a->scratch);
    }
    delete a;
}

static bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }
static int check_slots_host(const s3_arena *a, int32_t n, const int32_t *slot_id, const int32_t *pos_host);

extern "C" int s3_kv_append(s3_arena *a, int32_t layer, int32_t n, const int32_t *slot_id, const int32_t *pos_host,
                            const int64_t *slot_off, const int32_t *pos, const void *k_new, const void *v_new,
                            void *stream) {
    if (!a || !a->base || layer < 0 || layer >= a->cfg.n_layers || n < 0) return S3_ERR_INVALID;
    if (n == 0) return S3_OK;
    if (!slot_off || !pos || !k_new || !v_new || !aligned16(k_new) || !aligned16(v_new)) return S3_ERR_INVALID;
    const int rc = check_slots_host(a, n, slot_id, pos_host);
    if (rc != S3_OK) return rc;
    hipLaunchKernelGGL(append_kernel, dim3((unsigned)n, 2), dim3(256), 0, (hipStream_t)stream, a->plane(layer, 0),
                       a->plane(layer, 1), slot_off, pos, (const char *)k_new, (const char *)v_new, a->row_bytes,
                       a->n_tokens, a->cfg.max_len);
    HIP_TRY(hipGetLastError());
    return S3_OK;
}

static int check_slots_host(const s3_arena *a, int32_t n, const int32_t *slot_id, const int32_t *pos_host) {
    if (!slot_id || !pos_host) return S3_OK;  // the caller vouches for the positions
    bool full = false;
    for (int32_t b = 0; b < n; b++) {
        const s3_slot *s = s3i_live_slot(a, slot_id[b]);
        if (!s || pos_host[b] < 0 || pos_host[b] > s->cap) return S3_ERR_INVALID;
        if (pos_host[b] == s->cap) full = true;
    }
    return full ? S3_ERR_SLOT_FULL : S3_OK;
}

// Shared by s3_decode_attention (fused = false: partial kernel + merge kernel) and s3_decode_step
// (fused = true: one kernel that also appends, merges and publishes the new lengths).
static int launch_attention(s3_arena *a, int32_t layer, int32_t n, const void *q, const int64_t *slot_off,
                            const int32_t *len_or_pos, void *out, int32_t out_dtype, float scale, void *stream,
                            bool fused, const void *k_new, const void *v_new, int32_t *len_out) {
    const int D = a->cfg.head_dim, H = a->cfg.n_heads;
    const int variant = a->variant >= 0 ? a->variant : 1;
    const Variant &vr = kVariants[variant];
    const int chunk = a->chunk > 0 ? a->chunk : 128;
    if (chunk % vr.ts) return S3_ERR_INVALID;
    attn_fn fn = fused ? pick_kernel<true>(a->cfg.kv_dtype, D, variant) : pick_kernel<false>(a->cfg.kv_dtype, D, variant);
    if (!fn) return S3_ERR_INVALID;
    const int GH = 512 / D;
    const int n_hg = (H + GH - 1) / GH;

    AttnArgs args;
    args.kplane = a->plane(layer, 0);
    args.vplane = a->plane(layer, 1);
    args.q = (const char *)q;
    args.slot_off = slot_off;
    args.cur_len = len_or_pos;
    args.out = out;
    args.n_tokens = a->n_tokens;
    args.n = n;
    args.H = H;
    args.chunk = chunk;
    args.max_chunks = (a->cfg.max_len + chunk - 1) / chunk;
    args.out_dtype = out_dtype;
    args.max_len = a->cfg.max_len;
    args.len_add = fused ? 1 : 0;
    if (!(scale > 0.f)) scale = 1.0f / sqrtf((float)D);
    args.scale_log2e = scale * 1.4426950408889634f;
    args.k_new = (const char *)k_new;
    args.v_new = (const char *)v_new;
    args.len_out = len_out;

    // scratch: [arrival counters, fixed size][partial sums][partial (max, sum)]
    const size_t cnt_bytes = (((size_t)(S3_MAX_BATCH + 1) * n_hg * sizeof(unsigned int)) + 255) & ~(size_t)255;
    const size_t n_part = (size_t)n * args.max_chunks * H;
    const size_t acc_bytes = n_part * D * sizeof(float);
    const size_t need = cnt_bytes + acc_bytes + n_part * sizeof(float2);
    const int rc = ensure_scratch(a, need);
    if (rc != S3_OK) return rc;
    args.arrivals = (unsigned int *)a->scratch;
    args.part_acc = (float *)((char *)a->scratch + cnt_bytes);
    args.part_ml = (float2 *)((char *)a->scratch + cnt_bytes + acc_bytes);

    const int nw = vr.ts * vr.hs;
    const int cus = a->num_cus > 0 ? a->num_cus : 256;
    const int blocks = a->grid_blocks > 0 ? a->grid_blocks : cus * (32 / nw);
    const size_t dyn_lds = (size_t)(n + 1) * sizeof(int);
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
    if (a->profile) {
        for (int i = 0; i < 3; i++) {
            const int prc = prof_next_event(a, &ev[i]);
            if (prc != S3_OK) return prc;
        }
        HIP_TRY(hipEventRecord(ev[0], (hipStream_t)stream));
    }
    hipLaunchKernelGGL(fn, dim3((unsigned)blocks), dim3((unsigned)(nw * 64)), dyn_lds, (hipStream_t)stream, args);
    HIP_TRY(hipGetLastError());
    if (a->profile) HIP_TRY(hipEventRecord(ev[1], (hipStream_t)stream));
    if (!fused) {
        const unsigned mblocks = (unsigned)(((int64_t)n * n_hg + 3) / 4);
        void (*mfn)(const AttnArgs) =
            D == 64 ? attn_merge_kernel<64> : D == 128 ? attn_merge_kernel<128> : attn_merge_kernel<256>;
        hipLaunchKernelGGL(mfn, dim3(mblocks), dim3(256), 0, (hipStream_t)stream, args);
        HIP_TRY(hipGetLastError());
    }
    if (a->profile) HIP_TRY(hipEventRecord(ev[2], (hipStream_t)stream));
    return S3_OK;
}

extern "C" int s3_decode_attention(s3_arena *a, int32_t layer, int32_t n, const void *q, const int64_t *slot_off,
                                   const int32_t *cur_len, void *out, int32_t out_dtype, float scale, void *stream) {
    if (!a || !a->base || layer < 0 || layer >= a->cfg.n_layers || n < 0 || n > S3_MAX_BATCH) return S3_ERR_INVALID;
    if (n == 0) return S3_OK;
    if (!q || !slot_off || !cur_len || !out || !aligned16(q) || !aligned16(out)) return S3_ERR_INVALID;
    if (out_dtype != S3_F32 && out_dtype != S3_F16 && out_dtype != S3_BF16) return S3_ERR_INVALID;
    return launch_attention(a, layer, n, q, slot_off, cur_len, out, out_dtype, scale, stream, false, nullptr, nullptr,
                            nullptr);
}

extern "C" int s3_decode_step(s3_arena *a, int32_t layer, int32_t n, const int32_t *slot_id, const int32_t *pos_host,
                              const int64_t *slot_off, const int32_t *pos, const void *q, const void *k_new,
                              const void *v_new, void *out, int32_t out_dtype, float scale, int32_t *len_out,
                              void *stream) {
    if (!a || !a->base || layer < 0 || layer >= a->cfg.n_layers || n < 0 || n > S3_MAX_BATCH) return S3_ERR_INVALID;
    if (n == 0) return S3_OK;
    if (!q || !k_new || !v_new || !slot_off || !pos || !out) return S3_ERR_INVALID;
    if (!aligned16(q) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(out)) return S3_ERR_INVALID;
    if (len_out == pos) return S3_ERR_INVALID;  // other workgroups still read pos while len_out is written
    if (out_dtype != S3_F32 && out_dtype != S3_F16 && out_dtype != S3_BF16) return S3_ERR_INVALID;
    const int rc = check_slots_host(a, n, slot_id, pos_host);
    if (rc != S3_OK) return rc;
    return launch_attention(a, layer, n, q, slot_off, pos, out, out_dtype, scale, stream, true, k_new, v_new, len_out);
}

extern "C" int s3_kv_fill(s3_arena *a, int32_t slot_id, int32_t layer, int32_t first_row, int32_t n_rows,
                          const void *k_rows, const void *v_rows, void *stream) {
    const s3_slot *s = s3i_live_slot(a, slot_id);
    if (!s || !a->base || layer < 0 || layer >= a->cfg.n_layers || first_row < 0 || n_rows < 0) return S3_ERR_INVALID;
    if ((int64_t)first_row + n_rows > s->cap) return S3_ERR_SLOT_FULL;
    if (n_rows == 0) return S3_OK;
    if (!k_rows || !v_rows) return S3_ERR_INVALID;
    const size_t nbytes = (size_t)n_rows * a->row_bytes;
    const int64_t row0 = s->off + first_row;
    int rc = s3i_launch_copy_planes((const char *)k_rows, a->plane(layer, 0) + row0 * a->row_bytes, nbytes, 0, 0, 1,
                                    stream);
    if (rc != S3_OK) return rc;
    return s3i_launch_copy_planes((const char *)v_rows, a->plane(layer, 1) + row0 * a->row_bytes, nbytes, 0, 0, 1,
                                  stream);
}

extern "C" int s3_kv_read_rows(s3_arena *a, int32_t slot_id, int32_t layer, int32_t which, int32_t first_row,
                               int32_t n_rows, void *dst, void *stream) {
    const s3_slot *s = s3i_live_slot(a, slot_id);
    if (!s || !a->base || layer < 0 || layer >= a->cfg.n_layers || first_row < 0 || n_rows < 0 ||
        (which != 0 && which != 1))
        return S3_ERR_INVALID;
    if ((int64_t)first_row + n_rows > s->cap) return S3_ERR_INVALID;
    if (n_rows == 0) return S3_OK;
    if (!dst) return S3_ERR_INVALID;
    return s3i_launch_copy_planes(a->plane(layer, which) + (s->off + first_row) * a->row_bytes, (char *)dst,
                                  (size_t)n_rows * a->row_bytes, 0, 0, 1, stream);
}
