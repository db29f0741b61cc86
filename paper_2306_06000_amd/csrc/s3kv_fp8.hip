// Kernels for 8-bit cache rows of libs3kv, gfx950.  The paper's related-work section names
// quantisation, next to multi-query attention, as a complementary way to shrink the cache; here a
// row holds e4m3 codes (1 sign, 4 exponent bits with bias 7, 3 fraction bits, no infinities, largest
// value 448) while queries and new rows stay 16-bit.  A new row is rounded once when it is appended
// (nearest code, ties to even, saturating, NaN -> 0x7f); attention widens the codes exactly and runs
// the same softmax(q.K^T.scale).V in fp32 (section 2.1).
//
// Attention: a wave's 128-bit load covers 1 KiB of consecutive arena bytes = 16 elements per lane,
// D/16 lanes per head, 1024/D heads of one row (or, when a row has fewer heads, whole consecutive
// rows, each lane group with its own online-softmax state).  Work list, near-equal chunks,
// longest-first order, TS waves per item merging through LDS: as in the kernel for shared K/V heads;
// chunks of one context merge inside the kernel (arrival counter), so no second kernel follows, and in a
// decode step the kernel quantises and appends the new row itself: one launch per step.
#include "s3kv_device.h"

typedef float f32x2v __attribute__((ext_vector_type(2)));

// e4m3 codes -> fp32, exact, four codes of one 32-bit word (v_cvt_pk_f32_fp8 reads this format on gfx950).
__device__ __forceinline__ void widen4_e4m3(const unsigned w, float (&f)[4]) {
    const f32x2v lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false);
    const f32x2v hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true);
    f[0] = lo[0];
    f[1] = lo[1];
    f[2] = hi[0];
    f[3] = hi[1];
}

// Two fp32 values -> their e4m3 codes in one half of a 32-bit word (v_cvt_pk_fp8_f32 rounds to the nearest
// code, ties to even, subnormal codes included).  Magnitudes are clamped to 448 first, so nothing depends on
// the instruction's overflow mode, and NaN is forced to 0x7f afterwards (the clamp turns it into a number).
template <bool HI>
__device__ __forceinline__ unsigned quantize2_e4m3(const float x0, const float x1, const unsigned old) {
    const float c0 = fminf(fmaxf(x0, -448.f), 448.f), c1 = fminf(fmaxf(x1, -448.f), 448.f);
    unsigned w = (unsigned)__builtin_amdgcn_cvt_pk_fp8_f32(c0, c1, (int)old, HI);
    constexpr unsigned S = HI ? 16u : 0u;
    if (x0 != x0) w = (w & ~(0xFFu << S)) | (0x7Fu << S);
    if (x1 != x1) w = (w & ~(0xFF00u << S)) | (0x7F00u << S);
    return w;
}

template <int ACT>
__device__ __forceinline__ float widen16(const unsigned short h) {
    if (ACT == S3_F16) return (float)__builtin_bit_cast(_Float16, h);
    const unsigned w = (unsigned)h << 16;
    return __builtin_bit_cast(float, w);
}

// 16 consecutive 16-bit elements (two 128-bit words) -> their 16 codes in element order.
template <int ACT>
__device__ __forceinline__ u32x4 quantize16(const u32x4 lo, const u32x4 hi) {
    u32x4 out;
#pragma unroll
    for (int w = 0; w < 4; w++) {
        const unsigned a = w < 2 ? lo[2 * w] : hi[2 * w - 4], c = w < 2 ? lo[2 * w + 1] : hi[2 * w - 3];
        const unsigned lo2 = quantize2_e4m3<false>(widen16<ACT>((unsigned short)(a & 0xFFFFu)),
                                                   widen16<ACT>((unsigned short)(a >> 16)), 0u);
        out[w] = quantize2_e4m3<true>(widen16<ACT>((unsigned short)(c & 0xFFFFu)), widen16<ACT>((unsigned short)(c >> 16)), lo2);
    }
    return out;
}

// grid (n, 2): block (b, which) quantises one new row of H*D 16-bit elements into row off+pos.
template <int ACT>
__global__ void __launch_bounds__(256) append_fp8_kernel(char *kplane, char *vplane, const int64_t *slot_off,
                                                         const int32_t *pos, const char *k_new, const char *v_new,
                                                         int32_t row_elems, int64_t n_tokens, int32_t max_len) {
    const int b = blockIdx.x;
    const int64_t off = slot_off[b];
    const int64_t p = pos[b];
    if (off < 0 || p < 0 || p >= max_len || off + p >= n_tokens) return;  // never leave the arena
    const char *src = (blockIdx.y ? v_new : k_new) + (int64_t)b * row_elems * 2;
    char *dst = (blockIdx.y ? vplane : kplane) + (off + p) * (int64_t)row_elems;
    for (int i = threadIdx.x; i < row_elems / 16; i += 256) {  // 16 elements: 32 bytes in, 16 out
        const u32x4 lo = *(const u32x4 *)(src + (int64_t)i * 32), hi = *(const u32x4 *)(src + (int64_t)i * 32 + 16);
        const u32x4 out = quantize16<ACT>(lo, hi);
        *(u32x4 *)(dst + (int64_t)i * 16) = out;
    }
}

template <int ACT, int D, int TS, int U>
__global__ void __launch_bounds__(TS * 64) attn_fp8_kernel(const AttnArgs a) {
    constexpr int LPH = D / 16;   // lanes per head
    constexpr int GH = 64 / LPH;  // heads per wave load
    extern __shared__ __align__(16) char dyn_lds[];  // the batch view
    __shared__ int wave_sums[S3_MAX_CLASSES * S3_MAX_WAVES];
    __shared__ float comb[TS][18][64];
    const int lane = threadIdx.x & 63, ts = threadIdx.x >> 6;
    const int tpw = (a.H < GH && GH % a.H == 0) ? GH / a.H : 1;  // rows per wave load
    const int n_hg = (a.H + GH - 1) / GH;
    const BatchView bv = build_batch_view(a, dyn_lds, wave_sums);
    const int64_t total = (int64_t)bv.total * n_hg;
    // the new lengths, and a zero output row for empty or refused contexts, by the workgroups in turn
    for (int b = blockIdx.x; b < a.n; b += gridDim.x) {
        if (a.len_out && threadIdx.x == 0) a.len_out[b] = a.cur_len[b] + 1;
        if (bv.len[b] == 0) {
            const float z[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            for (int e = threadIdx.x; e < a.H * D / 8; e += TS * 64) store_out8(a.out, a.out_dtype, ((int64_t)b * a.H * D / 8 + e) * 8, z);
        }
    }

    const int slot = lane / LPH, dl = lane % LPH;
    const int tsub = tpw > 1 ? slot / a.H : 0;
    const unsigned rs32 = (unsigned)(a.H * D);  // bytes of one cached row
    for (int64_t item = blockIdx.x; item < total; item += gridDim.x) {
        const Item it = decode_item(a, bv, item, n_hg);
        const int h = tpw > 1 ? slot % a.H : it.hgb * GH + slot;
        const bool h_ok = h < a.H;
        const int hc = h_ok ? h : a.H - 1;
        const int start = it.c * it.clen, end = min(it.len, start + it.clen);
        // decode step: row len-1 is still a 16-bit row in k_new / v_new; the chunk that ends with it
        // streams the rows before it and takes the new row in its last wave (below)
        const bool has_new = a.k_new != nullptr && end == it.len;
        const int end_mem = has_new ? end - 1 : end;
        // the new row costs its wave one more memory round trip, about what a batch of four rows costs: its
        // share of the streamed rows is shorter by that much
        const int per = (end_mem - start + (has_new ? 4 : 0) + TS - 1) / TS;
        const int j0 = min(end_mem, start + ts * per), j1 = min(end_mem, j0 + per);
        const char *kp = a.kplane + it.off * (int64_t)rs32 + hc * D + dl * 16;
        const char *vp = a.vplane + it.off * (int64_t)rs32 + hc * D + dl * 16;
        float q[16];
        {
            const char *qp = a.q + (((int64_t)it.b * a.H + hc) * D + dl * 16) * 2;
            const u32x4 q0 = *(const u32x4 *)qp, q1 = *(const u32x4 *)(qp + 16);
#pragma unroll
            for (int i = 0; i < 8; i++) {
                const unsigned w = i < 4 ? q0[i] : q1[i - 4];
                q[2 * i] = widen16<ACT>((unsigned short)(w & 0xFFFFu)) * a.scale_log2e;  // scale folded into q
                q[2 * i + 1] = widen16<ACT>((unsigned short)(w >> 16)) * a.scale_log2e;
            }
        }
        float m = -INFINITY, l = 0.f, acc[16];
#pragma unroll
        for (int e = 0; e < 16; e++) acc[e] = 0.f;
        for (int j = j0; j < j1; j += U * tpw) {
            u32x4 kk[U], vv[U];
#pragma unroll
            for (int u = 0; u < U; u++)
                kk[u] = load16<true>(kp + (uint64_t)(unsigned)min(j + u * tpw + tsub, j1 - 1) * rs32);
#pragma unroll
            for (int u = 0; u < U; u++)
                vv[u] = load16<true>(vp + (uint64_t)(unsigned)min(j + u * tpw + tsub, j1 - 1) * rs32);
            float s[U], mb = -INFINITY;
#pragma unroll
            for (int u = 0; u < U; u++) {
                float d = 0.f;
#pragma unroll
                for (int w = 0; w < 4; w++) {
                    float f[4];
                    const unsigned word = kk[u][w];
                    widen4_e4m3(word, f);
#pragma unroll
                    for (int e = 0; e < 4; e++) d = fmaf(q[4 * w + e], f[e], d);
                }
                d = group_sum<LPH>(d);
                s[u] = (j + u * tpw + tsub < j1) ? d : -INFINITY;
                mb = fmaxf(mb, s[u]);
            }
            // a lane group whose rows of this batch are all past the end keeps its state
            const float mn = fmaxf(m, mb);
            const float alpha = (mn == -INFINITY) ? 1.f : fast_exp2(m - mn);
            l *= alpha;
#pragma unroll
            for (int e = 0; e < 16; e++) acc[e] *= alpha;
#pragma unroll
            for (int u = 0; u < U; u++) {
                const float p = (mn == -INFINITY) ? 0.f : fast_exp2(s[u] - mn);
                l += p;
#pragma unroll
                for (int w = 0; w < 4; w++) {
                    float f[4];
                    const unsigned word = vv[u][w];
                    widen4_e4m3(word, f);
#pragma unroll
                    for (int e = 0; e < 4; e++) acc[4 * w + e] = fmaf(p, f[e], acc[4 * w + e]);
                }
            }
            m = mn;
        }
        if (has_new && ts == TS - 1) {
            // The new row: rounded to codes exactly as the append kernel rounds it, written to the arena by
            // the lanes that own its bytes, and attended over as the codes widen (what a later step reads).
            const int64_t in_byte = (((int64_t)it.b * a.H + hc) * D + dl * 16) * 2;
            const u32x4 kc = quantize16<ACT>(*(const u32x4 *)(a.k_new + in_byte), *(const u32x4 *)(a.k_new + in_byte + 16));
            const u32x4 vc = quantize16<ACT>(*(const u32x4 *)(a.v_new + in_byte), *(const u32x4 *)(a.v_new + in_byte + 16));
            if (h_ok && tsub == 0) {
                const int64_t row_byte = (it.off + it.len - 1) * (int64_t)rs32 + h * D + dl * 16;
                *(u32x4 *)(a.kplane + row_byte) = kc;
                *(u32x4 *)(a.vplane + row_byte) = vc;
            }
            float d = 0.f;
#pragma unroll
            for (int w = 0; w < 4; w++) {
                float f[4];
                const unsigned word = kc[w];
                widen4_e4m3(word, f);
#pragma unroll
                for (int e = 0; e < 4; e++) d = fmaf(q[4 * w + e], f[e], d);
            }
            d = group_sum<LPH>(d);
            const float s_new = tsub == 0 ? d : -INFINITY;  // one row: the first lane group's
            const float mn = fmaxf(m, s_new);
            const float alpha = (mn == -INFINITY) ? 1.f : fast_exp2(m - mn);
            const float p = (mn == -INFINITY) ? 0.f : fast_exp2(s_new - mn);
            l = l * alpha + p;
#pragma unroll
            for (int w = 0; w < 4; w++) {
                float f[4];
                const unsigned word = vc[w];
                widen4_e4m3(word, f);
#pragma unroll
                for (int e = 0; e < 4; e++) acc[4 * w + e] = fmaf(p, f[e], acc[4 * w + e] * alpha);
            }
            m = mn;
        }
        comb[ts][0][lane] = m;
        comb[ts][1][lane] = l;
#pragma unroll
        for (int e = 0; e < 16; e++) comb[ts][2 + e][lane] = acc[e];
        __syncthreads();
        if (ts == 0 && h_ok && tsub == 0) {
            float o[16], mm = -INFINITY, ll = 0.f;
#pragma unroll
            for (int e = 0; e < 16; e++) o[e] = 0.f;
            // a chunk has at least one row, so the maximum over its waves and lane groups is finite
            for (int t = 0; t < TS; t++)
                for (int g = 0; g < tpw; g++) mm = fmaxf(mm, comb[t][0][lane + g * a.H * LPH]);
            for (int t = 0; t < TS; t++)
                for (int g = 0; g < tpw; g++) {
                    const int src = lane + g * a.H * LPH;
                    const float wt = fast_exp2(comb[t][0][src] - mm);
                    ll += wt * comb[t][1][src];
#pragma unroll
                    for (int e = 0; e < 16; e++) o[e] += wt * comb[t][2 + e][src];
                }
            if (it.nchunks <= 1) {
                const float inv = 1.f / ll;
                float o0[8], o1[8];
#pragma unroll
                for (int e = 0; e < 8; e++) {
                    o0[e] = o[e] * inv;
                    o1[e] = o[8 + e] * inv;
                }
                const int64_t e0 = ((int64_t)it.b * a.H + h) * D + dl * 16;
                store_out8(a.out, a.out_dtype, e0, o0);
                store_out8(a.out, a.out_dtype, e0 + 8, o1);
            } else {  // a chunk of a longer context: the partial goes out with write-through stores
                const int64_t pi = ((int64_t)it.b * a.max_chunks + it.c) * a.H + h;
                float *pa = a.part_acc + pi * D + dl * 16;
                if (dl == 0) put_partial2<true>((float *)a.part_ml + 2 * pi, (f32x2){mm, ll});
#pragma unroll
                for (int v4 = 0; v4 < 4; v4++)
                    put_partial4<true>(pa + 4 * v4, (f32x4){o[4 * v4], o[4 * v4 + 1], o[4 * v4 + 2], o[4 * v4 + 3]});
            }
        }
        if (ts == 0 && it.nchunks > 1) {
            // Chunks meet through an arrival counter per (sequence, head group), as in the fused multi-head
            // step: whoever delivers the last chunk merges them.  With the default chunk of 1024 rows this is
            // rare, which is what makes it cheaper than a merge launch after every attention launch.
            unsigned int *cnt = a.arrivals + (int64_t)it.b * n_hg + it.hgb;
            if (chunk_arrived(a, cnt, it.nchunks)) {
                if (h_ok && tsub == 0) {
                    merge_chunks<D, true>(a, a.H, it.b, h, 2 * dl, it.nchunks);
                    merge_chunks<D, true>(a, a.H, it.b, h, 2 * dl + 1, it.nchunks);
                }
            }
        }
        __syncthreads();  // comb is reused by the next item
    }
}

// Shapes: (TS waves per workgroup, U rows per load batch).
struct Fp8Shape {
    int ts, u;
};
static const Fp8Shape kFp8Shapes[] = {{8, 4}, {4, 4}, {8, 2}, {4, 8}};
int s3i_num_fp8_shapes() { return (int)(sizeof(kFp8Shapes) / sizeof(kFp8Shapes[0])); }

template <int ACT, int D>
static attn_fn pick_fp8_shape(int shape) {
    switch (shape) {
        case 0: return attn_fp8_kernel<ACT, D, 8, 4>;
        case 1: return attn_fp8_kernel<ACT, D, 4, 4>;
        case 2: return attn_fp8_kernel<ACT, D, 8, 2>;
        case 3: return attn_fp8_kernel<ACT, D, 4, 8>;
        default: return nullptr;
    }
}

attn_fn s3i_pick_fp8(int act, int d, int shape, int *threads) {
    if (shape < 0 || shape >= s3i_num_fp8_shapes()) shape = 2;  // measured best on MI355X: eight waves, two rows per round
    *threads = kFp8Shapes[shape].ts * 64;
    if (act == S3_F16) {
        if (d == 64) return pick_fp8_shape<S3_F16, 64>(shape);
        if (d == 128) return pick_fp8_shape<S3_F16, 128>(shape);
        if (d == 256) return pick_fp8_shape<S3_F16, 256>(shape);
    } else if (act == S3_BF16) {
        if (d == 64) return pick_fp8_shape<S3_BF16, 64>(shape);
        if (d == 128) return pick_fp8_shape<S3_BF16, 128>(shape);
        if (d == 256) return pick_fp8_shape<S3_BF16, 256>(shape);
    }
    return nullptr;
}

append_fp8_fn s3i_pick_append_fp8(int act) {
    return act == S3_F16 ? append_fp8_kernel<S3_F16> : act == S3_BF16 ? append_fp8_kernel<S3_BF16> : nullptr;
}
