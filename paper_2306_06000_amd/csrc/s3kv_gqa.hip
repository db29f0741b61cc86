// Attention kernel for shared key/value heads (grouped-query / multi-query attention) of libs3kv,
// gfx950.  Launched by the host code in s3kv_kernels.hip through the pointer s3i_pick_gqa returns.
#include "s3kv_device.h"

// Grouped-query / multi-query attention (n_kv_heads < n_heads; the paper's related-work section names
// multi-query attention as a complementary way to shrink the cache): K/V rows hold H heads, q and out
// Hq = H * group heads; K/V head k serves query heads k*group .. k*group+group-1.  A wave's 128-bit
// load covers 1 KiB of consecutive arena bytes as in the multi-head kernels: GH K/V heads of one row
// or, when a row has fewer than GH heads (H dividing GH), GH/H whole consecutive rows, each lane group
// then keeping its own online-softmax state for its share of the rows.  Every lane carries GQ query
// heads per K/V head; group/GQ items per K/V head group re-read the same rows.
// Work item = (sequence, chunk of its context, K/V head group, query sub-block), enumerated from the
// same LDS batch view (near-equal chunks, longest contexts first) as in the multi-head kernels; empty
// contexts have no item and get their zero rows from the merge kernel.  The TS waves of a workgroup
// split the chunk's rows and merge through LDS, one query head at a time; wave 0 writes the output (one chunk) or the chunk partial (whole 32-byte
// vector stores per lane: per-element device-scope stores as in the fused multi-head step cost more
// here than the extra launch), and attn_merge_kernel, launched after it with H = the query head
// count, finishes multi-chunk contexts.
// With len_add = 1 it is the attention half of a decode step whose append ran as its own launch before.
template <int DT, int D, int GQ, int TS, int U>
__global__ void __launch_bounds__(TS * 64) attn_gqa_kernel(const AttnArgs a) {
    constexpr int LPH = D / 8;
    constexpr int GH = 64 / LPH;
    extern __shared__ __align__(16) char dyn_lds[];  // the batch view
    __shared__ int wave_sums[S3_MAX_CLASSES * S3_MAX_WAVES];
    __shared__ float comb[TS][10][64];
    const int lane = threadIdx.x & 63, ts = threadIdx.x >> 6;
    const int group = a.Hq / a.H;
    const int tpw = (a.H < GH && GH % a.H == 0) ? GH / a.H : 1;  // rows per wave load
    const int n_kvhg = (a.H + GH - 1) / GH, n_qsub = group / GQ;
    const int per_seq = n_kvhg * n_qsub;
    const BatchView bv = build_batch_view(a, dyn_lds, wave_sums);
    const int64_t total = (int64_t)bv.total * per_seq;
    if (blockIdx.x == 0 && a.len_out)
        for (int b = threadIdx.x; b < a.n; b += TS * 64) a.len_out[b] = a.cur_len[b] + 1;

    const int slot = lane / LPH, dl = lane % LPH;
    const int tsub = tpw > 1 ? slot / a.H : 0;
    for (int64_t item = blockIdx.x; item < total; item += gridDim.x) {
        const Item it = decode_item(a, bv, item, per_seq);
        const int r = it.hgb, b = it.b, c = it.c, len = it.len, nchunks = it.nchunks, clen = it.clen;
        const int kvhg = r / n_qsub, qsub = r - kvhg * n_qsub;
        const int64_t off = it.off;
        const int hk = tpw > 1 ? slot % a.H : kvhg * GH + slot;
        const bool hk_ok = hk < a.H;
        const int hkc = hk_ok ? hk : a.H - 1;
        const int start = c * clen, end = min(len, start + clen);
        const int per = (end - start + TS - 1) / TS;
        const int j0 = min(end, start + ts * per), j1 = min(end, j0 + per);
        const int64_t rstride = (int64_t)a.H * D * 2;
        const int64_t lane_byte = ((int64_t)hkc * D + dl * 8) * 2;
        const char *kp = a.kplane + off * rstride + lane_byte;
        const char *vp = a.vplane + off * rstride + lane_byte;
        const int hq0 = hkc * group + qsub * GQ;  // first of this lane's GQ query heads
        u32x4 qv[GQ];
#pragma unroll
        for (int i = 0; i < GQ; i++)
            qv[i] = *(const u32x4 *)(a.q + (((int64_t)b * a.Hq + hq0 + i) * D + dl * 8) * 2);
        float m[GQ], l[GQ], acc[GQ][8];
#pragma unroll
        for (int i = 0; i < GQ; i++) {
            m[i] = -INFINITY;
            l[i] = 0.f;
#pragma unroll
            for (int e = 0; e < 8; e++) acc[i][e] = 0.f;
        }
        for (int j = j0; j < j1; j += U * tpw) {
            u32x4 kk[U], vv[U];
#pragma unroll
            for (int u = 0; u < U; u++) kk[u] = load16<true>(kp + (int64_t)min(j + u * tpw + tsub, j1 - 1) * rstride);
#pragma unroll
            for (int u = 0; u < U; u++) vv[u] = load16<true>(vp + (int64_t)min(j + u * tpw + tsub, j1 - 1) * rstride);
#pragma unroll
            for (int i = 0; i < GQ; i++) {
                float s[U], mb = -INFINITY;
#pragma unroll
                for (int u = 0; u < U; u++) {
                    const float d = group_sum<LPH>(dot8<DT>(qv[i], kk[u]));
                    s[u] = (j + u * tpw + tsub < j1) ? d * a.scale_log2e : -INFINITY;
                    mb = fmaxf(mb, s[u]);
                }
                // a lane group whose rows of this batch are all past the end keeps its state
                const float mn = fmaxf(m[i], mb);
                const float alpha = (mn == -INFINITY) ? 1.f : fast_exp2(m[i] - mn);
                l[i] *= alpha;
#pragma unroll
                for (int e = 0; e < 8; e++) acc[i][e] *= alpha;
#pragma unroll
                for (int u = 0; u < U; u++) {
                    const float p = (mn == -INFINITY) ? 0.f : fast_exp2(s[u] - mn);
                    l[i] += p;
                    axpy8<DT>(acc[i], p, vv[u]);
                }
                m[i] = mn;
            }
        }
        const bool writer = ts == 0 && hk_ok && tsub == 0;
#pragma unroll
        for (int i = 0; i < GQ; i++) {
            comb[ts][0][lane] = m[i];
            comb[ts][1][lane] = l[i];
#pragma unroll
            for (int e = 0; e < 8; e++) comb[ts][2 + e][lane] = acc[i][e];
            __syncthreads();
            if (writer) {
                float o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                float mm = -INFINITY, ll = 0.f;
                if (len > 0) {  // a chunk's rows start at wave 0, lane group 0, so the maximum is finite
                    for (int t = 0; t < TS; t++)
                        for (int g = 0; g < tpw; g++) mm = fmaxf(mm, comb[t][0][lane + g * a.H * LPH]);
                    for (int t = 0; t < TS; t++)
                        for (int g = 0; g < tpw; g++) {
                            const int src = lane + g * a.H * LPH;
                            const float wt = fast_exp2(comb[t][0][src] - mm);
                            ll += wt * comb[t][1][src];
#pragma unroll
                            for (int e = 0; e < 8; e++) o[e] += wt * comb[t][2 + e][src];
                        }
                }
                if (nchunks <= 1) {
                    const float inv = len > 0 ? 1.f / ll : 0.f;
#pragma unroll
                    for (int e = 0; e < 8; e++) o[e] *= inv;
                    store_out8(a.out, a.out_dtype, ((int64_t)b * a.Hq + hq0 + i) * D + dl * 8, o);
                } else {
                    const int64_t pi = ((int64_t)b * a.max_chunks + c) * a.Hq + hq0 + i;
                    float *pml = (float *)a.part_ml + 2 * pi;
                    float *pa = a.part_acc + pi * D + dl * 8;
                    if (dl == 0) *(float2 *)pml = make_float2(mm, ll);
                    ((f32x4 *)pa)[0] = (f32x4){o[0], o[1], o[2], o[3]};
                    ((f32x4 *)pa)[1] = (f32x4){o[4], o[5], o[6], o[7]};
                }
            }
            __syncthreads();  // comb is reused by the next query head and the next item
        }
    }
}

// Shapes of the shared-K/V kernel: (TS waves per workgroup, U rows per load batch).  Four-wave
// workgroups won every sweep on MI355X (the kernel needs 100-200 registers per lane, so small
// workgroups pack the CU better); more query heads per lane want fewer rows in flight per wave.
struct GqaShape {
    int ts, u;
};
static const GqaShape kGqaShapes[] = {{4, 4}, {4, 8}, {4, 2}};
static const int kNumGqaShapes = (int)(sizeof(kGqaShapes) / sizeof(kGqaShapes[0]));

template <int DT, int D, int GQ>
static attn_fn pick_gqa_shape(int shape) {
    switch (shape) {
        case 0: return attn_gqa_kernel<DT, D, GQ, 4, 4>;
        case 1: return attn_gqa_kernel<DT, D, GQ, 4, 8>;
        case 2: return attn_gqa_kernel<DT, D, GQ, 4, 2>;
        default: return nullptr;
    }
}

template <int DT, int D>
static attn_fn pick_gqa_width(int gq, int shape) {
    switch (gq) {
        case 1: return pick_gqa_shape<DT, D, 1>(shape);
        case 2: return pick_gqa_shape<DT, D, 2>(shape);
        case 4: return pick_gqa_shape<DT, D, 4>(shape);
        case 8: return pick_gqa_shape<DT, D, 8>(shape);
        default: return nullptr;
    }
}

int s3i_num_gqa_shapes() { return kNumGqaShapes; }

attn_fn s3i_pick_gqa(int dt, int d, int gq, int shape, int *threads) {
    if (shape < 0 || shape >= kNumGqaShapes) shape = gq == 8 ? 2 : gq == 4 ? 1 : 0;
    *threads = kGqaShapes[shape].ts * 64;
    if (dt == S3_F16) {
        if (d == 64) return pick_gqa_width<S3_F16, 64>(gq, shape);
        if (d == 128) return pick_gqa_width<S3_F16, 128>(gq, shape);
        if (d == 256) return pick_gqa_width<S3_F16, 256>(gq, shape);
    } else {
        if (d == 64) return pick_gqa_width<S3_BF16, 64>(gq, shape);
        if (d == 128) return pick_gqa_width<S3_BF16, 128>(gq, shape);
        if (d == 256) return pick_gqa_width<S3_BF16, 256>(gq, shape);
    }
    return nullptr;
}

