// Attention kernels for multi-head 16-bit caches (one cached head per query head), gfx950.  Included by
// s3kv_attn_inst.hip, which is compiled once per head dimension (the instantiations of one head dimension
// form one translation unit so that they build in parallel).
//
// Work decomposition.  The method is bound by HBM bandwidth (about one flop per byte), so the unit of
// parallelism is bytes, not sequences: every context is cut into near-equal chunks of at most `chunk`
// tokens and the (chunk, head-group) pairs of the whole ragged batch form one flat work list, longest
// contexts first, that a fixed grid walks with a stride.  A wavefront covers GH adjacent heads of one
// token per 128-bit load (64 lanes x 16 B = 1 KiB of contiguous memory; head_dim 96: four heads of twelve
// lanes each, 768 contiguous bytes, the other four lanes of every sixteen idle); the lanes of a head
// reduce their dot product with DPP row operations, keep a running maximum and sum in fp32, and
// accumulate their 8-element slice of the output.  The TS waves of a workgroup that share a head group
// split the chunk's tokens and merge through LDS; chunks of one context merge in a second kernel
// (s3_decode_attention) or, in the fused step, in the epilogue wave of whichever workgroup delivers the
// last chunk.  Score s_j = q.K_j * scale as in the section 2.1 equation of the S3 paper; softmax is
// max-subtracted; everything after the 16-bit loads is fp32.
#pragma once
#include "s3kv_device.h"

// Lanes of a wave that share one head.  A lane holds 8 elements (16 bytes), so a head needs D/8 lanes;
// they sit in a group of LPH adjacent lanes, LPH a power of two so that the DPP reductions apply: for
// D = 96 twelve of sixteen lanes are used.
template <int D>
struct HeadLanes {
    static constexpr int USED = D / 8;
    static constexpr int LPH = D == 96 ? 16 : D / 8;
    static constexpr int GH = 64 / LPH;  // heads per wave load
};

// One wave's share of an item: tokens [j0, j1) of head group hg, online softmax in fp32.
// DT: element type of q/K/V.  D: head_dim.  U: tokens per load batch.  NT: non-temporal loads.
// FUSED: row len-1 is still only in k_new / v_new: it is taken from there and, by the wave whose
// range holds it, written into the arena (the append).
// PF: software pipelining - the loads of the next batch of U tokens are issued before the current
// batch is reduced, so the wave always has loads in flight (two register sets, used alternately).
template <int DT, int D, int U, bool NT, bool FUSED>
struct TokenStream {
    static constexpr int LPH = HeadLanes<D>::LPH;
    static constexpr int GH = HeadLanes<D>::GH;
    const char *kp, *vp, *knew, *vnew;
    int64_t rstride;
    int jnew, j1;
    float scale_log2e;
    u32x4 qv;

    __device__ __forceinline__ void load(int j, u32x4 (&kk)[U], u32x4 (&vv)[U]) const {
#pragma unroll
        for (int u = 0; u < U; u++) {
            const int jj = min(j + u, j1 - 1);
            const char *src = kp + (int64_t)jj * rstride;
            if (FUSED) src = (jj == jnew) ? knew : src;
            kk[u] = load16<NT>(src);
        }
#pragma unroll
        for (int u = 0; u < U; u++) {
            const int jj = min(j + u, j1 - 1);
            const char *src = vp + (int64_t)jj * rstride;
            if (FUSED) src = (jj == jnew) ? vnew : src;
            vv[u] = load16<NT>(src);
        }
    }

    __device__ __forceinline__ void reduce(int j, const u32x4 (&kk)[U], const u32x4 (&vv)[U], float &m, float &l,
                                           float (&acc)[8]) const {
        float s[U];
#pragma unroll
        for (int u = 0; u < U; u++) s[u] = dot8<DT>(qv, kk[u]);
#pragma unroll
        for (int u = 0; u < U; u++) s[u] = group_sum<LPH>(s[u]);
        float mb = -INFINITY;
#pragma unroll
        for (int u = 0; u < U; u++) {
            s[u] = (j + u < j1) ? s[u] * scale_log2e : -INFINITY;
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
};

template <int DT, int D, int U, bool NT, bool FUSED, bool PF>
__device__ __forceinline__ void wave_tokens(const AttnArgs &a, const Item &it, int hg, int j0, int j1, float &m,
                                            float &l, float (&acc)[8]) {
    typedef TokenStream<DT, D, U, NT, FUSED> TS_t;
    typedef HeadLanes<D> HL;
    const int lane = threadIdx.x & 63;
    const int g = lane / HL::LPH, dl = lane % HL::LPH;
    const int h = hg * HL::GH + g;
    // lanes beyond the heads of the row, and the idle lanes of a head group (D = 96), stream the bytes of a
    // lane that exists (same cache lines, no extra memory traffic), contribute a zero query and never store
    const bool lane_ok = h < a.H && dl < HL::USED;
    const int hc = h < a.H ? h : a.H - 1;
    const int dc = dl < HL::USED ? dl : HL::USED - 1;
    const int64_t rstride = (int64_t)a.H * D * 2;
    const int64_t lane_byte = ((int64_t)hc * D + dc * 8) * 2;
    const int64_t in_byte = ((int64_t)it.b * a.H * D) * 2 + lane_byte;  // this lane's slice of row b of q/k_new/v_new
    TS_t st;
    st.kp = a.kplane + it.off * rstride + lane_byte;
    st.vp = a.vplane + it.off * rstride + lane_byte;
    st.knew = FUSED ? a.k_new + in_byte : nullptr;
    st.vnew = FUSED ? a.v_new + in_byte : nullptr;
    st.rstride = rstride;
    st.jnew = FUSED ? it.len - 1 : -1;
    st.j1 = j1;
    st.scale_log2e = a.scale_log2e;
    st.qv = *(const u32x4 *)(a.q + in_byte);
    if (HL::USED < HL::LPH && dl >= HL::USED) st.qv = (u32x4){0u, 0u, 0u, 0u};  // idle lanes add nothing to the head's dot product

    m = -INFINITY;
    l = 0.f;
#pragma unroll
    for (int i = 0; i < 8; i++) acc[i] = 0.f;
    if (!PF) {
        for (int j = j0; j < j1; j += U) {
            u32x4 kk[U], vv[U];
            st.load(j, kk, vv);
            st.reduce(j, kk, vv, m, l, acc);
        }
    } else if (j0 < j1) {
        u32x4 ka[U], va[U], kb[U], vb[U];
        st.load(j0, ka, va);
        for (int j = j0; j < j1; j += 2 * U) {
            const bool more = j + U < j1;
            if (more) st.load(j + U, kb, vb);
            st.reduce(j, ka, va, m, l, acc);
            if (more) {
                if (j + 2 * U < j1) st.load(j + 2 * U, ka, va);
                st.reduce(j + U, kb, vb, m, l, acc);
            }
        }
    }
    if (FUSED && lane_ok && j0 <= st.jnew && st.jnew < j1) {  // the append: this wave owns the new row's slice
        *(u32x4 *)(a.kplane + (it.off + st.jnew) * rstride + lane_byte) = *(const u32x4 *)(a.k_new + in_byte);
        *(u32x4 *)(a.vplane + (it.off + st.jnew) * rstride + lane_byte) = *(const u32x4 *)(a.v_new + in_byte);
    }
}

// Merge TS token splits (rows first..first+TS-1 of comb) lane by lane.
template <int TS>
__device__ __forceinline__ void combine_splits(const float (*comb)[10][64], int first, int lane, float &m, float &l,
                                               float (&acc)[8]) {
    m = comb[first][0][lane];
    for (int t = 1; t < TS; t++) m = fmaxf(m, comb[first + t][0][lane]);
    l = 0.f;
#pragma unroll
    for (int i = 0; i < 8; i++) acc[i] = 0.f;
    for (int t = 0; t < TS; t++) {  // split 0 is never empty, so m is finite; empty splits weigh exp2(-inf) = 0
        const float wt = fast_exp2(comb[first + t][0][lane] - m);
        l += wt * comb[first + t][1][lane];
#pragma unroll
        for (int i = 0; i < 8; i++) acc[i] += wt * comb[first + t][2 + i][lane];
    }
}

// Write one (chunk, head) result: the final output row slice if the context has a single chunk,
// else the partial (max, sum, weighted sum).
template <int D, bool COHERENT>
__device__ __forceinline__ void emit_chunk(const AttnArgs &a, const Item &it, int h, int dl, float m, float l,
                                           const float (&acc)[8]) {
    if (it.nchunks == 1) {
        const float inv = 1.f / l;
        float o[8];
#pragma unroll
        for (int i = 0; i < 8; i++) o[i] = acc[i] * inv;
        store_out8(a.out, a.out_dtype, ((int64_t)it.b * a.H + h) * D + dl * 8, o);
        return;
    }
    const int64_t pi = ((int64_t)it.b * a.max_chunks + it.c) * a.H + h;
    float *pml = (float *)a.part_ml + 2 * pi;
    float *pa = a.part_acc + pi * D + dl * 8;
    if (dl == 0) put_partial2<COHERENT>(pml, (f32x2){m, l});
    put_partial4<COHERENT>(pa, (f32x4){acc[0], acc[1], acc[2], acc[3]});
    put_partial4<COHERENT>(pa + 4, (f32x4){acc[4], acc[5], acc[6], acc[7]});
}

// Attention only (s3_decode_attention): TS*HS waves; the TS waves of a head group split the chunk's
// tokens and merge through LDS; multi-chunk contexts are finished by attn_merge_kernel.
template <int DT, int D, int TS, int HS, int U, bool NT, bool PF>
__global__ void __launch_bounds__(TS *HS * 64) attn_partial_kernel(const AttnArgs a) {
    constexpr int LPH = HeadLanes<D>::LPH, USED = HeadLanes<D>::USED, GH = HeadLanes<D>::GH;
    constexpr int NW = TS * HS;
    extern __shared__ __align__(16) char dyn_lds[];  // the batch view
    __shared__ int wave_sums[S3_MAX_CLASSES * S3_MAX_WAVES];
    __shared__ float comb[TS > 1 ? NW : 1][10][64];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ts = wave % TS, hs = wave / TS;
    const int n_hg = (a.H + GH - 1) / GH;
    const int n_hgb = (n_hg + HS - 1) / HS;
    const BatchView bv = build_batch_view(a, dyn_lds, wave_sums);
    const int64_t total = (int64_t)bv.total * n_hgb;

    for (int64_t item = blockIdx.x; item < total; item += gridDim.x) {
        const Item it = decode_item(a, bv, item, n_hgb);
        const int hg = it.hgb * HS + hs;
        int j0, j1;
        split_rows(it, ts, TS, j0, j1);
        float m, l, acc[8];
        wave_tokens<DT, D, U, NT, false, PF>(a, it, hg, j0, j1, m, l, acc);
        if (TS > 1) {
            comb[wave][0][lane] = m;
            comb[wave][1][lane] = l;
#pragma unroll
            for (int i = 0; i < 8; i++) comb[wave][2 + i][lane] = acc[i];
            __syncthreads();
            if (ts == 0) combine_splits<TS>(comb, wave, lane, m, l, acc);
        }
        const int h = hg * GH + lane / LPH;
        if (ts == 0 && h < a.H && lane % LPH < USED) emit_chunk<D, false>(a, it, h, lane % LPH, m, l, acc);
        if (TS > 1) __syncthreads();  // comb is reused by the next item
    }
}

// The whole layer-step in one launch (s3_decode_step): TS*HS compute waves plus ONE epilogue wave.
// Compute waves stream their token shares (taking the new row from k_new / v_new and appending it),
// drop (max, sum, weighted sum) into one of two LDS buffers and move on to the next item after a
// single barrier.  The epilogue wave merges the splits, writes the output or the chunk partial,
// announces the chunk on the context's arrival counter and, if it delivered the last chunk, merges
// the chunks; all its memory latencies overlap with the compute waves' next item.  len_out and the
// zero rows of empty contexts are published by the workgroups in turn.
template <int DT, int D, int TS, int HS, int U, bool NT, bool PF>
__global__ void __launch_bounds__((TS *HS + 1) * 64) attn_step_kernel(const AttnArgs a) {
    constexpr int LPH = HeadLanes<D>::LPH, USED = HeadLanes<D>::USED, GH = HeadLanes<D>::GH;
    constexpr int NWC = TS * HS;  // compute waves
    extern __shared__ __align__(16) char dyn_lds[];  // the batch view
    __shared__ int wave_sums[S3_MAX_CLASSES * S3_MAX_WAVES];
    __shared__ float comb[2][NWC][10][64];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool epilogue = wave == NWC;
    const int ts = wave % TS, hs = wave / TS;
    const int n_hg = (a.H + GH - 1) / GH;
    const int n_hgb = (n_hg + HS - 1) / HS;
    const BatchView bv = build_batch_view(a, dyn_lds, wave_sums);
    const int64_t total = (int64_t)bv.total * n_hgb;

    // Housekeeping that belongs to no item, spread over the workgroups (sequence b goes to workgroup
    // b mod grid) so that none of them starts its first item late: the new lengths, and a zero output
    // row for empty or refused contexts.
    for (int b = blockIdx.x; b < a.n; b += gridDim.x) {
        if (a.len_out && threadIdx.x == 0) a.len_out[b] = a.cur_len[b] + 1;
        if (bv.len[b] == 0) {
            const int per_row = a.H * D / 8;
            const float z[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            for (int e = threadIdx.x; e < per_row; e += (NWC + 1) * 64) store_out8(a.out, a.out_dtype, ((int64_t)b * per_row + e) * 8, z);
        }
    }

    int parity = 0;
    for (int64_t item = blockIdx.x; item < total; item += gridDim.x, parity ^= 1) {
        const Item it = decode_item(a, bv, item, n_hgb);
        if (!epilogue) {
            int j0, j1;
            split_rows(it, ts, TS, j0, j1);
            float m, l, acc[8];
            wave_tokens<DT, D, U, NT, true, PF>(a, it, it.hgb * HS + hs, j0, j1, m, l, acc);
            comb[parity][wave][0][lane] = m;
            comb[parity][wave][1][lane] = l;
#pragma unroll
            for (int i = 0; i < 8; i++) comb[parity][wave][2 + i][lane] = acc[i];
        }
        // The only barrier of an item.  Buffer `parity` is next written two items later, after the
        // barrier of item+1, which the epilogue wave reaches only when it is done reading it.
        __syncthreads();
        if (epilogue) {
            const bool dl_ok = lane % LPH < USED;
            for (int s = 0; s < HS; s++) {
                const int h = (it.hgb * HS + s) * GH + lane / LPH;
                if (h < a.H && dl_ok) {
                    float m, l, acc[8];
                    combine_splits<TS>(comb[parity], s * TS, lane, m, l, acc);
                    emit_chunk<D, true>(a, it, h, lane % LPH, m, l, acc);
                }
            }
            if (it.nchunks > 1) {
                unsigned int *cnt = a.arrivals + (int64_t)it.b * n_hgb + it.hgb;
                if (chunk_arrived(a, cnt, it.nchunks)) {  // every chunk of this context has arrived
                    for (int s = 0; s < HS; s++) {
                        const int h = (it.hgb * HS + s) * GH + lane / LPH;
                        if (h < a.H && dl_ok) merge_chunks<D, true>(a, a.H, it.b, h, lane % LPH, it.nchunks);
                    }
                }
            }
        }
    }
}

// One wave per (sequence, head group): merge the chunk partials of contexts longer than one
// chunk; write zeros for empty contexts; leave single-chunk contexts (already final) alone.
template <int D>
__global__ void __launch_bounds__(256) attn_merge_kernel(const AttnArgs a) {
    constexpr int LPH = HeadLanes<D>::LPH, USED = HeadLanes<D>::USED, GH = HeadLanes<D>::GH;
    const int lane = threadIdx.x & 63;
    const int n_hg = (a.H + GH - 1) / GH;
    const int64_t wid = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (wid >= (int64_t)a.n * n_hg) return;
    const int b = (int)(wid / n_hg), hg = (int)(wid % n_hg);
    const int h = hg * GH + lane / LPH, dl = lane % LPH;
    if (h >= a.H || dl >= USED) return;
    const int nchunks = chunks_of(a, b, a.chunk);
    if (nchunks == 1) return;
    if (nchunks > 1) {
        merge_chunks<D, false>(a, a.H, b, h, dl, nchunks);
        return;
    }
    const float z[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    store_out8(a.out, a.out_dtype, ((int64_t)b * a.H + h) * D + dl * 8, z);
}

// Kernel shapes: (index, TS token splits, HS head groups per workgroup, U rows per load batch, NT, PF).
#define S3_VARIANTS(X)            \
    X(0, 4, 1, 4, true, false)    \
    X(1, 8, 1, 4, true, false)    \
    X(2, 4, 2, 4, true, false)    \
    X(3, 1, 4, 4, true, false)    \
    X(4, 8, 1, 2, true, true)     \
    X(5, 2, 4, 4, true, false)    \
    X(6, 1, 8, 4, true, false)    \
    X(7, 7, 1, 4, true, true)     \
    X(8, 4, 1, 4, false, false)   \
    X(9, 15, 1, 2, true, true)
#define S3_DEFAULT_VARIANT 4

template <int DT, int D>
static attn_fn pick_variant(int v, bool fused) {
    switch (v) {
#define X(i, ts, hs, u, nt, pf) \
    case i: return fused ? (attn_fn)attn_step_kernel<DT, D, ts, hs, u, nt, pf> : (attn_fn)attn_partial_kernel<DT, D, ts, hs, u, nt, pf>;
        S3_VARIANTS(X)
#undef X
        default: return nullptr;
    }
}
