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


// ---- streaming through a per-wave LDS ring ------------------------------------------------------------------
// The rows in flight do not sit in vector registers: every 128-bit load of a row piece goes from global memory
// straight into the wave's ring in LDS (global_load_lds_dwordx4: lane l's 16 bytes land at base + 16*l, so one
// load deposits the same 1 KiB the register path would hold), and the wave reads a row back with ds_read_b128
// when its turn comes.  R rows of K and of V are kept in flight per wave (2 KiB per row) without a register per
// byte, which is what limits the depth of the register path.  The memory counter is managed by hand: loads
// return in issue order, so before rows [j, j+U) are read it is enough that at most the loads issued after
// them - 2 per row - are still outstanding.
typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void glb_void;

__device__ __forceinline__ void dma16_nt(const char *src, char *lds_dst) {
    // aux 2 = nt: the rows are read once (same hint as the register path's non-temporal loads)
    __builtin_amdgcn_global_load_lds((glb_void *)src, (lds_void *)lds_dst, 16, 0, 2);
}

template <int N>
__device__ __forceinline__ void wait_vm_then_read2(const char *s0, const char *s1, u32x4 &k0, u32x4 &v0, u32x4 &k1, u32x4 &v1) {
    const unsigned a0 = (unsigned)(uintptr_t)(lds_void *)s0, a1 = (unsigned)(uintptr_t)(lds_void *)s1;
    asm volatile(
        "s_waitcnt vmcnt(%6)\n\t"
        "ds_read_b128 %0, %4\n\t"
        "ds_read_b128 %1, %4 offset:1024\n\t"
        "ds_read_b128 %2, %5\n\t"
        "ds_read_b128 %3, %5 offset:1024\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(k0), "=&v"(v0), "=&v"(k1), "=&v"(v1)
        : "v"(a0), "v"(a1), "n"(N)
        : "memory");
}

template <int DT, int D, int R, bool FUSED>
__device__ __forceinline__ void wave_tokens_ring(const AttnArgs &a, const Item &it, int hg, int j0, int j1, char *ring,
                                                 float &m, float &l, float (&acc)[8]) {
    constexpr int U = 2;
    typedef TokenStream<DT, D, U, true, FUSED> TS_t;
    typedef HeadLanes<D> HL;
    const int lane = threadIdx.x & 63;
    const int g = lane / HL::LPH, dl = lane % HL::LPH;
    const int h = hg * HL::GH + g;
    const bool lane_ok = h < a.H && dl < HL::USED;
    const int hc = h < a.H ? h : a.H - 1;
    const int dc = dl < HL::USED ? dl : HL::USED - 1;
    const int64_t rstride = (int64_t)a.H * D * 2;
    const int64_t lane_byte = ((int64_t)hc * D + dc * 8) * 2;
    const int64_t in_byte = ((int64_t)it.b * a.H * D) * 2 + lane_byte;
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
    if (HL::USED < HL::LPH && dl >= HL::USED) st.qv = (u32x4){0u, 0u, 0u, 0u};

    m = -INFINITY;
    l = 0.f;
#pragma unroll
    for (int i = 0; i < 8; i++) acc[i] = 0.f;
    if (j0 < j1) {
        char *mine = ring + lane * 16;  // this lane's 16 bytes of every slot
        int issued = j0, islot = 0;     // next row to load and the slot it goes to
        auto issue = [&]() {
            const char *ks = st.kp + (int64_t)issued * rstride, *vs = st.vp + (int64_t)issued * rstride;
            if (FUSED && issued == st.jnew) {
                ks = st.knew;
                vs = st.vnew;
            }
            dma16_nt(ks, ring + islot * 2048);
            dma16_nt(vs, ring + islot * 2048 + 1024);
            issued++;
            islot = islot + 1 == R ? 0 : islot + 1;
        };
        for (int r = 0; r < R && issued < j1; r++) issue();
        int cslot = 0;
        for (int j = j0; j < j1; j += U) {
            // slots of rows j and j+1 (the tail batch of an odd share reads its one row twice; the second
            // copy is masked in reduce)
            const int s0 = cslot, s1 = (j + 1 < j1) ? (cslot + 1 == R ? 0 : cslot + 1) : cslot;
            u32x4 kk[U], vv[U];
            if (issued - j >= R) wait_vm_then_read2<2 * (R - U)>(mine + s0 * 2048, mine + s1 * 2048, kk[0], vv[0], kk[1], vv[1]);
            else wait_vm_then_read2<0>(mine + s0 * 2048, mine + s1 * 2048, kk[0], vv[0], kk[1], vv[1]);
            // the two slots are free again: refill them before the arithmetic
            if (issued < j1) issue();
            if (issued < j1) issue();
            cslot = cslot + U >= R ? cslot + U - R : cslot + U;
            st.reduce(j, kk, vv, m, l, acc);
        }
    }
    if (FUSED && lane_ok && j0 <= st.jnew && st.jnew < j1) {
        *(u32x4 *)(a.kplane + (it.off + st.jnew) * rstride + lane_byte) = *(const u32x4 *)(a.k_new + in_byte);
        *(u32x4 *)(a.vplane + (it.off + st.jnew) * rstride + lane_byte) = *(const u32x4 *)(a.v_new + in_byte);
    }
}

// Merge TS token splits (rows first..first+TS-1 of comb) lane by lane.  Two splits per round: unrolled over
// all of them the eighty values of eight splits would sit in registers at once and set the kernel's register
// count (which decides how many waves a SIMD holds) for the sake of the epilogue wave alone.
template <int TS>
__device__ __forceinline__ void combine_splits(const float (*comb)[10][64], int first, int lane, float &m, float &l,
                                               float (&acc)[8]) {
    m = comb[first][0][lane];
#pragma unroll
    for (int t = 1; t < TS; t++) m = fmaxf(m, comb[first + t][0][lane]);
    l = 0.f;
#pragma unroll
    for (int i = 0; i < 8; i++) acc[i] = 0.f;
#pragma unroll 2
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
// R > 0: the rows in flight go through a per-wave LDS ring of R rows (wave_tokens_ring) instead of registers.
// DYN: the work list is not walked with a fixed stride; after its first item a workgroup takes the next
// unclaimed position from a device-wide counter (fetched by the epilogue wave one item ahead, so that the
// round trip hides behind the streaming), which keeps every compute unit busy to the end whatever else
// occupies some of them, and makes the longest-first order of the list a longest-processing-time schedule.
template <int DT, int D, int TS, int HS, int U, bool NT, bool PF, int R, bool DYN>
__global__ void __launch_bounds__((TS *HS + 1) * 64) attn_step_kernel(const AttnArgs a) {
    constexpr int LPH = HeadLanes<D>::LPH, USED = HeadLanes<D>::USED, GH = HeadLanes<D>::GH;
    constexpr int NWC = TS * HS;  // compute waves
    extern __shared__ __align__(16) char dyn_lds[];  // the batch view, then the rings
    __shared__ int wave_sums[S3_MAX_CLASSES * S3_MAX_WAVES];
    __shared__ float comb[2][NWC][10][64];
    __shared__ long long next_pos[2];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool epilogue = wave == NWC;
    const int ts = wave % TS, hs = wave / TS;
    const int n_hg = (a.H + GH - 1) / GH;
    const int n_hgb = (n_hg + HS - 1) / HS;
    const BatchView bv = build_batch_view(a, dyn_lds, wave_sums);
    const int64_t total = (int64_t)bv.total * n_hgb;
    char *ring = R > 0 ? dyn_lds + ((batch_view_bytes(a.n, a.ncls) + 15) & ~(size_t)15) + (size_t)(epilogue ? 0 : wave) * (R * 2048)
                       : nullptr;

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

    // a work list no longer than the grid deals every position at launch: nothing to claim, no counter traffic
    const bool dyn = DYN && total > (int64_t)gridDim.x;
    int parity = 0;
    int64_t item = blockIdx.x;
    while (item < total) {
        const Item it = decode_item(a, bv, item, n_hgb);
        if (!epilogue) {
            int j0, j1;
            split_rows(it, ts, TS, j0, j1);
            float m, l, acc[8];
            if (R > 0) wave_tokens_ring<DT, D, R, true>(a, it, it.hgb * HS + hs, j0, j1, ring, m, l, acc);
            else wave_tokens<DT, D, U, NT, true, PF>(a, it, it.hgb * HS + hs, j0, j1, m, l, acc);
            comb[parity][wave][0][lane] = m;
            comb[parity][wave][1][lane] = l;
#pragma unroll
            for (int i = 0; i < 8; i++) comb[parity][wave][2 + i][lane] = acc[i];
        } else if (dyn) {
            // claim the position this workgroup works on after `item`; positions below gridDim.x were dealt
            // at launch.  next_pos[parity] was last read after the barrier two items ago.
            unsigned int got = 0;
            if (lane == 0) got = atomicAdd(a.queue, 1u);
            got = __builtin_amdgcn_readfirstlane(got);
            if (lane == 0) next_pos[parity] = (long long)gridDim.x + got;
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
        item = dyn ? (int64_t)next_pos[parity] : item + gridDim.x;
        parity ^= 1;
    }
    if (dyn && threadIdx.x == 0) {
        // the last workgroup to leave puts both counters back to zero for the next launch (nobody claims a
        // position after it has announced its exit)
        const unsigned int gone = atomicAdd(a.queue + 1, 1u);
        if (gone == gridDim.x - 1) {
            atomicExch(a.queue, 0u);
            atomicExch(a.queue + 1, 0u);
        }
    }
}

// ---- the fused step with the row stream carried across items ------------------------------------------------
// In attn_step_kernel a compute wave drains its loads at the end of every item (last rows, LDS hand-over,
// barrier, look-up of the next item, query load) before the first rows of the next item leave: with one
// workgroup per compute unit all eight waves of the unit do so at once and the unit has nothing in flight for
// about one memory round trip per item.  Here a wave keeps two cursors over the workgroup's item sequence: a
// LOADER that issues the row batches (U rows of K and of V into one of two register sets, alternately) and runs
// up to one item ahead, and a REDUCER that consumes the sets in the same order.  When the loader has issued the
// last batch of its share of an item it opens the next item at once (position, rows, query), so the first rows
// of item k+1 are already on their way while the last rows of item k are reduced, handed over and merged.
// Every set load is unconditional (a wave without further work re-reads its query row) so that the memory
// counter the compiler waits on always means the same thing: the other set stays in flight.
// All cursor state is wave-uniform and lives in scalar registers; a row address is a scalar base plus one
// per-lane 32-bit offset.  A share without rows (fewer rows than waves) still takes one batch, whose loads
// point at the query row and whose reduction is skipped.  The new row is stored from the registers it was
// streamed into.  With a dynamic list the epilogue wave claims positions two items ahead: position k+1 is read
// by the loaders between the barriers of items k-1 and k, and was published before the barrier of item k-1.
template <int DT, int D, int TS, int U, bool DYN>
__global__ void __launch_bounds__((TS + 1) * 64) attn_step_stream_kernel(const AttnArgs a) {
    typedef HeadLanes<D> HL;
    typedef TokenStream<DT, D, U, true, true> TS_t;
    constexpr int LPH = HL::LPH, USED = HL::USED, GH = HL::GH;
    constexpr int NO_ROW = -0x40000000;  // "no new row in this share": equal to no row index
    extern __shared__ __align__(16) char dyn_lds[];  // the batch view
    __shared__ int wave_sums[S3_MAX_CLASSES * S3_MAX_WAVES];
    __shared__ float comb[2][TS][10][64];
    __shared__ long long next_pos[2];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool epilogue = wave == TS;
    const int n_hgb = (a.H + GH - 1) / GH;
    // position 0 of a workgroup is its index, position 1 its first claim (visible behind the view's barrier)
    if (DYN && threadIdx.x == TS * 64) next_pos[1] = (long long)gridDim.x + atomicAdd(a.queue, 1u);
    const BatchView bv = build_batch_view(a, dyn_lds, wave_sums);
    // (scalar on purpose: every branch of the cursors below must be provably uniform)
    const int64_t total = uniform64((int64_t)bv.total * n_hgb);
    const int64_t grid = gridDim.x;

    for (int b = blockIdx.x; b < a.n; b += gridDim.x) {  // the new lengths; zero rows of empty or refused contexts
        if (a.len_out && threadIdx.x == 0) a.len_out[b] = a.cur_len[b] + 1;
        if (bv.len[b] == 0) {
            const int per_row = a.H * D / 8;
            const float z[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            for (int e = threadIdx.x; e < per_row; e += (TS + 1) * 64) store_out8(a.out, a.out_dtype, ((int64_t)b * per_row + e) * 8, z);
        }
    }

    if ((int64_t)blockIdx.x < total) {
        if (!epilogue) {
            const int g = lane / LPH, dl = lane % LPH;
            const int dc = dl < USED ? dl : USED - 1;
            const int64_t rstride = (int64_t)a.H * D * 2;

            // ---- loader cursor (wave-uniform except lane_l, ok_l, q_l)
            int seq_l = 0;
            int64_t pos_l = blockIdx.x;
            bool exhausted = false, fresh = false;
            Item it_l;
            int j0_l = 0, j_l = 0, j1_l = 0, jnew_l = NO_ROW;
            int64_t stride_l = 0;
            const char *kb_l = a.q, *vb_l = a.q, *kn_l = a.q, *vn_l = a.q;
            unsigned lane_l = 0;
            bool ok_l = false;
            u32x4 q_l = (u32x4){0u, 0u, 0u, 0u};
            auto open_item = [&]() {
                it_l = uniform_item(decode_item(a, bv, pos_l, n_hgb));
                split_rows(it_l, wave, TS, j0_l, j1_l);
                j_l = j0_l;
                fresh = true;
                const int h = it_l.hgb * GH + g;
                ok_l = h < a.H && dl < USED;
                const int hc = h < a.H ? h : a.H - 1;
                lane_l = (unsigned)((hc * D + dc * 8) * 2);
                const int64_t in_row = (int64_t)it_l.b * a.H * D * 2;  // row b of q / k_new / v_new
                q_l = *(const u32x4 *)(a.q + in_row + lane_l);
                if (USED < LPH && dl >= USED) q_l = (u32x4){0u, 0u, 0u, 0u};
                if (j0_l < j1_l) {
                    kb_l = a.kplane + it_l.off * rstride;
                    vb_l = a.vplane + it_l.off * rstride;
                    kn_l = a.k_new + in_row;
                    vn_l = a.v_new + in_row;
                    stride_l = rstride;
                    jnew_l = it_l.len - 1;
                } else {  // no rows for this wave: its one batch reads the query row and is not reduced
                    kb_l = vb_l = kn_l = vn_l = a.q + in_row;
                    stride_l = 0;
                    jnew_l = NO_ROW;
                }
            };
            auto issue = [&](u32x4(&kk)[U], u32x4(&vv)[U]) {
                if (!exhausted && !fresh && j_l >= j1_l) {  // this share is on its way: on to the next item
                    const int64_t nxt = DYN ? uniform64(next_pos[(seq_l + 1) & 1]) : pos_l + grid;
                    if (nxt < total) {
                        pos_l = nxt;
                        seq_l++;
                        open_item();
                    } else {
                        exhausted = true;
                        stride_l = 0;  // whatever is still issued re-reads one valid row
                        jnew_l = NO_ROW;
                    }
                }
#pragma unroll
                for (int u = 0; u < U; u++) {
                    const int jj = min(j_l + u, j1_l - 1);
                    const char *row = (jj == jnew_l) ? kn_l : kb_l + (int64_t)jj * stride_l;
                    kk[u] = load16<true>(row + (size_t)lane_l);
                }
#pragma unroll
                for (int u = 0; u < U; u++) {
                    const int jj = min(j_l + u, j1_l - 1);
                    const char *row = (jj == jnew_l) ? vn_l : vb_l + (int64_t)jj * stride_l;
                    vv[u] = load16<true>(row + (size_t)lane_l);
                }
                j_l += U;
                fresh = false;
            };

            // ---- reducer cursor
            TS_t st;
            st.scale_log2e = a.scale_log2e;
            int seq_r = 0, j_r = 0, jnew_r = NO_ROW, parity = 0;
            int64_t off_r = 0;
            unsigned lane_r = 0;
            bool ok_r = false;
            float m = -INFINITY, l = 0.f, acc[8];
            auto adopt = [&]() {  // the reducer enters the item the loader has open
                j_r = j0_l;
                st.j1 = j1_l;
                jnew_r = j0_l < j1_l ? it_l.len - 1 : NO_ROW;
                off_r = it_l.off;
                st.qv = q_l;
                lane_r = lane_l;
                ok_r = ok_l;
                m = -INFINITY;
                l = 0.f;
#pragma unroll
                for (int i = 0; i < 8; i++) acc[i] = 0.f;
            };
            // One set: reduce it, close the item if that was its last batch, refill the set.  The loop below has ONE
            // exit, at its bottom, and every trip through it issues the same loads in the same order (after the last
            // item a half only waits for its set and refills it with the query row): the compiler derives how many
            // loads may stay in flight at each wait from ALL paths that reach it, and a path that skipped a refill
            // would make it wait for the other set as well, i.e. drain the pipeline this kernel exists to keep full.
            bool done = false;
            auto half = [&](u32x4(&kk)[U], u32x4(&vv)[U]) {
                if (!done && j_r < st.j1) {
                    st.reduce(j_r, kk, vv, m, l, acc);
                    if (jnew_r >= j_r && jnew_r < j_r + U && jnew_r < st.j1 && ok_r) {  // the append
                        char *kd = a.kplane + (off_r + jnew_r) * rstride + (size_t)lane_r;
                        char *vd = a.vplane + (off_r + jnew_r) * rstride + (size_t)lane_r;
#pragma unroll
                        for (int u = 0; u < U; u++) {
                            if (j_r + u == jnew_r) {
                                *(u32x4 *)kd = kk[u];
                                *(u32x4 *)vd = vv[u];
                            }
                        }
                    }
                } else {
                    // a batch without rows: wait for its loads all the same, so that a set is never refilled
                    // with loads into it still pending
#pragma unroll
                    for (int u = 0; u < U; u++) asm volatile("" ::"v"(kk[u]), "v"(vv[u]));
                }
                j_r += U;
                if (!done && j_r >= st.j1) {
                    comb[parity][wave][0][lane] = m;
                    comb[parity][wave][1][lane] = l;
#pragma unroll
                    for (int i = 0; i < 8; i++) comb[parity][wave][2 + i][lane] = acc[i];
                    __syncthreads();  // the item's only barrier; buffer `parity` is written again two items later
                    parity ^= 1;
                    if (seq_l == seq_r) {
                        done = true;  // the loader opened nothing further: the list is exhausted
                    } else {
                        seq_r++;
                        adopt();
                    }
                }
                issue(kk, vv);
            };

            u32x4 ka[U], va[U], kb[U], vb[U];
            open_item();
            issue(ka, va);
            adopt();
            issue(kb, vb);
            do {
                half(ka, va);
                half(kb, vb);
            } while (!done);
        } else {
            const bool dl_ok = lane % LPH < USED;
            int64_t pos = blockIdx.x;
            int64_t pos1 = DYN ? uniform64(next_pos[1]) : pos + grid;
            int parity = 0;
            while (pos < total) {
                const Item it = decode_item(a, bv, pos, n_hgb);
                int64_t pos2 = pos1 + grid;
                if (DYN && pos1 < total) {  // the position after next; next_pos[parity] was last read before the previous barrier
                    unsigned int got = 0;
                    if (lane == 0) got = atomicAdd(a.queue, 1u);
                    got = __builtin_amdgcn_readfirstlane(got);
                    pos2 = grid + got;
                    if (lane == 0) next_pos[parity] = pos2;
                }
                __syncthreads();
                const int h = it.hgb * GH + lane / LPH;
                if (h < a.H && dl_ok) {
                    float m, l, acc[8];
                    combine_splits<TS>(comb[parity], 0, lane, m, l, acc);
                    emit_chunk<D, true>(a, it, h, lane % LPH, m, l, acc);
                }
                if (it.nchunks > 1) {
                    unsigned int *cnt = a.arrivals + (int64_t)it.b * n_hgb + it.hgb;
                    if (chunk_arrived(a, cnt, it.nchunks)) {  // every chunk of this context has arrived
                        if (h < a.H && dl_ok) merge_chunks<D, true>(a, a.H, it.b, h, lane % LPH, it.nchunks);
                    }
                }
                pos = pos1;
                pos1 = pos2;
                parity ^= 1;
            }
        }
    }
    if (DYN && threadIdx.x == 0) {
        // the last workgroup to leave puts both counters back to zero for the next launch (a workgroup has made
        // all its claims before the barrier of its last item)
        const unsigned int gone = atomicAdd(a.queue + 1, 1u);
        if (gone == gridDim.x - 1) {
            atomicExch(a.queue, 0u);
            atomicExch(a.queue + 1, 0u);
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

// Kernel shapes: (index, TS token splits, HS head groups per workgroup, U rows per load batch, NT, PF, R rows of
// the LDS ring (0: rows in flight sit in registers), DYN dynamic work list, XS row stream carried across items);
// R, DYN and XS concern the fused step kernel only (the attention-only kernel of such a shape is the register /
// fixed-stride one).
#define S3_VARIANTS(X)                            \
    X(0, 4, 1, 4, true, false, 0, false, false)   \
    X(1, 8, 1, 4, true, false, 0, false, false)   \
    X(2, 4, 2, 4, true, false, 0, false, false)   \
    X(3, 1, 4, 4, true, false, 0, false, false)   \
    X(4, 8, 1, 2, true, true, 0, false, false)    \
    X(5, 2, 4, 4, true, false, 0, false, false)   \
    X(6, 1, 8, 4, true, false, 0, false, false)   \
    X(7, 7, 1, 4, true, true, 0, false, false)    \
    X(8, 4, 1, 4, false, false, 0, false, false)  \
    X(9, 15, 1, 2, true, true, 0, false, false)   \
    X(10, 8, 1, 2, true, true, 0, true, false)    \
    X(11, 8, 1, 2, true, true, 6, false, false)   \
    X(12, 8, 1, 2, true, true, 6, true, false)    \
    X(13, 8, 1, 3, true, true, 0, true, false)    \
    X(14, 8, 1, 3, true, true, 0, true, true)     \
    X(15, 8, 1, 2, true, true, 0, true, true)     \
    X(16, 8, 1, 2, true, true, 0, false, true)    \
    X(17, 8, 1, 3, true, true, 0, false, true)
// Defaults (measured on MI355X): shape 4 with a fixed stride while the work list is about as long as the grid
// (batches of up to 128 sequences); beyond, the dynamic work list (+4 % to +7 % on batches of 512 and 700
// sequences; -5 % on a batch of 128 long contexts) with three rows per register set (shape 13: +1.5 % / +0.5 % over
// two rows there; on the small batches three or four rows per set are 1-5 % behind two).  The LDS-ring shapes stay
// selectable for comparison: they measured 2-3 % behind the register path.  So do the shapes that carry the row
// stream across items (14-17): with one workgroup per compute unit they measured level with shape 13 on the
// batch of 512 (0.770-0.775 of peak against 0.7725; two resident workgroups, which their lower register count
// allows, 0.750-0.757) and 1-3 % behind shape 4 on the small batches - the pause of a compute unit's loads at an
// item's end is not what bounds the kernel.  Shapes that were tried with the
// dynamic list and dropped: two or four head groups per workgroup with four or two waves each (0.756 / 0.745 of
// peak on the batch of 512 against 0.762), one workgroup per whole row (eight head groups, one wave each: 0.655).
#define S3_DEFAULT_VARIANT 4
#define S3_DEFAULT_VARIANT_LARGE 13

template <int DT, int D>
static attn_fn pick_variant(int v, bool fused) {
    switch (v) {
#define X(i, ts, hs, u, nt, pf, r, dyn, xs)                                                                       \
    case i:                                                                                                       \
        if (!fused) return (attn_fn)attn_partial_kernel<DT, D, ts, hs, u, nt, pf>;                                  \
        if constexpr (xs) return (attn_fn)attn_step_stream_kernel<DT, D, ts * hs, u, dyn>; /* XS shapes: hs = 1 */ \
        else return (attn_fn)attn_step_kernel<DT, D, ts, hs, u, nt, pf, r, dyn>;
        S3_VARIANTS(X)
#undef X
        default: return nullptr;
    }
}
