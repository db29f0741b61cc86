// Matrix-core attention kernel for shared key/value heads (multi-query / grouped-query attention,
// which the paper's related-work section names as a complementary way to shrink the cache), gfx950.
// Launched by the host code in s3kv_kernels.hip through the pointer s3i_pick_gqa_mfma returns.
//
// With one cached head serving `group` query heads, a decode step is no longer one dot product per
// cached row but a small dense contraction: scores S^T[rows x heads] = K[rows x D] . Q^T[D x heads]
// and output O^T[D x heads] = V^T[D x rows] . P^T[rows x heads].  The vector-ALU kernel repeats the
// dot / exp / accumulate work per query head and becomes instruction bound from about eight heads
// per cached head; here both products run on MFMA and every (row, head) score is handled by
// exactly one lane.
//
// One wave = one work item = (sequence, chunk of its context, K/V head, block of 16 query heads);
// the four waves of a workgroup are independent (no barrier after the batch-view prologue).  Per
// tile of 16 cached rows:
//   * K: lane (r = lane % 16, g = lane / 16) holds 16 bytes (8 elements) of row r at element offset
//     32*ks + 8*g, ks = 0 .. D/32-1 - loaded so directly with plain loads, or, in launches whose K rows
//     exceed the memory-side cache, loaded in whole rows with the streaming hint and brought into that
//     layout through a per-wave LDS buffer - : the A operand of
//     v_mfma_f32_16x16x32 (row r, contraction slots of lane group g); Q^T is the B operand, loaded
//     once per item with the same slot assignment (head = lane % 16), so whichever way the
//     instruction numbers its contraction slots, both operands agree.  The accumulator holds
//     S^T[row 4*g + i][head lane % 16], i < 4.
//   * softmax: scale into log2 units, mask rows past the end, tile maximum per head (over the four
//     registers, then across the four lane groups); the exponent reference m follows the maximum
//     lazily (see the loop), p = exp2(s - m), running sum.
//   * V: the accumulator layout of S^T is already the B-operand layout of v_mfma_f32_16x16x16
//     (4 contraction slots = rows 4*g .. 4*g+3, column = head), so P^T needs no shuffle.  The A
//     operand V^T (row of the product = output element d, contraction = cached rows) needs four
//     cached rows at ONE d per lane, while memory holds eight d of one row per 16-byte load: the V
//     tile goes through a per-wave LDS buffer (row-major, row stride padded by 8 bytes so that the
//     four lane groups hit different banks) and is read back as 16-bit gathers.  With 8-bit rows a
//     lane reads one 32-bit word (four consecutive d) from each of its four rows and transposes the
//     4 x 4 codes in registers (eight v_perm_b32), which feeds four products at once; the products'
//     operand rows are numbered accordingly (d = 64q + 4n + j) and the results leave in that order.
//   * p enters the second product as two 16-bit operands of the storage type, a high part (p rounded)
//     and a low part (the remainder, rounded), and the product is issued for both, which keeps the
//     weights' error near 2^-16 (bfloat16) / 2^-22 (fp16) instead of 2^-9 / 2^-12: with one part only,
//     values of magnitude 1e2 put the fp16 kernel outside the attention tolerance.
// Accumulators: O^T block db holds O^T[d = 16*db + 4*g + i][head], fp32.  Results leave as the
// final row (single-chunk contexts) or as a chunk partial (max, sum, unnormalised row).  Partials are
// finished either by attn_merge_kernel (a second launch) or, with merge_in_kernel, inside this launch:
// an arrival counter per (sequence, K/V head, query block), write-through partials, the wave that
// delivers the last chunk merges.  Done at once after every item this tripled the kernel's time (with
// one wave per item nothing hides the write-through and the counter's round trip); here the
// publication of an item trails the wave's work by two items - the counter is bumped at the end of the
// NEXT item, when the partial's stores have long completed, and its answer is looked at one item
// later still - so a wave never waits for either.  It still loses to the merge launch and is not the
// default: with 128-row chunks nearly every item leaves an 8 KiB partial, and written through to memory
// (as partials that cross XCDs inside one launch must be) they cost more than the launch they save -
// 32 query / 8 cached heads x 128, 256 sequences: kernel 74 -> 101 us, whole step 72 -> 89 us;
// multi-query 16/1 x 256: 29 -> 65 us.  In a decode step the new row is read from k_new / v_new and
// appended by the wave that owns it.
#include <type_traits>

#include "s3kv_device.h"

typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

template <int DT>
__device__ __forceinline__ f32x4 mfma_scores(const u32x4 a, const u32x4 b, const f32x4 c) {
    if (DT == S3_F16)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

template <int DT>
__device__ __forceinline__ f32x4 mfma_values(const u32x2 a, const u32x2 b, const f32x4 c) {
    if (DT == S3_F16)
        return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4, a), __builtin_bit_cast(f16x4, b), c, 0, 0, 0);
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(i16x4, a), __builtin_bit_cast(i16x4, b), c, 0, 0, 0);
}

__device__ __forceinline__ unsigned pack_f16(float lo, float hi) {
    const f16x2 h = {(_Float16)lo, (_Float16)hi};
    return __builtin_bit_cast(unsigned, h);
}
__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {  // round to nearest even (v_cvt_pk_bf16_f32)
    const bf16x2 h = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(unsigned, h);
}

// Four consecutive output elements starting at element index e.
__device__ __forceinline__ void store_out4(void *out, int out_dtype, int64_t e, const f32x4 v) {
    if (out_dtype == S3_F32) {
        *(f32x4 *)((float *)out + e) = v;
    } else {
        u32x2 w;
        if (out_dtype == S3_F16) {
            w[0] = pack_f16(v[0], v[1]);
            w[1] = pack_f16(v[2], v[3]);
        } else {
            w[0] = f32_to_bf16_rne(v[0]) | (f32_to_bf16_rne(v[1]) << 16);
            w[1] = f32_to_bf16_rne(v[2]) | (f32_to_bf16_rne(v[3]) << 16);
        }
        *(u32x2 *)((uint16_t *)out + e) = w;
    }
}

// Two e4m3 codes (bytes 2*half, 2*half+1 of w) -> one 32-bit word of two DT elements, exact: every e4m3 value
// is an fp16 and a bfloat16 number, and gfx950 converts a pair of codes to either type in one instruction
// (v_cvt_scalef32_pk_{f16,bf16}_fp8 with scale 1).
template <int DT>
__device__ __forceinline__ unsigned widen2_e4m3(const unsigned w, const bool upper) {
    if (DT == S3_F16) {
        const f16x2 h = upper ? __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w, 1.0f, true) : __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w, 1.0f, false);
        return __builtin_bit_cast(unsigned, h);
    }
    const bf16x2 h = upper ? __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, true) : __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, false);
    return __builtin_bit_cast(unsigned, h);
}

// Bytes j of four words -> one word, j = 0..3 (a 4 x 4 byte transpose in eight v_perm_b32; selector bytes 0-3
// pick from the second operand, 4-7 from the first).
__device__ __forceinline__ void transpose4x4_bytes(const unsigned w0, const unsigned w1, const unsigned w2, const unsigned w3,
                                                   unsigned (&t)[4]) {
    const unsigned a_lo = __builtin_amdgcn_perm(w1, w0, 0x05010400u);  // w0.0 w1.0 w0.1 w1.1
    const unsigned a_hi = __builtin_amdgcn_perm(w1, w0, 0x07030602u);  // w0.2 w1.2 w0.3 w1.3
    const unsigned b_lo = __builtin_amdgcn_perm(w3, w2, 0x05010400u);  // w2.0 w3.0 w2.1 w3.1
    const unsigned b_hi = __builtin_amdgcn_perm(w3, w2, 0x07030602u);
    t[0] = __builtin_amdgcn_perm(b_lo, a_lo, 0x05040100u);  // w0.0 w1.0 w2.0 w3.0
    t[1] = __builtin_amdgcn_perm(b_lo, a_lo, 0x07060302u);
    t[2] = __builtin_amdgcn_perm(b_hi, a_hi, 0x05040100u);
    t[3] = __builtin_amdgcn_perm(b_hi, a_hi, 0x07060302u);
}

// A chunk whose partial this wave has written and whose arrival is still to be counted / answered.
struct PendingChunk {
    unsigned int *cnt;  // the context's arrival counter; null: nothing pending
    int b, hq0, nheads, nchunks;
};

// The wave that delivered the last chunk of (sequence b, query heads hq0 .. hq0+nheads-1) merges their chunk
// partials: 64/(D/8) heads per pass, each lane its 8-element slice.
template <int D>
__device__ __forceinline__ void merge_pending(const AttnArgs &a, const PendingChunk &p, int lane) {
    constexpr int LPH = D / 8, HPP = 64 / LPH;
    for (int h0 = 0; h0 < p.nheads; h0 += HPP) {
        const int h = h0 + lane / LPH;
        if (h < p.nheads) merge_chunks<D, true>(a, a.Hq, p.b, p.hq0 + h, lane % LPH, p.nchunks);
    }
}

// KV8: the cache rows are e4m3 codes (one byte per element) and DT is the type of q; a 16-byte load then
// holds 16 elements, which are widened (exactly) to DT in registers and feed two contraction steps.
template <int DT, int D, bool KV8>
__global__ void __launch_bounds__(256, D <= 128 ? 2 : 1) attn_gqa_mfma_kernel(const AttnArgs a) {
    constexpr int EB = KV8 ? 1 : 2;       // bytes per cached element
    constexpr int KS = D / 32;            // contraction steps of the score product
    constexpr int KL = KV8 ? D / 64 : KS; // 16-byte K loads per lane and tile
    constexpr int DB = D / 16;            // 16-element blocks of an output row
    constexpr int PPR = D * EB / 16;      // 16-byte pieces per cached row of one head
    constexpr int VL = 16 * PPR / 64;     // 16-byte loads per lane for a 16-row V tile
    // LDS row stride of the V tile, bytes.  16-bit rows: 8 bytes of padding, so that the four lane groups' 16-bit
    // gathers hit different banks.  8-bit rows: 16 bytes, so that rows stay 16-byte aligned and the four lane
    // groups' 32-bit reads (rows 4g .. 4g+3, sixteen consecutive words each) cover the banks evenly.
    constexpr int VSTRIDE = KV8 ? D + 16 : D * 2 + 8;
    constexpr float RESCALE_LOG2 = 8.f;   // see the softmax step
    extern __shared__ __align__(16) char dyn_lds[];  // the batch view
    __shared__ int wave_sums[S3_MAX_CLASSES * S3_MAX_WAVES];
    // LDS row stride of the K tile: with 16 bytes of padding the 128-bit reads of sixteen rows cover every bank once
    constexpr int KSTRIDE = D * EB + 16;
    __shared__ __align__(16) char vtile[4][16 * VSTRIDE];
    __shared__ __align__(16) char ktile[4][16 * KSTRIDE];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int group = a.Hq / a.H;
    const int nqb = (group + 15) / 16;  // blocks of 16 query heads per K/V head
    const int per_seq = a.H * nqb;
    const BatchView bv = build_batch_view(a, dyn_lds, wave_sums);
    const int64_t total = (int64_t)bv.total * per_seq;
    if (blockIdx.x == 0) {
        if (a.len_out)
            for (int b = threadIdx.x; b < a.n; b += 256) a.len_out[b] = a.cur_len[b] + 1;
    }
    const bool ink = a.merge_in_kernel != 0;
    // Dynamic work list: a wave takes its first item by its index and then claims positions from a device-wide
    // counter, so that the waves end together whatever their items' lengths (the items of a ragged batch differ
    // by a factor of five and a fixed stride leaves the sum of a dozen of them to chance).
    // One device-wide counter serves a few million claims a second, far fewer than the waves of a large launch
    // ask for, so only the END of the list is dealt that way: the first dyn_list per cent of the positions (whole
    // rounds of the grid) go by stride.
    // Not the default: measured +2.4 % and +3.6 % on 1024 and 2048 sequences of 32q/8kv x 128 with three quarters of
    // the list by stride, -11 % on 1024 sequences with 8-bit rows (items half as long, claims twice as often) and
    // -40 % on 256 sequences (three rounds of the grid).
    const int static_pct = a.dyn_list > 0 ? a.dyn_list : 0;
    const bool dyn = static_pct > 0 && static_pct < 100 && a.queue != nullptr;
    if (ink) {  // no merge launch follows: the zero rows of empty or refused contexts are written here, by the workgroups in turn
        for (int b = blockIdx.x; b < a.n; b += gridDim.x) {
            if (bv.len[b] == 0) {
                const float z[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                for (int e = threadIdx.x; e < a.Hq * D / 8; e += 256) store_out8(a.out, a.out_dtype, ((int64_t)b * a.Hq * D / 8 + e) * 8, z);
            }
        }
    }
    // Chunks published by this wave whose bookkeeping is still due (wave-uniform): `told` has its partial in
    // flight to memory, `counted` has been counted on its context's arrival counter and awaits the answer.
    PendingChunk told, counted;
    told.cnt = counted.cnt = nullptr;
    unsigned int counted_old = 0;
    auto settle = [&](bool drain) {
        if (!told.cnt && !counted.cnt) return;
        // everything this wave stored or loaded before the current item's results has completed: the loads were
        // consumed, and the stores are older than they
        __builtin_amdgcn_s_waitcnt(0);
        for (int round = 0; round < (drain ? 2 : 1); round++) {
            if (counted.cnt) {
                if (__builtin_amdgcn_readfirstlane(counted_old) == (unsigned int)(counted.nchunks - 1)) {
                    if (lane == 0) atomicExch(counted.cnt, 0u);  // leave the counter clean for the next launch
                    if (a.merge_sync) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
                    merge_pending<D>(a, counted, lane);
                }
                counted.cnt = nullptr;
            }
            if (told.cnt) {
                if (a.merge_sync) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
                if (lane == 0) counted_old = atomicAdd(told.cnt, 1u);
                counted = told;
                told.cnt = nullptr;
            }
        }
    };

    char *vt = vtile[wave];
    char *kt = ktile[wave];
    const int64_t rstride = (int64_t)a.H * D * EB;
    const unsigned rs32 = (unsigned)rstride;  // a cached row of all K/V heads: below 2^32 bytes
    // SK: the K rows of this launch are more than the memory-side cache holds, so none of them survives until
    // the next step and they are read with the streaming hint like the V rows; otherwise with plain loads (a batch
    // whose K rows fit - 256 sequences of 32q/8kv x 128 - finds most of them still cached one step later: 0.76 of
    // peak against 0.63 with the hint; a batch of 1024 the other way round, 0.66 against 0.63).
    auto run_items = [&](auto stream_k_tag) {
    constexpr bool SK = decltype(stream_k_tag)::value;
    const int64_t n_waves = (int64_t)gridDim.x * 4;
    // positions below t_static (at least one round: a wave's first item is always its own index) go by stride
    const int64_t t_static = dyn ? max((int64_t)1, total * static_pct / 100 / n_waves) * n_waves : total;
    int64_t item = (int64_t)blockIdx.x * 4 + wave;
    while (item < total) {
        // dynamic part of the work list: the position after this one is claimed now and looked at when this item is done
        const bool claim_next = dyn && item + n_waves >= t_static;
        unsigned int claimed = 0;
        if (claim_next && lane == 0) claimed = atomicAdd(a.queue, 1u);
        const Item it = decode_item(a, bv, item, per_seq);
        const int hk = it.hgb / nqb, qb = it.hgb - hk * nqb;
        const int start = it.c * it.clen, end = min(it.len, start + it.clen);
        const int head = qb * 16 + n;  // query head of this lane's column, within the group
        const bool head_ok = head < group;
        const int hq = hk * group + (head_ok ? head : group - 1);

        u32x4 qop[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ks++) {
            // elements of contraction step ks held by lane group g: the same as the K operand's (a 16-byte K
            // load of 8-bit rows covers 16 elements = steps 2j and 2j+1 of lane group g)
            const int e0 = KV8 ? (ks >> 1) * 64 + g * 16 + (ks & 1) * 8 : ks * 32 + g * 8;
            qop[ks] = *(const u32x4 *)(a.q + (((int64_t)it.b * a.Hq + hq) * D + e0) * 2);
            if (!head_ok) qop[ks] = (u32x4){0u, 0u, 0u, 0u};  // padding columns: zero scores, never stored
        }
        char *kbase = a.kplane + it.off * rstride + (int64_t)hk * D * EB;
        char *vbase = a.vplane + it.off * rstride + (int64_t)hk * D * EB;
        // Decode step (len_add = 1): row len-1 is still only in k_new / v_new.  Every reader takes it from
        // there; the wave of query block 0 whose chunk holds it also writes it into the arena (the append).
        // (8-bit rows are quantised by the append kernel before this launch: nothing to take from k_new.)
        const int jnew = (a.len_add && !KV8) ? it.len - 1 : -1;
        const char *knew = a.k_new + ((int64_t)it.b * a.H + hk) * D * 2;
        const char *vnew = a.v_new + ((int64_t)it.b * a.H + hk) * D * 2;

        f32x4 o[DB];
#pragma unroll
        for (int db = 0; db < DB; db++) o[db] = (f32x4){0.f, 0.f, 0.f, 0.f};
        float m = -INFINITY, lsum = 0.f;

        // Loads of one 16-row tile (rows past the chunk's end are clamped to its last row and masked later).
        // V, and K when it streams (SK): whole rows per load instruction (16 bytes per lane, PPR lanes per row).
        // K otherwise: the operand layout directly (row n, 16 bytes at 64 ks + 16 g).
        auto load_tile = [&](int r0, u32x4 (&kld)[KL], u32x4 (&vv)[VL]) {
            static_assert(KL == VL, "K and V tiles are loaded with the same pattern");
            if (SK) {
#pragma unroll
                for (int i = 0; i < KL; i++) {
                    const int idx = i * 64 + lane;
                    const int rv = min(r0 + idx / PPR, end - 1);
                    kld[i] = load16<true>((rv == jnew ? knew : kbase + (uint64_t)(unsigned)rv * rs32) + (idx % PPR) * 16);
                }
            } else {
                const int rk = min(r0 + n, end - 1);
                const char *krow = (rk == jnew ? knew : kbase + (uint64_t)(unsigned)rk * rs32) + g * 16;
#pragma unroll
                for (int ks = 0; ks < KL; ks++) kld[ks] = load16<false>(krow + ks * 64);
            }
#pragma unroll
            for (int i = 0; i < VL; i++) {
                const int idx = i * 64 + lane;
                const int rv = min(r0 + idx / PPR, end - 1);
                vv[i] = load16<true>((rv == jnew ? vnew : vbase + (uint64_t)(unsigned)rv * rs32) + (idx % PPR) * 16);
            }
        };
        auto reduce_tile = [&](int r0, const u32x4 (&kld)[KL], const u32x4 (&vv)[VL]) {
            if (qb == 0 && jnew >= r0 && jnew < r0 + 16 && jnew < end) {  // this tile holds the new row: append it
                if (!SK && r0 + n == jnew) {
#pragma unroll
                    for (int ks = 0; ks < KL; ks++)
                        *(u32x4 *)(kbase + (uint64_t)(unsigned)jnew * rs32 + g * 16 + ks * 64) = kld[ks];
                }
#pragma unroll
                for (int i = 0; i < VL; i++) {
                    const int idx = i * 64 + lane;
                    if (r0 + idx / PPR == jnew) {
                        if (SK) *(u32x4 *)(kbase + (uint64_t)(unsigned)jnew * rs32 + (idx % PPR) * 16) = kld[i];
                        *(u32x4 *)(vbase + (uint64_t)(unsigned)jnew * rs32 + (idx % PPR) * 16) = vv[i];
                    }
                }
            }
            u32x4 kop[KL];
            if (SK) {
                // K tile through this wave's LDS buffer into operand layout, one 128-bit read per contraction load.
                // (Loading the operand layout directly is 64 separate 16-byte cache accesses per instruction and
                // fetches every 128-byte line twice, the second time from the L1 - which the streaming hint forgoes.)
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int i = 0; i < KL; i++) {
                    const int idx = i * 64 + lane;
                    *(u32x4 *)(kt + (idx / PPR) * KSTRIDE + (idx % PPR) * 16) = kld[i];
                }
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int ks = 0; ks < KL; ks++) kop[ks] = *(const u32x4 *)(kt + n * KSTRIDE + ks * 64 + g * 16);
                __builtin_amdgcn_wave_barrier();
            } else {
#pragma unroll
                for (int ks = 0; ks < KL; ks++) kop[ks] = kld[ks];
            }
            f32x4 s = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ks++) {
                u32x4 kk;
                if (KV8) {
                    const u32x4 raw = kop[ks >> 1];
#pragma unroll
                    for (int w = 0; w < 2; w++) {
                        const unsigned word = raw[(ks & 1) * 2 + w];
                        kk[2 * w] = widen2_e4m3<DT>(word, false);
                        kk[2 * w + 1] = widen2_e4m3<DT>(word, true);
                    }
                } else {
                    kk = kop[ks];
                }
                s = mfma_scores<DT>(kk, qop[ks], s);
            }

            float sv[4], mt = -INFINITY;
#pragma unroll
            for (int i = 0; i < 4; i++) {
                sv[i] = (r0 + 4 * g + i < end) ? s[i] * a.scale_log2e : -INFINITY;
                mt = fmaxf(mt, sv[i]);
            }
            mt = fmaxf(mt, __shfl_xor(mt, 16));
            mt = fmaxf(mt, __shfl_xor(mt, 32));
            // Lazy reference: m is the exponent reference of the running sums, not necessarily the
            // running maximum.  It moves (and the accumulators are rescaled) only when a tile's
            // maximum exceeds it by more than RESCALE_LOG2, so p stays below 2^RESCALE_LOG2 and the
            // rescale, which would otherwise run for almost every tile, runs for the first tile and
            // then hardly ever.  (max, sum, row) leave the kernel consistent with whatever m is, which
            // is all the merge of chunks needs.
            const bool move = mt > m + RESCALE_LOG2;  // first tile: m = -inf
            if (__builtin_amdgcn_ballot_w64(move) != 0) {
                const float mn = move ? mt : m;
                const float alpha = fast_exp2(m - mn);  // 1 where the reference stays, 0 on the first tile
                lsum *= alpha;
#pragma unroll
                for (int db = 0; db < DB; db++) o[db] *= alpha;
                m = mn;
            }
            float p[4];
#pragma unroll
            for (int i = 0; i < 4; i++) {
                p[i] = fast_exp2(sv[i] - m);
                lsum += p[i];
            }

            // The weights enter the second product as 16-bit operands: a high part (p rounded to the type) and
            // a low part (what the high part misses, rounded again), two products per value block.  Together
            // they carry about twice the type's mantissa, so the weighted sum is as exact as the fp32 weights
            // allow, also for values of large magnitude (one rounded part alone is off by 2^-12 of |p v|).
            u32x2 pop, pop_lo;
            float r[4];
            if (DT == S3_F16) {
#pragma unroll
                for (int i = 0; i < 4; i++) r[i] = p[i] - (float)(_Float16)p[i];
                pop[0] = pack_f16(p[0], p[1]);
                pop[1] = pack_f16(p[2], p[3]);
                pop_lo[0] = pack_f16(r[0], r[1]);
                pop_lo[1] = pack_f16(r[2], r[3]);
            } else {
#pragma unroll
                for (int i = 0; i < 4; i++) r[i] = p[i] - (float)(__bf16)p[i];
                pop[0] = pack_bf16(p[0], p[1]);
                pop[1] = pack_bf16(p[2], p[3]);
                pop_lo[0] = pack_bf16(r[0], r[1]);
                pop_lo[1] = pack_bf16(r[2], r[3]);
            }

            // V tile through this wave's LDS buffer.  The LDS unit serves one wave's operations in
            // issue order; the wave barriers only keep the compiler from moving them across.
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int i = 0; i < VL; i++) {
                const int idx = i * 64 + lane;
                char *dst = vt + (idx / PPR) * VSTRIDE + (idx % PPR) * 16;
                const u32x4 w = vv[i];
                if (KV8) {
                    *(u32x4 *)dst = w;
                } else {
                    *(u32x2 *)dst = (u32x2){w[0], w[1]};
                    *(u32x2 *)(dst + 8) = (u32x2){w[2], w[3]};
                }
            }
            __builtin_amdgcn_wave_barrier();
            if (KV8) {
                // Four products at a time: this lane's operand row m = n of products 4q .. 4q+3 is output element
                // d = 64q + 4n + j (j = 0..3), four consecutive codes = ONE 32-bit word per cached row; the words of
                // rows 4g .. 4g+3 are transposed in registers into the four operands (codes of four rows at one d).
#pragma unroll
                for (int q4 = 0; q4 < DB / 4; q4++) {
                    const unsigned *src = (const unsigned *)(vt + (4 * g) * VSTRIDE + q4 * 64) + n;
                    unsigned t[4];
                    transpose4x4_bytes(src[0], src[VSTRIDE / 4], src[2 * (VSTRIDE / 4)], src[3 * (VSTRIDE / 4)], t);
#pragma unroll
                    for (int j = 0; j < 4; j++) {
                        const u32x2 vop = (u32x2){widen2_e4m3<DT>(t[j], false), widen2_e4m3<DT>(t[j], true)};
                        o[4 * q4 + j] = mfma_values<DT>(vop, pop, o[4 * q4 + j]);
                        o[4 * q4 + j] = mfma_values<DT>(vop, pop_lo, o[4 * q4 + j]);
                    }
                }
            } else {
#pragma unroll
                for (int db = 0; db < DB; db++) {
                    const unsigned short *src = (const unsigned short *)(vt + (4 * g) * VSTRIDE) + db * 16 + n;
                    const unsigned v0 = src[0], v1 = src[VSTRIDE / 2], v2 = src[2 * (VSTRIDE / 2)], v3 = src[3 * (VSTRIDE / 2)];
                    const u32x2 vop = (u32x2){v0 | (v1 << 16), v2 | (v3 << 16)};
                    o[db] = mfma_values<DT>(vop, pop, o[db]);
                    o[db] = mfma_values<DT>(vop, pop_lo, o[db]);
                }
            }
            __builtin_amdgcn_wave_barrier();
        };
        // Two register sets used alternately: the next tile's loads are in flight while this one is reduced.
        // The loop takes tiles in pairs for as long as a further tile follows the pair, so that every load in it is
        // unconditional (the compiler then lets the other set's loads stay in flight at each wait); the last one
        // or two tiles follow outside, and no tile beyond the chunk's end is ever loaded.
        u32x4 k0[KL], v0[VL], k1[KL], v1[VL];
        load_tile(start, k0, v0);
        int r0 = start;
        while (r0 + 32 < end) {
            load_tile(r0 + 16, k1, v1);
            reduce_tile(r0, k0, v0);
            load_tile(r0 + 32, k0, v0);
            reduce_tile(r0 + 16, k1, v1);
            r0 += 32;
        }
        if (r0 + 16 < end) {
            load_tile(r0 + 16, k1, v1);
            reduce_tile(r0, k0, v0);
            reduce_tile(r0 + 16, k1, v1);
        } else {
            reduce_tile(r0, k0, v0);
        }

        lsum += __shfl_xor(lsum, 16);
        lsum += __shfl_xor(lsum, 32);
        if (ink) settle(false);
        if (head_ok) {
            // Four consecutive output elements per store.  16-bit rows: accumulator block t holds elements
            // 16t + 4g + i (i = 0..3).  8-bit rows (see the V product): register i of blocks 4q .. 4q+3 holds
            // elements 64q + 16g + 4i + j.
            auto piece = [&](int t, int &d0) -> f32x4 {
                if (!KV8) {
                    d0 = t * 16 + 4 * g;
                    return o[t];
                }
                const int q4 = t / 4, i = t % 4;
                d0 = q4 * 64 + 16 * g + 4 * i;
                return (f32x4){o[4 * q4][i], o[4 * q4 + 1][i], o[4 * q4 + 2][i], o[4 * q4 + 3][i]};
            };
            if (it.nchunks == 1) {
                const float inv = 1.f / lsum;
#pragma unroll
                for (int t = 0; t < DB; t++) {
                    int d0;
                    const f32x4 v = piece(t, d0);
                    store_out4(a.out, a.out_dtype, ((int64_t)it.b * a.Hq + hq) * D + d0, v * inv);
                }
            } else {
                const int64_t pi = ((int64_t)it.b * a.max_chunks + it.c) * a.Hq + hq;
                if (ink) {
                    if (g == 0) put_partial2<true>((float *)a.part_ml + 2 * pi, (f32x2){m, lsum});
                } else {
                    if (g == 0) a.part_ml[pi] = make_float2(m, lsum);
                }
#pragma unroll
                for (int t = 0; t < DB; t++) {
                    int d0;
                    const f32x4 v = piece(t, d0);
                    if (ink) put_partial4<true>(a.part_acc + pi * D + d0, v);
                    else *(f32x4 *)(a.part_acc + pi * D + d0) = v;
                }
            }
        }
        if (ink && it.nchunks > 1) {
            told.cnt = a.arrivals + (int64_t)it.b * per_seq + it.hgb;
            told.b = it.b;
            told.hq0 = hk * group + qb * 16;
            told.nheads = min(16, group - qb * 16);
            told.nchunks = it.nchunks;
        }
        item = claim_next ? t_static + (int64_t)__builtin_amdgcn_readfirstlane(claimed) : item + n_waves;
    }
    };
    // chunk counts bound the rows: (chunks - 1) * chunk < rows of a context <= chunks * chunk
    const int64_t k_bytes = (int64_t)bv.total * a.chunk * rstride;
    if (a.stream_k < 0 ? k_bytes > ((int64_t)256 << 20) : a.stream_k != 0) run_items(std::true_type{});
    else run_items(std::false_type{});
    if (ink) settle(true);  // the last one or two chunks of this wave
    if (dyn && lane == 0) {
        // the last wave to leave puts both counters back to zero for the next launch (a wave has made all its
        // claims before it announces its exit)
        const unsigned int gone = atomicAdd(a.queue + 1, 1u);
        if (gone == (unsigned int)(gridDim.x * 4 - 1)) {
            atomicExch(a.queue, 0u);
            atomicExch(a.queue + 1, 0u);
        }
    }
}

attn_fn s3i_pick_gqa_mfma(int dt, int d) {
    if (dt == S3_F16) {
        if (d == 64) return attn_gqa_mfma_kernel<S3_F16, 64, false>;
        if (d == 128) return attn_gqa_mfma_kernel<S3_F16, 128, false>;
        if (d == 256) return attn_gqa_mfma_kernel<S3_F16, 256, false>;
    } else {
        if (d == 64) return attn_gqa_mfma_kernel<S3_BF16, 64, false>;
        if (d == 128) return attn_gqa_mfma_kernel<S3_BF16, 128, false>;
        if (d == 256) return attn_gqa_mfma_kernel<S3_BF16, 256, false>;
    }
    return nullptr;
}

// The same kernel over 8-bit (e4m3) rows; act is the type of q.
attn_fn s3i_pick_gqa_mfma8(int act, int d) {
    if (act == S3_F16) {
        if (d == 64) return attn_gqa_mfma_kernel<S3_F16, 64, true>;
        if (d == 128) return attn_gqa_mfma_kernel<S3_F16, 128, true>;
        if (d == 256) return attn_gqa_mfma_kernel<S3_F16, 256, true>;
    } else if (act == S3_BF16) {
        if (d == 64) return attn_gqa_mfma_kernel<S3_BF16, 64, true>;
        if (d == 128) return attn_gqa_mfma_kernel<S3_BF16, 128, true>;
        if (d == 256) return attn_gqa_mfma_kernel<S3_BF16, 256, true>;
    }
    return nullptr;
}
