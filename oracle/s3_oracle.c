/*
 * CPU oracle for single-query (decode-step) attention.  TEST INFRASTRUCTURE ONLY:
 * nothing in the product path may call, link or import this file.
 *
 * What it computes (paper section 2.1, the self-attention equation):
 *     h_out = softmax(q . K^T / sqrt(d)) . V
 * for one query row q against the L cached key/value rows of its own sequence,
 * once per attention head (d = head dimension; with one head and d = model
 * dimension this is the paper's formula verbatim).
 *
 * It is the definition written out: a dot product per cached row, the maximum,
 * exponentials, their sum, the normalised weights, and a weighted sum of value
 * rows.  No tiling, no running ("online") softmax, no reordering.
 *
 * Inputs are the values as stored in the KV cache: 16-bit patterns of IEEE
 * binary16 (dtype 0) or bfloat16 (dtype 1), or 8-bit e4m3 codes (dtype 3, one code
 * in the low byte of each uint16_t; the query then has a 16-bit type of its own,
 * qdtype).  They are widened to REAL before any arithmetic.  The file is compiled twice: REAL = float (the fp32 oracle)
 * and REAL = double (its twin, used to bound the fp32 oracle's own error).
 *
 * Row addressing: element d of row j of a matrix is base[j * row_stride + d];
 * the caller chooses row_stride so that per-head slices of [rows][H][D] storage
 * can be addressed without copying.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#ifndef REAL
#error "compile with -DREAL=float -DSUF=f32 or -DREAL=double -DSUF=f64"
#endif
#define CAT_(a, b) a##_##b
#define CAT(a, b) CAT_(a, b)
#define FN(name) CAT(name, SUF)

/* IEEE binary16 -> REAL, exact (every binary16 value is a binary32 value).
 * binary16 = 1 sign, 5 exponent (bias 15), 10 fraction bits;
 * binary32 = 1 sign, 8 exponent (bias 127), 23 fraction bits. */
static REAL widen_f16(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) & 1u;
    uint32_t e = (uint32_t)(h >> 10) & 0x1fu;
    uint32_t f = (uint32_t)h & 0x3ffu;
    float v;
    if (e == 0) {
        v = (float)f * 5.9604644775390625e-8f; /* zero or subnormal: f * 2^-24, exact */
    } else {
        /* normal: same fraction, exponent re-biased by 127 - 15; e == 31 is inf / NaN */
        uint32_t bits = ((e == 31 ? 255u : e + 112u) << 23) | (f << 13);
        memcpy(&v, &bits, sizeof v);
    }
    return (REAL)(sign ? -v : v);
}

/* bfloat16 -> REAL, exact: a bfloat16 is the upper half of a binary32. */
static REAL widen_bf16(uint16_t h)
{
    uint32_t bits = (uint32_t)h << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (REAL)f;
}

/* 8-bit float e4m3 ("fn": finite + NaN, no infinities; the open 8-bit format most 8-bit caches use):
 * 1 sign, 4 exponent (bias 7), 3 fraction bits.  exponent 0: zero / subnormal f * 2^-9;
 * exponent 15 with fraction 7: NaN; everything else (1 + f/8) * 2^(e-7), largest 448. */
static REAL widen_e4m3(uint8_t b)
{
    int sign = b >> 7, e = (b >> 3) & 15, f = b & 7;
    double v;
    if (e == 15 && f == 7) return (REAL)NAN;
    if (e == 0) v = ldexp((double)f, -9);
    else v = ldexp(1.0 + f / 8.0, e - 7);
    return (REAL)(sign ? -v : v);
}

/* REAL-independent: nearest e4m3 code of a float, ties to the even code, magnitudes beyond the
 * largest finite value (448) saturate to it, NaN -> 0x7f.  Written as a search over the 127
 * non-negative finite codes so that it shares nothing with a bit-twiddling implementation. */
static uint8_t quantize_e4m3(float x)
{
    if (x != x) return 0x7f;
    uint8_t sign = (uint8_t)(signbit(x) ? 0x80 : 0);
    double a = fabs((double)x);
    if (a >= 448.0) return (uint8_t)(sign | 0x7e);
    int lo = 0, hi = 0x7e; /* codes are monotone in value: find the last code with value <= a */
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if ((double)widen_e4m3((uint8_t)mid) <= a) lo = mid; else hi = mid - 1;
    }
    if (lo == 0x7e) return (uint8_t)(sign | lo);
    double below = (double)widen_e4m3((uint8_t)lo), above = (double)widen_e4m3((uint8_t)(lo + 1));
    double dl = a - below, du = above - a;
    int code = dl < du ? lo : du < dl ? lo + 1 : ((lo & 1) ? lo + 1 : lo);
    return (uint8_t)(sign | code);
}

/* 16-bit storage types carry their pattern in a uint16_t; the 8-bit type (dtype 3, the number the
 * library's interface gives it) in its low byte. */
static REAL widen(uint16_t h, int dtype)
{
    return dtype == 0 ? widen_f16(h) : dtype == 1 ? widen_bf16(h) : widen_e4m3((uint8_t)h);
}

/* Exposed so that tests can pin the widening against an independent library. */
void FN(s3o_widen)(const uint16_t *src, int64_t n, int dtype, REAL *dst)
{
    for (int64_t i = 0; i < n; i++) dst[i] = widen(src[i], dtype);
}

/* Quantise n floats to e4m3 codes (what an 8-bit cache stores for a new row). */
void FN(s3o_quantize_e4m3)(const float *src, int64_t n, uint8_t *dst)
{
    for (int64_t i = 0; i < n; i++) dst[i] = quantize_e4m3(src[i]);
}

/* Step 1: s_j = scale * sum_d q[d] * K[j][d],  j = 0..L-1. */
void FN(s3o_scores)(const uint16_t *q, int qdtype, const uint16_t *K, int64_t row_stride, int L, int D,
                    int dtype, REAL scale, REAL *s)
{
    for (int j = 0; j < L; j++) {
        REAL dot = 0;
        for (int d = 0; d < D; d++) dot += widen(q[d], qdtype) * widen(K[(int64_t)j * row_stride + d], dtype);
        s[j] = dot * scale;
    }
}

/* Step 2: p = softmax(s): subtract the maximum, exponentiate, divide by the sum. */
void FN(s3o_softmax)(const REAL *s, int L, REAL *p)
{
    if (L <= 0) return;
    REAL m = s[0];
    for (int j = 1; j < L; j++)
        if (s[j] > m) m = s[j];
    REAL Z = 0;
    for (int j = 0; j < L; j++) {
        p[j] = (REAL)(sizeof(REAL) == 4 ? expf((float)(s[j] - m)) : exp((double)(s[j] - m)));
        Z += p[j];
    }
    for (int j = 0; j < L; j++) p[j] /= Z;
}

/* Step 3: o[d] = sum_j p_j * V[j][d]. */
void FN(s3o_weighted_sum)(const REAL *p, const uint16_t *V, int64_t row_stride, int L, int D, int dtype,
                          REAL *o)
{
    for (int d = 0; d < D; d++) o[d] = 0;
    for (int j = 0; j < L; j++)
        for (int d = 0; d < D; d++) o[d] += p[j] * widen(V[(int64_t)j * row_stride + d], dtype);
}

/* One (sequence, head): the three steps in order.  L == 0 (nothing cached) is
 * defined as an all-zero output row.  Returns 0, or -1 if scratch allocation fails. */
int FN(s3o_attend_one)(const uint16_t *q, int qdtype, const uint16_t *K, const uint16_t *V, int64_t row_stride,
                       int L, int D, int dtype, REAL scale, REAL *o)
{
    if (L <= 0) {
        for (int d = 0; d < D; d++) o[d] = 0;
        return 0;
    }
    REAL *s = (REAL *)malloc(sizeof(REAL) * (size_t)L * 2);
    if (!s) return -1;
    REAL *p = s + L;
    FN(s3o_scores)(q, qdtype, K, row_stride, L, D, dtype, scale, s);
    FN(s3o_softmax)(s, L, p);
    FN(s3o_weighted_sum)(p, V, row_stride, L, D, dtype, o);
    free(s);
    return 0;
}

/* A ragged batch.  Sequence b has its own K and V storage, K_ptr[b] / V_ptr[b],
 * laid out [rows][Hkv][D]; it attends over its first len[b] rows only (no padding).
 * q and out are [n][H][D].  Hkv == H is the paper's multi-head attention (section
 * 2.1).  Hkv < H (Hkv divides H) is multi-query attention, which the paper's
 * related-work section names as a way to shrink the cache, in its grouped form:
 * the H query heads are split into Hkv runs of H / Hkv consecutive heads, and run k
 * shares key/value head k; Hkv == 1 is multi-query attention proper (every head
 * reads the one key/value head).  Each query head still computes the same three
 * steps.  The (sequence, head) pairs are independent, so they may be spread over
 * `threads` OpenMP threads (1 = plain serial loops); the arithmetic of each pair
 * is the same either way.  Returns the number of threads used, or -1 on
 * allocation failure or if Hkv does not divide H. */
int FN(s3o_attention_batch)(int n, int H, int Hkv, int D, int dtype, int qdtype, const uint16_t *const *K_ptr,
                            const uint16_t *const *V_ptr, const int32_t *len, const uint16_t *q,
                            REAL scale, REAL *out, int threads)
{
    int used = 1, fail = 0;
    int64_t pairs = (int64_t)n * H;
    if (Hkv < 1 || H % Hkv) return -1;
    int heads_per_kv = H / Hkv;
#ifdef _OPENMP
    if (threads < 1) threads = 1;
    used = threads;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads) reduction(| : fail)
#endif
    for (int64_t i = 0; i < pairs; i++) {
        int b = (int)(i / H), h = (int)(i % H);
        int hk = h / heads_per_kv; /* the key/value head this query head reads */
        int rc = FN(s3o_attend_one)(q + ((int64_t)b * H + h) * D, qdtype, K_ptr[b] + (int64_t)hk * D,
                                    V_ptr[b] + (int64_t)hk * D, (int64_t)Hkv * D, len[b], D, dtype, scale,
                                    out + ((int64_t)b * H + h) * D);
        if (rc) fail |= 1;
    }
    return fail ? -1 : used;
}
