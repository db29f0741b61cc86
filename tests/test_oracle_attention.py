"""Pins of the CPU attention oracle against things other than itself.

The oracle follows the self-attention equation of section 2.1 of the paper.  Here it is
held to: an independent 16-bit widening (numpy / torch), closed forms (a golden file,
length-1 contexts, identical keys, zero query, one-hot values), invariants (weights sum
to one, shift invariance, permutation invariance, rows beyond the length are never read),
library routines it must reduce to (scipy softmax, torch scaled-dot-product attention),
brute force in pure Python floats, and its own float64 twin.
"""
import math
import os

import numpy as np
import pytest

from oracle import kv_oracle as orc
from paper_2306_06000_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bits(x, dtype):
    return wl.to_bits(np.asarray(x, np.float32), dtype)


def np_widen(b, dtype):
    """Independent widening: numpy's float16, or a shift into float32 done by numpy."""
    b = np.asarray(b, np.uint16)
    if dtype == orc.F16:
        return b.view(np.float16).astype(np.float64)
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


# ---------------------------------------------------------------- widening
def test_widen_f16_all_patterns_match_numpy():
    allb = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = orc.widen(allb, orc.F16, "f32")
    want = allb.view(np.float16).astype(np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))
    got64 = orc.widen(allb, orc.F16, "f64")
    assert np.array_equal(got64[~nan], want[~nan].astype(np.float64))


def test_widen_bf16_all_patterns_match_torch():
    import torch

    allb = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = orc.widen(allb, orc.BF16, "f32")
    want = torch.from_numpy(allb.view(np.int16).copy()).view(torch.bfloat16).float().numpy()
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def test_bf16_rounding_of_generator_matches_torch():
    import torch

    x = np.random.default_rng(1).standard_normal(100000).astype(np.float32)
    mine = wl.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(mine, ref)


# ---------------------------------------------------------------- golden closed form
def _read_golden():
    rows = {"K": [], "V": []}
    for line in open(os.path.join(GOLDEN, "attention_closed_form.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        vals = [float(v) for v in vals]
        if key in ("K", "V"):
            rows[key].append(vals)
        else:
            rows[key] = vals
    return rows


@pytest.mark.parametrize("dtype", [orc.F16, orc.BF16])
@pytest.mark.parametrize("precision", ["f32", "f64"])
def test_golden_closed_form(dtype, precision):
    g = _read_golden()
    q = bits(g["q"], dtype)
    K = bits(g["K"], dtype)
    V = bits(g["V"], dtype)
    s = orc.scores(q, K, dtype, 1.0 / math.sqrt(4), precision)
    assert np.allclose(s, [1.0, 0.0], atol=1e-7)
    p = orc.softmax(s, precision)
    assert np.allclose(p, g["p"], atol=2e-7)
    out, _ = orc.attention_ragged(q.reshape(1, 1, 4), [K.reshape(2, 1, 4)], [V.reshape(2, 1, 4)], [2], dtype,
                                  None, precision)
    assert np.allclose(out[0, 0], g["out"], atol=1e-6)


# ---------------------------------------------------------------- softmax
@pytest.mark.parametrize("precision", ["f32", "f64"])
def test_softmax_invariants_and_scipy(precision):
    from scipy.special import softmax as sp_softmax

    rng = np.random.default_rng(2)
    for L in (1, 2, 7, 64, 1000):
        s = rng.standard_normal(L) * 5
        p = orc.softmax(s, precision).astype(np.float64)
        tol = 1e-6 if precision == "f32" else 1e-13
        assert abs(p.sum() - 1.0) < tol * max(1, L / 50)
        assert (p > 0).all() and (p <= 1).all()
        assert np.allclose(p, sp_softmax(s.astype(np.float32 if precision == "f32" else np.float64).astype(
            np.float64)), atol=tol)
        shifted = orc.softmax(s + 3.25, precision)
        assert np.allclose(shifted, p, atol=20 * tol)


def test_softmax_huge_scores_are_finite_and_pick_the_max():
    s = np.array([1.0, -2.0, 3.0, 2.5]) * 1e4
    p = orc.softmax(s, "f32")
    assert np.isfinite(p).all()
    assert np.argmax(p) == 2 and abs(p[2] - 1.0) < 1e-6


# ---------------------------------------------------------------- special cases
@pytest.mark.parametrize("dtype", [orc.F16, orc.BF16])
def test_length_one_returns_v_exactly(dtype):
    rng = np.random.default_rng(3)
    H, D = 3, 16
    q = wl.normal_bits(rng, (2, H, D), dtype)
    K = [wl.normal_bits(rng, (4, H, D), dtype) for _ in range(2)]
    V = [wl.normal_bits(rng, (4, H, D), dtype) for _ in range(2)]
    out, _ = orc.attention_ragged(q, K, V, [1, 1], dtype)
    for b in range(2):
        assert np.array_equal(out[b].astype(np.float64), np_widen(V[b][0], dtype))


@pytest.mark.parametrize("dtype", [orc.F16, orc.BF16])
def test_identical_keys_and_zero_query_give_mean_of_v(dtype):
    rng = np.random.default_rng(4)
    H, D, L = 2, 32, 37
    q = wl.normal_bits(rng, (1, H, D), dtype)
    krow = wl.normal_bits(rng, (1, H, D), dtype)
    K = np.repeat(krow, L, axis=0)
    V = wl.normal_bits(rng, (L, H, D), dtype)
    mean = np_widen(V, dtype).mean(axis=0)
    out, _ = orc.attention_ragged(q, [K], [V], [L], dtype)
    assert np.allclose(out[0], mean, atol=2e-6)
    Kr = wl.normal_bits(rng, (L, H, D), dtype)
    out0, _ = orc.attention_ragged(np.zeros_like(q), [Kr], [V], [L], dtype)
    assert np.allclose(out0[0], mean, atol=2e-6)


def test_one_hot_values_read_back_the_softmax_weights():
    dtype = orc.F16
    rng = np.random.default_rng(5)
    L = D = 16
    q = wl.normal_bits(rng, (1, 1, D), dtype)
    K = wl.normal_bits(rng, (L, 1, D), dtype)
    V = bits(np.eye(L, D).reshape(L, 1, D), dtype)
    out, _ = orc.attention_ragged(q, [K], [V], [L], dtype)
    qf, kf = np_widen(q[0, 0], dtype), np_widen(K[:, 0], dtype)
    s = kf @ qf / math.sqrt(D)
    p = np.exp(s - s.max())
    p /= p.sum()
    assert np.allclose(out[0, 0], p, atol=1e-6)
    # a transposed product (rows of K indexed by d) would need L == D to even run; make sure
    # the answer is not symmetric under that mistake
    sT = kf.T @ qf / math.sqrt(D)
    pT = np.exp(sT - sT.max())
    pT /= pT.sum()
    assert not np.allclose(out[0, 0], pT, atol=1e-3)


def test_permuting_cached_rows_leaves_output_unchanged():
    dtype = orc.F16
    rng = np.random.default_rng(6)
    H, D, L = 4, 64, 211
    q = wl.normal_bits(rng, (1, H, D), dtype)
    K = wl.normal_bits(rng, (L, H, D), dtype)
    V = wl.normal_bits(rng, (L, H, D), dtype)
    perm = rng.permutation(L)
    a, _ = orc.attention_ragged(q, [K], [V], [L], dtype)
    b, _ = orc.attention_ragged(q, [K[perm]], [V[perm]], [L], dtype)
    assert np.allclose(a, b, atol=2e-6)
    assert not np.allclose(a, orc.attention_ragged(q, [K[perm]], [V], [L], dtype)[0], atol=1e-3)


def test_rows_beyond_length_are_never_read_and_empty_context_is_zero():
    dtype = orc.F16
    rng = np.random.default_rng(7)
    H, D = 2, 16
    q = wl.normal_bits(rng, (3, H, D), dtype)
    K = [wl.normal_bits(rng, (10, H, D), dtype) for _ in range(3)]
    V = [wl.normal_bits(rng, (10, H, D), dtype) for _ in range(3)]
    lens = [10, 4, 0]
    ref, _ = orc.attention_ragged(q, K, V, lens, dtype)
    for b in range(3):
        K[b][lens[b]:] = 0x7E00  # NaN
        V[b][lens[b]:] = 0x7E00
    got, _ = orc.attention_ragged(q, K, V, lens, dtype)
    assert np.array_equal(ref, got)
    assert np.isfinite(got).all()
    assert np.array_equal(got[2], np.zeros((H, D), np.float32))


# ---------------------------------------------------------------- brute force / library
def _brute(qf, Kf, Vf, scale):
    """Explicit score vector with Python floats and lists only."""
    L, D = len(Kf), len(qf)
    s = [sum(qf[d] * Kf[j][d] for d in range(D)) * scale for j in range(L)]
    m = max(s)
    w = [math.exp(x - m) for x in s]
    Z = sum(w)
    return [sum(w[j] / Z * Vf[j][d] for j in range(L)) for d in range(D)]


@pytest.mark.parametrize("dtype", [orc.F16, orc.BF16])
def test_brute_force_tiny(dtype):
    rng = np.random.default_rng(8)
    for B, H, D in ((1, 1, 4), (3, 2, 8), (2, 2, 5)):
        lens = [int(rng.integers(1, 6)) for _ in range(B)]
        q = wl.normal_bits(rng, (B, H, D), dtype)
        K = [wl.normal_bits(rng, (5, H, D), dtype) for _ in range(B)]
        V = [wl.normal_bits(rng, (5, H, D), dtype) for _ in range(B)]
        out32, _ = orc.attention_ragged(q, K, V, lens, dtype, None, "f32")
        out64, _ = orc.attention_ragged(q, K, V, lens, dtype, None, "f64")
        for b in range(B):
            for h in range(H):
                want = _brute(np_widen(q[b, h], dtype).tolist(),
                              np_widen(K[b][:lens[b], h], dtype).tolist(),
                              np_widen(V[b][:lens[b], h], dtype).tolist(), 1.0 / math.sqrt(D))
                assert np.allclose(out64[b, h], want, atol=1e-12)
                assert np.allclose(out32[b, h], want, atol=1e-6)


def test_single_head_matches_torch_sdpa():
    """One head with D = hidden size is the paper's formula verbatim; torch's CPU float64
    scaled-dot-product attention with a single query row is the textbook routine for it."""
    import torch

    dtype = orc.F16
    rng = np.random.default_rng(9)
    D, L = 128, 77
    q = wl.normal_bits(rng, (1, 1, D), dtype)
    K = wl.normal_bits(rng, (L, 1, D), dtype)
    V = wl.normal_bits(rng, (L, 1, D), dtype)
    tq = torch.from_numpy(np_widen(q, dtype)).reshape(1, 1, 1, D)
    tk = torch.from_numpy(np_widen(K, dtype)).reshape(1, 1, L, D)
    tv = torch.from_numpy(np_widen(V, dtype)).reshape(1, 1, L, D)
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).reshape(D).numpy()
    out64, _ = orc.attention_ragged(q, [K], [V], [L], dtype, None, "f64")
    out32, _ = orc.attention_ragged(q, [K], [V], [L], dtype, None, "f32")
    assert np.allclose(out64[0, 0], want, atol=1e-12)
    assert np.allclose(out32[0, 0], want, atol=1e-6)


def test_multi_head_matches_torch_sdpa_ragged():
    import torch

    dtype = orc.BF16
    rng = np.random.default_rng(10)
    H, D = 12, 128
    lens = [1, 63, 200]
    q = wl.normal_bits(rng, (3, H, D), dtype)
    K = [wl.normal_bits(rng, (L + 3, H, D), dtype) for L in lens]
    V = [wl.normal_bits(rng, (L + 3, H, D), dtype) for L in lens]
    out, _ = orc.attention_ragged(q, K, V, lens, dtype, None, "f32", threads=2)
    for b, L in enumerate(lens):
        tq = torch.from_numpy(np_widen(q[b], dtype)).reshape(1, H, 1, D)
        tk = torch.from_numpy(np_widen(K[b][:L], dtype)).permute(1, 0, 2).reshape(1, H, L, D)
        tv = torch.from_numpy(np_widen(V[b][:L], dtype)).permute(1, 0, 2).reshape(1, H, L, D)
        want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).reshape(H, D).numpy()
        assert np.allclose(out[b], want, atol=2e-6)


def test_explicit_scale_is_used():
    dtype = orc.F16
    rng = np.random.default_rng(11)
    D, L = 16, 9
    q = wl.normal_bits(rng, (1, 1, D), dtype)
    K = wl.normal_bits(rng, (L, 1, D), dtype)
    V = wl.normal_bits(rng, (L, 1, D), dtype)
    a, _ = orc.attention_ragged(q, [K], [V], [L], dtype, 0.7)
    want = _brute(np_widen(q[0, 0], dtype).tolist(), np_widen(K[:, 0], dtype).tolist(),
                  np_widen(V[:, 0], dtype).tolist(), 0.7)
    assert np.allclose(a[0, 0], want, atol=1e-6)


# ---------------------------------------------------------------- shared key/value heads
@pytest.mark.parametrize("H,Hkv", [(8, 2), (8, 1), (12, 4), (6, 6)])
def test_shared_kv_heads_match_torch_sdpa_with_repeated_heads(H, Hkv):
    """Grouped / multi-query attention (related work): query head h reads key/value head
    h // (H // Hkv).  Textbook routine: repeat every key/value head H // Hkv times in place and
    run ordinary multi-head attention.  A wrong head mapping (h % Hkv, a transposed group) or a
    wrong row stride fails here because all heads hold different numbers."""
    import torch

    dtype = orc.F16
    rng = np.random.default_rng(21)
    D = 64
    lens = [1, 37, 130]
    q = wl.normal_bits(rng, (3, H, D), dtype)
    K = [wl.normal_bits(rng, (L + 2, Hkv, D), dtype) for L in lens]
    V = [wl.normal_bits(rng, (L + 2, Hkv, D), dtype) for L in lens]
    out, _ = orc.attention_ragged(q, K, V, lens, dtype, None, "f64", threads=2)
    g = H // Hkv
    for b, L in enumerate(lens):
        tq = torch.from_numpy(np_widen(q[b], dtype)).reshape(1, H, 1, D)
        tk = torch.from_numpy(np_widen(K[b][:L], dtype)).permute(1, 0, 2).repeat_interleave(g, dim=0).reshape(1, H, L, D)
        tv = torch.from_numpy(np_widen(V[b][:L], dtype)).permute(1, 0, 2).repeat_interleave(g, dim=0).reshape(1, H, L, D)
        want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).reshape(H, D).numpy()
        assert np.allclose(out[b], want, atol=1e-12)


def test_shared_kv_heads_equal_multi_head_on_copied_heads():
    """The same thing without a library: materialise the shared heads as H separate (equal) heads
    and run the multi-head oracle; bit-equal because each head's arithmetic is the same."""
    dtype = orc.BF16
    rng = np.random.default_rng(22)
    H, Hkv, D = 8, 2, 32
    lens = [5, 64]
    q = wl.normal_bits(rng, (2, H, D), dtype)
    K = [wl.normal_bits(rng, (L, Hkv, D), dtype) for L in lens]
    V = [wl.normal_bits(rng, (L, Hkv, D), dtype) for L in lens]
    shared, _ = orc.attention_ragged(q, K, V, lens, dtype)
    full, _ = orc.attention_ragged(q, [np.repeat(k, H // Hkv, axis=1) for k in K],
                                   [np.repeat(v, H // Hkv, axis=1) for v in V], lens, dtype)
    assert np.array_equal(shared, full)


def test_kv_oracle_bytes_per_token_counts_kv_heads_only():
    """Cache bytes per token are 2 (K and V) * layers * kv heads * d * 2 bytes: with all heads this
    is the 4*l*d_h of section 2.1; sharing key/value heads divides it by the group size."""
    full = orc.KVOracle(28, 16, 256, orc.F16, 64, 2048, 1 << 30, store=False)
    mqa = orc.KVOracle(28, 16, 256, orc.F16, 64, 2048, 1 << 30, store=False, n_kv_heads=1)
    gqa = orc.KVOracle(28, 16, 256, orc.F16, 64, 2048, 1 << 30, store=False, n_kv_heads=4)
    assert full.bytes_per_token == 4 * 28 * 4096
    assert mqa.bytes_per_token * 16 == full.bytes_per_token
    assert gqa.bytes_per_token * 4 == full.bytes_per_token
    assert mqa.N == (1 << 30) // mqa.bytes_per_token


# ---------------------------------------------------------------- 8-bit (e4m3) cache rows
def test_e4m3_widening_matches_torch_for_all_codes():
    import torch

    codes = np.arange(256, dtype=np.uint16)
    got = orc.widen(codes, orc.E4M3, "f32")
    want = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy()
    nan = np.isnan(want)
    assert nan.sum() == 2 and np.array_equal(np.isnan(got), nan)      # 0x7f and 0xff
    assert np.array_equal(got[~nan], want[~nan])
    assert got[0x7e] == 448.0 and got[0x01] == 2.0 ** -9 and got[0x38] == 1.0  # the format's corner values


def test_e4m3_quantiser_matches_torch_below_overflow_and_saturates_above():
    """Nearest code, ties to even: torch's float8_e4m3fn conversion is the library routine for that
    wherever the value does not overflow (it yields NaN on overflow; the cache saturates instead)."""
    import torch

    rng = np.random.default_rng(31)
    x = np.concatenate([rng.standard_normal(200000).astype(np.float32) * 3,
                        rng.uniform(-464, 464, 50000).astype(np.float32),
                        (rng.standard_normal(20000) * 2.0 ** -8).astype(np.float32),   # subnormal range
                        np.array([0.0, -0.0, 2.0 ** -10, 3 * 2.0 ** -11, 2.0 ** -9, 17.0, 19.0, 448.0, 463.9], np.float32)])
    # every midpoint between neighbouring codes (ties) and both its float neighbours
    vals = orc.widen(np.arange(0x7f, dtype=np.uint16), orc.E4M3, "f64")
    mids = ((vals[:-1] + vals[1:]) / 2).astype(np.float32)
    x = np.concatenate([x, mids, -mids, np.nextafter(mids, np.float32(0)), np.nextafter(mids, np.float32(1e9))])
    got = orc.quantize_e4m3(x).astype(np.uint8)
    want = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(got, want)
    # overflow: saturate to the largest finite code with the sign kept; NaN stays NaN
    big = np.array([464.0, 465.0, 1e6, np.inf, -464.0, -1e30, -np.inf], np.float32)
    assert orc.quantize_e4m3(big).tolist() == [0x7e, 0x7e, 0x7e, 0x7e, 0xfe, 0xfe, 0xfe]
    assert orc.quantize_e4m3(np.array([np.nan], np.float32)).tolist() == [0x7f]
    # every finite code is a fixed point
    codes = np.array([c for c in range(256) if c not in (0x7f, 0xff)], np.uint16)
    back = orc.quantize_e4m3(orc.widen(codes, orc.E4M3, "f32"))
    assert np.array_equal(back[codes != 0x80], codes[codes != 0x80]) and back[codes == 0x80].tolist() == [0x80]


def test_e4m3_cache_attention_matches_torch_sdpa_on_widened_rows():
    import torch

    rng = np.random.default_rng(32)
    H, D, lens = 4, 64, [1, 50, 129]
    q = wl.normal_bits(rng, (3, H, D), orc.BF16)
    K = [orc.quantize_e4m3(rng.standard_normal((L, H, D)).astype(np.float32)) for L in lens]
    V = [orc.quantize_e4m3(rng.standard_normal((L, H, D)).astype(np.float32)) for L in lens]
    out, _ = orc.attention_ragged(q, K, V, lens, orc.E4M3, None, "f64", threads=2, q_dtype=orc.BF16)
    f8 = lambda c: torch.from_numpy(c.astype(np.uint8)).view(torch.float8_e4m3fn).double()
    for b, L in enumerate(lens):
        tq = torch.from_numpy(np_widen(q[b], orc.BF16)).reshape(1, H, 1, D)
        tk = f8(K[b]).permute(1, 0, 2).reshape(1, H, L, D)
        tv = f8(V[b]).permute(1, 0, 2).reshape(1, H, L, D)
        want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).reshape(H, D).numpy()
        assert np.allclose(out[b], want, atol=1e-12)
    # length 1 reads the stored codes back exactly
    assert np.array_equal(out[0], orc.widen(V[0][0], orc.E4M3, "f64"))


def test_e4m3_kv_oracle_quantises_on_append_and_halves_the_bytes():
    o16 = orc.KVOracle(2, 4, 64, orc.F16, 64, 256, 1 << 24)
    o8 = orc.KVOracle(2, 4, 64, orc.E4M3, 64, 256, 1 << 24, act_dtype=orc.F16)
    assert o8.bytes_per_token * 2 == o16.bytes_per_token and o8.N == 2 * o16.N
    assert o8.alloc([10])[0] == 1
    rng = np.random.default_rng(33)
    k = wl.normal_bits(rng, (4, 64), orc.F16)
    v = wl.normal_bits(rng, (4, 64), orc.F16)
    assert o8.append(0, 1, 0, k, v) == 0
    import torch
    want = torch.from_numpy(k.view(np.float16).astype(np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(o8.rows(0, 1, 0, 1)[0].astype(np.uint8), want)


# ---------------------------------------------------------------- oracle accuracy, split-K identity
def test_fp32_oracle_close_to_float64_twin_on_c0():
    w = wl.c0()
    rng = np.random.default_rng(w.seed)
    lens = [s.total for s in w.seqs]
    q = wl.normal_bits(rng, (w.batch, w.n_heads, w.head_dim), w.dtype)
    K = [wl.normal_bits(rng, (L, w.n_heads, w.head_dim), w.dtype) for L in lens]
    V = [wl.normal_bits(rng, (L, w.n_heads, w.head_dim), w.dtype) for L in lens]
    a, _ = orc.attention_ragged(q, K, V, lens, w.dtype, None, "f32", threads=4)
    b, _ = orc.attention_ragged(q, K, V, lens, w.dtype, None, "f64", threads=4)
    assert np.abs(a - b).max() <= 1e-5
    serial, used = orc.attention_ragged(q, K, V, lens, w.dtype, None, "f32", threads=1)
    assert used == 1 and np.array_equal(serial, a)  # threading never changes the arithmetic


@pytest.mark.parametrize("chunk", [1, 7, 64, 173])
def test_split_merge_identity(chunk):
    """Merging per-chunk (max, sum, weighted sum) equals the unsplit result (float64)."""
    dtype = orc.F16
    rng = np.random.default_rng(12)
    D, L = 32, 173
    q = wl.normal_bits(rng, (1, 1, D), dtype)
    K = wl.normal_bits(rng, (L, 1, D), dtype)
    V = wl.normal_bits(rng, (L, 1, D), dtype)
    whole, _ = orc.attention_ragged(q, [K], [V], [L], dtype, None, "f64")
    s = orc.scores(q[0, 0], K[:, 0], dtype, 1.0 / math.sqrt(D), "f64")
    vf = np_widen(V[:, 0], dtype)
    parts = []
    for j0 in range(0, L, chunk):
        sc = s[j0:j0 + chunk]
        m = sc.max()
        e = np.exp(sc - m)
        parts.append((m, e.sum(), e @ vf[j0:j0 + chunk]))
    assert np.allclose(orc.merge_partials(parts), whole[0, 0], atol=1e-12)


# ---------------------------------------------------------------- the store's attention wrapper
def test_kv_oracle_attention_reads_the_key_plane_for_scores_and_the_value_plane_for_the_sum():
    """Closed form: when all cached keys of a head are identical the weights are uniform and the output is
    the mean of that head's cached values (section 2.1 equation).  Every (layer, plane, sequence) of the
    store holds its own constant, so an output names the plane, layer and sequence it was read from."""
    dtype = orc.F16
    o = orc.KVOracle(3, 2, 8, dtype, 64, 256, 10**7)
    rng = np.random.default_rng(30)
    const = lambda layer, plane, sid: 1.0 + layer + 0.25 * plane + 0.03125 * sid  # exact in fp16
    ids = [o.alloc_one(p)[0] for p in (64, 128, 64)]
    for sid in ids:
        cap = o.slots[sid][1]
        for layer in range(3):
            k = np.full((cap, 2, 8), const(layer, 0, sid), np.float32)
            v = np.full((cap, 2, 8), const(layer, 1, sid), np.float32)
            assert o.fill(sid, layer, bits(k, dtype), bits(v, dtype)) == orc.OK
    q = wl.normal_bits(rng, (3, 2, 8), dtype)
    order, lens = [ids[2], ids[0], ids[1]], [5, 64, 17]  # batch order differs from id order
    for layer in range(3):
        for precision, tol in (("f32", 1e-6), ("f64", 1e-12)):
            out = o.attention(layer, order, lens, q, None, precision, 2)
            for b, sid in enumerate(order):
                assert np.allclose(out[b], const(layer, 1, sid), atol=tol), (layer, b)


def test_kv_oracle_attention_equals_attention_ragged_on_hand_built_lists():
    """Random rows, ragged lengths shorter than what is stored, rows written by fill and by append: the
    wrapper must hand exactly the sequences' own key and value rows of that layer, in batch order."""
    import torch

    for dtype, H, Hkv in ((orc.F16, 4, 4), (orc.BF16, 4, 2)):
        D, n_layers = 16, 2
        o = orc.KVOracle(n_layers, H, D, dtype, 64, 256, 10**7, n_kv_heads=Hkv)
        rng = np.random.default_rng(31)
        ids, kept = [], {}
        for pred, rows in ((64, 20), (128, 100), (64, 63)):
            sid = o.alloc_one(pred)[0]
            ids.append(sid)
            for layer in range(n_layers):
                k = wl.normal_bits(rng, (rows + 1, Hkv, D), dtype)
                v = wl.normal_bits(rng, (rows + 1, Hkv, D), dtype)
                assert o.fill(sid, layer, k[:rows], v[:rows]) == orc.OK
                assert o.append(sid, layer, rows, k[rows], v[rows]) == orc.OK
                kept[sid, layer] = (k, v)
        order = [ids[1], ids[2], ids[0]]
        lens = [101, 40, 21]
        q = wl.normal_bits(rng, (3, H, D), dtype)
        for layer in range(n_layers):
            out = o.attention(layer, order, lens, q, 0.3, "f64", 1)
            want, _ = orc.attention_ragged(q, [kept[s, layer][0] for s in order], [kept[s, layer][1] for s in order],
                                           lens, dtype, 0.3, "f64")
            assert np.array_equal(out, want)
            for b, sid in enumerate(order):  # and against the library routine, on the rows kept here
                L, g = lens[b], H // Hkv
                tq = torch.from_numpy(np_widen(q[b], dtype)).reshape(1, H, 1, D)
                tk = torch.from_numpy(np_widen(kept[sid, layer][0][:L], dtype)).permute(1, 0, 2).repeat_interleave(g, 0)
                tv = torch.from_numpy(np_widen(kept[sid, layer][1][:L], dtype)).permute(1, 0, 2).repeat_interleave(g, 0)
                ref = torch.nn.functional.scaled_dot_product_attention(tq, tk[None], tv[None], scale=0.3).reshape(H, D)
                assert np.allclose(out[b], ref.numpy(), atol=1e-12)
