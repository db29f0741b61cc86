"""GPU parity at the numeric edges of the softmax of the section 2.1 equation, for every kernel family
(multi-head, shared K/V heads on the vector ALU and on the matrix cores, 8-bit rows, 8-bit rows with shared
heads), against the fp32 oracle at max-abs 2e-3 / relative L2 1e-3: peaked softmax (queries scaled by 8 and
32, so that most weights underflow), one dominant key late (and early) in a context of several chunks (the
running maximum moves after accumulation has begun; chunk partials with very different maxima are merged),
keys and values of magnitude 1e2, all-equal scores over 16384 rows.  Plus 96-wide heads (the 64 x 96 model of
the paper's table 1) and a soak of the merge that happens inside one launch."""
import os

import numpy as np
import pytest

from oracle import kv_oracle as orc
from paper_2306_06000_amd import binding as s3
from paper_2306_06000_amd import workloads as wl
from tests.harness import MAX_ABS, REL_L2, assert_close, device_bits

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
DEV = "cuda:0"
TDT = {0: torch.float16, 1: torch.bfloat16}

# (name, query heads, cached heads, head dim, cache type, activation type, expected kernel kind)
FAMILIES = [
    ("multi-head f16", 16, 16, 256, s3.S3_F16, s3.S3_F16, 0),
    ("multi-head bf16", 12, 12, 128, s3.S3_BF16, s3.S3_BF16, 0),
    ("multi-head f16 d96", 8, 8, 96, s3.S3_F16, s3.S3_F16, 0),
    ("shared heads, vector ALU", 8, 4, 128, s3.S3_F16, s3.S3_F16, 1),
    ("shared heads, matrix cores f16", 16, 2, 128, s3.S3_F16, s3.S3_F16, 2),
    ("shared heads, matrix cores bf16", 32, 8, 128, s3.S3_BF16, s3.S3_BF16, 2),
    ("8-bit rows", 16, 16, 256, s3.S3_E4M3, s3.S3_F16, 3),
    ("8-bit rows, shared heads", 16, 4, 128, s3.S3_E4M3, s3.S3_BF16, 4),
]


@pytest.fixture(scope="module", autouse=True)
def need_gpu_and_lib():
    assert torch.cuda.is_available(), "these tests need the GPU box"
    assert os.path.exists(s3.LIB_PATH), "libs3kv.so must be built before the GPU tests run"
    s3.lib()


class EdgeRig:
    """One arena of any family over hand-made fp32 data; the same bit patterns go to the oracle."""

    def __init__(self, fam, lens, M=1024, G=64):
        self.name, self.H, self.Hkv, self.D, self.kvt, self.act, kind = fam
        self.lens = list(lens)
        self.cfg = s3.make_config(1, self.H, self.D, self.kvt, G, M, 0 if self.Hkv == self.H else self.Hkv,
                                  self.act if self.kvt == s3.S3_E4M3 else 0)
        bpt = s3.s3_kv_bytes_per_token(self.cfg)
        assert bpt > 0
        preds = [max(1, L + 1) for L in lens]
        caps = [s3.s3_kv_capacity_for(self.cfg, p) for p in preds]
        self.N = sum(caps) + M
        self.mem = torch.zeros(self.N * bpt, dtype=torch.uint8, device=DEV)
        st, self.a = s3.s3_kv_arena_init(self.cfg, self.mem, self.mem.numel())
        assert st == 0
        assert s3.s3_kv_get_param(self.a, "kernel_kind") == (0, kind), self.name
        self.o = orc.KVOracle(1, self.H, self.D, self.kvt, G, M, self.N * bpt,
                              n_kv_heads=None if self.Hkv == self.H else self.Hkv,
                              act_dtype=self.act if self.kvt == s3.S3_E4M3 else None)
        rc, self.ids, self.offs, self.caps = s3.s3_kv_alloc(self.a, preds)
        assert rc == len(preds) and self.o.alloc(preds)[0] == rc
        self.stream = torch.cuda.current_stream().cuda_stream
        self.off_d = torch.tensor(self.offs.tolist(), dtype=torch.int64, device=DEV)

    def cache_bits(self, x):
        if self.kvt == s3.S3_E4M3:
            return wl.to_bits(np.clip(x, -448.0, 448.0), wl.E4M3)
        return wl.to_bits(x, self.kvt)

    def put(self, K, V):
        """K[b], V[b]: fp32 [lens[b]][Hkv][D]."""
        tdt = None if self.kvt == s3.S3_E4M3 else TDT[self.kvt]
        for sid, k, v in zip(self.ids.tolist(), K, V):
            if k.shape[0] == 0:
                continue
            kb, vb = self.cache_bits(k), self.cache_bits(v)
            assert self.o.fill(sid, 0, kb, vb) == 0
            assert s3.s3_kv_fill(self.a, sid, 0, 0, k.shape[0], device_bits(kb, tdt, DEV), device_bits(vb, tdt, DEV),
                                 self.stream) == 0

    def attend(self, q, lens=None, out_dtype=s3.S3_F32):
        lens = self.lens if lens is None else lens
        qb = wl.to_bits(q, self.act)
        n = len(lens)
        len_d = torch.tensor(lens, dtype=torch.int32, device=DEV)
        odt = {s3.S3_F32: torch.float32, s3.S3_F16: torch.float16, s3.S3_BF16: torch.bfloat16}[out_dtype]
        out = torch.full((n, self.H, self.D), float("nan"), dtype=odt, device=DEV)
        st = s3.s3_decode_attention(self.a, 0, n, device_bits(qb, TDT[self.act], DEV), self.off_d, len_d, out, out_dtype,
                                    0.0, self.stream)
        assert st == 0, st
        torch.cuda.synchronize()
        return qb, out.float().cpu().numpy()

    def step(self, q, k_new, v_new):
        """s3_decode_step at pos = lens: appends the rows and attends over lens + 1 rows."""
        qb, kb, vb = (wl.to_bits(x, self.act) for x in (q, k_new, v_new))
        n = len(self.lens)
        pos_d = torch.tensor(self.lens, dtype=torch.int32, device=DEV)
        out = torch.full((n, self.H, self.D), float("nan"), dtype=torch.float32, device=DEV)
        len_out = torch.zeros(n, dtype=torch.int32, device=DEV)
        st = s3.s3_decode_step(self.a, 0, n, self.off_d, pos_d, *(device_bits(x, TDT[self.act], DEV) for x in (qb, kb, vb)),
                               out, s3.S3_F32, 0.0, len_out, self.stream, slot_id=self.ids, pos_host=self.lens)
        assert st == 0, st
        torch.cuda.synchronize()
        for b, sid in enumerate(self.ids.tolist()):
            assert self.o.append(sid, 0, self.lens[b], kb[b], vb[b]) == 0
        assert len_out.cpu().tolist() == [L + 1 for L in self.lens]
        return qb, out.cpu().numpy()

    def want(self, qb, lens=None, precision="f32"):
        return self.o.attention(0, self.ids.tolist(), self.lens if lens is None else lens, qb, None, precision, 8)

    def close(self):
        torch.cuda.synchronize()
        s3.s3_kv_arena_destroy(self.a)


def errors(got, want):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    return float(np.abs(got - want).max()), float(np.linalg.norm((got - want).ravel()) / max(np.linalg.norm(want.ravel()), 1e-30))


def check_cases(rig, q, tag, bad, chunks, via_twin=False):
    """Attention of the rig's batch at several chunk sizes against the fp32 oracle; failures are collected
    (with the oracle's own distance to its float64 twin) so that one run reports every case.
    via_twin: for outputs of magnitude 1e2 under a hard arg-max the fp32 definition itself is only determined
    to about 2e-2 (near ties between scores of magnitude 1e2 turn one ulp of a score into 1e-5 of a weight,
    times values of 1e2: measured as the fp32 oracle's distance to its float64 twin), so an absolute 2e-3
    against the fp32 oracle would test the oracle's rounding, not the kernel.  There the kernel is held to the
    float64 twin instead: no further from it than 2e-3 plus twice the fp32 oracle's own distance; the relative
    L2 bound against the fp32 oracle stays as it is."""
    for chunk in chunks:
        assert s3.s3_kv_set_param(rig.a, "chunk", chunk) == 0
        qb, got = rig.attend(q)
        want = rig.want(qb)
        ma, rel = errors(got, want)
        ok = np.isfinite(got).all() and rel <= REL_L2
        oa = orel = 0.0
        if ok and via_twin:
            twin = rig.want(qb, precision="f64")
            oa, orel = errors(want, twin)
            ok = errors(got, twin)[0] <= MAX_ABS + 2.0 * oa
        elif ok:
            ok = ma <= MAX_ABS
        if not ok:
            if not via_twin:
                oa, orel = errors(want, rig.want(qb, precision="f64"))
            bad.append(f"{rig.name} / {tag} / chunk {chunk}: max-abs {ma:.3e} rel-L2 {rel:.3e} "
                       f"(fp32 oracle vs float64 twin: {oa:.3e} {orel:.3e})")


@pytest.mark.parametrize("fam", FAMILIES, ids=[f[0] for f in FAMILIES])
def test_peaked_softmax_dominant_keys_and_large_magnitudes(fam):
    name, H, Hkv, D, kvt, act, kind = fam
    rng = np.random.default_rng(500 + kind + D)
    lens = [300, 301, 64, 1, 517, 129]
    n, g = len(lens), H // Hkv
    bad = []
    chunks = (64, 0) if kind != 2 and kind != 4 else (32, 64, 0)
    K = [rng.standard_normal((L, Hkv, D), dtype=np.float32) for L in lens]
    V = [rng.standard_normal((L, Hkv, D), dtype=np.float32) for L in lens]
    q = rng.standard_normal((n, H, D), dtype=np.float32)

    # 1. queries scaled by 8 and by 32: the softmax is peaked, most weights underflow to zero
    rig = EdgeRig(fam, lens)
    rig.put(K, V)
    for s in (8.0, 32.0):
        check_cases(rig, q * s, f"q x{s:g}", bad, chunks)
    rig.close()

    # 2. one dominant key: row j* of every cached head is 4 x the first query of that head's group, so that
    # its score exceeds all others by tens of units; late in the context (last chunk, after four others),
    # early (row 2), and in the middle
    for where in ("late", "early", "middle"):
        K2 = [k.copy() for k in K]
        for b, L in enumerate(lens):
            j = {"late": L - 3, "early": 2, "middle": L // 2}[where]
            j = min(max(j, 0), L - 1)
            K2[b][j] = 4.0 * q[b, ::g]  # [Hkv][D]
        rig = EdgeRig(fam, lens)
        rig.put(K2, V)
        check_cases(rig, q, f"dominant key {where}", bad, chunks)
        rig.close()

    # 3. keys of magnitude 1e2 (scores of magnitude 1e2: a hard arg-max with near ties now and then), values
    # of magnitude 1; then both at 1e2 (held to the float64 twin, see check_cases)
    rig = EdgeRig(fam, lens)
    rig.put([100.0 * k for k in K], V)
    check_cases(rig, q, "K x100", bad, chunks)
    rig.close()
    rig = EdgeRig(fam, lens)
    rig.put([100.0 * k for k in K], [100.0 * v for v in V])
    check_cases(rig, q, "K, V x100", bad, chunks, via_twin=True)
    rig.close()

    # 4. values of magnitude 1e2 under a flat softmax (tiny queries): sums of large terms
    rig = EdgeRig(fam, lens)
    rig.put(K, [100.0 * v for v in V])
    check_cases(rig, q * 0.01, "V x100, q x0.01", bad, chunks)
    rig.close()
    assert not bad, "\n".join(bad)


@pytest.mark.parametrize("fam", [FAMILIES[0], FAMILIES[4], FAMILIES[6]], ids=[FAMILIES[i][0] for i in (0, 4, 6)])
def test_all_equal_scores_over_16384_rows(fam):
    """Identical keys: every weight is 1/L, the output is the mean of the values (closed form), over the
    longest context the library is tested at; the sum of 16384 equal weights must not lose the small ones."""
    name, H, Hkv, D, kvt, act, kind = fam
    if D == 256:
        fam = (name, 4, 4, D, kvt, act, kind)  # four heads keep the arena small
        H = Hkv = 4
    rng = np.random.default_rng(600 + kind)
    L = 16384
    lens = [L, L - 1, 5000]
    rig = EdgeRig(fam, lens, M=L)
    krow = rng.standard_normal((1, Hkv, D), dtype=np.float32)
    V = [rng.standard_normal((x, Hkv, D), dtype=np.float32) for x in lens]
    rig.put([np.repeat(krow, x, axis=0) for x in lens], V)
    q = rng.standard_normal((3, H, D), dtype=np.float32) * 4.0
    bad = []
    for chunk in ((1024, 128, 0) if kind in (0, 3) else (128, 0)):
        assert s3.s3_kv_set_param(rig.a, "chunk", chunk) == 0
        qb, got = rig.attend(q)
        ma, rel = errors(got, rig.want(qb))
        if not (ma <= MAX_ABS and rel <= REL_L2):
            bad.append(f"{name} chunk {chunk}: {ma:.3e} {rel:.3e}")
        for b in range(3):  # closed form: the mean of the stored values, per cached head
            stored = orc.widen(rig.o.data[int(rig.ids[b])][0, 1, :lens[b]], kvt, "f64").mean(axis=0)  # [Hkv][D]
            mean = np.repeat(stored, H // Hkv, axis=0)
            assert np.abs(got[b] - mean).max() < 2e-4, (name, chunk, b)
    rig.close()
    assert not bad, "\n".join(bad)


@pytest.mark.parametrize("fam", [FAMILIES[0], FAMILIES[1], FAMILIES[2], FAMILIES[6]],
                         ids=[FAMILIES[i][0] for i in (0, 1, 2, 6)])
def test_decode_step_with_a_dominant_new_row_merges_chunks_with_very_different_maxima(fam):
    """The fused step merges the chunks of a context inside the launch.  The NEW row (taken from k_new, not
    yet in the arena) is the dominant key, so the last chunk's maximum exceeds the others' by tens of units;
    and the other way round (dominant key in the first chunk, new row ordinary)."""
    name, H, Hkv, D, kvt, act, kind = fam
    rng = np.random.default_rng(700 + D)
    lens = [299, 64, 0, 511, 130]
    n = len(lens)
    bad = []
    for where in ("new row", "first chunk"):
        K = [rng.standard_normal((L, Hkv, D), dtype=np.float32) for L in lens]
        V = [rng.standard_normal((L, Hkv, D), dtype=np.float32) for L in lens]
        q = rng.standard_normal((n, H, D), dtype=np.float32)
        k_new = rng.standard_normal((n, Hkv, D), dtype=np.float32)
        v_new = rng.standard_normal((n, Hkv, D), dtype=np.float32)
        if where == "new row":
            k_new = 4.0 * q
        else:
            for b, L in enumerate(lens):
                if L:
                    K[b][min(1, L - 1)] = 4.0 * q[b]
        for chunk in (64, 128, 0):
            for sync in (0, 1):
                rig = EdgeRig(fam, lens)
                rig.put(K, V)
                assert s3.s3_kv_set_param(rig.a, "chunk", chunk) == 0
                assert s3.s3_kv_set_param(rig.a, "merge_sync", sync) == 0
                qb, got = rig.step(q, k_new, v_new)
                ma, rel = errors(got, rig.want(qb, [L + 1 for L in lens]))
                if not (np.isfinite(got).all() and ma <= MAX_ABS and rel <= REL_L2):
                    bad.append(f"{name} / dominant {where} / chunk {chunk} / merge_sync {sync}: {ma:.3e} {rel:.3e}")
                rig.close()
    assert not bad, "\n".join(bad)


# ---------------------------------------------------------------- 96-wide heads
@pytest.mark.parametrize("dtype", [s3.S3_F16, s3.S3_BF16])
@pytest.mark.parametrize("H", [1, 3, 5, 64])
def test_head_dim_96_every_variant_and_chunk_size(H, dtype):
    """The 64-head x 96 model of the paper's table 1 (and head counts that leave the last wave's head group
    partly empty): twelve of every sixteen lanes carry a head."""
    lens = [0, 1, 2, 17, 63, 64, 65, 100, 129, 300, 515, 40]
    fam = ("d96", H, H, 96, dtype, dtype, 0)
    rig = EdgeRig(fam, lens)
    rng = np.random.default_rng(96 + H + dtype)
    rig.put([rng.standard_normal((L, H, 96), dtype=np.float32) for L in lens],
            [rng.standard_normal((L, H, 96), dtype=np.float32) for L in lens])
    q = rng.standard_normal((len(lens), H, 96), dtype=np.float32)
    nv = s3.s3_kv_get_param(rig.a, "n_variants")[1]
    for variant in range(nv):
        assert s3.s3_kv_set_param(rig.a, "variant", variant) == 0
        for chunk in (32, 128, 0):
            assert s3.s3_kv_set_param(rig.a, "chunk", chunk) == 0
            qb, got = rig.attend(q)
            assert_close(got, rig.want(qb), f"d96 H{H} dt{dtype} variant {variant} chunk {chunk}")
            assert not got[0].any()
    # 16-bit outputs: fp16 within the tolerance, bf16 = the fp32 result rounded once
    assert s3.s3_kv_set_param(rig.a, "variant", -1) == 0
    qb, got32 = rig.attend(q)
    _, got16 = rig.attend(q, out_dtype=s3.S3_F16)
    assert_close(got16, rig.want(qb), "d96 fp16 output")
    _, gotbf = rig.attend(q, out_dtype=s3.S3_BF16)
    assert np.array_equal(gotbf, torch.from_numpy(got32).to(torch.bfloat16).float().numpy())
    rig.close()


def test_head_dim_96_decode_step_appends_bit_exactly_and_equals_append_then_attention():
    H, D, dtype = 64, 96, s3.S3_F16
    lens = [0, 1, 63, 64, 200, 511, 1000]
    rng = np.random.default_rng(9600)
    K = [rng.standard_normal((L, H, D), dtype=np.float32) for L in lens]
    V = [rng.standard_normal((L, H, D), dtype=np.float32) for L in lens]
    q, k_new, v_new = (rng.standard_normal((len(lens), H, D), dtype=np.float32) for _ in range(3))
    fam = ("d96 step", H, H, D, dtype, dtype, 0)
    outs = []
    for chunk in (0, 128):
        rig = EdgeRig(fam, lens, M=2048)
        rig.put(K, V)
        assert s3.s3_kv_set_param(rig.a, "chunk", chunk) == 0
        snap_before = rig.mem.clone()
        qb, got = rig.step(q, k_new, v_new)
        assert_close(got, rig.want(qb, [L + 1 for L in lens]), f"d96 step chunk {chunk}")
        # the appended rows, and only they, changed; they equal the oracle's rows bit for bit
        for b, sid in enumerate(rig.ids.tolist()):
            for which in (0, 1):
                dst = torch.empty((lens[b] + 1, H, D), dtype=torch.int16, device=DEV)
                assert s3.s3_kv_read_rows(rig.a, sid, 0, which, 0, lens[b] + 1, dst, rig.stream) == 0
                assert np.array_equal(dst.cpu().numpy().view(np.uint16), rig.o.rows(sid, 0, which, lens[b] + 1))
        changed = (rig.mem != snap_before).sum().item()
        assert 0 < changed <= 2 * len(lens) * H * D * 2
        # the unfused pair on the same data gives the same bits
        rig2 = EdgeRig(fam, lens, M=2048)
        rig2.put(K, V)
        assert s3.s3_kv_set_param(rig2.a, "chunk", chunk) == 0
        kb, vb = wl.to_bits(k_new, dtype), wl.to_bits(v_new, dtype)
        pos_d = torch.tensor(lens, dtype=torch.int32, device=DEV)
        assert s3.s3_kv_append(rig2.a, 0, len(lens), rig2.off_d, pos_d, device_bits(kb, TDT[dtype], DEV),
                               device_bits(vb, TDT[dtype], DEV), rig2.stream, slot_id=rig2.ids, pos_host=lens) == 0
        _, got2 = rig2.attend(q, [L + 1 for L in lens])
        assert np.array_equal(got, got2)
        outs.append(got)
        rig.close()
        rig2.close()


def test_worked_example_model_shape_runs_through_the_library():
    """One layer of the 44-layer / 6144-wide / 64-head model of sections 2.1-2.2 (table 1): 24 576 bytes per
    token and layer, ragged batch, against the oracle."""
    H, D = 64, 96
    cfg44 = s3.make_config(44, H, D, s3.S3_F16, 64, 2048)
    assert s3.s3_kv_bytes_per_token(cfg44) == 1081344  # 4 * l * d_h: "1 MB per token"
    lens = [50, 700, 2047, 333]
    fam = ("worked example", H, H, D, s3.S3_F16, s3.S3_F16, 0)
    rig = EdgeRig(fam, lens, M=2048)
    assert s3.s3_kv_bytes_per_token(rig.cfg) * 44 == 1081344
    rng = np.random.default_rng(44)
    rig.put([rng.standard_normal((L, H, D), dtype=np.float32) for L in lens],
            [rng.standard_normal((L, H, D), dtype=np.float32) for L in lens])
    q = rng.standard_normal((4, H, D), dtype=np.float32)
    qb, got = rig.attend(q)
    assert_close(got, rig.want(qb), "64 x 96")
    rig.close()


# ---------------------------------------------------------------- the merge inside one launch, many times
@pytest.mark.parametrize("sync,launches,variant", [(0, 200, -1), (1, 40, -1), (0, 120, 10), (1, 20, 10), (0, 40, 12),
                                                   (0, 120, 14), (1, 20, 14), (0, 40, 16)])
def test_soak_of_the_in_kernel_merge_equals_the_two_kernel_path(sync, launches, variant):
    """Many contexts of many chunks, a grid that covers every compute unit (all XCDs), the same step
    launched again and again: the output of the fused step (chunks meet through arrival counters and
    write-through partials inside the launch) must equal, bit for bit, the two-kernel path (partials with
    plain stores, merged by a second launch) every time.  Stops at the first mismatch.  Also with the dynamic
    work list (variant 10: positions claimed from a device-wide counter that every launch must leave at zero)
    and with rows staged through the LDS ring (variant 12), on grids smaller and larger than the list; and with
    the row stream carried from one item into the next (variants 14, 16: positions claimed two items ahead)."""
    H, D, dtype = 16, 256, s3.S3_F16
    rng = np.random.default_rng(800)
    lens = [int(x) for x in rng.integers(200, 1000, size=96)]
    n = len(lens)
    fam = ("soak", H, H, D, dtype, dtype, 0)
    rig = EdgeRig(fam, lens)
    rig.put([rng.standard_normal((L, H, D), dtype=np.float32) for L in lens],
            [rng.standard_normal((L, H, D), dtype=np.float32) for L in lens])
    assert s3.s3_kv_set_param(rig.a, "chunk", 64) == 0  # 4 to 16 chunks per context, about 9000 items
    assert s3.s3_kv_set_param(rig.a, "merge_sync", sync) == 0
    assert s3.s3_kv_set_param(rig.a, "variant", variant) == 0
    cus = s3.s3_kv_get_param(rig.a, "num_cus")[1]
    assert cus >= 8
    q, k_new, v_new = (device_bits(wl.normal_bits(rng, (n, H, D), dtype), TDT[dtype], DEV) for _ in range(3))
    pos_d = torch.tensor(lens, dtype=torch.int32, device=DEV)
    len1_d = pos_d + 1
    len_out = torch.zeros(n, dtype=torch.int32, device=DEV)
    # reference: append, then attention + merge kernel
    assert s3.s3_kv_append(rig.a, 0, n, rig.off_d, pos_d, k_new, v_new, rig.stream) == 0
    ref = torch.empty((n, H, D), dtype=torch.float32, device=DEV)
    assert s3.s3_decode_attention(rig.a, 0, n, q, rig.off_d, len1_d, ref, s3.S3_F32, 0.0, rig.stream) == 0
    torch.cuda.synchronize()
    out = torch.empty_like(ref)
    for grid in (0, 2 * cus, 8 * cus, 7, 100000):
        assert s3.s3_kv_set_param(rig.a, "grid_blocks", grid) == 0
        for i in range(launches if grid == 0 else launches // 2 if grid in (2 * cus, 8 * cus) else 6):
            out.fill_(float("nan"))
            assert s3.s3_decode_step(rig.a, 0, n, rig.off_d, pos_d, q, k_new, v_new, out, s3.S3_F32, 0.0, len_out,
                                     rig.stream) == 0
            assert torch.equal(out, ref), f"merge_sync {sync} grid {grid}: launch {i} differs from the two-kernel path"
    rig.close()


@pytest.mark.parametrize("variant", [14, 15, 16, 17])
@pytest.mark.parametrize("H,D,dtype", [(16, 256, s3.S3_F16), (12, 128, s3.S3_BF16), (8, 96, s3.S3_F16), (3, 64, s3.S3_BF16)])
def test_row_stream_carried_across_items_equals_the_two_kernel_path(variant, H, D, dtype):
    """Kernel shapes whose waves start loading the rows of their next item while the current one is still being
    reduced.  Grids far smaller than the work list, so that every workgroup walks many items; contexts from one row
    up, so that the list holds items whose trailing waves have no rows at all, shares of a single load batch and
    shares of many; chunk sizes from the smallest.  The fused step must leave the same rows and the same output
    bits as append + attention + merge, launch after launch (the claim counters must come back to zero)."""
    rng = np.random.default_rng(900 + variant)
    lens = [1, 2, 3, 5, 7, 8, 9, 15, 16, 17, 31, 32, 33, 63, 64, 65, 100, 129, 255, 256, 257, 300, 511, 640, 777, 1000,
            4, 1, 66, 12]
    n = len(lens)
    rig = EdgeRig(("stream", H, H, D, dtype, dtype, 0), lens)
    rig.put([rng.standard_normal((L, H, D), dtype=np.float32) for L in lens],
            [rng.standard_normal((L, H, D), dtype=np.float32) for L in lens])
    assert s3.s3_kv_set_param(rig.a, "variant", variant) == 0
    q, k_new, v_new = (device_bits(wl.normal_bits(rng, (n, H, D), dtype), TDT[dtype], DEV) for _ in range(3))
    pos_d = torch.tensor(lens, dtype=torch.int32, device=DEV)
    len_out = torch.zeros(n, dtype=torch.int32, device=DEV)
    assert s3.s3_kv_append(rig.a, 0, n, rig.off_d, pos_d, k_new, v_new, rig.stream) == 0
    ref = torch.empty((n, H, D), dtype=torch.float32, device=DEV)
    out = torch.empty_like(ref)
    for chunk in (32, 64, 256):
        assert s3.s3_kv_set_param(rig.a, "chunk", chunk) == 0
        assert s3.s3_kv_set_param(rig.a, "grid_blocks", 0) == 0
        assert s3.s3_decode_attention(rig.a, 0, n, q, rig.off_d, pos_d + 1, ref, s3.S3_F32, 0.0, rig.stream) == 0
        torch.cuda.synchronize()
        for grid in (1, 2, 5, 64, 0):
            assert s3.s3_kv_set_param(rig.a, "grid_blocks", grid) == 0
            for i in range(3):
                out.fill_(float("nan"))
                len_out.zero_()
                assert s3.s3_decode_step(rig.a, 0, n, rig.off_d, pos_d, q, k_new, v_new, out, s3.S3_F32, 0.0, len_out,
                                         rig.stream) == 0
                assert torch.equal(out, ref), f"chunk {chunk} grid {grid} launch {i}"
                assert len_out.cpu().tolist() == [L + 1 for L in lens]
    rig.close()


@pytest.mark.parametrize("fam", [FAMILIES[4], FAMILIES[5], FAMILIES[7]], ids=[FAMILIES[i][0] for i in (4, 5, 7)])
def test_matrix_core_kernel_merging_chunks_inside_the_launch_equals_the_merge_launch(fam):
    """The matrix-core kernel for shared heads can finish multi-chunk contexts itself (arrival counters, the
    publication of a chunk trailing the wave's work by two items) instead of leaving them to a merge launch:
    same bits as the two-launch path, for attention and for the decode step, on a dominant-key batch (chunks with
    very different maxima), launch after launch (the counters must come back to zero), and within the tolerance
    of the oracle."""
    name, H, Hkv, D, kvt, act, kind = fam
    rng = np.random.default_rng(900 + D + kind)
    lens = [300, 0, 301, 64, 1, 517, 129, 1000, 33]
    n, g = len(lens), H // Hkv
    K = [rng.standard_normal((L, Hkv, D), dtype=np.float32) for L in lens]
    V = [rng.standard_normal((L, Hkv, D), dtype=np.float32) for L in lens]
    q = rng.standard_normal((n, H, D), dtype=np.float32)
    for b, L in enumerate(lens):
        if L:
            K[b][max(L - 3, 0)] = 4.0 * q[b, ::g]
    k_new = rng.standard_normal((n, Hkv, D), dtype=np.float32)
    v_new = rng.standard_normal((n, Hkv, D), dtype=np.float32)
    for chunk in (32, 64, 0, 512):
        outs = {}
        for merge in (0, 1):
            rig = EdgeRig(fam, lens, M=2048)
            rig.put(K, V)
            assert s3.s3_kv_set_param(rig.a, "chunk", chunk) == 0
            assert s3.s3_kv_set_param(rig.a, "gqa_merge", merge) == 0
            assert s3.s3_kv_get_param(rig.a, "gqa_merge") == (0, merge)
            got = []
            for rep in range(6 if merge else 1):  # again and again on the same counters
                qb, o = rig.attend(q)
                got.append(o)
            assert all(np.array_equal(got[0], x) for x in got[1:]), (name, chunk)
            assert_close(got[0], rig.want(qb), f"{name} chunk {chunk} gqa_merge {merge}")
            assert not got[0][1].any()  # the empty context: zeros, written by whoever finishes the contexts
            qb, step = rig.step(q, k_new, v_new)
            assert_close(step, rig.want(qb, [L + 1 for L in lens]), f"{name} step chunk {chunk} gqa_merge {merge}")
            outs[merge] = (got[0], step)
            rig.close()
        assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1]), (name, chunk)


STREAM_FAMILIES = [FAMILIES[4], FAMILIES[5], FAMILIES[7],
                   ("shared heads, matrix cores d64", 16, 4, 64, s3.S3_F16, s3.S3_F16, 2),
                   ("multi-query, matrix cores d256", 16, 1, 256, s3.S3_BF16, s3.S3_BF16, 2),
                   ("8-bit rows, shared heads d256", 8, 2, 256, s3.S3_E4M3, s3.S3_F16, 4)]


@pytest.mark.parametrize("fam", STREAM_FAMILIES, ids=[f[0] for f in STREAM_FAMILIES])
def test_matrix_core_kernel_streaming_k_rows_equals_plain_loads(fam):
    """The matrix-core kernel reads K either straight into operand layout with plain loads or, when a launch's K
    rows exceed the memory-side cache, in whole rows with the streaming hint and through LDS (`gqa_stream`): the
    operands hold the same bits either way, so attention and the decode step (whose append takes the new row from
    differently laid out registers) must give the same output bits, the appended row must read back the same, and
    both must meet the oracle's tolerance."""
    name, H, Hkv, D, kvt, act, kind = fam
    rng = np.random.default_rng(950 + D + kind)
    lens = [300, 0, 301, 64, 1, 517, 129, 1000, 33, 15, 16, 17]
    n = len(lens)
    K = [rng.standard_normal((L, Hkv, D), dtype=np.float32) for L in lens]
    V = [rng.standard_normal((L, Hkv, D), dtype=np.float32) for L in lens]
    q = rng.standard_normal((n, H, D), dtype=np.float32)
    k_new = rng.standard_normal((n, Hkv, D), dtype=np.float32)
    v_new = rng.standard_normal((n, Hkv, D), dtype=np.float32)
    for chunk in (32, 0, 512):
        outs = {}
        for stream in (0, 1):
            rig = EdgeRig(fam, lens, M=2048)
            rig.put(K, V)
            assert s3.s3_kv_set_param(rig.a, "chunk", chunk) == 0
            assert s3.s3_kv_set_param(rig.a, "gqa_stream", stream) == 0
            assert s3.s3_kv_get_param(rig.a, "gqa_stream") == (0, stream)
            qb, att = rig.attend(q)
            assert_close(att, rig.want(qb), f"{name} chunk {chunk} gqa_stream {stream}")
            qb, step = rig.step(q, k_new, v_new)
            longer = [L + 1 for L in lens]
            assert_close(step, rig.want(qb, longer), f"{name} step chunk {chunk} gqa_stream {stream}")
            _, again = rig.attend(q, lens=longer)  # the appended rows, now read from the arena
            assert np.array_equal(again, step), (name, chunk, stream)
            outs[stream] = (att, step)
            rig.close()
        assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1]), (name, chunk)
    a_rig = EdgeRig(fam, [4])
    assert s3.s3_kv_set_param(a_rig.a, "gqa_stream", 2) == s3.S3_ERR_INVALID
    assert s3.s3_kv_set_param(a_rig.a, "gqa_stream", -1) == 0
    a_rig.close()


@pytest.mark.parametrize("fam", STREAM_FAMILIES[:3], ids=[f[0] for f in STREAM_FAMILIES[:3]])
def test_matrix_core_kernel_claiming_the_end_of_its_work_list_equals_the_fixed_stride(fam):
    """`gqa_dynamic`: the waves of the matrix-core kernel take the first part of the work list by stride and claim
    the rest from a device-wide counter that every launch must leave at zero.  Grids far smaller than the list, so
    that most positions are claimed; launch after launch; attention and decode step; same bits as the fixed
    stride."""
    name, H, Hkv, D, kvt, act, kind = fam
    rng = np.random.default_rng(970 + D + kind)
    lens = [300, 0, 301, 64, 1, 517, 129, 1000, 33, 15, 16, 17, 700, 45]
    n = len(lens)
    K = [rng.standard_normal((L, Hkv, D), dtype=np.float32) for L in lens]
    V = [rng.standard_normal((L, Hkv, D), dtype=np.float32) for L in lens]
    q = rng.standard_normal((n, H, D), dtype=np.float32)
    rig = EdgeRig(fam, lens, M=2048)
    rig.put(K, V)
    assert s3.s3_kv_set_param(rig.a, "chunk", 64) == 0
    assert s3.s3_kv_set_param(rig.a, "gqa_dynamic", 0) == 0
    qb, ref = rig.attend(q)
    assert_close(ref, rig.want(qb), name)
    for grid in (1, 3, 0):
        assert s3.s3_kv_set_param(rig.a, "grid_blocks", grid) == 0
        for pct in (1, 50, 99, -1):
            assert s3.s3_kv_set_param(rig.a, "gqa_dynamic", pct) == 0
            for rep in range(3):
                _, got = rig.attend(q)
                assert np.array_equal(got, ref), (name, grid, pct, rep)
    assert s3.s3_kv_set_param(rig.a, "gqa_dynamic", 101) == s3.S3_ERR_INVALID
    # the decode step, half of the list claimed, against the step by stride on a twin arena
    k_new = rng.standard_normal((n, Hkv, D), dtype=np.float32)
    v_new = rng.standard_normal((n, Hkv, D), dtype=np.float32)
    twin = EdgeRig(fam, lens, M=2048)
    twin.put(K, V)
    steps = []
    for r, pct in ((rig, 50), (twin, 0)):
        assert s3.s3_kv_set_param(r.a, "chunk", 64) == 0
        assert s3.s3_kv_set_param(r.a, "grid_blocks", 2) == 0
        assert s3.s3_kv_set_param(r.a, "gqa_dynamic", pct) == 0
        steps.append(r.step(q, k_new, v_new)[1])
    assert np.array_equal(steps[0], steps[1]), name
    rig.close()
    twin.close()
