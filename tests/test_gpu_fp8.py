"""GPU parity for 8-bit (e4m3) cache rows: the HIP path through the C ABI against the CPU oracle.
Stored codes must be bit-exact (the append's quantisation included); attention within max-abs 2e-3
and relative L2 1e-3 of the fp32 oracle, which widens the same codes."""
import os

import numpy as np
import pytest

from oracle import kv_oracle as orc
from paper_2306_06000_amd import binding as s3
from paper_2306_06000_amd import workloads as wl
from tests.harness import OracleReplay, assert_close, device_bits, make_sources

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
DEV = "cuda:0"
TDT = {0: torch.float16, 1: torch.bfloat16}


@pytest.fixture(scope="module", autouse=True)
def need_gpu_and_lib():
    assert torch.cuda.is_available(), "these tests need the GPU box"
    assert os.path.exists(s3.LIB_PATH), "libs3kv.so must be built before the GPU tests run"
    s3.lib()


class Rig8:
    """A small 8-bit arena with hand-placed sequences, mirrored in the oracle."""

    def __init__(self, n_layers, H, D, act, G, M, preds, seed, Hkv=None, arena_tokens=None):
        self.n_layers, self.Hq, self.D, self.act = n_layers, H, D, act
        self.H = Hkv or H  # heads of a cached row
        self.cfg = s3.make_config(n_layers, H, D, s3.S3_E4M3, G, M, 0 if Hkv is None else Hkv, act)
        bpt = s3.s3_kv_bytes_per_token(self.cfg)
        assert bpt == 2 * n_layers * self.H * D
        caps = [min(M, max(G, -(-p // G) * G)) for p in preds]
        self.N = arena_tokens or (sum(caps) + 3 * M)
        self.mem = torch.zeros(self.N * bpt, dtype=torch.uint8, device=DEV)
        st, self.a = s3.s3_kv_arena_init(self.cfg, self.mem, self.mem.numel())
        assert st == 0
        assert s3.s3_kv_get_param(self.a, "kernel_kind") == (0, 3 if self.H == H else 4)
        self.o = orc.KVOracle(n_layers, H, D, orc.E4M3, G, M, self.N * bpt, act_dtype=act, n_kv_heads=Hkv)
        assert bpt == self.o.bytes_per_token
        rc, self.ids, self.offs, self.caps = s3.s3_kv_alloc(self.a, preds)
        n_o, ids_o, offs_o, caps_o = self.o.alloc(preds)
        assert rc == n_o == len(preds)
        assert self.ids.tolist() == ids_o and self.offs.tolist() == offs_o and self.caps.tolist() == caps_o
        self.rng = np.random.default_rng(seed)
        self.stream = torch.cuda.current_stream().cuda_stream

    def fill(self, lens, layer=0, rows=None):
        for i, (sid, L) in enumerate(zip(self.ids.tolist(), lens)):
            if L == 0:
                continue
            if rows is None:
                k = wl.normal_bits(self.rng, (L, self.H, self.D), wl.E4M3)
                v = wl.normal_bits(self.rng, (L, self.H, self.D), wl.E4M3)
            else:
                k, v = rows[i]
            assert self.o.fill(sid, layer, k, v) == 0
            assert s3.s3_kv_fill(self.a, sid, layer, 0, L, device_bits(k, None, DEV), device_bits(v, None, DEV),
                                 self.stream) == 0

    def read(self, sid, layer, which, rows):
        dst = torch.empty((int(rows), self.H, self.D), dtype=torch.uint8, device=DEV)
        assert s3.s3_kv_read_rows(self.a, sid, layer, which, 0, int(rows), dst, self.stream) == 0
        return dst.cpu().numpy()

    def attend(self, lens, layer=0, out_dtype=s3.S3_F32, scale=0.0):
        n = len(lens)
        q = wl.normal_bits(self.rng, (n, self.Hq, self.D), self.act)
        qd = device_bits(q, TDT[self.act], DEV)
        off_d = torch.tensor(self.offs.tolist(), dtype=torch.int64, device=DEV)
        len_d = torch.tensor(lens, dtype=torch.int32, device=DEV)
        odt = {s3.S3_F32: torch.float32, s3.S3_F16: torch.float16, s3.S3_BF16: torch.bfloat16}[out_dtype]
        out = torch.full((n, self.Hq, self.D), float("nan"), dtype=odt, device=DEV)
        st = s3.s3_decode_attention(self.a, layer, n, qd, off_d, len_d, out, out_dtype, scale, self.stream)
        assert st == 0, st
        torch.cuda.synchronize()
        return q, out.float().cpu().numpy()

    def oracle_attend(self, q, lens, layer=0, scale=None):
        return self.o.attention(layer, self.ids.tolist(), lens, q, scale, "f32", threads=8)

    def close(self):
        torch.cuda.synchronize()
        s3.s3_kv_arena_destroy(self.a)


def test_config_rules_for_8_bit_rows():
    ok = s3.make_config(1, 16, 256, s3.S3_E4M3, 64, 2048, 0, s3.S3_BF16)
    assert s3.s3_kv_bytes_per_token(ok) == 2 * 16 * 256
    for bad in (s3.make_config(1, 16, 256, s3.S3_E4M3, 64, 2048, 0, s3.S3_F32),
                s3.make_config(1, 16, 256, s3.S3_E4M3, 64, 2048, 5, s3.S3_F16),   # 5 does not divide 16
                s3.make_config(1, 16, 256, 4, 64, 2048)):
        assert s3.s3_kv_bytes_per_token(bad) == s3.S3_ERR_INVALID


@pytest.mark.parametrize("D", [64, 128, 256])
def test_length_one_context_reads_every_finite_code_back_exactly(D):
    """softmax over one row is 1, so out = V widened: all 254 finite codes must come back as the
    values the format defines (this is what pins the kernel's widening instruction)."""
    H = 1024 // D * 2
    rig = Rig8(1, H, D, s3.S3_F16, 64, 64, [1], seed=1)
    codes = np.arange(H * D, dtype=np.uint32) % 256
    codes[(codes & 0x7f) == 0x7f] = 0x3c          # the two NaN codes
    v = codes.astype(np.uint8).reshape(1, H, D)
    k = wl.normal_bits(rig.rng, (1, H, D), wl.E4M3)
    rig.fill([1], rows=[(k, v)])
    q, got = rig.attend([1])
    want = orc.widen(v[0].astype(np.uint16), orc.E4M3, "f32")
    assert np.array_equal(got[0], want)
    assert {int(c) for c in v.ravel()} >= set(range(256)) - {0x7f, 0xff}
    rig.close()


@pytest.mark.parametrize("act", [s3.S3_F16, s3.S3_BF16])
def test_append_quantises_bit_exactly(act):
    """New 16-bit rows become e4m3 codes: nearest, ties to even, saturating, NaN -> 0x7f; every code
    must equal the oracle's, including midpoints between codes, subnormals, overflow and specials."""
    H, D = 4, 128
    n = 6
    rig = Rig8(2, H, D, act, 64, 128, [64] * n, seed=2)
    pos = [0, 1, 5, 17, 62, 63]
    vals = orc.widen(np.arange(0x7f, dtype=np.uint16), orc.E4M3, "f64")
    mids = (vals[:-1] + vals[1:]) / 2
    special = np.concatenate([mids, -mids, vals, [0.0, -0.0, 448.0, 464.0, 465.0, 1e4, 65504.0, -1e4, np.inf, -np.inf,
                                                 np.nan, 2.0 ** -10, 3 * 2.0 ** -11, 2.0 ** -11, 6e-8, -6e-8]])
    x = (rig.rng.standard_normal((2, n, H, D)) * rig.rng.choice([0.01, 1.0, 30.0, 300.0], (2, n, H, 1))).astype(np.float32)
    x.reshape(2, -1)[:, :special.size] = special.astype(np.float32)
    with np.errstate(over="ignore", invalid="ignore"):
        kb, vb = wl.to_bits(x[0], act), wl.to_bits(x[1], act)
    if act == s3.S3_BF16:  # the generator's bf16 rounding is for finite inputs: patch the specials in by hand
        for arr, src in ((kb, x[0]), (vb, x[1])):
            arr[np.isnan(src)] = 0x7FC0
            arr[np.isposinf(src)] = 0x7F80
            arr[np.isneginf(src)] = 0xFF80
    off_d = torch.tensor(rig.offs.tolist(), dtype=torch.int64, device=DEV)
    pos_d = torch.tensor(pos, dtype=torch.int32, device=DEV)
    st = s3.s3_kv_append(rig.a, 1, n, off_d, pos_d, device_bits(kb, TDT[act], DEV), device_bits(vb, TDT[act], DEV),
                         rig.stream, slot_id=rig.ids, pos_host=pos)
    assert st == 0
    for b, sid in enumerate(rig.ids.tolist()):
        assert rig.o.append(sid, 1, pos[b], kb[b], vb[b]) == 0
        for which in (0, 1):
            got = rig.read(sid, 1, which, 64)
            assert np.array_equal(got, rig.o.data[sid][1, which].astype(np.uint8)), (b, which)
            assert not rig.read(sid, 0, which, 64).any()  # the other layer is untouched
    rig.close()


RAGGED = [0, 1, 2, 3, 15, 16, 17, 31, 33, 64, 100, 255, 257, 600, 1000, 1, 5]


@pytest.mark.parametrize("act", [s3.S3_F16, s3.S3_BF16])
@pytest.mark.parametrize("D", [64, 128, 256])
@pytest.mark.parametrize("H", [1, 2, 3, 8, 16, 20])
def test_attention_over_8_bit_rows(H, D, act):
    rig = Rig8(2, H, D, act, 64, 1024, [max(1, L) for L in RAGGED], seed=10 + H + D)
    rig.fill(RAGGED, layer=1)
    q, got = rig.attend(RAGGED, layer=1)
    assert_close(got, rig.oracle_attend(q, RAGGED, layer=1), f"e4m3 {H}x{D}")
    assert not got[0].any()  # empty context: zeros
    for shape in range(s3.s3_kv_get_param(rig.a, "n_variants")[1]):
        assert s3.s3_kv_set_param(rig.a, "variant", shape) == 0
        for chunk in (32, 160, 1024):
            assert s3.s3_kv_set_param(rig.a, "chunk", chunk) == 0
            q, got = rig.attend(RAGGED, layer=1)
            assert_close(got, rig.oracle_attend(q, RAGGED, layer=1), f"e4m3 {H}x{D} shape {shape} chunk {chunk}")
    q, got = rig.attend(RAGGED, layer=1, out_dtype=s3.S3_F16, scale=0.05)
    assert np.abs(got - rig.oracle_attend(q, RAGGED, layer=1, scale=0.05)).max() <= 2e-3
    rig.close()


@pytest.mark.parametrize("act", [s3.S3_F16, s3.S3_BF16])
def test_decode_step_quantises_appends_and_attends(act):
    H, D = 16, 256
    pos = [0, 1, 31, 63, 64, 100, 255, 513, 5]
    caps = [p + 1 for p in pos]
    rig = Rig8(1, H, D, act, 64, 1024, caps, seed=40)
    rig.fill(pos)
    n = len(pos)
    q, k, v = (wl.normal_bits(rig.rng, (n, H, D), act) for _ in range(3))
    qd, kd, vd = (device_bits(x, TDT[act], DEV) for x in (q, k, v))
    off_d = torch.tensor(rig.offs.tolist(), dtype=torch.int64, device=DEV)
    pos_d = torch.tensor(pos, dtype=torch.int32, device=DEV)
    out = torch.full((n, H, D), float("nan"), dtype=torch.float32, device=DEV)
    len_out = torch.zeros(n, dtype=torch.int32, device=DEV)
    assert s3.s3_decode_step(rig.a, 0, n, off_d, pos_d, qd, kd, vd, out, s3.S3_F32, 0.0, len_out, rig.stream,
                             slot_id=rig.ids, pos_host=rig.caps.tolist()) == s3.S3_ERR_SLOT_FULL
    assert s3.s3_decode_step(rig.a, 0, n, off_d, pos_d, qd, kd, vd, out, s3.S3_F32, 0.0, len_out, rig.stream,
                             slot_id=rig.ids, pos_host=pos) == 0
    torch.cuda.synchronize()
    assert len_out.cpu().tolist() == caps
    for b, sid in enumerate(rig.ids.tolist()):
        assert rig.o.append(sid, 0, pos[b], k[b], v[b]) == 0
        for which in (0, 1):
            assert np.array_equal(rig.read(sid, 0, which, rig.caps[b]), rig.o.data[sid][0, which].astype(np.uint8))
    assert_close(out.cpu().numpy(), rig.oracle_attend(q, caps), "e4m3 step")
    rig.close()


@pytest.mark.parametrize("act", [s3.S3_F16, s3.S3_BF16])
@pytest.mark.parametrize("D", [64, 128, 256])
def test_decode_step_rounds_finite_special_values_like_the_append(D, act):
    """The decode step rounds the new row inside the attention kernel: midpoints between codes, subnormal
    codes, values at and beyond the largest code must give the oracle's codes there too."""
    H = 2048 // D
    pos = [0, 3, 64, 700]
    rig = Rig8(1, H, D, act, 64, 1024, [p + 1 for p in pos], seed=45 + D)
    rig.fill(pos)
    n = len(pos)
    vals = orc.widen(np.arange(0x7f, dtype=np.uint16), orc.E4M3, "f64")
    mids = (vals[:-1] + vals[1:]) / 2
    special = np.concatenate([mids, -mids, vals, -vals, [0.0, -0.0, 448.0, 464.0, 465.0, 1e4, 65504.0, -1e4, 2.0 ** -10,
                                                         3 * 2.0 ** -11, 2.0 ** -11, 6e-8, -6e-8, 2.0 ** -9 * 0.75]])
    x = (rig.rng.standard_normal((2, n, H, D)) * rig.rng.choice([0.01, 1.0, 30.0], (2, n, H, 1))).astype(np.float32)
    assert special.size <= H * D
    for b in range(n):
        x[0, b].reshape(-1)[:special.size] = np.roll(special, 7 * b).astype(np.float32)
        x[1, b].reshape(-1)[-special.size:] = np.roll(special, 3 * b).astype(np.float32)
    kb, vb = wl.to_bits(x[0], act), wl.to_bits(x[1], act)
    q = wl.normal_bits(rig.rng, (n, H, D), act)
    qd, kd, vd = (device_bits(t, TDT[act], DEV) for t in (q, kb, vb))
    off_d = torch.tensor(rig.offs.tolist(), dtype=torch.int64, device=DEV)
    pos_d = torch.tensor(pos, dtype=torch.int32, device=DEV)
    out = torch.full((n, H, D), float("nan"), dtype=torch.float32, device=DEV)
    len_out = torch.zeros(n, dtype=torch.int32, device=DEV)
    assert s3.s3_decode_step(rig.a, 0, n, off_d, pos_d, qd, kd, vd, out, s3.S3_F32, 0.0, len_out, rig.stream,
                             slot_id=rig.ids, pos_host=pos) == 0
    torch.cuda.synchronize()
    assert len_out.cpu().tolist() == [p + 1 for p in pos]
    for b, sid in enumerate(rig.ids.tolist()):
        assert rig.o.append(sid, 0, pos[b], kb[b], vb[b]) == 0
        for which in (0, 1):
            assert np.array_equal(rig.read(sid, 0, which, pos[b] + 1), rig.o.rows(sid, 0, which, pos[b] + 1).astype(np.uint8)), (b, which)
    got = out.cpu().numpy()
    want = rig.oracle_attend(q, [p + 1 for p in pos])
    assert np.isfinite(got).all()
    assert np.linalg.norm(got - want) <= 1e-3 * np.linalg.norm(want)
    rig.close()


SHARED8 = [(32, 8, 128), (16, 1, 256), (8, 1, 64), (8, 2, 64), (12, 4, 128), (6, 3, 256), (64, 8, 128), (40, 2, 128), (9, 3, 64)]


@pytest.mark.parametrize("act", [s3.S3_F16, s3.S3_BF16])
@pytest.mark.parametrize("H,Hkv,D", SHARED8)
def test_shared_heads_over_8_bit_rows(H, Hkv, D, act):
    """Both footprint variants at once: e4m3 rows of Hkv cached heads, H query heads; the matrix-core
    kernel widens the codes in registers.  (40, 2, 128) has 20 query heads per cached head: two blocks
    of 16 columns, the second partly padding."""
    rig = Rig8(2, H, D, act, 64, 1024, [max(1, L) for L in RAGGED], seed=60 + H + Hkv, Hkv=Hkv)
    rig.fill(RAGGED, layer=1)
    for chunk in (0, 32, 160, 1024):
        assert s3.s3_kv_set_param(rig.a, "chunk", chunk) == 0
        q, got = rig.attend(RAGGED, layer=1)
        assert_close(got, rig.oracle_attend(q, RAGGED, layer=1), f"e4m3 shared {H}/{Hkv}x{D} chunk {chunk}")
        assert not got[0].any()
    rig.close()


@pytest.mark.parametrize("H,Hkv,D,act", [(32, 8, 128, s3.S3_BF16), (16, 1, 256, s3.S3_F16)])
def test_shared_heads_over_8_bit_rows_decode_step(H, Hkv, D, act):
    pos = [0, 1, 31, 63, 64, 100, 255, 513, 5]
    caps = [p + 1 for p in pos]
    rig = Rig8(1, H, D, act, 64, 1024, caps, seed=80 + H, Hkv=Hkv)
    rig.fill(pos)
    n = len(pos)
    q = wl.normal_bits(rig.rng, (n, H, D), act)
    k = wl.normal_bits(rig.rng, (n, Hkv, D), act)
    v = wl.normal_bits(rig.rng, (n, Hkv, D), act)
    qd, kd, vd = (device_bits(x, TDT[act], DEV) for x in (q, k, v))
    off_d = torch.tensor(rig.offs.tolist(), dtype=torch.int64, device=DEV)
    pos_d = torch.tensor(pos, dtype=torch.int32, device=DEV)
    out = torch.full((n, H, D), float("nan"), dtype=torch.float32, device=DEV)
    len_out = torch.zeros(n, dtype=torch.int32, device=DEV)
    assert s3.s3_decode_step(rig.a, 0, n, off_d, pos_d, qd, kd, vd, out, s3.S3_F32, 0.0, len_out, rig.stream,
                             slot_id=rig.ids, pos_host=pos) == 0
    torch.cuda.synchronize()
    assert len_out.cpu().tolist() == caps
    for b, sid in enumerate(rig.ids.tolist()):
        assert rig.o.append(sid, 0, pos[b], k[b], v[b]) == 0
        for which in (0, 1):
            assert np.array_equal(rig.read(sid, 0, which, rig.caps[b]), rig.o.data[sid][0, which].astype(np.uint8))
    assert_close(out.cpu().numpy(), rig.oracle_attend(q, caps), "e4m3 shared step")
    rig.close()


@pytest.mark.parametrize("seed", range(16))
def test_random_configuration_over_8_bit_rows(seed):
    """A seeded draw over head shape and sharing, query type, batch, ragged lengths, chunk, kernel shape,
    classes and grid size, for attention over e4m3 rows."""
    rng = np.random.default_rng(3000 + seed)
    D = int(rng.choice([64, 128, 256]))
    act = int(rng.choice([s3.S3_F16, s3.S3_BF16]))
    Hkv = int(rng.choice([1, 2, 3, 4, 8]))
    group = int(rng.choice([1, 1, 2, 4, 5, 8, 16]))
    H = Hkv * group
    n = int(rng.choice([1, 2, 7, 33, 64, 65, 130]))
    lens = [int(x) for x in rng.choice([0, 1, 2, 15, 16, 17, 63, 64, 65, 200, 511, 700, 1024], n)]
    rig = Rig8(1, H, D, act, 64, 1024, [max(1, L) for L in lens], seed=4000 + seed, Hkv=None if group == 1 else Hkv)
    rig.fill(lens)
    nv = s3.s3_kv_get_param(rig.a, "n_variants")[1]
    for _ in range(2):
        assert s3.s3_kv_set_param(rig.a, "variant", int(rng.integers(-1, nv))) == 0
        assert s3.s3_kv_set_param(rig.a, "chunk", int(rng.choice([0, 32, 96, 256, 1024]))) == 0
        assert s3.s3_kv_set_param(rig.a, "classes", int(rng.integers(0, 9))) == 0
        assert s3.s3_kv_set_param(rig.a, "grid_blocks", int(rng.choice([0, 1, 3, 64, 300, 2048]))) == 0
        q, got = rig.attend(lens)
        assert_close(got, rig.oracle_attend(q, lens), f"random e4m3 {seed}: H{H} Hkv{Hkv} D{D} n{n}")
        for b, L in enumerate(lens):
            if L == 0:
                assert not got[b].any()
    rig.close()


def test_8_bit_contexts_up_to_a_long_maximum_length():
    """max_len = 16384 over e4m3 rows: a full context, one a row short of it and short ones; 128 chunks per
    context (chunk 128) merge inside the kernel; the decode step rounds and appends the last row of the
    nearly full slot."""
    H, D, act, M = 4, 128, s3.S3_BF16, 16384
    lens = [M, M - 1, 1, 700, 0, 5000]
    rig = Rig8(1, H, D, act, 128, M, [max(1, L) for L in lens], seed=89)
    rig.fill(lens)
    for chunk in (0, 128, 2048):
        assert s3.s3_kv_set_param(rig.a, "chunk", chunk) == 0
        q, got = rig.attend(lens)
        assert_close(got, rig.oracle_attend(q, lens), f"long e4m3 contexts, chunk {chunk}")
    assert s3.s3_kv_set_param(rig.a, "chunk", 0) == 0
    keep = [1, 2, 3, 5]
    ids = rig.ids[keep]
    pos = [lens[b] for b in keep]
    m = len(keep)
    q, k, v = (wl.normal_bits(rig.rng, (m, H, D), act) for _ in range(3))
    qd, kd, vd = (device_bits(x, TDT[act], DEV) for x in (q, k, v))
    off_d = torch.tensor(rig.offs[keep].tolist(), dtype=torch.int64, device=DEV)
    pos_d = torch.tensor(pos, dtype=torch.int32, device=DEV)
    out = torch.full((m, H, D), float("nan"), dtype=torch.float32, device=DEV)
    len_out = torch.zeros(m, dtype=torch.int32, device=DEV)
    assert s3.s3_decode_step(rig.a, 0, m, off_d, pos_d, qd, kd, vd, out, s3.S3_F32, 0.0, len_out, rig.stream,
                             slot_id=ids, pos_host=pos) == 0
    torch.cuda.synchronize()
    assert len_out.cpu().tolist() == [p + 1 for p in pos]
    for j, sid in enumerate(ids.tolist()):
        assert rig.o.append(sid, 0, pos[j], k[j], v[j]) == 0
        for which in (0, 1):
            assert np.array_equal(rig.read(sid, 0, which, pos[j] + 1), rig.o.rows(sid, 0, which, pos[j] + 1).astype(np.uint8))
    want = rig.o.attention(0, ids.tolist(), [p + 1 for p in pos], q, None, "f32", threads=8)
    assert_close(out.cpu().numpy(), want, "e4m3 decode step at the maximum length")
    rig.close()


def test_8_bit_slot_whose_rows_lie_beyond_4_gib_of_its_plane():
    """32 KiB rows of codes, slots that start more than 4 GiB into the plane; a decode step there."""
    H, D, act = 128, 256, s3.S3_F16
    row_bytes = H * D
    filler = 2 ** 32 // row_bytes + 500
    rig = Rig8(1, H, D, act, 64, 2 * 2 ** 32 // row_bytes, [filler, 100, 64], seed=96, arena_tokens=filler + 4000)
    assert int(rig.offs[1]) * row_bytes > 2 ** 32
    ids, offs, lens = rig.ids[1:], rig.offs[1:], [100, 63]
    for sid, L in zip(ids.tolist(), lens):
        k = wl.normal_bits(rig.rng, (L, H, D), wl.E4M3)
        v = wl.normal_bits(rig.rng, (L, H, D), wl.E4M3)
        assert rig.o.fill(sid, 0, k, v) == 0
        assert s3.s3_kv_fill(rig.a, sid, 0, 0, L, device_bits(k, None, DEV), device_bits(v, None, DEV), rig.stream) == 0
    n = 2
    q, k, v = (wl.normal_bits(rig.rng, (n, H, D), act) for _ in range(3))
    qd, kd, vd = (device_bits(x, TDT[act], DEV) for x in (q, k, v))
    off_d = torch.tensor(offs.tolist(), dtype=torch.int64, device=DEV)
    pos_d = torch.tensor(lens, dtype=torch.int32, device=DEV)
    out = torch.full((n, H, D), float("nan"), dtype=torch.float32, device=DEV)
    len_out = torch.zeros(n, dtype=torch.int32, device=DEV)
    assert s3.s3_decode_step(rig.a, 0, n, off_d, pos_d, qd, kd, vd, out, s3.S3_F32, 0.0, len_out, rig.stream,
                             slot_id=ids, pos_host=lens) == 0
    torch.cuda.synchronize()
    for j, sid in enumerate(ids.tolist()):
        assert rig.o.append(sid, 0, lens[j], k[j], v[j]) == 0
        for which in (0, 1):
            assert np.array_equal(rig.read(sid, 0, which, lens[j] + 1), rig.o.rows(sid, 0, which, lens[j] + 1).astype(np.uint8))
    want = rig.o.attention(0, ids.tolist(), [L + 1 for L in lens], q, None, "f32", threads=8)
    assert_close(out.cpu().numpy(), want, "e4m3 rows beyond 4 GiB")
    rig.close()


@pytest.mark.parametrize("H,Hkv", [(4, None), (8, 2)])
def test_8_bit_step_refuses_full_slots_and_skips_bad_entries(H, Hkv):
    """The decode step over 8-bit rows (which appends inside the attention kernel, or with the quantising
    append before the matrix-core kernel) writes nothing for a refused call or a device entry that would
    leave the arena: zero output row, arena untouched except the valid neighbour's new row."""
    D, act = 128, s3.S3_F16
    lens = [64, 10]
    rig = Rig8(1, H, D, act, 64, 256, [64, 64], seed=23, Hkv=Hkv, arena_tokens=1024)
    rig.fill(lens)
    n, kvh = 2, Hkv or H
    q = device_bits(wl.normal_bits(rig.rng, (n, H, D), act), TDT[act], DEV)
    k, v = (device_bits(wl.normal_bits(rig.rng, (n, kvh, D), act), TDT[act], DEV) for _ in range(2))
    off_d = torch.tensor(rig.offs.tolist(), dtype=torch.int64, device=DEV)
    pos_d = torch.tensor(lens, dtype=torch.int32, device=DEV)
    out = torch.zeros((n, H, D), dtype=torch.float32, device=DEV)
    snap = rig.mem.clone()
    assert s3.s3_decode_step(rig.a, 0, n, off_d, pos_d, q, k, v, out, s3.S3_F32, 0.0, None, rig.stream,
                             slot_id=rig.ids, pos_host=lens) == s3.S3_ERR_SLOT_FULL
    torch.cuda.synchronize()
    assert torch.equal(snap, rig.mem)
    for bad in ([rig.N - 5, int(rig.offs[1])], [-1, int(rig.offs[1])]):
        bad_off = torch.tensor(bad, dtype=torch.int64, device=DEV)
        out.fill_(float("nan"))
        assert s3.s3_decode_step(rig.a, 0, n, bad_off, pos_d, q, k, v, out, s3.S3_F32, 0.0, None, rig.stream) == 0
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert not got[0].any() and np.isfinite(got[1]).all()
        changed = (snap != rig.mem).nonzero().flatten().cpu().numpy()
        row_bytes = kvh * D
        lo = (int(rig.offs[1]) + lens[1]) * row_bytes  # the valid neighbour's new K row; its V row is one plane on
        plane = rig.N * row_bytes
        assert changed.size and all(lo <= c % plane < lo + row_bytes for c in changed.tolist())
    rig.close()


def test_grow_and_evict_move_8_bit_rows_bit_exactly():
    H, D = 8, 128
    rig = Rig8(2, H, D, s3.S3_BF16, 64, 512, [64, 100, 64], seed=50)
    lens = [64, 90, 10]
    for layer in (0, 1):
        rig.fill(lens, layer=layer)
    sid = int(rig.ids[0])
    got = s3.s3_kv_grow(rig.a, sid, 64, rig.stream)
    assert got == rig.o.grow(sid, 64) and got[2] == 128
    for layer in (0, 1):
        for which in (0, 1):
            assert np.array_equal(rig.read(sid, layer, which, 64), rig.o.rows(sid, layer, which, 64).astype(np.uint8))
    other = int(rig.ids[1])
    for layer in (0, 1):
        for which in (0, 1):
            assert np.array_equal(rig.read(other, layer, which, 90), rig.o.rows(other, layer, which, 90).astype(np.uint8))
    assert s3.s3_kv_evict_bytes(rig.a, 90) == 2 * 2 * 90 * H * D
    rig.close()


def test_c6_trace_with_grow_free_and_refill():
    from paper_2306_06000_amd.engine import DecodeEngine

    w = wl.c6(batch=48, steps=40)
    eng = DecodeEngine(w)
    prefill, tensors_for = make_sources(w, eng)
    eng.start(prefill)
    got = {}
    for t in range(w.steps):
        out = eng.step(tensors_for(t), prefill, check_host=True)
        if t in (0, 20, 39):
            got[t] = out.float().cpu().numpy()
    rep = OracleReplay(w, eng.arena_tokens)
    outs = rep.replay(eng.events, attend_steps={0, 20, 39})
    for t, g in got.items():
        assert_close(g, outs[t][2], f"{w.name} step {t}")
    for a in eng.active:
        sid = rep.sid[a.serial]
        assert sid == a.slot and rep.o.slots[sid] == [a.off, a.cap] and rep.len[a.serial] == a.len
        for which in (0, 1):
            assert np.array_equal(eng.read_slot(a, 0, which), rep.o.rows(sid, 0, which, a.len).astype(np.uint8))
    assert s3.s3_kv_stats(eng.arena) == (0, *rep.o.stats())
    assert s3.s3_kv_get_param(eng.arena, "n_grows")[1] == rep.o.n_grows
    eng.close()
