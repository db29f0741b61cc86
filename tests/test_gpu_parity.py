"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Integers (ids, offsets, capacities) and stored rows must be bit-exact;
attention must be within max-abs 2e-3 and relative L2 1e-3 of the fp32 oracle."""
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


class Rig:
    """A small arena with hand-placed sequences, mirrored in the oracle."""

    def __init__(self, n_layers, H, D, dtype, G, M, preds, seed, arena_tokens=None, Hkv=None):
        self.n_layers, self.H, self.D, self.dtype = n_layers, H, D, dtype
        self.Hkv = Hkv or H  # heads of a cached row
        self.cfg = s3.make_config(n_layers, H, D, dtype, G, M, 0 if Hkv is None else Hkv)
        bpt = s3.s3_kv_bytes_per_token(self.cfg)
        caps = [min(M, max(G, -(-p // G) * G)) for p in preds]
        self.N = arena_tokens or (sum(caps) + 3 * M)
        self.mem = torch.zeros(self.N * bpt, dtype=torch.uint8, device=DEV)
        st, self.a = s3.s3_kv_arena_init(self.cfg, self.mem, self.mem.numel())
        assert st == 0
        self.o = orc.KVOracle(n_layers, H, D, dtype, G, M, self.N * bpt, n_kv_heads=Hkv)
        assert bpt == self.o.bytes_per_token
        rc, self.ids, self.offs, self.caps = s3.s3_kv_alloc(self.a, preds)
        n_o, ids_o, offs_o, caps_o = self.o.alloc(preds)
        assert rc == n_o == len(preds)
        assert self.ids.tolist() == ids_o and self.offs.tolist() == offs_o and self.caps.tolist() == caps_o
        self.rng = np.random.default_rng(seed)
        self.stream = torch.cuda.current_stream().cuda_stream

    def fill(self, lens, layer=0):
        for sid, L in zip(self.ids.tolist(), lens):
            if L == 0:
                continue
            k = wl.normal_bits(self.rng, (L, self.Hkv, self.D), self.dtype)
            v = wl.normal_bits(self.rng, (L, self.Hkv, self.D), self.dtype)
            assert self.o.fill(sid, layer, k, v) == 0
            st = s3.s3_kv_fill(self.a, sid, layer, 0, L, device_bits(k, TDT[self.dtype], DEV),
                               device_bits(v, TDT[self.dtype], DEV), self.stream)
            assert st == 0

    def attend(self, lens, layer=0, out_dtype=s3.S3_F32, scale=0.0, offs=None, q=None):
        n = len(lens)
        if q is None:
            q = wl.normal_bits(self.rng, (n, self.H, self.D), self.dtype)
        qd = device_bits(q, TDT[self.dtype], DEV)
        off_d = torch.tensor(self.offs.tolist() if offs is None else offs, dtype=torch.int64, device=DEV)
        len_d = torch.tensor(lens, dtype=torch.int32, device=DEV)
        odt = {s3.S3_F32: torch.float32, s3.S3_F16: torch.float16, s3.S3_BF16: torch.bfloat16}[out_dtype]
        out = torch.full((n, self.H, self.D), float("nan"), dtype=odt, device=DEV)
        st = s3.s3_decode_attention(self.a, layer, n, qd, off_d, len_d, out, out_dtype, scale, self.stream)
        assert st == 0, st
        torch.cuda.synchronize()
        return q, out.float().cpu().numpy()

    def oracle_attend(self, q, lens, layer=0, scale=None):
        return self.o.attention(layer, self.ids.tolist(), lens, q, scale, "f32", threads=8)

    def close(self):
        torch.cuda.synchronize()
        s3.s3_kv_arena_destroy(self.a)


def n_variants(a):
    return s3.s3_kv_get_param(a, "n_variants")[1]


# ---------------------------------------------------------------- C0, the whole config
@pytest.mark.parametrize("fused", [True, False])
def test_c0_one_append_and_attention_step(fused):
    from paper_2306_06000_amd.engine import DecodeEngine

    w = wl.c0()
    eng = DecodeEngine(w, arena_tokens=512, fused=fused)
    prefill, tensors_for = make_sources(w, eng)
    eng.start(prefill)
    assert [a.cap for a in eng.active] == [64, 64, 128, 128] and [a.off for a in eng.active] == [0, 64, 128, 256]
    out = eng.step(tensors_for(0), prefill, check_host=True)
    got = out.float().cpu().numpy()
    rep = OracleReplay(w, 512)
    outs = rep.replay(eng.events, attend_steps={0})
    serials, lens, want = outs[0]
    assert lens == [17, 64, 100, 128]
    assert_close(got, want, "C0")
    # the step retired all four sequences (each generated its one token); rows were checked by replay
    assert eng.active == [] and s3.s3_kv_stats(eng.arena)[1] == 0
    eng.close()


def test_c0_read_as_pre_append_lengths_needs_two_grows():
    """Other reading of the config: {17,64,100,128} rows are cached BEFORE the step with capacities
    {64,64,128,128}: sequences 1 and 3 are full, append reports it, grow doubles them."""
    rig = Rig(1, 16, 256, s3.S3_F16, 64, 2048, [17, 64, 100, 128], seed=5)
    lens = [17, 64, 100, 128]
    rig.fill(lens)
    n = 4
    k = wl.normal_bits(rig.rng, (n, 16, 256), 0)
    v = wl.normal_bits(rig.rng, (n, 16, 256), 0)
    kd, vd = device_bits(k, torch.float16, DEV), device_bits(v, torch.float16, DEV)
    off_d = torch.tensor(rig.offs.tolist(), dtype=torch.int64, device=DEV)
    pos_d = torch.tensor(lens, dtype=torch.int32, device=DEV)
    before = [rig_read(rig, sid, 0, w_, c) for sid, c in zip(rig.ids.tolist(), rig.caps.tolist()) for w_ in (0, 1)]
    st = s3.s3_kv_append(rig.a, 0, n, off_d, pos_d, kd, vd, rig.stream, slot_id=rig.ids, pos_host=lens)
    assert st == s3.S3_ERR_SLOT_FULL
    after = [rig_read(rig, sid, 0, w_, c) for sid, c in zip(rig.ids.tolist(), rig.caps.tolist()) for w_ in (0, 1)]
    assert all(np.array_equal(x, y) for x, y in zip(before, after))  # nothing was written
    for b in (1, 3):
        sid = int(rig.ids[b])
        assert rig.o.append(sid, 0, lens[b], k[b], v[b]) == orc.ERR_SLOT_FULL
        got = s3.s3_kv_grow(rig.a, sid, lens[b], rig.stream)
        assert got == rig.o.grow(sid, lens[b])
        rig.offs[b], rig.caps[b] = got[1], got[2]
    assert rig.caps.tolist() == [64, 128, 128, 256]
    off_d = torch.tensor(rig.offs.tolist(), dtype=torch.int64, device=DEV)
    st = s3.s3_kv_append(rig.a, 0, n, off_d, pos_d, kd, vd, rig.stream, slot_id=rig.ids, pos_host=lens)
    assert st == 0
    for b, sid in enumerate(rig.ids.tolist()):
        assert rig.o.append(sid, 0, lens[b], k[b], v[b]) == 0
        for which in (0, 1):
            assert np.array_equal(rig_read(rig, sid, 0, which, rig.caps[b]), rig.o.data[sid][0, which])
    lens1 = [L + 1 for L in lens]
    q, got = rig.attend(lens1)
    assert_close(got, rig.oracle_attend(q, lens1), "C0 pre-append reading")
    rig.close()


def rig_read(rig, sid, layer, which, rows):
    dst = torch.empty((int(rows), rig.Hkv, rig.D), dtype=torch.int16, device=DEV)
    assert s3.s3_kv_read_rows(rig.a, sid, layer, which, 0, int(rows), dst, rig.stream) == 0
    return dst.cpu().numpy().view(np.uint16)


# ---------------------------------------------------------------- kernel variants, chunk sizes, shapes
RAGGED = [1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 200, 255, 256, 257, 300, 511, 777, 1000, 1, 5, 64]


def test_every_variant_and_chunk_size_on_a_ragged_batch():
    rig = Rig(1, 16, 256, s3.S3_F16, 64, 2048, RAGGED, seed=11)
    rig.fill(RAGGED)
    q = wl.normal_bits(rig.rng, (len(RAGGED), 16, 256), 0)
    want = rig.oracle_attend(q, RAGGED)
    for variant in range(n_variants(rig.a)):
        for chunk in (32, 64, 128, 256, 1024):
            assert s3.s3_kv_set_param(rig.a, "variant", variant) == 0
            assert s3.s3_kv_set_param(rig.a, "chunk", chunk) == 0
            _, got = rig.attend(RAGGED, q=q)
            assert_close(got, want, f"variant {variant} chunk {chunk}")
    # a grid much smaller than the work list (every workgroup walks many items) and a huge one
    s3.s3_kv_set_param(rig.a, "variant", 1)
    s3.s3_kv_set_param(rig.a, "chunk", 64)
    for blocks in (1, 7, 100000):
        s3.s3_kv_set_param(rig.a, "grid_blocks", blocks)
        _, got = rig.attend(RAGGED, q=q)
        assert_close(got, want, f"grid {blocks}")
    rig.close()


@pytest.mark.parametrize("dtype", [s3.S3_F16, s3.S3_BF16])
@pytest.mark.parametrize("D", [64, 128, 256])
@pytest.mark.parametrize("H", [1, 3, 12, 16])
def test_shapes_and_types(dtype, D, H):
    lens = [1, 17, 64, 100, 128, 129, 515, 40]
    rig = Rig(1, H, D, dtype, 64, 1024, lens, seed=100 * D + 10 * H + dtype)
    rig.fill(lens)
    q = wl.normal_bits(rig.rng, (len(lens), H, D), dtype)
    want = rig.oracle_attend(q, lens)
    for variant in (0, 1, 3, 6):
        s3.s3_kv_set_param(rig.a, "variant", variant)
        _, got = rig.attend(lens, q=q)
        assert_close(got, want, f"H{H} D{D} dt{dtype} v{variant}")
    rig.close()


def test_multi_layer_planes_are_independent():
    lens = [70, 130, 5]
    rig = Rig(3, 4, 128, s3.S3_BF16, 64, 512, lens, seed=3)
    for layer in range(3):
        rig.fill(lens, layer)
    for layer in range(3):
        q, got = rig.attend(lens, layer)
        assert_close(got, rig.oracle_attend(q, lens, layer), f"layer {layer}")
    rig.close()


def test_explicit_scale_and_output_types():
    lens = [9, 150, 64]
    rig = Rig(1, 2, 128, s3.S3_F16, 64, 512, lens, seed=4)
    rig.fill(lens)
    q, got = rig.attend(lens, scale=0.05)
    assert_close(got, rig.oracle_attend(q, lens, scale=0.05), "scale 0.05")
    want = rig.oracle_attend(q, lens)
    _, got16 = rig.attend(lens, out_dtype=s3.S3_F16, q=q)
    assert_close(got16, want, "fp16 output")
    # a bfloat16 output cannot meet 2e-3 by rounding alone (half an ulp is 3.9e-3 in [1, 2)):
    # it must equal the fp32 result rounded once
    _, got32 = rig.attend(lens, q=q)
    _, gotbf = rig.attend(lens, out_dtype=s3.S3_BF16, q=q)
    rounded = torch.from_numpy(got32).to(torch.bfloat16).float().numpy()
    assert np.array_equal(gotbf, rounded)
    rig.close()


# ---------------------------------------------------------------- edge cases
def test_empty_context_length_one_and_max_length():
    M = 2048
    lens = [0, 1, M, 0, 2047]
    rig = Rig(1, 16, 256, s3.S3_F16, 64, M, [64, 64, M, 64, M], seed=6)
    rig.fill(lens)
    for chunk in (128, 2048, 32):
        s3.s3_kv_set_param(rig.a, "chunk", chunk)
        q, got = rig.attend(lens)
        want = rig.oracle_attend(q, lens)
        assert_close(got, want, f"edges chunk {chunk}")
        assert not got[0].any() and not got[3].any()  # empty context: zero row
        v0 = rig.o.rows(int(rig.ids[1]), 0, 1, 1)[0].view(np.float16).astype(np.float32)
        assert np.array_equal(got[1], v0)  # one cached row: the output is that value row exactly
    rig.close()


def test_identical_keys_give_the_mean_value_and_permutation_invariance():
    H, D, L = 16, 256, 333
    rig = Rig(1, H, D, s3.S3_F16, 64, 2048, [L, L], seed=8)
    rng = rig.rng
    krow = wl.normal_bits(rng, (1, H, D), 0)
    k = np.repeat(krow, L, axis=0)
    v = wl.normal_bits(rng, (L, H, D), 0)
    perm = rng.permutation(L)
    k2 = wl.normal_bits(rng, (L, H, D), 0)
    for sid, (kk, vv) in zip(rig.ids.tolist(), [(k, v), (k2, v)]):
        s3.s3_kv_fill(rig.a, sid, 0, 0, L, device_bits(kk, torch.float16, DEV), device_bits(vv, torch.float16, DEV),
                      rig.stream)
    q, got = rig.attend([L, L])
    mean = v.view(np.float16).astype(np.float64).mean(axis=0)
    assert np.abs(got[0] - mean).max() < 1e-4
    s3.s3_kv_fill(rig.a, int(rig.ids[0]), 0, 0, L, device_bits(k2[perm], torch.float16, DEV),
                  device_bits(v[perm], torch.float16, DEV), rig.stream)
    q2 = np.stack([q[1], q[1]])
    _, got2 = rig.attend([L, L], q=q2)
    assert np.abs(got2[0] - got2[1]).max() < 1e-5  # same rows in another order
    rig.close()


def test_bad_device_entries_are_skipped_not_followed():
    """Offsets / lengths that would address rows outside the arena are refused inside the
    kernels: attention returns a zero row, append writes nothing."""
    lens = [50, 60, 70, 80]
    rig = Rig(1, 4, 128, s3.S3_F16, 64, 256, lens, seed=9, arena_tokens=1024)
    rig.fill(lens)
    offs = rig.offs.tolist()
    bad_offs = [offs[0], -64, rig.N - 10, offs[3]]
    bad_lens = [50, 60, 70, 257]  # 1: negative offset, 2: runs past the arena, 3: longer than max_len
    q, got = rig.attend(bad_lens, offs=bad_offs)
    want = rig.oracle_attend(q, lens)
    assert_close(got[0], want[0], "good row beside bad ones")
    assert not got[1].any() and not got[2].any() and not got[3].any()
    snap = rig.mem.clone()
    k = device_bits(wl.normal_bits(rig.rng, (4, 4, 128), 0), torch.float16, DEV)
    off_d = torch.tensor([-1, rig.N, rig.N - 1, offs[0]], dtype=torch.int64, device=DEV)
    pos_d = torch.tensor([0, 0, 5, 256], dtype=torch.int32, device=DEV)
    assert s3.s3_kv_append(rig.a, 0, 4, off_d, pos_d, k, k, rig.stream) == 0
    torch.cuda.synchronize()
    assert torch.equal(snap, rig.mem)
    rig.close()


def test_append_writes_exactly_the_addressed_rows():
    lens = [10, 64, 127]
    rig = Rig(2, 12, 128, s3.S3_BF16, 64, 512, [64, 128, 128], seed=10)
    for layer in range(2):
        rig.fill(lens, layer)
    n = 3
    k = wl.normal_bits(rig.rng, (n, 12, 128), 1)
    v = wl.normal_bits(rig.rng, (n, 12, 128), 1)
    off_d = torch.tensor(rig.offs.tolist(), dtype=torch.int64, device=DEV)
    pos_d = torch.tensor(lens, dtype=torch.int32, device=DEV)
    st = s3.s3_kv_append(rig.a, 1, n, off_d, pos_d, device_bits(k, torch.bfloat16, DEV),
                         device_bits(v, torch.bfloat16, DEV), rig.stream, slot_id=rig.ids, pos_host=lens)
    assert st == 0
    for b, sid in enumerate(rig.ids.tolist()):
        assert rig.o.append(sid, 1, lens[b], k[b], v[b]) == 0
    for b, sid in enumerate(rig.ids.tolist()):
        for layer in range(2):
            for which in (0, 1):
                assert np.array_equal(rig_read(rig, sid, layer, which, rig.caps[b]), rig.o.data[sid][layer, which])
    # host-side refusal: unknown id, negative position
    assert s3.s3_kv_append(rig.a, 0, n, off_d, pos_d, device_bits(k, torch.bfloat16, DEV),
                           device_bits(v, torch.bfloat16, DEV), rig.stream, slot_id=[0, 1, 9], pos_host=lens) == -1
    rig.close()


def test_grow_moves_rows_bit_exactly_and_leaves_other_slots_alone():
    lens = [64, 100, 128, 30]
    rig = Rig(2, 16, 256, s3.S3_F16, 64, 2048, [64, 100, 128, 30], seed=12)
    for layer in range(2):
        rig.fill(lens, layer)
    for b in (0, 2):
        sid = int(rig.ids[b])
        got = s3.s3_kv_grow(rig.a, sid, lens[b], rig.stream)
        assert got == rig.o.grow(sid, lens[b]) and got[2] == 2 * rig.caps[b]
        rig.offs[b], rig.caps[b] = got[1], got[2]
    for b, sid in enumerate(rig.ids.tolist()):
        for layer in range(2):
            for which in (0, 1):
                assert np.array_equal(rig_read(rig, sid, layer, which, lens[b]), rig.o.rows(sid, layer, which, lens[b]))
    q, got = rig.attend(lens, layer=1)
    assert_close(got, rig.oracle_attend(q, lens, layer=1), "after grow")
    assert s3.s3_kv_stats(rig.a) == (0, *rig.o.stats())
    rig.close()


def test_fused_step_equals_append_then_attention_bit_for_bit():
    """s3_decode_step is defined as s3_kv_append + s3_decode_attention over pos+1 rows: same arena
    rows, len_out = pos + 1 and the same output bits (both cut the contexts into the same chunks and
    the work order does not enter the arithmetic).  For every variant, a few chunk sizes and class counts."""
    pos = [0, 1, 30, 31, 63, 64, 127, 128, 255, 256, 700, 1023, 5, 64]
    caps = [p + 1 for p in pos]
    H, D, dt = 16, 256, s3.S3_F16
    n = len(pos)
    rigs = [Rig(1, H, D, dt, 64, 1024, caps, seed=21) for _ in range(2)]  # same seed: same contents
    for r in rigs:
        r.fill(pos)
    rng = np.random.default_rng(22)
    for variant in range(n_variants(rigs[0].a)):
        for chunk in (64, 128, 512):
            q, k, v = (device_bits(wl.normal_bits(rng, (n, H, D), dt), torch.float16, DEV) for _ in range(3))
            outs, rows = [], []
            for r, fused in zip(rigs, (False, True)):
                s3.s3_kv_set_param(r.a, "variant", variant)
                s3.s3_kv_set_param(r.a, "chunk", chunk)
                assert s3.s3_kv_set_param(r.a, "classes", (variant + chunk // 64) % 9) == 0
                off_d = torch.tensor(r.offs.tolist(), dtype=torch.int64, device=DEV)
                pos_d = torch.tensor(pos, dtype=torch.int32, device=DEV)
                out = torch.full((n, H, D), float("nan"), dtype=torch.float32, device=DEV)
                if fused:
                    len_out = torch.zeros(n, dtype=torch.int32, device=DEV)
                    assert s3.s3_decode_step(r.a, 0, n, off_d, pos_d, q, k, v, out, s3.S3_F32, 0.0, len_out, r.stream,
                                             slot_id=r.ids, pos_host=pos) == 0
                    assert len_out.cpu().tolist() == [p + 1 for p in pos]
                    assert s3.s3_decode_step(r.a, 0, n, off_d, pos_d, q, k, v, out, s3.S3_F32, 0.0, pos_d,
                                             r.stream) == s3.S3_ERR_INVALID  # len_out must not alias pos
                else:
                    assert s3.s3_kv_append(r.a, 0, n, off_d, pos_d, k, v, r.stream, slot_id=r.ids, pos_host=pos) == 0
                    assert s3.s3_decode_attention(r.a, 0, n, q, off_d, pos_d + 1, out, s3.S3_F32, 0.0, r.stream) == 0
                torch.cuda.synchronize()
                outs.append(out.cpu().numpy())
                rows.append([rig_read(r, sid, 0, w_, c) for sid, c in zip(r.ids.tolist(), caps) for w_ in (0, 1)])
            assert np.array_equal(outs[0], outs[1]), (variant, chunk)
            assert all(np.array_equal(x, y) for x, y in zip(rows[0], rows[1])), (variant, chunk)
    for r in rigs:
        r.close()


@pytest.mark.parametrize("H,Hkv", [(4, None), (8, 2), (4, 2)])
def test_fused_step_refuses_full_slots_and_skips_bad_entries(H, Hkv):
    """Multi-head step kernel, matrix-core kernel (appends inside) and vector-ALU shared-head kernel
    (append launch before it)."""
    lens = [64, 10]
    rig = Rig(1, H, 128, s3.S3_F16, 64, 256, [64, 64], seed=23, arena_tokens=1024, Hkv=Hkv)
    rig.fill(lens)
    n, kvh = 2, Hkv or H
    q = device_bits(wl.normal_bits(rig.rng, (n, H, 128), 0), torch.float16, DEV)
    k, v = (device_bits(wl.normal_bits(rig.rng, (n, kvh, 128), 0), torch.float16, DEV) for _ in range(2))
    off_d = torch.tensor(rig.offs.tolist(), dtype=torch.int64, device=DEV)
    pos_d = torch.tensor(lens, dtype=torch.int32, device=DEV)
    out = torch.zeros((n, H, 128), dtype=torch.float32, device=DEV)
    snap = rig.mem.clone()
    assert s3.s3_decode_step(rig.a, 0, n, off_d, pos_d, q, k, v, out, s3.S3_F32, 0.0, None, rig.stream,
                             slot_id=rig.ids, pos_host=lens) == s3.S3_ERR_SLOT_FULL
    torch.cuda.synchronize()
    assert torch.equal(snap, rig.mem)
    # device entries that would leave the arena: zero row, nothing written, neighbours unaffected
    bad_off = torch.tensor([rig.N - 5, int(rig.offs[1])], dtype=torch.int64, device=DEV)
    out.fill_(float("nan"))
    assert s3.s3_decode_step(rig.a, 0, n, bad_off, pos_d, q, k, v, out, s3.S3_F32, 0.0, None, rig.stream) == 0
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert not got[0].any() and np.isfinite(got[1]).all()
    rig.close()


def test_compact_moves_rows_bit_exactly_including_overlapping_moves():
    """Holes left by finished sequences are closed by sliding the live slots down; a slot larger than
    the hole in front of it overlaps its own destination and is moved in pieces."""
    preds = [64, 2048, 64, 700, 128, 64, 300]
    lens = [64, 2000, 10, 650, 128, 1, 257]
    rig = Rig(2, 16, 256, s3.S3_F16, 64, 2048, preds, seed=31)
    for layer in range(2):
        rig.fill(lens, layer)
    for b in (0, 2, 5):  # holes of 64 rows in front of the 2048-row slot, between and behind
        sid = int(rig.ids[b])
        assert s3.s3_kv_free(rig.a, sid) == rig.o.free(sid) == 0
    live = [1, 3, 4, 6]
    ids = [int(rig.ids[b]) for b in live]
    st, new_off, moved = s3.s3_kv_compact(rig.a, ids, [lens[b] for b in live], rig.stream)
    want, want_moved = rig.o.compact()
    assert st == 0 and moved == want_moved == 4 and new_off.tolist() == [want[i] for i in ids]
    assert s3.s3_kv_stats(rig.a) == (0, *rig.o.stats())
    for b, sid in zip(live, ids):
        assert s3.s3_kv_slot_info(rig.a, sid) == (0, *rig.o.slots[sid])
        for layer in range(2):
            for which in (0, 1):
                assert np.array_equal(rig_read(rig, sid, layer, which, lens[b]), rig.o.rows(sid, layer, which, lens[b]))
    # attention over the moved slots
    rig.ids = np.array(ids, np.int32)
    rig.offs = new_off.copy()
    q, got = rig.attend([lens[b] for b in live], layer=1)
    assert_close(got, rig.oracle_attend(q, [lens[b] for b in live], layer=1), "after compaction")
    rig.close()


@pytest.mark.parametrize("pinned", [True, False])
def test_evict_to_host_and_restore_with_doubled_reservation(pinned):
    """Pinned memory makes the copies asynchronous; pageable memory works too: same bytes either way."""
    preds = [300, 128, 64]
    lens = [257, 128, 40]
    rig = Rig(2, 12, 128, s3.S3_BF16, 64, 512, preds, seed=33, arena_tokens=640)  # 320 + 128 + 64 used
    for layer in range(2):
        rig.fill(lens, layer)
    sid = int(rig.ids[1])
    assert s3.s3_kv_grow(rig.a, sid, 128, rig.stream)[0] == s3.S3_ERR_NOMEM  # 256 needed, 128 free
    nbytes = s3.s3_kv_evict_bytes(rig.a, 128)
    assert nbytes == 2 * 2 * 128 * 12 * 128 * 2
    host = torch.empty(nbytes, dtype=torch.uint8)
    if pinned:
        host = host.pin_memory()
    assert s3.s3_kv_evict(rig.a, sid, 128, host, rig.stream) == 0
    st_o, blob = rig.o.evict(sid, 128)
    assert st_o == 0 and s3.s3_kv_stats(rig.a) == (0, *rig.o.stats())
    torch.cuda.synchronize()
    assert np.array_equal(host.numpy().view(np.uint16).reshape(2, 2, 128, 12, 128), blob)
    assert s3.s3_kv_evict(rig.a, sid, 1, host, rig.stream) == s3.S3_ERR_INVALID  # already gone
    # the second sequence finishes; now the doubled reservation fits
    assert s3.s3_kv_restore(rig.a, 256, 128, host, rig.stream)[0] == s3.S3_ERR_NOMEM
    assert rig.o.restore(256, blob)[0] == orc.ERR_NOMEM
    assert s3.s3_kv_free(rig.a, int(rig.ids[2])) == rig.o.free(int(rig.ids[2])) == 0
    got = s3.s3_kv_restore(rig.a, 256, 128, host, rig.stream)
    assert got == rig.o.restore(256, blob) and got[3] == 256
    new_id = got[1]
    for layer in range(2):
        for which in (0, 1):
            assert np.array_equal(rig_read(rig, new_id, layer, which, 128), rig.o.rows(new_id, layer, which, 128))
            assert np.array_equal(rig_read(rig, int(rig.ids[0]), layer, which, 257),
                                  rig.o.rows(int(rig.ids[0]), layer, which, 257))
    assert s3.s3_kv_restore(rig.a, 100, 128, host, rig.stream)[0] == s3.S3_ERR_INVALID
    rig.close()


def test_gather_and_scatter_rows_are_the_device_side_halves_of_evict_and_restore():
    """An eviction staged through device memory: gather into a contiguous buffer (same layout and bits as the
    host buffer of s3_kv_evict, i.e. the oracle's evicted rows), free, reserve the doubled slot, scatter back;
    nothing else in the arena changes."""
    preds = [300, 128, 64]
    lens = [257, 128, 40]
    rig = Rig(2, 12, 128, s3.S3_BF16, 64, 512, preds, seed=34, arena_tokens=896)
    for layer in range(2):
        rig.fill(lens, layer)
    sid = int(rig.ids[1])
    nbytes = s3.s3_kv_evict_bytes(rig.a, 128)
    stage = torch.full((nbytes + 64,), 0xAB, dtype=torch.uint8, device=DEV)
    assert s3.s3_kv_gather_rows(rig.a, sid, 129, stage, rig.stream) == s3.S3_ERR_INVALID  # more rows than the slot holds
    assert s3.s3_kv_gather_rows(rig.a, 7, 1, stage, rig.stream) == s3.S3_ERR_INVALID
    assert s3.s3_kv_gather_rows(rig.a, sid, 128, stage[8:], rig.stream) == s3.S3_ERR_INVALID  # misaligned
    assert s3.s3_kv_gather_rows(rig.a, sid, 128, stage, rig.stream) == 0
    assert s3.s3_kv_free(rig.a, sid) == 0
    st_o, blob = rig.o.evict(sid, 128)
    assert st_o == 0 and s3.s3_kv_stats(rig.a) == (0, *rig.o.stats())
    torch.cuda.synchronize()
    assert np.array_equal(stage[:nbytes].cpu().numpy().view(np.uint16).reshape(2, 2, 128, 12, 128), blob)
    assert (stage[nbytes:] == 0xAB).all()  # nothing beyond the rows was written
    # over the host link and back with the small-grid copy kernel (pinned host memory, any grid size)
    host = torch.zeros(nbytes, dtype=torch.uint8).pin_memory()
    back = torch.full((nbytes + 64,), 0xCD, dtype=torch.uint8, device=DEV)
    assert s3.s3_kv_link_copy(host, stage, nbytes, 16, rig.stream) == 0
    assert s3.s3_kv_link_copy(back, host, nbytes, 3, rig.stream) == 0
    assert s3.s3_kv_link_copy(back, host, nbytes + 8, 3, rig.stream) == s3.S3_ERR_INVALID
    assert s3.s3_kv_link_copy(back, host, nbytes, 0, rig.stream) == s3.S3_ERR_INVALID
    torch.cuda.synchronize()
    assert np.array_equal(host.numpy().view(np.uint16).reshape(2, 2, 128, 12, 128), blob)
    assert torch.equal(back[:nbytes], stage[:nbytes]) and (back[nbytes:] == 0xCD).all()
    stage = back
    # the freed room is overwritten by a newcomer before the sequence returns
    rc, ids, offs, caps = s3.s3_kv_alloc(rig.a, [128])
    assert (rc, int(ids[0]), int(offs[0]), int(caps[0])) == (1, *rig.o.alloc_one(128))
    other = wl.normal_bits(rig.rng, (128, 12, 128), 1)
    for layer in range(2):
        assert rig.o.fill(int(ids[0]), layer, other, other) == 0
        assert s3.s3_kv_fill(rig.a, int(ids[0]), layer, 0, 128, device_bits(other, torch.bfloat16, DEV),
                             device_bits(other, torch.bfloat16, DEV), rig.stream) == 0
    want_cap = s3.s3_kv_grown_capacity(rig.cfg, 128)
    rc, ids2, offs2, caps2 = s3.s3_kv_alloc(rig.a, [want_cap])
    got_o = rig.o.restore(want_cap, blob)
    assert (0 if rc == 1 else -2, int(ids2[0]), int(offs2[0]), int(caps2[0])) == got_o and caps2[0] == 256
    snap = rig.mem.clone()
    assert s3.s3_kv_scatter_rows(rig.a, int(ids2[0]), 257, stage, rig.stream) == s3.S3_ERR_INVALID
    assert s3.s3_kv_scatter_rows(rig.a, int(ids2[0]), 128, stage, rig.stream) == 0
    torch.cuda.synchronize()
    changed = (rig.mem != snap).sum().item()
    assert 0 < changed <= nbytes
    for slot, rows in ((int(ids2[0]), 128), (int(ids[0]), 128), (int(rig.ids[0]), 257), (int(rig.ids[2]), 40)):
        for layer in range(2):
            for which in (0, 1):
                assert np.array_equal(rig_read(rig, slot, layer, which, rows), rig.o.rows(slot, layer, which, rows))
    rig.close()


def test_fill_batch_equals_fills_plus_patch():
    """s3_kv_fill_batch = the s3_kv_fill of every newcomer + the s3_kv_batch_patch of their batch entries,
    in one launch (more than 16 newcomers: several); arguments are checked before anything is enqueued."""
    H, D, dt = 4, 128, s3.S3_BF16
    preds = [64, 200, 64, 130, 64, 64, 500, 64, 90, 64, 64, 64, 300, 64, 64, 64, 64, 64, 77, 64]
    rig = Rig(2, H, D, dt, 64, 512, preds, seed=31)
    rows = [1, 200, 0, 130, 64, 3, 500, 17, 90, 64, 2, 5, 300, 9, 33, 64, 1, 8, 77, 60]
    n = len(preds)
    ks = [wl.normal_bits(rig.rng, (max(r, 1), H, D), dt) for r in rows]
    vs = [wl.normal_bits(rig.rng, (max(r, 1), H, D), dt) for r in rows]
    kd = [device_bits(k, TDT[dt], DEV) for k in ks]
    vd = [device_bits(v, TDT[dt], DEV) for v in vs]
    batch_n = 32
    off_d = torch.full((batch_n,), -7, dtype=torch.int64, device=DEV)
    len_d = torch.full((batch_n,), -7, dtype=torch.int32, device=DEV)
    idx = [(3 * i + 1) % batch_n for i in range(n)]
    assert len(set(idx)) == n
    bad_rows = list(rows)
    bad_rows[6] = 513  # more than the slot holds: refused as a whole
    assert s3.s3_kv_fill_batch(rig.a, 1, rig.ids, bad_rows, kd, vd, rig.stream, slot_off=off_d, length=len_d,
                               batch_n=batch_n, batch_idx=idx) == s3.S3_ERR_SLOT_FULL
    assert s3.s3_kv_fill_batch(rig.a, 1, rig.ids, rows, kd, vd, rig.stream, slot_off=off_d, length=len_d,
                               batch_n=batch_n, batch_idx=[99] * n) == s3.S3_ERR_INVALID
    torch.cuda.synchronize()
    assert (off_d.cpu().numpy() == -7).all() and not rig_read(rig, int(rig.ids[1]), 1, 0, 200).any()
    assert s3.s3_kv_fill_batch(rig.a, 1, rig.ids, rows, kd, vd, rig.stream, slot_off=off_d, length=len_d,
                               batch_n=batch_n, batch_idx=idx) == 0
    torch.cuda.synchronize()
    got_off, got_len = off_d.cpu().numpy(), len_d.cpu().numpy()
    for i, sid in enumerate(rig.ids.tolist()):
        assert got_off[idx[i]] == rig.offs[i] and got_len[idx[i]] == rows[i]
        if rows[i]:
            assert rig.o.fill(sid, 1, ks[i][:rows[i]], vs[i][:rows[i]]) == 0
        for which in (0, 1):
            assert np.array_equal(rig_read(rig, sid, 1, which, rig.caps[i]), rig.o.data[sid][1, which])
            assert not rig_read(rig, sid, 0, which, rig.caps[i]).any()  # the other layer is untouched
    untouched = sorted(set(range(batch_n)) - set(idx))
    assert (got_off[untouched] == -7).all() and (got_len[untouched] == -7).all()
    # without the batch arrays it is the fills alone
    assert s3.s3_kv_fill_batch(rig.a, 0, rig.ids[:3], rows[:3], kd[:3], vd[:3], rig.stream) == 0
    torch.cuda.synchronize()
    assert np.array_equal(rig_read(rig, int(rig.ids[1]), 0, 0, 200), ks[1])
    rig.close()


def test_batch_patch_rewrites_only_the_named_entries():
    n = 100
    off = torch.arange(n, dtype=torch.int64, device=DEV) * 64
    ln = torch.arange(n, dtype=torch.int32, device=DEV)
    idx = list(range(0, 100, 3))  # 34 updates: more than one launch's worth
    new_off = [7000 + i for i in idx]
    new_len = [900 + i for i in idx]
    st = torch.cuda.current_stream().cuda_stream
    assert s3.s3_kv_batch_patch(n, off, ln, idx, new_off, new_len, st) == 0
    want_off = (np.arange(n) * 64).astype(np.int64)
    want_len = np.arange(n).astype(np.int32)
    want_off[idx] = new_off
    want_len[idx] = new_len
    assert off.cpu().numpy().tolist() == want_off.tolist() and ln.cpu().numpy().tolist() == want_len.tolist()
    assert s3.s3_kv_batch_patch(n, off, None, [5], [1], None, st) == 0  # offsets only
    assert int(off[5]) == 1 and int(ln[5]) == want_len[5]
    assert s3.s3_kv_batch_patch(n, off, ln, [100], [1], [1], st) == s3.S3_ERR_INVALID
    assert s3.s3_kv_batch_patch(n, None, None, [1], [1], [1], st) == s3.S3_ERR_INVALID


# ---------------------------------------------------------------- traces
def run_trace(w, steps, attend_steps, arena_tokens=None, variant=None, chunk=None, sample=None, fused=True, admission="fifo"):
    from paper_2306_06000_amd.engine import DecodeEngine

    eng = DecodeEngine(w, arena_tokens=arena_tokens, fused=fused, admission=admission)
    if variant is not None:
        s3.s3_kv_set_param(eng.arena, "variant", variant)
    if chunk is not None:
        s3.s3_kv_set_param(eng.arena, "chunk", chunk)
    prefill, tensors_for = make_sources(w, eng)
    eng.start(prefill)
    got = {}
    for t in range(steps):
        out = eng.step(tensors_for(t), prefill, check_host=True)
        if t in attend_steps:
            got[t] = out.float().cpu().numpy()
    rep = OracleReplay(w, eng.arena_tokens)
    outs = rep.replay(eng.events, attend_steps=set(attend_steps))
    for t in attend_steps:
        serials, lens, want = outs[t]
        assert_close(got[t], want, f"{w.name} step {t}")
    # every live slot holds exactly the rows the oracle holds
    live = eng.active if sample is None else eng.active[:sample]
    for a in live:
        sid = rep.sid[a.serial]
        assert sid == a.slot and rep.o.slots[sid] == [a.off, a.cap] and rep.len[a.serial] == a.len
        for layer in range(w.n_layers):
            for which in (0, 1):
                assert np.array_equal(eng.read_slot(a, layer, which), rep.o.rows(sid, layer, which, a.len))
    assert s3.s3_kv_stats(eng.arena) == (0, *rep.o.stats())
    stats = dict(grows=s3.s3_kv_get_param(eng.arena, "n_grows")[1], frees=sum(e[0] == "free" for e in eng.events),
                 evicted=eng.n_evicted)
    assert stats["grows"] == rep.o.n_grows
    eng.close()
    return stats


# ---------------------------------------------------------------- shared key/value heads
GQA_SHAPES = [  # (query heads, kv heads, head dim)
    (32, 8, 128), (16, 1, 256), (8, 1, 64), (8, 2, 64), (12, 4, 128), (6, 3, 256), (24, 8, 64), (64, 8, 128),
    (16, 16, 128), (12, 2, 128), (9, 3, 64), (40, 5, 128),
]


@pytest.mark.parametrize("dtype", [s3.S3_F16, s3.S3_BF16])
@pytest.mark.parametrize("H,Hkv,D", GQA_SHAPES)
def test_shared_kv_heads_attention(H, Hkv, D, dtype):
    """n_kv_heads < n_heads (grouped-query; 1 = multi-query, related work): rows hold Hkv heads,
    query head h reads head h // (H // Hkv).  Ragged lengths incl. empty, one row and a tail that
    is no multiple of the rows a wave load covers.  (16, 16, 128) with the field set explicitly is
    plain multi-head attention and takes the multi-head kernels."""
    lens = [0, 1, 2, 3, 7, 8, 9, 31, 33, 64, 100, 255, 257, 600, 1, 5]
    rig = Rig(2, H, D, dtype, 64, 1024, [max(1, L) for L in lens], seed=70 + H + Hkv, Hkv=Hkv)
    rig.fill(lens, layer=1)
    q, got = rig.attend(lens, layer=1)
    want = rig.oracle_attend(q, lens, layer=1)
    assert_close(got, want, f"shared kv {H}/{Hkv} d{D}")
    assert not got[0].any()  # empty context: zeros
    # 16-bit outputs follow the same rule as the multi-head kernels: fp16 within the tolerance; a bf16 output
    # cannot meet 2e-3 by rounding alone and must equal the fp32 result rounded once
    _, got16 = rig.attend(lens, layer=1, out_dtype=s3.S3_F16, q=q)
    assert_close(got16, want, f"shared kv {H}/{Hkv} d{D} fp16 output")
    _, gotbf = rig.attend(lens, layer=1, out_dtype=s3.S3_BF16, q=q)
    assert np.array_equal(gotbf, torch.from_numpy(got).to(torch.bfloat16).float().numpy())
    # every kernel shape; chunk sizes from contexts in up to 19 pieces (merged by the second kernel)
    # to all in one piece
    shapes = n_variants(rig.a) if Hkv < H else 1
    for shape in range(shapes):
        if Hkv < H:
            assert s3.s3_kv_set_param(rig.a, "variant", shape) == 0
        for chunk in (32, 160, 1024):
            assert s3.s3_kv_set_param(rig.a, "chunk", chunk) == 0
            q, got = rig.attend(lens, layer=1)
            assert_close(got, rig.oracle_attend(q, lens, layer=1), f"shared kv {H}/{Hkv} d{D} shape {shape} chunk {chunk}")
    if Hkv < H:
        assert s3.s3_kv_set_param(rig.a, "variant", shapes) == s3.S3_ERR_INVALID
    rig.close()


@pytest.mark.parametrize("H,Hkv,D,dtype", [(32, 8, 128, s3.S3_BF16), (16, 1, 256, s3.S3_F16), (8, 2, 64, s3.S3_F16)])
def test_shared_kv_heads_decode_step_appends_then_attends(H, Hkv, D, dtype):
    """s3_decode_step with shared heads: the new [Hkv][D] rows land at row pos of both planes
    (bit-exact against the oracle's rows), len_out = pos + 1, attention over pos + 1 rows within
    tolerance; a full slot is refused on the host with nothing written."""
    pos = [0, 1, 31, 63, 64, 100, 255, 513, 5]
    caps = [p + 1 for p in pos]
    rig = Rig(1, H, D, dtype, 64, 1024, caps, seed=90 + H, Hkv=Hkv)
    rig.fill(pos)
    n = len(pos)
    q = wl.normal_bits(rig.rng, (n, H, D), dtype)
    k = wl.normal_bits(rig.rng, (n, Hkv, D), dtype)
    v = wl.normal_bits(rig.rng, (n, Hkv, D), dtype)
    qd, kd, vd = (device_bits(x, TDT[dtype], DEV) for x in (q, k, v))
    off_d = torch.tensor(rig.offs.tolist(), dtype=torch.int64, device=DEV)
    pos_d = torch.tensor(pos, dtype=torch.int32, device=DEV)
    out = torch.full((n, H, D), float("nan"), dtype=torch.float32, device=DEV)
    len_out = torch.zeros(n, dtype=torch.int32, device=DEV)
    full = list(rig.caps.tolist())
    assert s3.s3_decode_step(rig.a, 0, n, off_d, pos_d, qd, kd, vd, out, s3.S3_F32, 0.0, len_out, rig.stream,
                             slot_id=rig.ids, pos_host=full) == s3.S3_ERR_SLOT_FULL
    assert s3.s3_decode_step(rig.a, 0, n, off_d, pos_d, qd, kd, vd, out, s3.S3_F32, 0.0, len_out, rig.stream,
                             slot_id=rig.ids, pos_host=pos) == 0
    torch.cuda.synchronize()
    assert len_out.cpu().tolist() == caps
    for b, sid in enumerate(rig.ids.tolist()):
        assert rig.o.append(sid, 0, pos[b], k[b], v[b]) == 0
        for which in (0, 1):
            assert np.array_equal(rig_read(rig, sid, 0, which, rig.caps[b]), rig.o.data[sid][0, which])
    assert_close(out.cpu().numpy(), rig.oracle_attend(q, caps), f"shared kv step {H}/{Hkv}")
    rig.close()


@pytest.mark.parametrize("fused", [True, False])
def test_c5_shared_kv_trace_with_grow_free_and_refill(fused):
    w = wl.c5(batch=48, steps=48)
    stats = run_trace(w, w.steps, attend_steps=[0, 20, 47], fused=fused)
    assert stats["frees"] >= 1


def test_c5_multi_query_trace():
    w = wl.c5(batch=32, steps=24, n_heads=16, n_kv_heads=1, head_dim=256, dtype=wl.F16)
    run_trace(w, w.steps, attend_steps=[0, 23])


@pytest.mark.parametrize("fused", [True, False])
def test_c1_trace_128_steps_with_grow_free_and_refill(fused):
    w = wl.c1()
    stats = run_trace(w, w.steps, attend_steps=[0, 1, 40, 127], fused=fused)
    assert stats["grows"] >= 1 and stats["frees"] >= 1 and stats["evicted"] == 0


@pytest.mark.parametrize("fused", [True, False])
def test_c2_shape_shortened_trace_with_mispredictions(fused):
    w = wl.c2(batch=192, steps=40)
    stats = run_trace(w, w.steps, attend_steps=[0, 39], sample=48, fused=fused)
    assert stats["grows"] >= 1


def test_c4_shape_long_contexts_bf16():
    w = wl.c4(batch=24, steps=6)
    run_trace(w, w.steps, attend_steps=[0, 5], sample=6)


def test_c3_shape_small_arena_28_layers():
    w = wl.c3(target_bytes=0)
    w.seqs = w.seqs[:6]
    w.arena_bytes = 0
    run_trace(w, 1, attend_steps=[0])


def tight_workload(seed, n=12, n_layers=2, H=4, D=64, dtype=wl.F16, steps=260):
    """Under-predicted sequences in an arena that cannot hold all their doubled reservations: the
    doubling runs out of room, which is the supervisor's case (section 3)."""
    rng = np.random.default_rng(seed)

    def draw():
        p, o = int(rng.integers(20, 60)), int(rng.integers(90, 240))
        return wl.Seq(prompt=p, output=o, predicted=p + int(rng.integers(4, 40)))

    return wl.Workload(f"tight-{seed}", 40 + seed, n_layers, H, D, dtype, 32, 512, n, steps, [draw() for _ in range(n)],
                       [draw() for _ in range(3 * n)], True)


def test_c1_trace_with_the_scheduler_admitting():
    """The batch is chosen by the library's scheduler (largest reservation first, from the initial
    candidates and the refill pool together) instead of in arrival order; the oracle's scheduler must
    pick the same requests and get the same slots at every iteration."""
    w = wl.c1(batch=24, steps=64)
    run_trace(w, w.steps, attend_steps=[0, 30, 63], admission="dff")  # the longest come first: few finish here;
    # refills through the scheduler are exercised by the tight-arena trace below


@pytest.mark.parametrize("seed,arena_tokens,admission", [(1, 1536, "fifo"), (2, 1280, "fifo"), (3, 2048, "fifo"), (1, 1536, "dff")])
def test_supervisor_path_compacts_evicts_and_readmits(seed, arena_tokens, admission):
    """Mispredictions in a tight arena: a doubling that finds no extent first compacts (when the free
    space is only fragmented), else the sequence goes to pinned host memory and returns with the doubled
    reservation once a finished sequence has made room.  Every id, offset and capacity the library
    answered, the rows of every live slot and the attention outputs must equal the oracle's replay."""
    from paper_2306_06000_amd.engine import DecodeEngine

    w = tight_workload(seed)
    eng = DecodeEngine(w, arena_tokens=arena_tokens, admission=admission)
    prefill, tensors_for = make_sources(w, eng)
    eng.start(prefill, stop_when_full=True)
    attend = sorted({0, 60, 130, 200, w.steps - 1})
    got = {}
    for t in range(w.steps):
        if eng.n_active == 0 and not eng.swapped and not eng.n_returning:
            break
        out = eng.step(tensors_for(t), prefill, check_host=True)
        if t in attend and out is not None:
            got[t] = out.float().cpu().numpy()
    eng.finish_restores()  # sequences whose rows are still on their way back join the batch: their rows are checked too
    kinds = [e[0] for e in eng.events]
    print(f"tight {seed}: grows {eng.n_grown} compactions {eng.n_compactions} out {eng.n_swapped_out} in {eng.n_swapped_in} "
          f"still on host {len(eng.swapped)} batch {eng.n_active}")
    rep = OracleReplay(w, eng.arena_tokens)
    outs = rep.replay(eng.events, attend_steps=set(got))
    for t in got:
        assert_close(got[t], outs[t][2], f"{w.name} step {t}")
    for a in eng.active:
        sid = rep.sid[a.serial]
        assert sid == a.slot and rep.o.slots[sid] == [a.off, a.cap] and rep.len[a.serial] == a.len
        for layer in range(w.n_layers):
            for which in (0, 1):
                assert np.array_equal(eng.read_slot(a, layer, which), rep.o.rows(sid, layer, which, a.len))
    assert s3.s3_kv_stats(eng.arena) == (0, *rep.o.stats())
    assert eng.n_swapped_out >= 1 and eng.n_swapped_in >= 1 and "restore" in kinds
    assert {r.serial for r in eng.swapped} == set(rep.blobs)
    eng.close()


@pytest.mark.parametrize("H,Hkv", [(2, None), (4, 1)])
def test_largest_batch_one_call_takes(H, Hkv):
    """4095 sequences in one call (the documented maximum; one more is refused), short ragged contexts,
    attention and a decode step, with the default work order and with eight length classes requested
    (the library keeps as many as fit its workgroup memory).  Multi-head kernels, and the matrix-core
    kernel for shared heads."""
    n, D, dt = 4095, 64, s3.S3_F16
    rng = np.random.default_rng(77)
    lens = [int(x) for x in rng.integers(0, 48, n)]
    lens[:4] = [0, 1, 47, 33]
    rig = Rig(1, H, D, dt, 64, 64, [64] * n, seed=78, Hkv=Hkv)
    kvh = Hkv or H
    rig.fill(lens)
    for classes in (0, 8):
        assert s3.s3_kv_set_param(rig.a, "classes", classes) == 0
        q, got = rig.attend(lens)
        assert_close(got, rig.oracle_attend(q, lens), f"batch of {n}, classes {classes}")
    q = wl.normal_bits(rig.rng, (n, H, D), dt)
    k = wl.normal_bits(rig.rng, (n, kvh, D), dt)
    v = wl.normal_bits(rig.rng, (n, kvh, D), dt)
    qd, kd, vd = (device_bits(x, TDT[dt], DEV) for x in (q, k, v))
    off_d = torch.tensor(rig.offs.tolist(), dtype=torch.int64, device=DEV)
    pos_d = torch.tensor(lens, dtype=torch.int32, device=DEV)
    out = torch.full((n, H, D), float("nan"), dtype=torch.float32, device=DEV)
    len_out = torch.zeros(n, dtype=torch.int32, device=DEV)
    assert s3.s3_decode_step(rig.a, 0, n, off_d, pos_d, qd, kd, vd, out, s3.S3_F32, 0.0, len_out, rig.stream) == 0
    torch.cuda.synchronize()
    assert len_out.cpu().tolist() == [L + 1 for L in lens]
    for b, sid in enumerate(rig.ids.tolist()):
        assert rig.o.append(sid, 0, lens[b], k[b], v[b]) == 0
    want = rig.o.attention(0, rig.ids.tolist(), [L + 1 for L in lens], q, None, "f32", threads=8)
    assert_close(out.cpu().numpy(), want, f"decode step on a batch of {n}")
    for b in (0, 1, 2, 3, n - 1):
        for which in (0, 1):
            assert np.array_equal(rig_read(rig, int(rig.ids[b]), 0, which, lens[b] + 1), rig.o.rows(int(rig.ids[b]), 0, which, lens[b] + 1))
    # one more sequence than a call takes
    big = torch.zeros(n + 1, dtype=torch.int64, device=DEV)
    big_len = torch.zeros(n + 1, dtype=torch.int32, device=DEV)
    q1 = torch.zeros((n + 1, H, D), dtype=torch.float16, device=DEV)
    o1 = torch.zeros((n + 1, H, D), dtype=torch.float32, device=DEV)
    assert s3.s3_decode_attention(rig.a, 0, n + 1, q1, big, big_len, o1, s3.S3_F32, 0.0, rig.stream) == s3.S3_ERR_INVALID
    rig.close()


@pytest.mark.parametrize("H,Hkv", [(2, None), (8, 2)])
def test_contexts_up_to_a_long_maximum_length(H, Hkv):
    """max_len = 16384: one context that fills it, one a row short of it, short ones beside them; up to
    128 chunks per context merge (chunk 128) and the default chunking; a decode step appends the last
    row of the nearly full slot."""
    D, dt, M = 128, s3.S3_BF16, 16384
    lens = [M, M - 1, 1, 700, 0, 5000]
    rig = Rig(1, H, D, dt, 128, M, [max(1, L) for L in lens], seed=88, Hkv=Hkv)
    kvh = Hkv or H
    rig.fill(lens)
    assert s3.s3_kv_set_param(rig.a, "chunk", 4096) == s3.S3_ERR_INVALID  # 2048 is the largest chunk
    for chunk in (0, 128, 2048):
        assert s3.s3_kv_set_param(rig.a, "chunk", chunk) == 0
        q, got = rig.attend(lens)
        assert_close(got, rig.oracle_attend(q, lens), f"long contexts, chunk {chunk}")
    assert s3.s3_kv_set_param(rig.a, "chunk", 0) == 0
    keep = [1, 2, 3, 5]  # the ones with room for one more row
    ids = rig.ids[keep]
    pos = [lens[b] for b in keep]
    m = len(keep)
    q = wl.normal_bits(rig.rng, (m, H, D), dt)
    k = wl.normal_bits(rig.rng, (m, kvh, D), dt)
    v = wl.normal_bits(rig.rng, (m, kvh, D), dt)
    qd, kd, vd = (device_bits(x, TDT[dt], DEV) for x in (q, k, v))
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
            assert np.array_equal(rig_read(rig, sid, 0, which, pos[j] + 1), rig.o.rows(sid, 0, which, pos[j] + 1))
    want = rig.o.attention(0, ids.tolist(), [p + 1 for p in pos], q, None, "f32", threads=8)
    assert_close(out.cpu().numpy(), want, "decode step at the maximum length")
    # the full slot takes no further row
    full = torch.tensor([int(rig.offs[0])], dtype=torch.int64, device=DEV)
    assert s3.s3_decode_step(rig.a, 0, 1, full, torch.tensor([M], dtype=torch.int32, device=DEV), qd, kd, vd, out, s3.S3_F32,
                             0.0, len_out, rig.stream, slot_id=rig.ids[:1], pos_host=[M]) == s3.S3_ERR_SLOT_FULL
    rig.close()


@pytest.mark.parametrize("H,D", [(96, 128), (128, 256)])
def test_wide_rows(H, D):
    """Rows of 24 KiB (96 heads of 128, the largest model of table 1) and 64 KiB: many head groups per
    sequence, byte offsets beyond 32 bits inside the arena."""
    dt = s3.S3_F16
    lens = [0, 1, 100, 513, 64]
    rig = Rig(2, H, D, dt, 64, 1024, [max(1, L + 1) for L in lens], seed=93, arena_tokens=70000)
    assert 3 * rig.N * H * D * 2 > 2 ** 32  # the planes of layer 1 start beyond 4 GiB
    rig.fill(lens, layer=1)
    for chunk in (0, 96):
        assert s3.s3_kv_set_param(rig.a, "chunk", chunk) == 0
        q, got = rig.attend(lens, layer=1)
        assert_close(got, rig.oracle_attend(q, lens, layer=1), f"wide rows {H}x{D} chunk {chunk}")
    rig.close()


@pytest.mark.parametrize("Hkv", [None, 32])
def test_slot_whose_rows_lie_beyond_4_gib_of_its_plane(Hkv):
    """64 KiB rows (16 KiB with shared heads), slots that start more than 4 GiB into the plane: every row
    address needs more than 32 bits relative to the plane.  A doubling (whose copy also lands up there) and
    a decode step, for the multi-head and the matrix-core kernel."""
    H, D, dt = 128, 256, s3.S3_F16
    row_bytes = (Hkv or H) * D * 2
    filler = 2 ** 32 // row_bytes + 500
    M = 2 * 2 ** 32 // row_bytes
    rig = Rig(1, H, D, dt, 64, M, [filler, 100, 64], seed=95, arena_tokens=filler + 4000, Hkv=Hkv)  # slot 0 is only a filler
    assert int(rig.offs[1]) * row_bytes > 2 ** 32
    H_rows = Hkv or H
    ids, offs = rig.ids[1:], rig.offs[1:]
    lens = [100, 64]
    for sid, L in zip(ids.tolist(), lens):
        k = wl.normal_bits(rig.rng, (L, H_rows, D), dt)
        v = wl.normal_bits(rig.rng, (L, H_rows, D), dt)
        assert rig.o.fill(sid, 0, k, v) == 0
        assert s3.s3_kv_fill(rig.a, sid, 0, 0, L, device_bits(k, TDT[dt], DEV), device_bits(v, TDT[dt], DEV), rig.stream) == 0
    st, off2, cap2 = s3.s3_kv_grow(rig.a, int(ids[1]), 64, rig.stream)  # 64 -> 128 rows: lands behind the first one
    assert (st, off2, cap2) == rig.o.grow(int(ids[1]), 64) and off2 * row_bytes > 2 ** 32
    offs = np.array([int(offs[0]), off2], np.int64)
    n = 2
    q = wl.normal_bits(rig.rng, (n, H, D), dt)
    k, v = (wl.normal_bits(rig.rng, (n, H_rows, D), dt) for _ in range(2))
    qd, kd, vd = (device_bits(x, TDT[dt], DEV) for x in (q, k, v))
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
            assert np.array_equal(rig_read(rig, sid, 0, which, lens[j] + 1), rig.o.rows(sid, 0, which, lens[j] + 1))
    want = rig.o.attention(0, ids.tolist(), [L + 1 for L in lens], q, None, "f32", threads=8)
    assert_close(out.cpu().numpy(), want, "rows beyond 4 GiB")
    rig.close()


@pytest.mark.parametrize("H,Hkv,chunk", [(16, None, 0), (16, None, 64), (32, 8, 0)])
def test_decode_step_recorded_in_a_graph_replays_exactly(H, Hkv, chunk):
    """A decode step whose launches were recorded into a HIP graph (after one eager call, so that the
    library's scratch exists and nothing allocates during the recording) gives the eager result on every
    replay, with other work in between: the arrival counters of the chunk merge clean up after themselves."""
    D, dt = 128, s3.S3_BF16
    lens = [0, 1, 63, 200, 511, 700, 64, 5]
    rig = Rig(1, H, D, dt, 64, 1024, [L + 1 for L in lens], seed=97, Hkv=Hkv)
    rig.fill(lens)
    assert s3.s3_kv_set_param(rig.a, "chunk", chunk) == 0
    n, kvh = len(lens), Hkv or H
    q = device_bits(wl.normal_bits(rig.rng, (n, H, D), dt), TDT[dt], DEV)
    k, v = (device_bits(wl.normal_bits(rig.rng, (n, kvh, D), dt), TDT[dt], DEV) for _ in range(2))
    off_d = torch.tensor(rig.offs.tolist(), dtype=torch.int64, device=DEV)
    pos_d = torch.tensor(lens, dtype=torch.int32, device=DEV)
    len_out = torch.zeros(n, dtype=torch.int32, device=DEV)
    eager = torch.full((n, H, D), float("nan"), dtype=torch.float32, device=DEV)
    assert s3.s3_decode_step(rig.a, 0, n, off_d, pos_d, q, k, v, eager, s3.S3_F32, 0.0, len_out, rig.stream) == 0
    torch.cuda.synchronize()
    want = eager.clone()
    out = torch.full((n, H, D), float("nan"), dtype=torch.float32, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        st = s3.s3_decode_step(rig.a, 0, n, off_d, pos_d, q, k, v, out, s3.S3_F32, 0.0, len_out,
                               torch.cuda.current_stream().cuda_stream)
    assert st == 0
    for rep in range(4):
        out.fill_(float("nan"))
        len_out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want), f"replay {rep}"
        assert len_out.cpu().tolist() == [L + 1 for L in lens]
        # the program's own eager work between replays, on the same arena
        again = torch.full((n, H, D), float("nan"), dtype=torch.float32, device=DEV)
        assert s3.s3_decode_step(rig.a, 0, n, off_d, pos_d, q, k, v, again, s3.S3_F32, 0.0, len_out, rig.stream) == 0
        torch.cuda.synchronize()
        assert torch.equal(again, want)
    rig.close()


# ---------------------------------------------------------------- seeded random configurations
@pytest.mark.parametrize("seed", range(24))
def test_random_configuration_against_the_oracle(seed):
    """A seeded draw over everything a caller can choose inside the documented limits: head shape and
    sharing, types, batch size, ragged lengths (empty ones included), chunk size, kernel variant, length
    classes and grid size; attention through s3_decode_attention and a decode step after it."""
    rng = np.random.default_rng(1000 + seed)
    D = int(rng.choice([64, 128, 256]))
    dt = int(rng.choice([s3.S3_F16, s3.S3_BF16]))
    Hkv = int(rng.choice([1, 2, 3, 4, 8]))
    group = int(rng.choice([1, 1, 2, 4, 5, 8, 16]))
    H = Hkv * group
    n = int(rng.choice([1, 2, 7, 33, 64, 65, 130]))
    M = 1024
    lens = [int(x) for x in rng.choice([0, 1, 2, 15, 16, 17, 63, 64, 65, 200, 511, 700, 1023], n)]
    rig = Rig(1, H, D, dt, 64, M, [min(M, L + 1) for L in lens], seed=2000 + seed, Hkv=None if group == 1 else Hkv)
    rig.fill(lens)
    nv = n_variants(rig.a)
    for _ in range(2):
        assert s3.s3_kv_set_param(rig.a, "variant", int(rng.integers(-1, nv))) == 0
        assert s3.s3_kv_set_param(rig.a, "chunk", int(rng.choice([0, 32, 96, 256, 1024]))) == 0
        assert s3.s3_kv_set_param(rig.a, "classes", int(rng.integers(0, 9))) == 0
        assert s3.s3_kv_set_param(rig.a, "grid_blocks", int(rng.choice([0, 1, 3, 64, 300, 2048]))) == 0
        q, got = rig.attend(lens)
        assert_close(got, rig.oracle_attend(q, lens), f"random {seed}: H{H} Hkv{Hkv} D{D} n{n}")
        for b, L in enumerate(lens):
            if L == 0:
                assert not got[b].any()
    # one decode step on the sequences that still have room
    pos = [L for L in lens if L < M]
    keep = [b for b, L in enumerate(lens) if L < M]
    ids = rig.ids[keep]
    m = len(keep)
    kvh = Hkv if group > 1 else H
    q = wl.normal_bits(rig.rng, (m, H, D), dt)
    k = wl.normal_bits(rig.rng, (m, kvh, D), dt)
    v = wl.normal_bits(rig.rng, (m, kvh, D), dt)
    qd, kd, vd = (device_bits(x, TDT[dt], DEV) for x in (q, k, v))
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
            assert np.array_equal(rig_read(rig, sid, 0, which, pos[j] + 1), rig.o.rows(sid, 0, which, pos[j] + 1))
    want = rig.o.attention(0, ids.tolist(), [p + 1 for p in pos], q, None, "f32", threads=8)
    assert_close(out.cpu().numpy(), want, f"random {seed} step")
    rig.close()
