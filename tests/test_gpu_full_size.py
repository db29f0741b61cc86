"""GPU parity at the full sizes of the workloads the benchmark times (C2, C3, C4), in the launch
configuration the benchmark uses (library defaults, one s3_decode_step per layer): every integer the
library returns against the oracle, stored rows bit-exact and attention within tolerance on sampled
steps / sequences / layers that the oracle can compute one by one."""
import os

import numpy as np
import pytest

from oracle import kv_oracle as orc
from paper_2306_06000_amd import binding as s3
from paper_2306_06000_amd import workloads as wl
from tests.harness import OracleReplay, assert_close, device_bits, make_sources

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module", autouse=True)
def need_gpu_and_lib():
    assert torch.cuda.is_available() and os.path.exists(s3.LIB_PATH)
    s3.lib()


def full_trace(w, steps, attend_steps, sample_rows):
    from paper_2306_06000_amd.engine import DecodeEngine

    src = wl.PooledSource(w, len(w.seqs))
    eng = DecodeEngine(w)
    prefill, tensors_for = make_sources(w, eng, src)
    eng.start(prefill)
    got = {}
    for t in range(steps):
        out = eng.step(tensors_for(t), prefill, check_host=(t % 16 == 0))
        if t in attend_steps:
            got[t] = out.float().cpu().numpy()
    rep = OracleReplay(w, eng.arena_tokens, src)
    outs = rep.replay(eng.events, attend_steps=set(attend_steps))
    for t in attend_steps:
        assert_close(got[t], outs[t][2], f"{w.name} step {t}")
    live = eng.active
    for a in live[:: max(1, len(live) // sample_rows)]:
        sid = rep.sid[a.serial]
        assert sid == a.slot and rep.o.slots[sid] == [a.off, a.cap] and rep.len[a.serial] == a.len
        for which in (0, 1):
            assert np.array_equal(eng.read_slot(a, 0, which), rep.o.rows(sid, 0, which, a.len))
    assert s3.s3_kv_stats(eng.arena) == (0, *rep.o.stats())
    grows = s3.s3_kv_get_param(eng.arena, "n_grows")[1]
    assert grows == rep.o.n_grows
    frees = sum(e[0] == "free" for e in eng.events)
    eng.close()
    return grows, frees


def test_c2_full_batch_512_256_steps():
    w = wl.c2()
    grows, frees = full_trace(w, w.steps, attend_steps=[0, 100, 255], sample_rows=24)
    assert grows >= 20 and frees >= 200  # the under-predicted tenth outgrows its slots; many sequences finish


def test_c4_full_batch_128_long_contexts_64_steps():
    w = wl.c4()
    full_trace(w, 63, attend_steps=[0, 31, 62], sample_rows=12)


def test_c3_full_200GB_arena_28_layers_sampled():
    from paper_2306_06000_amd.engine import DecodeEngine

    w = wl.c3()
    src = wl.PooledSource(w, 1024)
    eng = DecodeEngine(w)
    assert eng.arena_mem.numel() >= 199 * 10**9
    tdt = eng.kv_dtype_torch()
    dev_rows = device_bits(src.rows, tdt, eng.dev)

    def prefill(serial, layer, rows):  # windows of the pool already resident on the device
        start = (serial * 37 + layer * 11) % 128
        return dev_rows[0, start:start + rows], dev_rows[1, start:start + rows]

    eng.start(prefill, stop_when_full=True)
    n = eng.n_active
    assert 600 <= n <= 1024
    # integers: the same admissions on the oracle (no storage)
    o = orc.KVOracle(w.n_layers, w.n_heads, w.head_dim, w.dtype, w.granule, w.max_len,
                     eng.arena_tokens * w.bytes_per_token, store=False)
    for ev in eng.events:
        if ev[0] == "alloc":
            assert o.alloc_one(ev[2]) == (ev[3], ev[4], ev[5])
    assert s3.s3_kv_stats(eng.arena) == (0, *o.stats())
    assert o.stats()[0] * w.bytes_per_token > 0.97 * w.arena_bytes  # the arena is full

    # one decode step over all 28 layers, the outputs of three layers kept
    eng._sync_arrays()
    st = torch.cuda.current_stream().cuda_stream
    layers = [0, 13, 27]
    outs, ins = {}, {}
    for layer in range(w.n_layers):
        q, k, v = src.step_tensors(0, layer, n)
        qd, kd, vd = (device_bits(x, tdt, eng.dev) for x in (q, k, v))
        out = torch.full((n, w.n_heads, w.head_dim), float("nan"), dtype=torch.float32, device=eng.dev)
        assert s3.s3_decode_step(eng.arena, layer, n, eng.slot_off_dev, eng.len_dev, qd, kd, vd, out, s3.S3_F32, 0.0,
                                 eng.len_next, st) == 0
        if layer in layers:
            outs[layer], ins[layer] = out, (q, k, v)
    torch.cuda.synchronize()
    assert (eng.len_next.cpu().numpy() == eng.len + 1).all()
    acts = eng.active
    order = np.argsort(eng.len)
    sample = sorted({0, n - 1, int(order[0]), int(order[-1]), int(order[n // 2]), n // 3})
    for layer in layers:
        q, k, v = ins[layer]
        got = outs[layer].cpu().numpy()
        assert np.isfinite(got).all()
        Ks, Vs, lens = [], [], []
        for b in sample:
            a = acts[b]
            pk, pv = src.prefill_rows(a.serial, layer, a.len)
            Ks.append(np.concatenate([pk, k[b:b + 1]]))
            Vs.append(np.concatenate([pv, v[b:b + 1]]))
            lens.append(a.len + 1)
        want, _ = orc.attention_ragged(q[sample], Ks, Vs, lens, w.dtype, None, "f32", threads=8)
        assert_close(got[sample], want, f"C3 layer {layer}")
        for j, b in enumerate(sample[:3]):  # stored rows, the appended one included
            a = acts[b]
            for which, ref in ((0, Ks[j]), (1, Vs[j])):
                assert np.array_equal(eng.read_slot(a, layer, which, a.len + 1), ref)
    eng.close()


def test_c5_shared_heads_at_the_benchmarked_batch():
    """C5 as bench.py times it (batch 256, 32 query / 8 cached heads, matrix-core kernel by default)."""
    w = wl.c5()
    assert w.batch == 256
    grows, frees = full_trace(w, 64, attend_steps=[0, 33, 63], sample_rows=16)
    assert frees >= 10


def test_c6_8_bit_rows_at_the_benchmarked_batch():
    """C6 as bench.py times it (batch 128, e4m3 rows, fp16 queries)."""
    w = wl.c6()
    assert w.batch == 128
    grows, frees = full_trace(w, 64, attend_steps=[0, 33, 63], sample_rows=16)
    assert frees >= 5
