"""CPU-side checks of libs3kv.so: it loads, exports every declared symbol, and its host
bookkeeping (slot table, first fit, doubling) agrees bit for bit with the oracle on random
traces.  A metadata-only arena (no device memory) is used, so no GPU call is made."""
import os
import re

import numpy as np
import pytest

from oracle import kv_oracle as orc
from paper_2306_06000_amd import binding as s3
from paper_2306_06000_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def built():
    if not os.path.exists(s3.LIB_PATH):
        from paper_2306_06000_amd.build import build_lib

        build_lib()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "s3kv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(s3_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    names = declared_symbols()
    assert {"s3_kv_arena_init", "s3_kv_alloc", "s3_kv_append", "s3_decode_attention", "s3_kv_grow", "s3_kv_free",
            "s3_kv_stats"} <= set(names)
    lib = s3.lib()
    for n in names:
        assert hasattr(lib, n), n
        assert n in s3.SIGNATURES, n
    assert sorted(s3.SIGNATURES) == names


def meta_arena(n_layers, H, D, dtype, G, M, nbytes):
    cfg = s3.make_config(n_layers, H, D, dtype, G, M)
    st, a = s3.s3_kv_arena_init(cfg, None, nbytes)
    assert st == s3.S3_OK
    return cfg, a


def test_bytes_per_token_matches_the_paper_example():
    cfg = s3.make_config(44, 64, 64, s3.S3_F16, 64, 2048)  # hidden 4096: 4*44*4096
    assert s3.s3_kv_bytes_per_token(cfg) == 4 * 44 * 4096
    bad = s3.make_config(44, 64, 80, s3.S3_F16, 64, 2048)  # head_dim 80 is not supported by the kernels
    assert s3.s3_kv_bytes_per_token(bad) == s3.S3_ERR_INVALID
    gptj = s3.make_config(28, 16, 256, s3.S3_BF16, 64, 2048)
    assert s3.s3_kv_bytes_per_token(gptj) == 458752
    # shared key/value heads (multi-query attention, related work): only the cached heads count
    assert s3.s3_kv_bytes_per_token(s3.make_config(28, 16, 256, s3.S3_BF16, 64, 2048, 16)) == 458752
    assert s3.s3_kv_bytes_per_token(s3.make_config(28, 16, 256, s3.S3_BF16, 64, 2048, 4)) == 458752 // 4
    assert s3.s3_kv_bytes_per_token(s3.make_config(28, 16, 256, s3.S3_BF16, 64, 2048, 1)) == 458752 // 16


def test_worked_example_of_the_paper_through_the_library():
    """Sections 2.1 and 2.2: the 44-layer model with hidden size 6144 (64 heads x 96, table 1) holds
    4 * l * d_h bytes per token, a maximum-length reservation of 2048 tokens takes about 2.2 GB, and the
    memory that is left on a 40 GB card admits fewer than twenty of them (golden file)."""
    g = {}
    for line in open(os.path.join(ROOT, "tests", "golden", "kv_bytes_worked_example.txt")):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            g[k] = int(v)
    cfg = s3.make_config(g["n_layers"], 64, 96, s3.S3_F16, 64, g["max_len"])
    assert 64 * 96 == g["hidden"]
    assert s3.s3_kv_bytes_per_token(cfg) == g["bytes_per_token"] == 1081344
    assert s3.s3_kv_bytes_per_token(cfg) * g["max_len"] == g["bytes_per_max_reservation"]
    for key_bytes, key_batch in (("free_bytes_decimal", "max_batch_decimal"), ("free_bytes_binary", "max_batch_binary")):
        st, a = s3.s3_kv_arena_init(cfg, None, g[key_bytes])
        assert st == s3.S3_OK
        rc, ids, offs, caps = s3.s3_kv_alloc(a, [2048] * 25)
        assert rc == g[key_batch] < 20
        assert ids[:rc].tolist() == list(range(rc)) and (ids[rc:] == -1).all()
        assert offs[:rc].tolist() == [2048 * i for i in range(rc)]
        s3.s3_kv_arena_destroy(a)
        # the same memory holds many more 50-token sequences when each reserves what is predicted
        st, a = s3.s3_kv_arena_init(cfg, None, g[key_bytes])
        many, *_ = s3.s3_kv_alloc(a, [50] * 1000)
        assert many == min(1000, (g[key_bytes] // g["bytes_per_token"]) // 64) and many > 10 * rc
        s3.s3_kv_arena_destroy(a)
    # 96-wide heads are a multi-head 16-bit shape only
    assert s3.s3_kv_bytes_per_token(s3.make_config(1, 64, 96, s3.S3_F16, 64, 2048, 8)) == s3.S3_ERR_INVALID
    assert s3.s3_kv_bytes_per_token(s3.make_config(1, 64, 96, s3.S3_E4M3, 64, 2048, 0, s3.S3_F16)) == s3.S3_ERR_INVALID


def test_reservation_rules_equal_the_oracles():
    """Capacity for a prediction (sections 1, 2.3) and the doubled reservation (section 3, supervisor
    paragraph) as the library exports them, against the oracle's."""
    for G, M in ((64, 2048), (128, 2048), (64, 320), (32, 16384)):
        cfg = s3.make_config(1, 2, 64, s3.S3_F16, G, M)
        o = orc.KVOracle(1, 2, 64, orc.F16, G, M, 10**6, store=False)
        for p in list(range(0, 3 * G + 2)) + [M - 1, M, M + 1, 10**6, 2**31 - 1]:
            assert s3.s3_kv_capacity_for(cfg, p) == o.capacity_for(p), (G, M, p)
        for cap in range(0, M + G, G):
            assert s3.s3_kv_grown_capacity(cfg, cap) == o.grown_capacity(cap), (G, M, cap)
        assert s3.s3_kv_capacity_for(cfg, -1) == s3.S3_ERR_INVALID
        assert s3.s3_kv_grown_capacity(cfg, -1) == s3.S3_ERR_INVALID
    bad = s3.make_config(1, 2, 64, s3.S3_F16, 64, 100)
    assert s3.s3_kv_capacity_for(bad, 1) == s3.S3_ERR_INVALID and s3.s3_kv_grown_capacity(bad, 64) == s3.S3_ERR_INVALID


def test_config_validation():
    for bad in [(0, 16, 256, 0, 64, 2048), (1, 0, 256, 0, 64, 2048), (1, 16, 100, 0, 64, 2048),
                (1, 16, 256, 2, 64, 2048), (1, 16, 256, 0, 0, 2048), (1, 16, 256, 0, 64, 2000),
                (1, 16, 256, 0, 64, 2048, 3), (1, 16, 256, 0, 64, 2048, 32), (1, 16, 256, 0, 64, 2048, -1)]:
        st, a = s3.s3_kv_arena_init(s3.make_config(*bad), None, 1 << 20)
        assert st == s3.S3_ERR_INVALID and a is None


def test_status_strings():
    assert s3.lib().s3_status_str(0) == b"S3_OK"
    assert s3.lib().s3_status_str(-3) == b"S3_ERR_SLOT_FULL"
    assert s3.lib().s3_last_hip_error() == b""


def test_c0_slots_and_stats():
    w = wl.c0()
    cfg, a = meta_arena(w.n_layers, w.n_heads, w.head_dim, w.dtype, w.granule, w.max_len, 512 * w.bytes_per_token)
    rc, ids, offs, caps = s3.s3_kv_alloc(a, [s.predicted for s in w.seqs])
    assert rc == 4 and ids.tolist() == [0, 1, 2, 3]
    assert caps.tolist() == [64, 64, 128, 128] and offs.tolist() == [0, 64, 128, 256]
    assert s3.s3_kv_stats(a) == (0, 384, 128, 128, 512)
    assert s3.s3_kv_slot_info(a, 2) == (0, 128, 128)
    assert s3.s3_kv_slot_info(a, 9)[0] == s3.S3_ERR_INVALID
    s3.s3_kv_arena_destroy(a)


def test_errors_leave_state_unchanged():
    cfg, a = meta_arena(1, 1, 64, 0, 64, 256, 256 * 256)  # 256 tokens
    rc, ids, offs, caps = s3.s3_kv_alloc(a, [128, 64])
    assert rc == 2
    before = s3.s3_kv_stats(a)
    assert s3.s3_kv_alloc(a, [5, -1])[0] == s3.S3_ERR_INVALID
    assert s3.s3_kv_grow(a, 0, 128)[0] == s3.S3_ERR_NOMEM
    assert s3.s3_kv_grow(a, 0, 129)[0] == s3.S3_ERR_INVALID
    assert s3.s3_kv_grow(a, 5, 1)[0] == s3.S3_ERR_INVALID
    assert s3.s3_kv_free(a, 7) == s3.S3_ERR_INVALID
    assert s3.s3_kv_stats(a) == before
    rc, ids2, offs2, caps2 = s3.s3_kv_alloc(a, [64, 64, 64])  # only one more fits
    assert rc == 1 and ids2.tolist() == [2, -1, -1] and offs2.tolist() == [192, -1, -1] and caps2.tolist() == [64, 0, 0]
    assert s3.s3_kv_free(a, 0) == s3.S3_OK
    assert s3.s3_kv_grow(a, 1, 64) == (s3.S3_OK, 0, 128)
    assert s3.s3_kv_grow(a, 1, 10)[0] == s3.S3_ERR_NOMEM  # 256 needed, 64 free
    s3.s3_kv_arena_destroy(a)


def test_grow_to_max_len_then_maxlen_error():
    cfg, a = meta_arena(1, 1, 64, 0, 64, 320, 4096 * 256)
    rc, ids, offs, caps = s3.s3_kv_alloc(a, [192])
    assert s3.s3_kv_grow(a, 0, 192)[2] == 320  # min(2*192, M)
    assert s3.s3_kv_grow(a, 0, 0)[0] == s3.S3_ERR_MAXLEN
    # rows cannot be touched through a metadata-only arena
    assert s3.s3_kv_fill(a, 0, 0, 0, 1, 16, 16) == s3.S3_ERR_INVALID
    assert s3.s3_kv_append(a, 0, 1, 16, 16, 16, 16) == s3.S3_ERR_INVALID
    assert s3.s3_decode_attention(a, 0, 1, 16, 16, 16, 16) == s3.S3_ERR_INVALID
    s3.s3_kv_arena_destroy(a)


def test_set_param_validation():
    cfg, a = meta_arena(1, 1, 64, 0, 64, 256, 1 << 20)
    assert s3.s3_kv_set_param(a, "chunk", 128) == s3.S3_OK
    assert s3.s3_kv_get_param(a, "chunk") == (0, 128)
    assert s3.s3_kv_set_param(a, "chunk", 100) == s3.S3_ERR_INVALID
    assert s3.s3_kv_set_param(a, "nonsense", 1) == s3.S3_ERR_INVALID
    st, nv = s3.s3_kv_get_param(a, "n_variants")
    assert st == 0 and nv >= 1
    assert s3.s3_kv_set_param(a, "variant", nv) == s3.S3_ERR_INVALID
    assert s3.s3_kv_set_param(a, "variant", nv - 1) == s3.S3_OK
    s3.s3_kv_arena_destroy(a)


@pytest.mark.parametrize("seed,granule,tokens", [(0, 64, 64 * 300), (1, 128, 128 * 97), (2, 64, 64 * 41)])
def test_random_trace_bit_exact_against_oracle(seed, granule, tokens):
    rng = np.random.default_rng(100 + seed)
    M = 2048
    bpt = 2 * 1 * 1 * 64 * 2
    o = orc.KVOracle(1, 1, 64, orc.F16, granule, M, tokens * bpt + 17, store=False)
    cfg, a = meta_arena(1, 1, 64, 0, granule, M, tokens * bpt + 17)
    live = []
    for step in range(10000 if seed == 0 else 3000):
        r = rng.random()
        if r > 0.995:
            lens = [int(rng.integers(0, o.slots[sid][1] + 1)) for sid in live]
            st, new_off, moved = s3.s3_kv_compact(a, live, lens)
            want, want_moved = o.compact()
            assert st == 0 and moved == want_moved and new_off.tolist() == [want[sid] for sid in live]
        elif r < 0.45 or not live:
            k = int(rng.integers(1, 5))
            preds = [int(rng.integers(0, 2400)) if rng.random() < 0.5 else int(rng.integers(1, 300)) for _ in range(k)]
            n_o, ids_o, offs_o, caps_o = o.alloc(preds)
            rc, ids, offs, caps = s3.s3_kv_alloc(a, preds)
            assert rc == n_o and ids.tolist() == ids_o and offs.tolist() == offs_o and caps.tolist() == caps_o
            live += [i for i in ids_o if i >= 0]
        elif r < 0.75:
            sid = live.pop(int(rng.integers(len(live))))
            assert s3.s3_kv_free(a, sid) == o.free(sid) == 0
        else:
            sid = live[int(rng.integers(len(live)))]
            length = int(rng.integers(0, o.slots[sid][1] + 1))
            assert s3.s3_kv_grow(a, sid, length) == o.grow(sid, length)
        assert s3.s3_kv_stats(a) == (0, *o.stats())
        if step % 97 == 0:
            for sid in live:
                assert s3.s3_kv_slot_info(a, sid) == (0, *o.slots[sid])
    assert s3.s3_kv_get_param(a, "n_grows") == (0, o.n_grows)
    s3.s3_kv_arena_destroy(a)


def test_profile_percentiles_are_zero_without_timed_launches():
    cfg, a = meta_arena(1, 16, 256, s3.S3_F16, 64, 2048, 1 << 24)
    for q in (10, 50, 90):
        assert s3.s3_kv_get_param(a, f"profile_p{q}_ns") == (0, 0)
    assert s3.s3_kv_get_param(a, "profile_p75_ns")[0] == s3.S3_ERR_INVALID
    assert s3.s3_kv_get_param(a, "kernel_kind") == (0, 0)
    s3.s3_kv_arena_destroy(a)
    st, b = s3.s3_kv_arena_init(s3.make_config(1, 16, 256, s3.S3_F16, 64, 2048, 8), None, 1 << 24)
    assert st == 0 and s3.s3_kv_get_param(b, "kernel_kind") == (0, 1)   # two query heads per cached head
    assert s3.s3_kv_set_param(b, "variant", s3.s3_kv_get_param(b, "n_variants")[1] - 1) == 0
    assert s3.s3_kv_get_param(b, "kernel_kind") == (0, 2)               # the last index is the matrix-core kernel
    s3.s3_kv_arena_destroy(b)
    st, c = s3.s3_kv_arena_init(s3.make_config(1, 16, 256, s3.S3_F16, 64, 2048, 1), None, 1 << 24)
    assert st == 0 and s3.s3_kv_get_param(c, "kernel_kind") == (0, 2)
    s3.s3_kv_arena_destroy(c)


def test_8_bit_cache_config_on_the_host():
    """e4m3 rows (quantisation, related work): one byte per element, 16-bit activation type required,
    shared K/V heads shrink it further; the allocator works in tokens as before."""
    ok = s3.make_config(28, 16, 256, s3.S3_E4M3, 64, 2048, 0, s3.S3_BF16)
    assert s3.s3_kv_bytes_per_token(ok) == 458752 // 2
    for bad in (s3.make_config(1, 16, 256, s3.S3_E4M3, 64, 2048, 0, s3.S3_F32),
                s3.make_config(1, 16, 256, s3.S3_E4M3, 64, 2048, 0, s3.S3_E4M3),
                s3.make_config(1, 16, 256, s3.S3_E4M3, 64, 2048, 5, s3.S3_F16),
                s3.make_config(1, 16, 256, 4, 64, 2048)):
        assert s3.s3_kv_bytes_per_token(bad) == s3.S3_ERR_INVALID
        assert s3.s3_kv_arena_init(bad, None, 1 << 20)[0] == s3.S3_ERR_INVALID
    st, a = s3.s3_kv_arena_init(ok, None, 100 * 229376)
    assert st == 0 and s3.s3_kv_stats(a)[4] == 100
    assert s3.s3_kv_get_param(a, "kernel_kind") == (0, 3)
    both = s3.make_config(28, 16, 256, s3.S3_E4M3, 64, 2048, 4, s3.S3_F16)  # 8-bit rows of 4 cached heads
    assert s3.s3_kv_bytes_per_token(both) == 458752 // 8
    st, b = s3.s3_kv_arena_init(both, None, 1 << 24)
    assert st == 0 and s3.s3_kv_get_param(b, "kernel_kind") == (0, 4) and s3.s3_kv_get_param(b, "n_variants") == (0, 1)
    s3.s3_kv_arena_destroy(b)
    o = orc.KVOracle(28, 16, 256, orc.E4M3, 64, 2048, 100 * 229376, store=False, act_dtype=orc.BF16)
    rc, ids, offs, caps = s3.s3_kv_alloc(a, [10, 65, 3000])
    assert (rc, ids.tolist(), offs.tolist(), caps.tolist()) == o.alloc([10, 65, 3000])
    s3.s3_kv_arena_destroy(a)


def test_compact_validation():
    cfg, a = meta_arena(1, 1, 64, 0, 64, 256, 1024 * 256)
    rc, ids, offs, caps = s3.s3_kv_alloc(a, [64, 64, 128])
    assert s3.s3_kv_free(a, 0) == 0
    before = s3.s3_kv_stats(a)
    assert s3.s3_kv_compact(a, [1, 7], [1, 1])[0] == s3.S3_ERR_INVALID
    assert s3.s3_kv_compact(a, [1], [65])[0] == s3.S3_ERR_INVALID
    assert s3.s3_kv_stats(a) == before and s3.s3_kv_slot_info(a, 1) == (0, 64, 64)
    st, new_off, moved = s3.s3_kv_compact(a, [2], [100])
    assert (st, new_off.tolist(), moved) == (0, [64], 2)
    assert s3.s3_kv_slot_info(a, 1) == (0, 0, 64) and s3.s3_kv_stats(a) == (0, 192, 832, 832, 1024)
    s3.s3_kv_arena_destroy(a)


def test_write_through_partials_carry_the_cache_bits_the_in_kernel_merge_relies_on(tmp_path):
    """Chunks of one context that meet inside one launch exchange their partial sums through memory between
    workgroups on different XCDs (each with its own L2).  The default ordering relies on `volatile` vector
    stores and loads being emitted as write-through / cache-bypassing accesses on gfx950 (cache bits sc0 sc1)
    and on the fence-based ordering emitting an L2 write-back before and an invalidate after the counter.
    This compiles the library's own helpers and reads the bits off the emitted code, so that a compiler
    change shows up here and not as a rare wrong merge."""
    import shutil
    import subprocess

    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc here")
    src = tmp_path / "probe.hip"
    src.write_text('''
#include <hip/hip_runtime.h>
#include "s3kv_device.h"
__global__ void probe_put(float *p, float x) {
    put_partial4<true>(p + 4 * threadIdx.x, (f32x4){x, x, x, x});
    put_partial2<true>(p + 4096 + 2 * threadIdx.x, (f32x2){x, x});
}
__global__ void probe_get(const float *p, float *out) {
    const f32x4 a = get_partial4<true>(p + 4 * threadIdx.x);
    const f32x2 b = get_partial2<true>(p + 4096 + 2 * threadIdx.x);
    out[threadIdx.x] = a[0] + a[1] + a[2] + a[3] + b[0] + b[1];
}
__global__ void probe_plain(float *p, float x) { put_partial4<false>(p + 4 * threadIdx.x, (f32x4){x, x, x, x}); }
__global__ void probe_arrive(AttnArgs a, unsigned int *cnt, int *flag) {
    if (chunk_arrived(a, cnt, 2)) flag[threadIdx.x] = 1;
}
''')
    csrc = os.path.join(ROOT, "paper_2306_06000_amd", "csrc")
    asm = tmp_path / "probe.s"
    subprocess.run([hipcc, "-O3", "-std=c++17", "--offload-arch=gfx950", "--cuda-device-only", "-S", "-I", csrc, "-I",
                    os.path.join(ROOT, "include"), "-x", "hip", str(src), "-o", str(asm)], check=True,
                   stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    text = asm.read_text()

    def body(kernel):
        m = re.search(r"^_Z\d+" + kernel + r"\w*:[^\n]*\n(.*?)s_endpgm", text, flags=re.S | re.M)
        assert m, kernel
        return m.group(1)

    put = body("probe_put")
    assert re.search(r"(global|flat)_store_dwordx4 .*\bsc0\b.*\bsc1\b", put), put
    assert re.search(r"(global|flat)_store_dwordx2 .*\bsc0\b.*\bsc1\b", put), put
    get = body("probe_get")
    assert re.search(r"(global|flat)_load_dwordx4 .*\bsc0\b.*\bsc1\b", get), get
    assert re.search(r"(global|flat)_load_dwordx2 .*\bsc0\b.*\bsc1\b", get), get
    plain = body("probe_plain")
    assert "_store_dwordx4" in plain and "sc0" not in plain  # the bits come from `volatile`, not from every store
    arrive = body("probe_arrive")
    # both orderings are in the code (merge_sync picks one at run time): the fenced one writes the L2 back before
    # the count and invalidates after it; the default drains the wave's memory counter before the count
    assert "buffer_wbl2" in arrive and "buffer_inv" in arrive and "global_atomic_add" in arrive
    assert re.search(r"s_waitcnt vmcnt\(0\).*global_atomic_add", arrive, flags=re.S)


def test_calls_that_touch_rows_refuse_a_metadata_only_arena_without_any_device_call():
    """The entry points added beside the core path make no HIP call before their argument checks: on an arena
    without device memory they answer S3_ERR_INVALID (this runs where no GPU exists)."""
    cfg, a = meta_arena(2, 4, 128, s3.S3_BF16, 64, 512, 1 << 24)
    rc, ids, offs, caps = s3.s3_kv_alloc(a, [100])
    assert rc == 1
    sid = int(ids[0])
    fake = 1 << 20  # an aligned address that is never dereferenced
    assert s3.s3_kv_gather_rows(a, sid, 10, fake) == s3.S3_ERR_INVALID
    assert s3.s3_kv_scatter_rows(a, sid, 10, fake) == s3.S3_ERR_INVALID
    assert s3.s3_kv_reserve_scratch(a, 64) == s3.S3_ERR_INVALID
    assert s3.s3_decode_step_static(a, 0, 1, fake, fake, fake, fake, fake, fake) == s3.S3_ERR_INVALID
    assert s3.s3_decode_step(a, 0, 1, fake, fake, fake, fake, fake, fake) == s3.S3_ERR_INVALID
    # the link copy checks sizes, alignment and the grid before it launches anything
    assert s3.s3_kv_link_copy(fake, fake + 4096, 0, 8) == s3.S3_OK  # nothing to copy
    assert s3.s3_kv_link_copy(fake, fake + 4096, 24, 8) == s3.S3_ERR_INVALID
    assert s3.s3_kv_link_copy(fake + 8, fake + 4096, 32, 8) == s3.S3_ERR_INVALID
    assert s3.s3_kv_link_copy(fake, fake + 4096, 32, 0) == s3.S3_ERR_INVALID
    assert s3.s3_kv_link_copy(fake, fake + 4096, 32, 1025) == s3.S3_ERR_INVALID
    assert s3.s3_kv_link_copy(None, fake, 32, 8) == s3.S3_ERR_INVALID
    # parameters of the new knobs
    assert s3.s3_kv_set_param(a, "merge_sync", 1) == s3.S3_OK and s3.s3_kv_get_param(a, "merge_sync") == (0, 1)
    assert s3.s3_kv_set_param(a, "merge_sync", 2) == s3.S3_ERR_INVALID
    st, dv = s3.s3_kv_get_param(a, "default_variant")
    st2, nv = s3.s3_kv_get_param(a, "n_variants")
    assert st == 0 and st2 == 0 and 0 <= dv < nv
    assert s3.lib().s3_status_str(s3.S3_ERR_SCRATCH) == b"S3_ERR_SCRATCH"
    s3.s3_kv_arena_destroy(a)


def test_committed_counter_summaries_carry_same_run_traffic_and_algorithmic_bytes():
    """bench.py prints `roofline.traffic` from the committed rocprofv3 counter summary of each target workload
    together with THAT run's own algorithmic bytes: both must be present, and every cached byte is read once
    (traffic within a few per cent of the algorithmic bytes)."""
    import bench

    for wl_name in ("c1", "c2", "c3", "c4"):
        traffic, algorithmic = bench.read_traffic("attn_step_kernel", wl_name)
        assert traffic and algorithmic, wl_name
        assert 0.97 <= traffic / algorithmic <= 1.03, (wl_name, traffic, algorithmic)
    assert bench.read_traffic("attn_step_kernel", "c9") == (None, None)
