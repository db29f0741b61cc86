"""Shared test plumbing: feed the same seeded inputs to the HIP engine and to the CPU oracle,
replay the engine's event log on the oracle, and compare."""
import numpy as np

from oracle import kv_oracle as orc
from paper_2306_06000_amd import workloads as wl

MAX_ABS, REL_L2 = 2e-3, 1e-3  # attention tolerance against the fp32 oracle (fp16 / bf16 storage)


def assert_close(got, want, what=""):
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    max_abs = np.abs(got - want).max() if got.size else 0.0
    denom = np.linalg.norm(want.ravel())
    rel = np.linalg.norm((got - want).ravel()) / denom if denom > 0 else np.linalg.norm(got.ravel())
    assert max_abs <= MAX_ABS and rel <= REL_L2, f"{what}: max-abs {max_abs:.3e} rel-L2 {rel:.3e}"
    return max_abs, rel


def device_bits(bits, torch_dtype, device):
    """uint16 patterns (numpy) -> device tensor of the 16-bit float type, bit-preserving; uint8 codes
    (8-bit cache rows) go up as they are."""
    import torch

    bits = np.ascontiguousarray(bits)
    if bits.dtype == np.uint8:
        return torch.from_numpy(bits).to(device)
    return torch.from_numpy(bits.view(np.int16)).to(device).view(torch_dtype)


def make_sources(w, engine, source=None):
    """prefill(serial, layer, rows) and tensors_for(step) closures that upload the seeded inputs.
    source: a workloads.PooledSource for full-size runs (default: fresh draws per call)."""
    tdt, adt = engine.kv_dtype_torch(), engine.act_dtype_torch()
    get_rows = source.prefill_rows if source else (lambda serial, layer, rows: wl.prefill_rows(w, serial, layer, rows))
    get_step = source.step_tensors if source else (lambda step, layer, n: wl.step_tensors(w, step, layer, n))

    def prefill(serial, layer, rows):
        k, v = get_rows(serial, layer, rows)
        return device_bits(k, tdt, engine.dev), device_bits(v, tdt, engine.dev)

    def tensors_for(step):
        def tensors(layer, n):
            q, k, v = get_step(step, layer, n)
            return tuple(device_bits(x, adt, engine.dev) for x in (q, k, v))

        return tensors

    return prefill, tensors_for


class OracleReplay:
    """Replays an engine event log on the CPU oracle; every integer the library returned must
    equal the oracle's.  Keeps serial -> oracle id so that rows can be compared afterwards."""

    def __init__(self, w, arena_tokens, source=None):
        self.w = w
        self.get_rows = source.prefill_rows if source else (lambda serial, layer, rows: wl.prefill_rows(w, serial, layer, rows))
        self.get_step = source.step_tensors if source else (lambda step, layer, n: wl.step_tensors(w, step, layer, n))
        self.o = orc.KVOracle(w.n_layers, w.n_heads, w.head_dim, w.dtype, w.granule, w.max_len,
                              arena_tokens * w.bytes_per_token, n_kv_heads=w.n_kv_heads,
                              act_dtype=None if w.act_dtype < 0 else w.act_dtype)
        self.sid = {}   # serial -> slot id
        self.len = {}   # serial -> rows cached
        self.blobs = {} # serial -> rows of a sequence that is on the host
        self.sched = None
        self.step_idx = 0

    def replay(self, events, attend_steps=(), threads=8, precision="f32"):
        """Returns {step index: (serials, lens, oracle attention output of the last layer)}."""
        w, o = self.w, self.o
        outs = {}
        for ev in events:
            kind = ev[0]
            if kind == "alloc":
                _, serial, pred, sid, off, cap = ev
                got = o.alloc_one(pred)
                assert got == (sid, off, cap), ("alloc", serial, got, (sid, off, cap))
                if sid >= 0:
                    self.sid[serial] = sid
            elif kind == "fill":
                _, serial, sid, rows = ev
                for layer in range(w.n_layers):
                    k, v = self.get_rows(serial, layer, rows)
                    assert o.fill(sid, layer, k, v) == orc.OK
                self.len[serial] = rows
            elif kind == "grow":
                _, serial, sid, length, st, off, cap = ev
                assert length == self.len[serial] == o.slots[sid][1]  # grown exactly when full
                got = o.grow(sid, length)
                assert got == (st, off, cap), ("grow", serial, got, (st, off, cap))
            elif kind == "sched_admit":
                _, max_out, serials, rids, sids, offs, caps = ev
                if self.sched is None:  # every request waits in the scheduler from the start
                    self.sched = orc.SchedulerOracle(o)
                    for rid, r in enumerate(list(w.seqs) + list(w.pool)):
                        self.sched.submit(rid, r.predicted)
                got = self.sched.admit(max_out)
                assert got == list(zip(rids, sids, offs, caps)), ("sched_admit", got, ev)
                for serial, sid in zip(serials, sids):
                    self.sid[serial] = sid
            elif kind == "compact":
                _, ids, new_off, moved = ev
                offs, want_moved = o.compact()
                assert [offs[i] for i in ids] == new_off and moved == want_moved, ("compact", moved, want_moved)
            elif kind == "evict":
                _, serial, sid, length = ev
                assert self.sid.pop(serial) == sid and length == self.len[serial]
                st, blob = o.evict(sid, length)
                assert st == orc.OK
                self.blobs[serial] = blob
            elif kind == "restore":
                _, serial, want, length, st, sid, off, cap = ev
                assert length == self.len[serial]
                got = o.restore(want, self.blobs[serial])
                assert got == (st, sid, off, cap), ("restore", serial, got, (st, sid, off, cap))
                if st == orc.OK:
                    self.sid[serial] = sid
                    del self.blobs[serial]
            elif kind == "free":
                _, serial, sid = ev
                assert self.sid.pop(serial) == sid
                assert o.free(sid) == orc.OK
                self.len.pop(serial)
            elif kind == "step":
                _, serials, lens = ev
                n = len(serials)
                t = self.step_idx
                last = None
                for layer in range(w.n_layers):
                    q, k, v = self.get_step(t, layer, n)
                    for b, serial in enumerate(serials):
                        assert o.append(self.sid[serial], layer, self.len[serial], k[b], v[b]) == orc.OK
                    if t in attend_steps and layer == w.n_layers - 1:
                        ids = [self.sid[s] for s in serials]
                        last = o.attention(layer, ids, lens, q, None, precision, threads)
                for b, serial in enumerate(serials):
                    self.len[serial] += 1
                    assert self.len[serial] == lens[b]
                if last is not None:
                    outs[t] = (list(serials), list(lens), last)
                self.step_idx += 1
            else:
                raise AssertionError(kind)
        return outs
