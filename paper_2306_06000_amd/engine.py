"""Decode-loop plumbing over the C ABI: owns the arena tensor and the per-batch device arrays,
decides WHEN to call alloc / fill / grow / free / append / attention for a synthetic workload,
and records what the library answered.  It computes nothing of the method itself.

Per decode step (iteration-level scheduling, section 3 of the S3 paper):
  1. every active sequence whose slot is full and which is not finished is grown (doubling);
  2. the new token's K/V row is appended at row len, len += 1;
  3. attention over the len rows now cached (append-then-attend: the new token attends to itself);
  4. sequences that reached their true total length are freed; with refill on, the next
     candidate of the pool is admitted into the freed room and its prompt rows are written.
When a reservation cannot be doubled because no extent is large enough (supervisor paragraph of
section 3): if the free space is merely fragmented the arena is compacted and the doubling repeated;
otherwise the sequence's rows go to pinned host memory, its slot is freed, and it comes back with the
doubled reservation as soon as a finished sequence has made room (before any newcomer).  The host link never
sits on the decode stream: an eviction gathers the rows into a device staging buffer with one kernel on the
decode stream (the slot is free right behind it), the buffer crosses to the host in one copy on a side stream;
a re-admission reserves its slot at once, brings the rows into a staging buffer on the side stream, and the
sequence joins the batch at the first step that finds that copy complete (one scatter kernel).
The event log lets a test replay the same decisions on the CPU oracle and compare every id,
offset and capacity bit for bit.  Host-side state is kept in numpy arrays so that a step costs
a few vector operations however large the batch is.
"""
from types import SimpleNamespace

import numpy as np
import torch

from . import binding as s3

_TORCH_DT = {s3.S3_F16: torch.float16, s3.S3_BF16: torch.bfloat16, s3.S3_F32: torch.float32}


class DecodeEngine:
    COMPACT_RATIO = 48  # live tokens per token of the wanted slot up to which compaction is preferred to a swap

    def __init__(self, w, arena_tokens=None, device="cuda:0", out_dtype=s3.S3_F32, log_events=True, fused=True,
                 on_nomem="swap", admission="fifo"):
        self.w = w
        # "fifo": candidates in pool order, each admitted iff it fits; "dff": the library's scheduler picks
        # them, largest reservation first, from everything that waits (section 3, scheduler paragraph)
        self.admission = admission
        self.sched = None
        self.fused = fused  # True: one s3_decode_step launch per layer; False: append + attention calls
        # "swap": compact, else evict to the host and re-admit later (the paper's supervisor); "drop": free
        self.on_nomem = on_nomem
        self.swapped = []     # evicted sequences waiting for room, oldest first
        self._restoring = []  # re-admitted sequences whose rows are still on their way back, oldest first
        self._host_free = []  # pinned buffers ready for reuse
        self._stage = []      # [event or None, device staging buffer, held]: free once the event has passed and no
                              # returning sequence holds it
        self._side = None     # stream on which evicted rows cross the host link, beside the decode steps
        self.n_swapped_out = self.n_swapped_in = self.n_compactions = 0
        self.capacity = 0     # entries the device arrays can hold (the largest batch so far)
        self.dev = torch.device(device)
        self.cfg = s3.make_config(w.n_layers, w.n_heads, w.head_dim, w.dtype, w.granule, w.max_len, w.n_kv_heads, max(w.act_dtype, 0))
        self.bpt = s3.s3_kv_bytes_per_token(self.cfg)
        if arena_tokens is None:
            if w.arena_bytes:
                arena_tokens = w.arena_bytes // self.bpt
            else:
                caps = [s3.s3_kv_capacity_for(self.cfg, s.predicted) for s in w.seqs]
                arena_tokens = int(1.5 * sum(caps)) + 2 * w.max_len
        self.arena_tokens = int(arena_tokens)
        self.arena_mem = torch.empty(self.arena_tokens * self.bpt, dtype=torch.uint8, device=self.dev)
        st, self.arena = s3.s3_kv_arena_init(self.cfg, self.arena_mem, self.arena_mem.numel())
        s3.check(st, "s3_kv_arena_init")
        if admission == "dff":
            st, self.sched = s3.s3_sched_create(self.arena)
            s3.check(st, "s3_sched_create")
            self._requests = list(w.seqs) + list(w.pool)  # request id = position in this list
            for rid, r in enumerate(self._requests):
                s3.check(s3.s3_sched_submit(self.sched, rid, r.predicted), "s3_sched_submit")
        if on_nomem == "swap":  # pinning is slow: six buffers of a quarter of the longest sequence are pinned up front
            self._side = torch.cuda.Stream(self.dev)
            quarter = max(w.granule, w.max_len // 4) * self.bpt
            self._host_free = [torch.empty(quarter, dtype=torch.uint8, pin_memory=True) for _ in range(6)]
            # and two that hold the longest sequence: pinning memory in the middle of a run maps it into the
            # device's address space, which stalls the kernels that are running
            self._host_free += [torch.empty(w.max_len * self.bpt, dtype=torch.uint8, pin_memory=True) for _ in range(2)]
            # device staging: four buffers that hold the longest sequence (allocating one mid-run would synchronise)
            self._stage = [[None, torch.empty(w.max_len * self.bpt, dtype=torch.uint8, device=self.dev), False]
                           for _ in range(4)]
        self.out_dtype = out_dtype
        self._row_term, self._seq_term = self._byte_terms()  # bytes per cached row and per sequence of one layer-step
        self.events = [] if log_events else None
        self.next_serial = 0
        self.pool_pos = 0
        self.n_evicted = 0
        self.n_grown = 0
        self.n_retired = 0
        # per active sequence, batch order
        self.serial = np.zeros(0, np.int64)
        self.slot = np.zeros(0, np.int32)
        self.off = np.zeros(0, np.int64)
        self.cap = np.zeros(0, np.int32)
        self.len = np.zeros(0, np.int32)
        self.total = np.zeros(0, np.int32)
        self.slot_off_dev = None
        self.len_dev = None
        self.len_next = None
        self._dirty = True   # the device arrays must be rebuilt (batch membership or order changed)
        self._patch = set()  # entries whose offset / length changed in place
        self.out = None
        self._out_n = -1     # batch size self.out was cut for
        # steps until some sequence fills its slot / reaches its total length (the per-step checks run only
        # then), and the rows the batch holds; refreshed by _recount() whenever membership or lengths change
        self._to_full = self._to_done = 0
        self._rows = 0

    # -- helpers ----------------------------------------------------------
    def close(self):
        if self.arena is not None:
            torch.cuda.synchronize(self.dev)
            self._restoring.clear()
            if self.sched is not None:
                s3.s3_sched_destroy(self.sched)
                self.sched = None
            s3.s3_kv_arena_destroy(self.arena)
            self.arena = None

    def _log(self, *ev):
        if self.events is not None:
            self.events.append(ev)

    def _stream_ptr(self):
        return torch.cuda.current_stream(self.dev).cuda_stream

    LINK_WORKGROUPS = 2  # workgroups (one compute unit each) of a copy over the host link: about 30 GB/s, and few
                         # enough writes queued for the link at once that the decode steps beside it run at full speed
    MAX_RETURNING = 2  # sequences on their way back at once; each holds a staging buffer until it has joined

    def _stage_buffer(self, block=True):
        """A device staging buffer that no returning sequence holds and whose last use has completed (if all
        that are not held are busy: blocks on one, or returns None; at least two never are held)."""
        idle = [e for e in self._stage if not e[2]]
        for entry in idle:
            if entry[0] is None or entry[0].query():
                entry[0] = None
                return entry
        if not block:
            return None
        entry = idle[0]
        entry[0].synchronize()
        entry[0] = None
        return entry

    def kv_dtype_torch(self):
        """torch type of cache rows handed to fill (8-bit caches: raw codes)."""
        return torch.uint8 if self.w.dtype == s3.S3_E4M3 else _TORCH_DT[self.w.dtype]

    def act_dtype_torch(self):
        """torch type of q, k_new, v_new."""
        return _TORCH_DT[self.w.q_dtype]

    @property
    def n_active(self):
        return int(self.slot.size)

    @property
    def active(self):
        """Read-only view of the batch as records (for tests and reports)."""
        return [SimpleNamespace(serial=int(self.serial[i]), slot=int(self.slot[i]), off=int(self.off[i]),
                                cap=int(self.cap[i]), len=int(self.len[i]), total=int(self.total[i]))
                for i in range(self.n_active)]

    def _pinned(self, arr):
        # torch's pinned-memory allocator does not reuse a block before the copy that reads it has
        # completed, so the staging tensor needs no lifetime management here
        return torch.from_numpy(arr.copy()).pin_memory()

    def _sync_arrays(self):
        if not self._dirty and self._patch:
            idx = np.fromiter(self._patch, np.int32)
            s3.check(s3.s3_kv_batch_patch(self.n_active, self.slot_off_dev, self.len_dev, idx, self.off[idx],
                                          self.len[idx], self._stream_ptr()), "s3_kv_batch_patch")
        self._patch.clear()
        n = self.n_active
        if self._dirty:  # a new batch (or every offset changed): upload; a batch that shrinks later uses a prefix
            if n > self.capacity or self.slot_off_dev is None:
                self.capacity = max(n, self.capacity)
                self.slot_off_dev = torch.empty(self.capacity, dtype=torch.int64, device=self.dev)
                self.len_dev = torch.empty(self.capacity, dtype=torch.int32, device=self.dev)
                self.len_next = torch.empty_like(self.len_dev)
                self.out_full = torch.empty((self.capacity, self.w.n_heads, self.w.head_dim),
                                            dtype=_TORCH_DT[self.out_dtype], device=self.dev)
                self._out_n = -1
                # the library's scratch is sized here, once per batch capacity, so that no decode step allocates
                s3.check(s3.s3_kv_reserve_scratch(self.arena, self.capacity), "s3_kv_reserve_scratch")
            self.slot_off_dev[:n].copy_(self._pinned(self.off), non_blocking=True)
            self.len_dev[:n].copy_(self._pinned(self.len), non_blocking=True)
            self._dirty = False
            self._out_n = -1
        if n != self._out_n:
            self.out = self.out_full[:n]
            self._out_n = n

    def _recount(self):
        n = self.n_active
        if n:
            self._to_full = int((self.cap - self.len).min())
            self._to_done = int((self.total - self.len).min())
            self._rows = int(self.len.sum())
        else:
            self._to_full = self._to_done = 1 << 30
            self._rows = 0

    def _set_batch(self, recs):
        self.serial = np.array([r[0] for r in recs], np.int64)
        self.slot = np.array([r[1] for r in recs], np.int32)
        self.off = np.array([r[2] for r in recs], np.int64)
        self.cap = np.array([r[3] for r in recs], np.int32)
        self.len = np.array([r[4] for r in recs], np.int32)
        self.total = np.array([r[5] for r in recs], np.int32)
        self._dirty = True
        self._recount()

    # -- admission --------------------------------------------------------
    def admit(self, seqs, prefill, fill=True):
        """Reserve slots for `seqs` in order (one s3_kv_alloc call) and write their cached rows
        (fill=False: the caller writes them, see retire_and_refill).
        prefill(serial, layer, rows) -> (k_rows, v_rows) device tensors [rows][H][D].
        Returns (serial, slot, off, cap, len, total) of the admitted ones."""
        preds = [s.predicted for s in seqs]
        rc, ids, offs, caps = s3.s3_kv_alloc(self.arena, preds)
        s3.check(rc, "s3_kv_alloc")
        admitted = []
        for s, sid, off, cap in zip(seqs, ids.tolist(), offs.tolist(), caps.tolist()):
            serial = self.next_serial
            self.next_serial += 1
            self._log("alloc", serial, s.predicted, sid, off, cap)
            if sid < 0:
                continue
            rows = s.start
            self._log("fill", serial, sid, rows)
            admitted.append((serial, sid, off, cap, rows, s.total))
        if fill:
            self._fill_admitted(admitted, prefill)
        return admitted

    def _fill_admitted(self, admitted, prefill):
        """Prompt rows of newly admitted sequences: one s3_kv_fill_batch call per layer (sixteen newcomers
        per launch) instead of one launch per sequence and layer."""
        if not admitted:
            return
        sids = np.array([r[1] for r in admitted], np.int32)
        rows = np.array([r[4] for r in admitted], np.int32)
        st = self._stream_ptr()
        for layer in range(self.w.n_layers):
            kv = [prefill(r[0], layer, r[4]) for r in admitted]
            s3.check(s3.s3_kv_fill_batch(self.arena, layer, sids, rows, [x[0] for x in kv], [x[1] for x in kv], st),
                     "s3_kv_fill_batch")

    def admit_scheduled(self, max_out, prefill, fill=True):
        """Let the scheduler admit up to max_out waiting requests (decreasing first fit).  Same return value
        as admit()."""
        if max_out <= 0 or s3.s3_sched_pool_size(self.sched) == 0:
            return []
        rc, rids, sids, offs, caps = s3.s3_sched_admit(self.sched, max_out)
        s3.check(rc, "s3_sched_admit")
        serials = list(range(self.next_serial, self.next_serial + len(rids)))
        self.next_serial += len(rids)
        self._log("sched_admit", max_out, serials, rids.tolist(), sids.tolist(), offs.tolist(), caps.tolist())
        admitted = []
        for serial, rid, sid, off, cap in zip(serials, rids.tolist(), sids.tolist(), offs.tolist(), caps.tolist()):
            r = self._requests[rid]
            self._log("fill", serial, sid, r.start)
            admitted.append((serial, sid, off, cap, r.start, r.total))
        if fill:
            self._fill_admitted(admitted, prefill)
        return admitted

    def start(self, prefill, stop_when_full=False):
        recs = []
        if self.admission == "dff":
            recs = self.admit_scheduled(self.w.batch, prefill)
        elif stop_when_full:  # admit candidates one by one until the arena refuses one; then write their rows
            for s in self.w.seqs:
                got = self.admit([s], prefill, fill=False)
                if not got:
                    break
                recs += got
            self._fill_admitted(recs, prefill)
        else:
            recs = self.admit(self.w.seqs, prefill)
        self._set_batch(recs)

    # -- one decode step --------------------------------------------------
    def grow_full_slots(self):
        full = np.nonzero(self.len == self.cap)[0]
        if full.size == 0:
            return
        drop, out = [], []
        for i in full.tolist():
            st, off, cap = self._grow(i)
            if st == s3.S3_ERR_NOMEM and self.on_nomem == "swap" and self._compact_for(
                    s3.s3_kv_grown_capacity(self.cfg, int(self.cap[i]))):
                st, off, cap = self._grow(i)
            if st == s3.S3_OK:
                self.off[i], self.cap[i] = off, cap
                self.n_grown += 1
                self._patch.add(i)
            elif st == s3.S3_ERR_NOMEM and self.on_nomem == "swap":
                out.append(i)
            elif st in (s3.S3_ERR_NOMEM, s3.S3_ERR_MAXLEN):
                drop.append(i)  # cannot continue: at the maximum length (or no host swap wanted)
            else:
                s3.check(st, "s3_kv_grow")
        for i in out:
            self._evict(i)
        for i in drop:
            s3.check(s3.s3_kv_free(self.arena, int(self.slot[i])), "s3_kv_free")
            self._log("free", int(self.serial[i]), int(self.slot[i]))
            self.n_evicted += 1
        if drop or out:
            self._remove(drop + out)
        self._recount()

    def _grow(self, i):
        st, off, cap = s3.s3_kv_grow(self.arena, int(self.slot[i]), int(self.len[i]), self._stream_ptr())
        self._log("grow", int(self.serial[i]), int(self.slot[i]), int(self.len[i]), st, off, cap)
        return st, off, cap

    def _compact_for(self, want):
        """Free space that is only fragmented: close the holes (every live slot belongs to the batch).
        True if an extent of `want` tokens exists afterwards."""
        st, used, free, largest, total = s3.s3_kv_stats(self.arena)
        s3.check(st, "s3_kv_stats")
        if free < want or largest >= want:
            return False
        # Compaction moves up to every live row through HBM; swapping one sequence moves its rows over the
        # host link twice, some fifty times slower per byte: compact only while that is the cheaper of the two.
        if used > self.COMPACT_RATIO * want:
            return False
        st, new_off, moved = s3.s3_kv_compact(self.arena, self.slot, self.len, self._stream_ptr())
        s3.check(st, "s3_kv_compact")
        self._log("compact", self.slot.tolist(), new_off.tolist(), moved)
        self.off[:] = new_off
        self.n_compactions += 1
        self._dirty = True
        return True

    def _evict(self, i):
        """Rows of batch entry i to pinned host memory; the slot is freed (the entry is removed by the caller).
        One gather kernel on the decode stream puts the rows into a device staging buffer, after which the slot's
        room can be reused in stream order; the staging buffer crosses the host link in one copy on the side
        stream, beside the decode steps that follow."""
        length, sid = int(self.len[i]), int(self.slot[i])
        nbytes = s3.s3_kv_evict_bytes(self.arena, length)
        host = self._host_buffer(nbytes)
        entry = self._stage_buffer()
        main = torch.cuda.current_stream(self.dev)
        s3.check(s3.s3_kv_gather_rows(self.arena, sid, length, entry[1], main.cuda_stream), "s3_kv_gather_rows")
        s3.check(s3.s3_kv_free(self.arena, sid), "s3_kv_free")
        ready, done = torch.cuda.Event(), torch.cuda.Event()
        ready.record(main)
        self._side.wait_event(ready)
        s3.check(s3.s3_kv_link_copy(host, entry[1], nbytes, self.LINK_WORKGROUPS, self._side.cuda_stream), "s3_kv_link_copy")
        done.record(self._side)
        entry[0] = done
        self._log("evict", int(self.serial[i]), sid, length)
        self.swapped.append(SimpleNamespace(serial=int(self.serial[i]), len=length, total=int(self.total[i]), nbytes=nbytes,
                                            want=s3.s3_kv_grown_capacity(self.cfg, int(self.cap[i])), host=host))
        self.n_swapped_out += 1

    def _host_buffer(self, nbytes):
        """Pinned staging memory for one evicted sequence (pinning memory costs far more than the copy it serves:
        buffers are reused once their sequence is back on the device)."""
        fits = [k for k, h in enumerate(self._host_free) if h.numel() >= nbytes]
        if fits:  # the smallest that fits
            return self._host_free.pop(min(fits, key=lambda k: self._host_free[k].numel()))
        return torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)

    def _restore_oldest(self):
        """Start bringing the longest-waiting evicted sequence back: its slot (the doubled reservation) is
        reserved now, its rows start their way into a device staging buffer on the side stream, and it joins the
        batch at the first step that finds them there (_join_restored).  -> True, or False (no room yet)."""
        if len(self._restoring) >= self.MAX_RETURNING:
            return False
        entry = self._stage_buffer(block=False)
        if entry is None:  # every staging buffer still carries an eviction to the host: try again at the next retirement
            return False
        rec = self.swapped[0]
        rc, ids, offs, caps = s3.s3_kv_alloc(self.arena, [rec.want])
        s3.check(rc, "s3_kv_alloc")
        st = s3.S3_OK if rc == 1 else s3.S3_ERR_NOMEM
        self._log("restore", rec.serial, rec.want, rec.len, st, int(ids[0]), int(offs[0]), int(caps[0]))
        if st == s3.S3_ERR_NOMEM:
            return False
        self.swapped.pop(0)
        entry[2] = True  # held until the rows have been scattered into the slot
        # on the side stream, i.e. behind this sequence's own copy to the host, which ran there
        s3.check(s3.s3_kv_link_copy(entry[1], rec.host, rec.nbytes, self.LINK_WORKGROUPS, self._side.cuda_stream),
                 "s3_kv_link_copy")
        back = torch.cuda.Event()
        back.record(self._side)
        entry[0] = back
        self._restoring.append(SimpleNamespace(event=back, entry=entry, host=rec.host, nbytes=rec.nbytes,
                                               rec=(rec.serial, int(ids[0]), int(offs[0]), int(caps[0]), rec.len, rec.total)))
        self.n_swapped_in += 1
        return True

    @property
    def n_returning(self):
        """Re-admitted sequences whose rows are still on their way back from the host."""
        return len(self._restoring)

    def finish_restores(self):
        """Block until every re-admitted sequence has its rows and is part of the batch again."""
        while self._restoring and self.n_active < max(self.capacity, 1):
            self._join_restored(wait=True)

    def _join_restored(self, wait=False):
        """Sequences whose rows have arrived in their staging buffer: scatter them into the reserved slot (one
        kernel on the decode stream) and append them to the batch."""
        joined = False
        while self._restoring and self.n_active < max(self.capacity, 1):
            r = self._restoring[0]
            if not r.event.query():
                if not wait:
                    break
                r.event.synchronize()
            self._restoring.pop(0)
            serial, sid, off, cap, length, total = r.rec
            main = torch.cuda.current_stream(self.dev)
            s3.check(s3.s3_kv_scatter_rows(self.arena, sid, length, r.entry[1], main.cuda_stream), "s3_kv_scatter_rows")
            used = torch.cuda.Event()
            used.record(main)
            r.entry[0], r.entry[2] = used, False
            self._host_free.append(r.host)
            self._append_entry(r.rec)
            joined = True
            wait = False
        if joined:
            self._recount()

    def _remove(self, gone):
        """Take entries out of the batch without re-uploading it: the last entry moves into each hole
        (one patched entry of the device arrays per hole) and the batch becomes a shorter prefix."""
        fields = ("serial", "slot", "off", "cap", "len", "total")
        n = self.n_active
        for i in sorted(gone, reverse=True):  # descending: the last entry is never a hole still to come
            last = n - 1
            if i != last:
                for name in fields:
                    getattr(self, name)[i] = getattr(self, name)[last]
                self._patch.add(i)
            self._patch.discard(last)
            n -= 1
        for name in fields:
            setattr(self, name, getattr(self, name)[:n].copy())

    def launch_step(self, tensors, check_host=False):
        """append + attention for every layer on the current batch.  tensors(layer, n) ->
        (q, k_new, v_new) device tensors.  Returns the output tensor of the LAST layer."""
        self._sync_arrays()
        n = self.n_active
        if n == 0:
            return None
        st = self._stream_ptr()
        ids = self.slot if check_host else None
        pos = self.len if check_host else None
        if not self.fused:
            torch.add(self.len_dev, 1, out=self.len_next)
        for layer in range(self.w.n_layers):
            q, k_new, v_new = tensors(layer, n)
            if self.fused:
                s3.check(s3.s3_decode_step(self.arena, layer, n, self.slot_off_dev, self.len_dev, q, k_new, v_new,
                                           self.out, self.out_dtype, 0.0, self.len_next, st, slot_id=ids,
                                           pos_host=pos), "s3_decode_step")
            else:
                s3.check(s3.s3_kv_append(self.arena, layer, n, self.slot_off_dev, self.len_dev, k_new, v_new, st,
                                         slot_id=ids, pos_host=pos), "s3_kv_append")
                s3.check(s3.s3_decode_attention(self.arena, layer, n, q, self.slot_off_dev, self.len_next, self.out,
                                                self.out_dtype, 0.0, st), "s3_decode_attention")
        self.len_dev, self.len_next = self.len_next, self.len_dev
        self.len += 1
        self._rows += n
        self._to_full -= 1
        self._to_done -= 1
        return self.out

    def retire_and_refill(self, prefill):
        done = np.nonzero(self.len >= self.total)[0]
        if done.size == 0 and not (self.swapped and self.n_active == 0):
            self._recount()
            return  # nothing was freed (a batch that is entirely on the host must come back, though)
        keep = np.ones(self.n_active, bool)
        for i in done.tolist():
            s3.check(s3.s3_kv_free(self.arena, int(self.slot[i])), "s3_kv_free")
            self._log("free", int(self.serial[i]), int(self.slot[i]))
            self.n_retired += 1
            keep[i] = False
        new = []  # batch entries that received a newcomer
        room = True  # an evicted sequence comes back before any newcomer; one refusal ends the attempts of this step
        for i in done.tolist():
            if self.swapped and room:
                room = self._restore_oldest()
                if room:
                    continue  # the entry stays open for the returning sequence, which joins when its rows are back
            if self.admission == "fifo" and self.w.refill and self.pool_pos < len(self.w.pool):
                got = self.admit([self.w.pool[self.pool_pos]], prefill, fill=False)
                self.pool_pos += 1
                if got:
                    (self.serial[i], self.slot[i], self.off[i], self.cap[i], self.len[i], self.total[i]) = got[0]
                    keep[i] = True
                    new.append(i)
        if self.admission == "dff" and self.w.refill:  # one scheduler pass for all entries that are still open
            holes = np.nonzero(~keep)[0].tolist()
            for i, got in zip(holes, self.admit_scheduled(len(holes), prefill, fill=False)):
                (self.serial[i], self.slot[i], self.off[i], self.cap[i], self.len[i], self.total[i]) = got
                keep[i] = True
                new.append(i)
        if new:
            # the prompt rows of all newcomers of this step in one launch per layer; if the batch keeps its
            # shape, the first launch also writes their entries of the device arrays
            in_place = bool(keep.all()) and not self._dirty and self.slot_off_dev is not None
            for layer in range(self.w.n_layers):
                rows = [prefill(int(self.serial[i]), layer, int(self.len[i])) for i in new]
                patch = dict(slot_off=self.slot_off_dev, length=self.len_dev, batch_n=self.n_active,
                             batch_idx=new) if in_place and layer == 0 else {}
                s3.check(s3.s3_kv_fill_batch(self.arena, layer, self.slot[new], self.len[new], [r[0] for r in rows],
                                             [r[1] for r in rows], self._stream_ptr(), **patch), "s3_kv_fill_batch")
            if not in_place:
                self._patch.update(new)
        if not keep.all():
            self._remove(np.nonzero(~keep)[0].tolist())
        while self.swapped and room and self.n_active + len(self._restoring) < self.capacity:
            room = self._restore_oldest()
        self._recount()

    def _append_entry(self, rec):
        for name, v in zip(("serial", "slot", "off", "cap", "len", "total"), rec):
            arr = getattr(self, name)
            setattr(self, name, np.append(arr, np.asarray([v], arr.dtype)))
        self._patch.add(self.n_active - 1)

    def step(self, tensors, prefill, check_host=False):
        if self._restoring:
            self._join_restored(wait=self.n_active == 0)
        if self._to_full <= 0:  # some slot is full: double it (or compact / swap / drop)
            self.grow_full_slots()
        out = self.launch_step(tensors, check_host)
        self.last_step_bytes = (self._row_term * self._rows + self._seq_term * self.n_active) * self.w.n_layers
        self.last_step_seqs = self.n_active
        if self.events is not None:
            self._log("step", self.serial.tolist(), self.len.tolist())
        if self._to_done <= 0 or (self.swapped and self.n_active == 0):  # some sequence has finished
            self.retire_and_refill(prefill)
        return out

    # -- accounting -------------------------------------------------------
    def algorithmic_bytes(self):
        """Bytes one layer-step of the CURRENT batch must move, counted after the append (the
        lengths attention sees): K and V rows read once, q read, out written, new k/v read and
        written."""
        e = 2                    # q, new k and v: 16-bit
        ec = self.w.elem_bytes   # cache rows
        e_out = {s3.S3_F32: 4, s3.S3_F16: 2, s3.S3_BF16: 2}[self.out_dtype]
        hd = self.w.n_heads * self.w.head_dim
        kvd = self.w.kv_heads * self.w.head_dim  # elements of one cached row
        B = self.n_active
        return 2 * kvd * ec * int(self.len.sum()) + B * hd * e + B * hd * e_out + 2 * B * kvd * (e + ec)

    def _byte_terms(self):
        """The same count as two factors: bytes per cached row, bytes per sequence (one layer-step)."""
        e, ec = 2, self.w.elem_bytes
        e_out = {s3.S3_F32: 4, s3.S3_F16: 2, s3.S3_BF16: 2}[self.out_dtype]
        hd = self.w.n_heads * self.w.head_dim
        kvd = self.w.kv_heads * self.w.head_dim
        return 2 * kvd * ec, hd * e + hd * e_out + 2 * kvd * (e + ec)

    def read_slot(self, a, layer, which, n_rows=None):
        n_rows = a.len if n_rows is None else n_rows
        eight_bit = self.w.dtype == s3.S3_E4M3
        dst = torch.empty((n_rows, self.w.kv_heads, self.w.head_dim), dtype=torch.uint8 if eight_bit else torch.int16,
                          device=self.dev)
        s3.check(s3.s3_kv_read_rows(self.arena, a.slot, layer, which, 0, n_rows, dst, self._stream_ptr()),
                 "s3_kv_read_rows")
        return dst.cpu().numpy() if eight_bit else dst.cpu().numpy().view(np.uint16)
