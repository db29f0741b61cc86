"""Decode-loop plumbing over the C ABI: owns the arena tensor and the per-batch device arrays,
decides WHEN to call alloc / fill / grow / free / append / attention for a synthetic workload,
and records what the library answered.  It computes nothing of the method itself.

Per decode step (iteration-level scheduling, section 3 of the S3 paper):
  1. every active sequence whose slot is full and which is not finished is grown (doubling);
  2. the new token's K/V row is appended at row len, len += 1;
  3. attention over the len rows now cached (append-then-attend: the new token attends to itself);
  4. sequences that reached their true total length are freed; with refill on, the next
     candidate of the pool is admitted into the freed room and its prompt rows are written.
The event log lets a test replay the same decisions on the CPU oracle and compare every id,
offset and capacity bit for bit.
"""
import numpy as np
import torch

from . import binding as s3

_TORCH_DT = {s3.S3_F16: torch.float16, s3.S3_BF16: torch.bfloat16, s3.S3_F32: torch.float32}


class Active:
    __slots__ = ("serial", "seq", "slot", "off", "cap", "len")

    def __init__(self, serial, seq, slot, off, cap, length):
        self.serial, self.seq, self.slot, self.off, self.cap, self.len = serial, seq, slot, off, cap, length


class DecodeEngine:
    def __init__(self, w, arena_tokens=None, device="cuda:0", out_dtype=s3.S3_F32, log_events=True):
        self.w = w
        self.dev = torch.device(device)
        self.cfg = s3.make_config(w.n_layers, w.n_heads, w.head_dim, w.dtype, w.granule, w.max_len)
        self.bpt = s3.s3_kv_bytes_per_token(self.cfg)
        if arena_tokens is None:
            if w.arena_bytes:
                arena_tokens = w.arena_bytes // self.bpt
            else:
                caps = [min(w.max_len, -(-max(s.predicted, 1) // w.granule) * w.granule) for s in w.seqs]
                arena_tokens = int(1.5 * sum(caps)) + 2 * w.max_len
        self.arena_tokens = int(arena_tokens)
        self.arena_mem = torch.empty(self.arena_tokens * self.bpt, dtype=torch.uint8, device=self.dev)
        st, self.arena = s3.s3_kv_arena_init(self.cfg, self.arena_mem, self.arena_mem.numel())
        s3.check(st, "s3_kv_arena_init")
        self.out_dtype = out_dtype
        self.active = []
        self.events = [] if log_events else None
        self.next_serial = 0
        self.pool_pos = 0
        self.n_evicted = 0
        self.slot_off_dev = None
        self.len_dev = None
        self._dirty = True
        self.out = None
        self.stream = 0  # torch's current (default) stream

    # -- helpers ----------------------------------------------------------
    def close(self):
        if self.arena is not None:
            torch.cuda.synchronize(self.dev)
            s3.s3_kv_arena_destroy(self.arena)
            self.arena = None

    def _log(self, *ev):
        if self.events is not None:
            self.events.append(ev)

    def _stream_ptr(self):
        return torch.cuda.current_stream(self.dev).cuda_stream

    def kv_dtype_torch(self):
        return _TORCH_DT[self.w.dtype]

    def _upload(self, values, dtype):
        # torch's pinned-memory allocator does not reuse a block before the copy that reads it has
        # completed, so the staging tensor needs no lifetime management here
        host = torch.tensor(values, dtype=dtype).pin_memory()
        return host.to(self.dev, non_blocking=True)

    def _sync_arrays(self):
        if self._dirty:
            self.slot_off_dev = self._upload([a.off for a in self.active], torch.int64)
            self.len_dev = self._upload([a.len for a in self.active], torch.int32)
            n = len(self.active)
            odt = _TORCH_DT[self.out_dtype]
            if self.out is None or self.out.shape[0] != n:
                self.out = torch.empty((n, self.w.n_heads, self.w.head_dim), dtype=odt, device=self.dev)
            self._dirty = False

    # -- admission --------------------------------------------------------
    def admit(self, seqs, prefill):
        """Reserve slots for `seqs` in order (one s3_kv_alloc call) and write their cached rows.
        prefill(serial, layer, rows) -> (k_rows, v_rows) device tensors [rows][H][D].
        Returns the Active records of the admitted ones."""
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
            for layer in range(self.w.n_layers):
                k_rows, v_rows = prefill(serial, layer, rows)
                s3.check(s3.s3_kv_fill(self.arena, sid, layer, 0, rows, k_rows, v_rows, self._stream_ptr()),
                         "s3_kv_fill")
            self._log("fill", serial, sid, rows)
            admitted.append(Active(serial, s, sid, off, cap, rows))
        return admitted

    def start(self, prefill, stop_when_full=False):
        if stop_when_full:  # admit candidates one by one until the arena refuses one
            for s in self.w.seqs:
                got = self.admit([s], prefill)
                if not got:
                    break
                self.active += got
        else:
            self.active = self.admit(self.w.seqs, prefill)
        self._dirty = True

    # -- one decode step --------------------------------------------------
    def grow_full_slots(self):
        for a in self.active:
            if a.len == a.cap:
                st, off, cap = s3.s3_kv_grow(self.arena, a.slot, a.len, self._stream_ptr())
                self._log("grow", a.serial, a.slot, a.len, st, off, cap)
                if st == s3.S3_OK:
                    a.off, a.cap = off, cap
                    self._dirty = True
                elif st in (s3.S3_ERR_NOMEM, s3.S3_ERR_MAXLEN):
                    a.len = -1  # cannot continue on the device: dropped (the paper evicts to the host)
                else:
                    s3.check(st, "s3_kv_grow")
        if any(a.len < 0 for a in self.active):
            for a in self.active:
                if a.len < 0:
                    s3.check(s3.s3_kv_free(self.arena, a.slot), "s3_kv_free")
                    self._log("free", a.serial, a.slot)
                    self.n_evicted += 1
            self.active = [a for a in self.active if a.len >= 0]
            self._dirty = True

    def launch_step(self, tensors, check_host=False):
        """append + attention for every layer on the current batch.  tensors(layer, n) ->
        (q, k_new, v_new) device tensors.  Returns the output tensor of the LAST layer."""
        self._sync_arrays()
        n = len(self.active)
        if n == 0:
            return None
        st = self._stream_ptr()
        ids = [a.slot for a in self.active] if check_host else None
        pos = [a.len for a in self.active] if check_host else None
        for layer in range(self.w.n_layers):
            q, k_new, v_new = tensors(layer, n)
            s3.check(s3.s3_kv_append(self.arena, layer, n, self.slot_off_dev, self.len_dev, k_new, v_new, st,
                                     slot_id=ids, pos_host=pos), "s3_kv_append")
            if layer == 0:
                self.len_plus1 = self.len_dev + 1
            s3.check(s3.s3_decode_attention(self.arena, layer, n, q, self.slot_off_dev, self.len_plus1, self.out,
                                            self.out_dtype, 0.0, st), "s3_decode_attention")
        self.len_dev = self.len_plus1
        for a in self.active:
            a.len += 1
        return self.out

    def retire_and_refill(self, prefill):
        done = [i for i, a in enumerate(self.active) if a.len >= a.seq.total]
        if not done:
            return
        for i in done:
            a = self.active[i]
            s3.check(s3.s3_kv_free(self.arena, a.slot), "s3_kv_free")
            self._log("free", a.serial, a.slot)
            self.active[i] = None
        if self.w.refill:
            for i in done:
                if self.pool_pos >= len(self.w.pool):
                    break
                got = self.admit([self.w.pool[self.pool_pos]], prefill)
                self.pool_pos += 1
                if got:
                    self.active[i] = got[0]
        self.active = [a for a in self.active if a is not None]
        self._dirty = True

    def step(self, tensors, prefill, check_host=False):
        self.grow_full_slots()
        out = self.launch_step(tensors, check_host)
        self._log("step", [a.serial for a in self.active], [a.len for a in self.active])
        self.retire_and_refill(prefill)
        return out

    # -- accounting -------------------------------------------------------
    def algorithmic_bytes(self):
        """Bytes one layer-step of the CURRENT batch must move (lengths before the append):
        K and V rows read once, q read, out written, new k/v read and written."""
        e = 2
        e_out = {s3.S3_F32: 4, s3.S3_F16: 2, s3.S3_BF16: 2}[self.out_dtype]
        hd = self.w.n_heads * self.w.head_dim
        B = len(self.active)
        sum_len = sum(a.len + 1 for a in self.active)
        return 2 * hd * e * sum_len + B * hd * e + B * hd * e_out + 4 * B * hd * e

    def read_slot(self, a, layer, which, n_rows=None):
        n_rows = a.len if n_rows is None else n_rows
        dst = torch.empty((n_rows, self.w.n_heads, self.w.head_dim), dtype=torch.int16, device=self.dev)
        s3.check(s3.s3_kv_read_rows(self.arena, a.slot, layer, which, 0, n_rows, dst, self._stream_ptr()),
                 "s3_kv_read_rows")
        return dst.cpu().numpy().view(np.uint16)
