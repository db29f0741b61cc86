"""CPU oracle for the prediction-sized KV cache and decode-step attention.

TEST INFRASTRUCTURE ONLY.  Only the tests, the smoke check and the benchmark's
CPU-baseline leg may import this module; the product path must never reach it.
It shares no code, header, table or layout with the HIP library.

What it models, with the passage of the paper each part follows:

* KV-cache size: ``4 * l * d_h`` bytes per token in half precision, i.e. two
  matrices (K and V) of ``d_h`` two-byte numbers per layer (section 2.1).
* Reservation by predicted length instead of the maximum sequence length
  (sections 1 and 2.3), admitted in caller order while the cache still fits in
  what is left of the memory (the admission loop of section 3, scheduler
  paragraph; the decreasing sort that precedes it is the scheduler's, not ours).
* Append-only filling of a reserved region (section 2.2).
* A sequence that has used up its reservation but is not finished gets twice
  the memory (section 3, supervisor paragraph).
* The supervisor's report of available memory (section 3, supervisor paragraph).
* Attention of one query row against the sequence's own cached rows, no
  padding (section 2.1 equation; section 3 on irregular batches); the arithmetic
  lives in ``s3_oracle.c``.

Storage is deliberately *not* an arena: every live sequence owns a private
array ``[n_layers][2][cap][H][D]`` of 16-bit patterns.  Offsets into the shared
token space are tracked as plain integers with a sorted free-extent list so that
they can be compared bit for bit with the library's answers.

Readings where the paper is silent (all restated in the design document):
capacity = predicted total length rounded UP to the granule, at least one
granule, at most ``max_len``; placement = first fit at the lowest offset; a grown
slot is placed while the old one is still reserved, so the two never overlap,
then the old one is released; growing a slot already at ``max_len`` is an error;
an empty context gives an all-zero output row.
"""
import ctypes
import os

import numpy as np

OK, ERR_INVALID, ERR_NOMEM, ERR_SLOT_FULL, ERR_MAXLEN = 0, -1, -2, -3, -4
F16, BF16 = 0, 1
E4M3 = 3  # 8-bit cache rows: one e4m3 code in the low byte of each uint16 the oracle stores

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        path = os.path.join(_HERE, "libs3oracle.so")
        if not os.path.exists(path):
            from oracle.build import build_oracle

            build_oracle()
        _LIB = ctypes.CDLL(path)
    return _LIB


def _c(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


_REAL = {"f32": (np.float32, ctypes.c_float), "f64": (np.float64, ctypes.c_double)}


def widen(bits, dtype, precision="f32"):
    """Stored 16-bit patterns -> real numbers, through the oracle's own C conversion."""
    npt, ct = _REAL[precision]
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.empty(bits.shape, npt)
    getattr(_lib(), f"s3o_widen_{precision}")(_c(bits, ctypes.c_uint16), ctypes.c_int64(bits.size),
                                              ctypes.c_int(dtype), _c(out, ct))
    return out


def quantize_e4m3(x):
    """float32 values -> e4m3 codes (uint16 array, code in the low byte): nearest, ties to even,
    saturating at +-448, NaN -> 0x7f.  What an 8-bit cache stores for a new row."""
    x = np.ascontiguousarray(x, np.float32)
    out = np.empty(x.shape, np.uint8)
    _lib().s3o_quantize_e4m3_f32(_c(x, ctypes.c_float), ctypes.c_int64(x.size), _c(out, ctypes.c_uint8))
    return out.astype(np.uint16)


def scores(q, K, dtype, scale, precision="f32", q_dtype=None):
    """Step 1 for one head: q [D], K [L][D] (stored patterns) -> s [L]."""
    npt, ct = _REAL[precision]
    q = np.ascontiguousarray(q, np.uint16)
    K = np.ascontiguousarray(K, np.uint16)
    L, D = K.shape
    s = np.empty(L, npt)
    getattr(_lib(), f"s3o_scores_{precision}")(_c(q, ctypes.c_uint16), dtype if q_dtype is None else q_dtype,
                                               _c(K, ctypes.c_uint16), ctypes.c_int64(D), L, D, dtype, ct(scale),
                                               _c(s, ct))
    return s


def softmax(s, precision="f32"):
    """Step 2: max-subtracted softmax of a score vector."""
    npt, ct = _REAL[precision]
    s = np.ascontiguousarray(s, npt)
    p = np.empty_like(s)
    getattr(_lib(), f"s3o_softmax_{precision}")(_c(s, ct), int(s.size), _c(p, ct))
    return p


def weighted_sum(p, V, dtype, precision="f32"):
    """Step 3 for one head: p [L], V [L][D] -> o [D]."""
    npt, ct = _REAL[precision]
    p = np.ascontiguousarray(p, npt)
    V = np.ascontiguousarray(V, np.uint16)
    L, D = V.shape
    o = np.empty(D, npt)
    getattr(_lib(), f"s3o_weighted_sum_{precision}")(_c(p, ct), _c(V, ctypes.c_uint16), ctypes.c_int64(D),
                                                     L, D, dtype, _c(o, ct))
    return o


def attention_ragged(q, K_list, V_list, lens, dtype, scale=None, precision="f32", threads=1, q_dtype=None):
    """softmax(q K^T * scale) V per (sequence, head) over each sequence's own length.

    q: [n][H][D] 16-bit patterns.  K_list[b], V_list[b]: [rows_b][Hkv][D] 16-bit
    patterns with rows_b >= lens[b]; only the first lens[b] rows are read.
    Hkv == H is multi-head attention (section 2.1); Hkv < H is the grouped form
    of the multi-query attention the related-work section names: query head h
    reads key/value head h // (H // Hkv).
    dtype is the storage type of K and V; q has the same type unless q_dtype says otherwise (8-bit
    caches keep 16-bit queries).  scale None means 1/sqrt(D).  Returns (out [n][H][D] real, threads used).
    """
    npt, ct = _REAL[precision]
    q = np.ascontiguousarray(q, np.uint16)
    n, H, D = q.shape
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    lens = np.ascontiguousarray(lens, np.int32)
    Ks = [np.ascontiguousarray(k, np.uint16) for k in K_list]
    Vs = [np.ascontiguousarray(v, np.uint16) for v in V_list]
    Hkv = Ks[0].shape[1] if n else H
    assert 1 <= Hkv <= H and H % Hkv == 0
    for b in range(n):
        assert Ks[b].shape[1:] == (Hkv, D) and Vs[b].shape[1:] == (Hkv, D)
        assert 0 <= lens[b] <= Ks[b].shape[0] and lens[b] <= Vs[b].shape[0]
    PT = ctypes.POINTER(ctypes.c_uint16)
    kp = (PT * max(n, 1))(*[_c(k, ctypes.c_uint16) for k in Ks])
    vp = (PT * max(n, 1))(*[_c(v, ctypes.c_uint16) for v in Vs])
    out = np.zeros((n, H, D), npt)
    used = getattr(_lib(), f"s3o_attention_batch_{precision}")(
        n, H, Hkv, D, dtype, dtype if q_dtype is None else q_dtype, kp, vp, _c(lens, ctypes.c_int32), _c(q, ctypes.c_uint16), ct(scale), _c(out, ct),
        int(threads))
    if used < 0:
        raise MemoryError("oracle scratch allocation failed")
    return out, used


def merge_partials(parts):
    """Merge softmax partials of disjoint pieces of one context (float64).

    parts: list of (m_c, l_c, acc_c) where, for piece c, m_c is the maximum
    score, l_c = sum_j exp(s_j - m_c) and acc_c[d] = sum_j exp(s_j - m_c) V[j][d].
    Result: o = sum_c acc_c e^{m_c - m*} / sum_c l_c e^{m_c - m*}, m* = max_c m_c,
    which is algebraically the unsplit softmax-weighted sum.
    """
    m_star = max(p[0] for p in parts)
    Z = 0.0
    o = np.zeros_like(np.asarray(parts[0][2], np.float64))
    for m_c, l_c, acc_c in parts:
        w = np.exp(np.float64(m_c) - np.float64(m_star))
        Z += np.float64(l_c) * w
        o += np.asarray(acc_c, np.float64) * w
    return o / Z


class KVOracle:
    """Slot allocator + per-sequence KV storage, step by step as the header describes."""

    def __init__(self, n_layers, n_heads, head_dim, dtype, granule, max_len, arena_bytes, store=True,
                 n_kv_heads=None, act_dtype=None):
        assert granule > 0 and max_len > 0 and max_len % granule == 0
        self.n_layers, self.H, self.D, self.dtype = n_layers, n_heads, head_dim, dtype
        # key/value heads per cached row: all heads (section 2.1) unless the model shares them
        # between query heads (multi-query attention, related work)
        self.Hkv = n_heads if not n_kv_heads else n_kv_heads
        assert n_heads % self.Hkv == 0
        self.G, self.M = granule, max_len
        # 8-bit cache rows (quantised cache, related work): queries and new rows stay 16-bit (act_dtype)
        # and a new row is quantised once, when it is appended
        self.act_dtype = dtype if act_dtype is None else act_dtype
        assert dtype != E4M3 or self.act_dtype in (F16, BF16)
        self.elem_bytes = 1 if dtype == E4M3 else 2
        # K and V, every layer, Hkv*D numbers of elem_bytes each: the paper's 4*l*d_h for 2-byte numbers
        # when Hkv*D = d_h
        self.bytes_per_token = 2 * n_layers * self.Hkv * head_dim * self.elem_bytes
        self.N = arena_bytes // self.bytes_per_token  # token rows the memory can hold
        self.free_list = [[0, self.N]] if self.N > 0 else []  # sorted by offset, coalesced
        self.slots = {}  # id -> [off, cap]
        self.data = {}  # id -> uint16 [n_layers][2][cap][H][D]
        self.store = store
        self.n_grows = 0

    # -- integers ---------------------------------------------------------
    def capacity_for(self, predicted_len):
        g = self.G
        cap = -(-int(predicted_len) // g) * g  # round up to the granule
        cap = max(g, cap)
        return min(self.M, cap)

    def grown_capacity(self, cap):
        """Reservation of a sequence that used up `cap` tokens and is not finished: twice the memory
        (section 3, supervisor paragraph), never more than the maximum sequence length."""
        return min(2 * int(cap), self.M)

    def _first_fit(self, cap):
        for i, (off, size) in enumerate(self.free_list):
            if size >= cap:
                return i
        return -1

    def _carve(self, cap):
        i = self._first_fit(cap)
        if i < 0:
            return -1
        off, size = self.free_list[i]
        if size == cap:
            del self.free_list[i]
        else:
            self.free_list[i] = [off + cap, size - cap]
        return off

    def _release(self, off, cap):
        fl = self.free_list
        i = 0
        while i < len(fl) and fl[i][0] < off:
            i += 1
        fl.insert(i, [off, cap])
        if i + 1 < len(fl) and fl[i][0] + fl[i][1] == fl[i + 1][0]:  # merge with the next extent
            fl[i][1] += fl[i + 1][1]
            del fl[i + 1]
        if i > 0 and fl[i - 1][0] + fl[i - 1][1] == fl[i][0]:  # merge with the previous extent
            fl[i - 1][1] += fl[i][1]
            del fl[i]

    def _new_id(self):
        i = 0
        while i in self.slots:
            i += 1
        return i

    def alloc_one(self, predicted_len):
        """-> (id, off, cap); (-1, -1, 0) when it does not fit (state unchanged)."""
        cap = self.capacity_for(predicted_len)
        off = self._carve(cap)
        if off < 0:
            return -1, -1, 0
        sid = self._new_id()
        self.slots[sid] = [off, cap]
        if self.store:
            self.data[sid] = np.zeros((self.n_layers, 2, cap, self.Hkv, self.D), np.uint16)
        return sid, off, cap

    def alloc(self, predicted_lens):
        """Caller order; each sequence admitted iff it fits in what is left."""
        if any(int(p) < 0 for p in predicted_lens):
            return ERR_INVALID, [], [], []
        ids, offs, caps = [], [], []
        for p in predicted_lens:
            sid, off, cap = self.alloc_one(p)
            ids.append(sid)
            offs.append(off)
            caps.append(cap)
        return sum(1 for s in ids if s >= 0), ids, offs, caps

    def free(self, sid):
        if sid not in self.slots:
            return ERR_INVALID
        off, cap = self.slots.pop(sid)
        self.data.pop(sid, None)
        self._release(off, cap)
        return OK

    def grow(self, sid, length):
        """-> (status, new_off, new_cap).  Doubles the reservation, keeps rows [0, length)."""
        if sid not in self.slots:
            return ERR_INVALID, -1, 0
        off, cap = self.slots[sid]
        if length < 0 or length > cap:
            return ERR_INVALID, -1, 0
        if cap >= self.M:
            return ERR_MAXLEN, -1, 0
        new_cap = self.grown_capacity(cap)
        new_off = self._carve(new_cap)  # the old extent is still reserved here
        if new_off < 0:
            return ERR_NOMEM, -1, 0
        if self.store:
            fresh = np.zeros((self.n_layers, 2, new_cap, self.Hkv, self.D), np.uint16)
            fresh[:, :, :length] = self.data[sid][:, :, :length]
            self.data[sid] = fresh
        self._release(off, cap)
        self.slots[sid] = [new_off, new_cap]
        self.n_grows += 1
        return OK, new_off, new_cap

    def evict(self, sid, length):
        """Move a sequence's rows [0, length) out of the cache (to the request pool in host memory, as
        the paper's supervisor does with a sequence that ran out of room) and free its slot.
        -> (status, rows [n_layers][2][length][H][D])."""
        if sid not in self.slots or length < 0 or length > self.slots[sid][1]:
            return ERR_INVALID, None
        blob = self.data[sid][:, :, :length].copy()
        self.free(sid)
        return OK, blob

    def restore(self, predicted_len, blob):
        """Re-admit an evicted sequence with a new (the paper: doubled) reservation.
        -> (status, id, off, cap)."""
        length = blob.shape[2]
        if predicted_len < length:
            return ERR_INVALID, -1, -1, 0
        sid, off, cap = self.alloc_one(predicted_len)
        if sid < 0:
            return ERR_NOMEM, -1, -1, 0
        self.data[sid][:, :, :length] = blob
        return OK, sid, off, cap

    def compact(self):
        """Slide every live slot down, in order of offset, so that no hole is left (the paper's
        supervisor shifts the rows below a blank up); the free space becomes one extent at the end.
        Each sequence's private rows are untouched.  -> {id: new_off}."""
        cursor = 0
        moved = 0
        for sid in sorted(self.slots, key=lambda i: self.slots[i][0]):
            if self.slots[sid][0] != cursor:
                moved += 1
            self.slots[sid][0] = cursor
            cursor += self.slots[sid][1]
        self.free_list = [[cursor, self.N - cursor]] if cursor < self.N else []
        return {sid: oc[0] for sid, oc in self.slots.items()}, moved

    def stats(self):
        """-> (used, free, largest_free, capacity), all in tokens."""
        used = sum(cap for _, cap in self.slots.values())
        free = sum(size for _, size in self.free_list)
        largest = max([size for _, size in self.free_list], default=0)
        return used, free, largest, self.N

    # -- rows -------------------------------------------------------------
    def append(self, sid, layer, pos, k_row, v_row):
        """Write the new token's key and value ([H][D] patterns) into row pos.  An 8-bit cache gets
        the 16-bit values rounded to the nearest e4m3 code (ties to even, saturating)."""
        if sid not in self.slots or not (0 <= layer < self.n_layers) or pos < 0:
            return ERR_INVALID
        off, cap = self.slots[sid]
        if pos >= cap:
            return ERR_SLOT_FULL
        if self.dtype == E4M3:
            k_row = quantize_e4m3(widen(k_row, self.act_dtype))
            v_row = quantize_e4m3(widen(v_row, self.act_dtype))
        self.data[sid][layer, 0, pos] = k_row
        self.data[sid][layer, 1, pos] = v_row
        return OK

    def fill(self, sid, layer, k_rows, v_rows):
        """Bulk write of rows [0, len) (the stand-in for the prompt phase)."""
        n = k_rows.shape[0]
        off, cap = self.slots[sid]
        if n > cap:
            return ERR_SLOT_FULL
        self.data[sid][layer, 0, :n] = k_rows
        self.data[sid][layer, 1, :n] = v_rows
        return OK

    def rows(self, sid, layer, which, length):
        return self.data[sid][layer, which, :length]

    def attention(self, layer, ids, lens, q, scale=None, precision="f32", threads=1):
        Ks = [self.data[s][layer, 0] for s in ids]
        Vs = [self.data[s][layer, 1] for s in ids]
        return attention_ragged(q, Ks, Vs, lens, self.dtype, scale, precision, threads, q_dtype=self.act_dtype)[0]


class SchedulerOracle:
    """Decreasing first fit with a single bin, step by step as the paper's scheduler paragraph (section 3)
    states it: sort the pool by KV-cache size, largest first (equal sizes keep arrival order - the paper
    does not say); walk it once; a request whose cache fits the memory that is left joins the batch and
    the memory shrinks by its size; stop when no memory is left or the pool has been walked.  "Fits"
    is asked from the slot allocator (first fit), so fragmentation can refuse what the total would hold."""

    def __init__(self, kv: "KVOracle"):
        self.kv = kv
        self.pool = []  # (request id, predicted total length), arrival order

    def submit(self, request_id, predicted_len):
        self.pool.append((request_id, predicted_len))

    def admit(self, max_out):
        order = sorted(range(len(self.pool)), key=lambda i: -self.kv.capacity_for(self.pool[i][1]))  # stable
        admitted, taken = [], set()
        for i in order:
            if len(admitted) >= max_out or self.kv.stats()[1] <= 0:
                break
            rid, pred = self.pool[i]
            sid, off, cap = self.kv.alloc_one(pred)
            if sid < 0:
                continue
            admitted.append((rid, sid, off, cap))
            taken.add(i)
        self.pool = [r for i, r in enumerate(self.pool) if i not in taken]
        return admitted
