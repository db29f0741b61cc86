"""Thin ctypes binding of libs3kv.so: same names as the C ABI, argument marshalling only.

Device arrays are passed as torch tensors (their ``data_ptr()`` is used) or raw integer
addresses; host arrays as numpy arrays / sequences.  Nothing here computes: every step of
the hot path runs inside the library's kernels.  The library must have been built
(``python -m paper_2306_06000_amd.build`` or ``__graft_entry__.build()``); loading fails
loudly otherwise - there is no fallback.
"""
import ctypes
import os

import numpy as np

S3_F16, S3_BF16, S3_F32, S3_E4M3 = 0, 1, 2, 3
S3_OK, S3_ERR_INVALID, S3_ERR_NOMEM, S3_ERR_SLOT_FULL, S3_ERR_MAXLEN, S3_ERR_HIP, S3_ERR_SCRATCH = 0, -1, -2, -3, -4, -5, -6
S3_STATIC_SCRATCH_BYTES = 32 << 20

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("S3KV_LIB") or os.path.join(_HERE, "libs3kv.so")  # S3KV_LIB: a diagnostic build
_lib = None


class s3_kv_config(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("n_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("kv_dtype", ctypes.c_int32), ("granule", ctypes.c_int32), ("max_len", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("act_dtype", ctypes.c_int32)]


_vp, _i32, _i64, _f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
_pi32, _pi64 = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64)

SIGNATURES = {
    "s3_kv_bytes_per_token": (_i64, [ctypes.POINTER(s3_kv_config)]),
    "s3_kv_capacity_for": (_i32, [ctypes.POINTER(s3_kv_config), _i32]),
    "s3_kv_grown_capacity": (_i32, [ctypes.POINTER(s3_kv_config), _i32]),
    "s3_kv_reserve_scratch": (ctypes.c_int, [_vp, _i32]),
    "s3_kv_arena_init": (ctypes.c_int, [ctypes.POINTER(_vp), ctypes.POINTER(s3_kv_config), _vp, ctypes.c_size_t]),
    "s3_kv_arena_destroy": (None, [_vp]),
    "s3_kv_alloc": (ctypes.c_int, [_vp, _i32, _pi32, _pi32, _pi64, _pi32]),
    "s3_kv_free": (ctypes.c_int, [_vp, _i32]),
    "s3_kv_slot_info": (ctypes.c_int, [_vp, _i32, _pi64, _pi32]),
    "s3_kv_append": (ctypes.c_int, [_vp, _i32, _i32, _pi32, _pi32, _vp, _vp, _vp, _vp, _vp]),
    "s3_decode_attention": (ctypes.c_int, [_vp, _i32, _i32, _vp, _vp, _vp, _vp, _i32, _f32, _vp]),
    "s3_decode_step": (ctypes.c_int, [_vp, _i32, _i32, _pi32, _pi32, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _f32, _vp, _vp]),
    "s3_decode_step_static": (ctypes.c_int, [_vp, _i32, _i32, _pi32, _pi32, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _f32, _vp, _vp]),
    "s3_kv_grow": (ctypes.c_int, [_vp, _i32, _i32, _pi64, _pi32, _vp]),
    "s3_kv_compact": (ctypes.c_int, [_vp, _i32, _pi32, _pi32, _pi64, _pi32, _vp]),
    "s3_kv_evict_bytes": (_i64, [_vp, _i32]),
    "s3_kv_evict": (ctypes.c_int, [_vp, _i32, _i32, _vp, _vp]),
    "s3_kv_restore": (ctypes.c_int, [_vp, _i32, _i32, _vp, _pi32, _pi64, _pi32, _vp]),
    "s3_kv_gather_rows": (ctypes.c_int, [_vp, _i32, _i32, _vp, _vp]),
    "s3_kv_scatter_rows": (ctypes.c_int, [_vp, _i32, _i32, _vp, _vp]),
    "s3_kv_link_copy": (ctypes.c_int, [_vp, _vp, ctypes.c_size_t, _i32, _vp]),
    "s3_sched_create": (ctypes.c_int, [ctypes.POINTER(_vp), _vp]),
    "s3_sched_destroy": (None, [_vp]),
    "s3_sched_submit": (ctypes.c_int, [_vp, _i64, _i32]),
    "s3_sched_admit": (ctypes.c_int, [_vp, _i32, _pi64, _pi32, _pi64, _pi32]),
    "s3_sched_pool_size": (ctypes.c_int, [_vp]),
    "s3_kv_stats": (ctypes.c_int, [_vp, _pi64, _pi64, _pi64, _pi64]),
    "s3_kv_fill": (ctypes.c_int, [_vp, _i32, _i32, _i32, _i32, _vp, _vp, _vp]),
    "s3_kv_batch_patch": (ctypes.c_int, [_i32, _vp, _vp, _i32, _pi32, _pi64, _pi32, _vp]),
    "s3_kv_fill_batch": (ctypes.c_int, [_vp, _i32, _i32, _pi32, _pi32, ctypes.POINTER(_vp), ctypes.POINTER(_vp), _i32, _vp,
                                        _vp, _pi32, _vp]),
    "s3_kv_read_rows": (ctypes.c_int, [_vp, _i32, _i32, _i32, _i32, _i32, _vp, _vp]),
    "s3_kv_probe_bandwidth": (ctypes.c_int, [_vp, ctypes.c_size_t, _i32, _i32, ctypes.POINTER(ctypes.c_double)]),
    "s3_kv_set_param": (ctypes.c_int, [_vp, ctypes.c_char_p, _i64]),
    "s3_kv_get_param": (ctypes.c_int, [_vp, ctypes.c_char_p, _pi64]),
    "s3_last_hip_error": (ctypes.c_char_p, []),
    "s3_status_str": (ctypes.c_char_p, [ctypes.c_int]),
}


def lib():
    """Load libs3kv.so once.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2306_06000_amd.build`; "
                               "there is no CPU fallback")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def _ptr(x):
    """Device/host address of a torch tensor, numpy array, int or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    raise TypeError(type(x))


def _host_i32(x):
    if x is None:
        return None, None
    arr = np.ascontiguousarray(x, np.int32)
    return arr, arr.ctypes.data_as(_pi32)


class S3Error(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        detail = lib().s3_last_hip_error().decode() if status == S3_ERR_HIP else ""
        super().__init__(f"{where}: {lib().s3_status_str(status).decode()} {detail}".strip())


def make_config(n_layers, n_heads, head_dim, kv_dtype, granule, max_len, n_kv_heads=0, act_dtype=0):
    return s3_kv_config(n_layers, n_heads, head_dim, kv_dtype, granule, max_len, n_kv_heads, act_dtype)


def s3_kv_bytes_per_token(cfg):
    return int(lib().s3_kv_bytes_per_token(ctypes.byref(cfg)))


def s3_kv_capacity_for(cfg, predicted_len):
    return int(lib().s3_kv_capacity_for(ctypes.byref(cfg), int(predicted_len)))


def s3_kv_grown_capacity(cfg, cap):
    return int(lib().s3_kv_grown_capacity(ctypes.byref(cfg), int(cap)))


def s3_kv_reserve_scratch(arena, max_batch):
    return lib().s3_kv_reserve_scratch(arena, int(max_batch))


def s3_kv_arena_init(cfg, dev_base, dev_bytes):
    """-> (status, arena handle).  dev_base: torch uint8 tensor / address / None (metadata only)."""
    h = _vp()
    st = lib().s3_kv_arena_init(ctypes.byref(h), ctypes.byref(cfg), _ptr(dev_base), int(dev_bytes))
    return st, (h if st == S3_OK else None)


def s3_kv_arena_destroy(arena):
    lib().s3_kv_arena_destroy(arena)


def s3_kv_alloc(arena, predicted_len):
    """-> (admitted or status, slot_id[n], slot_off[n], slot_cap[n]) as numpy arrays."""
    pl, plp = _host_i32(predicted_len)
    n = int(pl.size)
    ids = np.full(n, -2, np.int32)
    offs = np.full(n, -2, np.int64)
    caps = np.full(n, -2, np.int32)
    rc = lib().s3_kv_alloc(arena, n, plp, ids.ctypes.data_as(_pi32), offs.ctypes.data_as(_pi64),
                           caps.ctypes.data_as(_pi32))
    return rc, ids, offs, caps


def s3_kv_free(arena, slot_id):
    return lib().s3_kv_free(arena, int(slot_id))


def s3_kv_slot_info(arena, slot_id):
    off, cap = _i64(-1), _i32(0)
    st = lib().s3_kv_slot_info(arena, int(slot_id), ctypes.byref(off), ctypes.byref(cap))
    return st, off.value, cap.value


def s3_kv_append(arena, layer, n, slot_off, pos, k_new, v_new, stream=0, slot_id=None, pos_host=None):
    _a, idp = _host_i32(slot_id)
    _b, php = _host_i32(pos_host)
    return lib().s3_kv_append(arena, int(layer), int(n), idp, php, _ptr(slot_off), _ptr(pos), _ptr(k_new),
                              _ptr(v_new), stream or None)


def s3_decode_attention(arena, layer, n, q, slot_off, cur_len, out, out_dtype=S3_F32, scale=0.0, stream=0):
    return lib().s3_decode_attention(arena, int(layer), int(n), _ptr(q), _ptr(slot_off), _ptr(cur_len), _ptr(out),
                                     int(out_dtype), float(scale), stream or None)


def s3_decode_step(arena, layer, n, slot_off, pos, q, k_new, v_new, out, out_dtype=S3_F32, scale=0.0, len_out=None,
                   stream=0, slot_id=None, pos_host=None):
    _a, idp = _host_i32(slot_id)
    _b, php = _host_i32(pos_host)
    return lib().s3_decode_step(arena, int(layer), int(n), idp, php, _ptr(slot_off), _ptr(pos), _ptr(q), _ptr(k_new),
                                _ptr(v_new), _ptr(out), int(out_dtype), float(scale), _ptr(len_out), stream or None)


def s3_decode_step_static(arena, layer, n, slot_off, pos, q, k_new, v_new, out, out_dtype=S3_F32, scale=0.0, len_out=None,
                          stream=0, slot_id=None, pos_host=None):
    """s3_decode_step for callers that cannot allocate: the library's fixed device scratch is used."""
    _a, idp = _host_i32(slot_id)
    _b, php = _host_i32(pos_host)
    return lib().s3_decode_step_static(arena, int(layer), int(n), idp, php, _ptr(slot_off), _ptr(pos), _ptr(q),
                                       _ptr(k_new), _ptr(v_new), _ptr(out), int(out_dtype), float(scale), _ptr(len_out),
                                       stream or None)


def s3_kv_grow(arena, slot_id, length, stream=0):
    """-> (status, new_off, new_cap)."""
    off, cap = _i64(-1), _i32(0)
    st = lib().s3_kv_grow(arena, int(slot_id), int(length), ctypes.byref(off), ctypes.byref(cap), stream or None)
    return st, off.value, cap.value


def s3_kv_compact(arena, slot_id, length, stream=0):
    """-> (status, new_off[n], n_moved)."""
    ids, idp = _host_i32(slot_id)
    lens, lp = _host_i32(length)
    n = int(ids.size) if ids is not None else 0
    new_off = np.full(n, -1, np.int64)
    moved = _i32(0)
    st = lib().s3_kv_compact(arena, n, idp, lp, new_off.ctypes.data_as(_pi64), ctypes.byref(moved), stream or None)
    return st, new_off, moved.value


def s3_kv_evict_bytes(arena, length):
    return int(lib().s3_kv_evict_bytes(arena, int(length)))


def s3_kv_evict(arena, slot_id, length, host_buf, stream=0):
    """host_buf: CPU tensor / numpy array (pinned for asynchronous copies) of s3_kv_evict_bytes bytes."""
    return lib().s3_kv_evict(arena, int(slot_id), int(length), _ptr(host_buf), stream or None)


def s3_kv_restore(arena, predicted_len, length, host_buf, stream=0):
    """-> (status, slot_id, off, cap)."""
    sid, off, cap = _i32(-1), _i64(-1), _i32(0)
    st = lib().s3_kv_restore(arena, int(predicted_len), int(length), _ptr(host_buf), ctypes.byref(sid),
                             ctypes.byref(off), ctypes.byref(cap), stream or None)
    return st, sid.value, off.value, cap.value


def s3_kv_gather_rows(arena, slot_id, length, dev_buf, stream=0):
    return lib().s3_kv_gather_rows(arena, int(slot_id), int(length), _ptr(dev_buf), stream or None)


def s3_kv_scatter_rows(arena, slot_id, length, dev_buf, stream=0):
    return lib().s3_kv_scatter_rows(arena, int(slot_id), int(length), _ptr(dev_buf), stream or None)


def s3_kv_link_copy(dst, src, nbytes, workgroups=16, stream=0):
    return lib().s3_kv_link_copy(_ptr(dst), _ptr(src), int(nbytes), int(workgroups), stream or None)


def s3_sched_create(arena):
    h = _vp()
    st = lib().s3_sched_create(ctypes.byref(h), arena)
    return st, (h if st == S3_OK else None)


def s3_sched_destroy(sched):
    lib().s3_sched_destroy(sched)


def s3_sched_submit(sched, request_id, predicted_len):
    return lib().s3_sched_submit(sched, int(request_id), int(predicted_len))


def s3_sched_admit(sched, max_out):
    """-> (admitted or status, request_id[], slot_id[], slot_off[], slot_cap[]) trimmed to the admitted ones."""
    rid = np.zeros(max_out, np.int64)
    sid = np.zeros(max_out, np.int32)
    off = np.zeros(max_out, np.int64)
    cap = np.zeros(max_out, np.int32)
    rc = lib().s3_sched_admit(sched, int(max_out), rid.ctypes.data_as(_pi64), sid.ctypes.data_as(_pi32),
                              off.ctypes.data_as(_pi64), cap.ctypes.data_as(_pi32))
    k = max(rc, 0)
    return rc, rid[:k], sid[:k], off[:k], cap[:k]


def s3_sched_pool_size(sched):
    return lib().s3_sched_pool_size(sched)


def s3_kv_stats(arena):
    """-> (status, used, free, largest_free, capacity) in tokens."""
    v = [_i64(0) for _ in range(4)]
    st = lib().s3_kv_stats(arena, *[ctypes.byref(x) for x in v])
    return (st, *[x.value for x in v])


def s3_kv_fill(arena, slot_id, layer, first_row, n_rows, k_rows, v_rows, stream=0):
    return lib().s3_kv_fill(arena, int(slot_id), int(layer), int(first_row), int(n_rows), _ptr(k_rows), _ptr(v_rows),
                            stream or None)


def s3_kv_fill_batch(arena, layer, slot_ids, n_rows, k_rows, v_rows, stream=0, slot_off=None, length=None, batch_n=0,
                     batch_idx=None):
    """k_rows / v_rows: sequences of device tensors (or addresses), one per newcomer."""
    s_arr, sp = _host_i32(slot_ids)
    r_arr, rp = _host_i32(n_rows)
    n = int(s_arr.size)
    kp = (_vp * max(n, 1))(*[_ptr(t) for t in k_rows])
    vp = (_vp * max(n, 1))(*[_ptr(t) for t in v_rows])
    if batch_idx is not None:
        b_arr, bp = _host_i32(batch_idx)
    else:
        b_arr, bp = None, None
    return lib().s3_kv_fill_batch(arena, int(layer), n, sp, rp, kp, vp, int(batch_n), _ptr(slot_off), _ptr(length), bp,
                                  stream or None)


def s3_kv_batch_patch(n, slot_off, length, idx, new_off, new_len, stream=0):
    i_arr, ip = _host_i32(idx)
    o_arr = np.ascontiguousarray(new_off, np.int64) if new_off is not None else None
    l_arr, lp = _host_i32(new_len)
    op = o_arr.ctypes.data_as(_pi64) if o_arr is not None else None
    return lib().s3_kv_batch_patch(int(n), _ptr(slot_off), _ptr(length), int(i_arr.size), ip, op, lp, stream or None)


def s3_kv_read_rows(arena, slot_id, layer, which, first_row, n_rows, dst, stream=0):
    return lib().s3_kv_read_rows(arena, int(slot_id), int(layer), int(which), int(first_row), int(n_rows), _ptr(dst),
                                 stream or None)


def s3_kv_probe_bandwidth(arena, nbytes, mode=0, reps=10):
    """-> (status, GB/s) of a plain streaming read (mode 0) or copy (mode 1) over the arena's first bytes."""
    g = ctypes.c_double(0.0)
    st = lib().s3_kv_probe_bandwidth(arena, int(nbytes), int(mode), int(reps), ctypes.byref(g))
    return st, g.value


def s3_kv_set_param(arena, name, value):
    return lib().s3_kv_set_param(arena, name.encode(), int(value))


def s3_kv_get_param(arena, name):
    v = _i64(0)
    st = lib().s3_kv_get_param(arena, name.encode(), ctypes.byref(v))
    return st, v.value


def check(status, where="s3kv"):
    if status < 0:
        raise S3Error(status, where)
    return status
