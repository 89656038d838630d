"""ctypes binding of oracle/pasta_oracle.c (TEST INFRASTRUCTURE; see the C file's header).

Pools, K/V rows and Q are numpy arrays: float32 for the fp32 pool, uint16 holding bf16 bit
patterns for the bf16 pool.  Outputs are float64.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pasta_oracle.c")
_LIB = os.path.join(_HERE, "libpasta_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (fp64, OpenMP). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-Wall", "-Wextra",
               _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _CGeom(C.Structure):
    _fields_ = [
        ("dtype", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
        ("head_dim", C.c_int32), ("max_requests", C.c_int32), ("page_tokens", C.c_int32),
        ("head_major", C.c_int32), ("n_phys_pages", C.c_int32), ("pages_per_request", C.c_int32),
        ("pad_", C.c_int32), ("pool_tokens", C.c_int64), ("page_table", C.c_void_p),
    ]


def _load():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        P = C.c_void_p
        L.oracle_num_threads.restype = C.c_int
        L.oracle_rows_per_layer.restype = C.c_int64
        L.oracle_rows_per_layer.argtypes = [P]
        L.oracle_phys_row.restype = C.c_int64
        L.oracle_phys_row.argtypes = [P, C.c_int32, C.c_int64]
        L.oracle_elem_offset.restype = C.c_int64
        L.oracle_elem_offset.argtypes = [P, C.c_int64, C.c_int32]
        L.oracle_append.restype = C.c_int
        L.oracle_append.argtypes = [P, P, P, C.c_int32, P, P, P, P, P]
        L.oracle_gather_map.restype = C.c_int64
        L.oracle_gather_map.argtypes = [P, C.c_int32, C.c_int32, C.c_int32, P, P, P, P]
        L.oracle_attention.restype = C.c_int
        L.oracle_attention.argtypes = [P, P, P, C.c_int32, P, P, P, P, P, P, P, C.c_double, P, P]
        L.oracle_attention_q64.restype = C.c_int
        L.oracle_attention_q64.argtypes = [P, P, P, C.c_int32, P, P, P, P, P, P, P, C.c_double, P, P]
        L.oracle_rope.restype = None
        L.oracle_rope.argtypes = [P, C.c_int64, C.c_int32, C.c_int32, P, C.c_double, P]
        L.oracle_round_pool.restype = None
        L.oracle_round_pool.argtypes = [P, C.c_int64, C.c_int32, P]
        L.oracle_visible_events.restype = C.c_int
        L.oracle_visible_events.argtypes = [C.c_int64, P, P, P, P, P, C.c_int32, C.c_int64, P]
        L.oracle_partial.restype = C.c_int
        L.oracle_partial.argtypes = [P, P, P, C.c_int64, P, P, C.c_int32, C.c_double, P, P, P]
        L.oracle_merge.restype = C.c_int
        L.oracle_merge.argtypes = [C.c_int32, C.c_int32, P, P, P, P, P]
        L.oracle_visible_dense.restype = C.c_int
        L.oracle_visible_dense.argtypes = [C.c_int64, P, C.c_int32, P, P, C.c_int32, P]
        L.oracle_attention_dense.restype = C.c_int
        L.oracle_attention_dense.argtypes = [P, P, P, C.c_int32, C.c_int64, P, P, C.c_double, P, P]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


class Geom:
    """Shape and pool layout of one handle, as the oracle sees it."""

    def __init__(self, dtype, n_q_heads, n_kv_heads, head_dim, max_requests=1, page_tokens=0,
                 head_major=False, n_phys_pages=0, pages_per_request=0, pool_tokens=0,
                 page_table=None):
        assert dtype in ("f32", "bf16")
        self.dtype = dtype
        self.np_dtype = np.float32 if dtype == "f32" else np.uint16
        self.Hq, self.Hkv, self.D = n_q_heads, n_kv_heads, head_dim
        self.page_table = None if page_table is None else _i32(page_table).reshape(
            max_requests, pages_per_request)
        self.c = _CGeom(0 if dtype == "f32" else 1, n_q_heads, n_kv_heads, head_dim, max_requests,
                        page_tokens, 1 if head_major else 0, n_phys_pages, pages_per_request, 0,
                        pool_tokens, None if self.page_table is None else self.page_table.ctypes.data)
        self.max_requests = max_requests

    @property
    def ref(self):
        return C.addressof(self.c)

    def rows_per_layer(self):
        return rows_per_layer(self)

    def new_pool(self):
        """Zero-filled K (or V) pool of one layer, flat."""
        return np.zeros(self.rows_per_layer() * self.Hkv * self.D, dtype=self.np_dtype)


def num_threads() -> int:
    return _load().oracle_num_threads()


def rows_per_layer(g: Geom) -> int:
    return _load().oracle_rows_per_layer(g.ref)


def phys_row(g: Geom, req: int, slot: int) -> int:
    return _load().oracle_phys_row(g.ref, req, slot)


def elem_offset(g: Geom, phys: int, head: int) -> int:
    return _load().oracle_elem_offset(g.ref, phys, head)


def append(g: Geom, k_pool, v_pool, request_id, k_new, v_new, tail):
    """Appends rows in call order; tail (int64 [max_requests]) is updated in place.
    Returns (status, slots)."""
    request_id = _i32(request_id)
    n = request_id.shape[0]
    k_new = np.ascontiguousarray(k_new, dtype=g.np_dtype)
    v_new = np.ascontiguousarray(v_new, dtype=g.np_dtype)
    assert k_new.size == n * g.Hkv * g.D and v_new.size == k_new.size
    assert tail.dtype == np.int64 and tail.shape[0] == g.max_requests
    slots = np.full(n, -1, dtype=np.int32)
    rc = _load().oracle_append(g.ref, _p(k_pool), _p(v_pool), n, _p(request_id), _p(k_new), _p(v_new),
                               _p(tail), _p(slots))
    return rc, slots


def gather_map(g: Geom, req, prefix_len, start, count, stride):
    start, count, stride = _i32(start), _i32(count), _i32(stride)
    n = _load().oracle_gather_map(g.ref, req, prefix_len, start.shape[0], _p(start), _p(count),
                                  _p(stride), None)
    if n < 0:
        raise ValueError("slot outside the request's pool")
    rows = np.empty(n, dtype=np.int64)
    _load().oracle_gather_map(g.ref, req, prefix_len, start.shape[0], _p(start), _p(count), _p(stride),
                              _p(rows))
    return rows


def attention(g: Geom, k_pool, v_pool, request_id, prefix_len, range_offsets, range_start, range_count,
              range_stride, q, scale):
    """Returns (out [n][Hq][D] float64, lse [n][Hq] float64)."""
    request_id, prefix_len, range_offsets = _i32(request_id), _i32(prefix_len), _i32(range_offsets)
    rs, rc_, rst = _i32(range_start), _i32(range_count), _i32(range_stride)
    n = request_id.shape[0]
    q = np.ascontiguousarray(q, dtype=g.np_dtype)
    assert q.size == n * g.Hq * g.D
    out = np.empty((n, g.Hq, g.D), dtype=np.float64)
    lse = np.empty((n, g.Hq), dtype=np.float64)
    rc = _load().oracle_attention(g.ref, _p(k_pool), _p(v_pool), n, _p(request_id), _p(prefix_len),
                                  _p(range_offsets), _p(rs), _p(rc_), _p(rst), _p(q), float(scale),
                                  _p(out), _p(lse))
    if rc != 0:
        raise ValueError(f"oracle_attention failed: {rc}")
    return out, lse


def attention_q64(g: Geom, k_pool, v_pool, request_id, prefix_len, range_offsets, range_start, range_count,
                  range_stride, q64, scale):
    """attention() with the queries given in float64 (rotated queries)."""
    request_id, prefix_len, range_offsets = _i32(request_id), _i32(prefix_len), _i32(range_offsets)
    rs, rc_, rst = _i32(range_start), _i32(range_count), _i32(range_stride)
    n = request_id.shape[0]
    q = np.ascontiguousarray(q64, dtype=np.float64)
    assert q.size == n * g.Hq * g.D
    out = np.empty((n, g.Hq, g.D), dtype=np.float64)
    lse = np.empty((n, g.Hq), dtype=np.float64)
    rc = _load().oracle_attention_q64(g.ref, _p(k_pool), _p(v_pool), n, _p(request_id), _p(prefix_len),
                                      _p(range_offsets), _p(rs), _p(rc_), _p(rst), _p(q), float(scale),
                                      _p(out), _p(lse))
    if rc != 0:
        raise ValueError(f"oracle_attention_q64 failed: {rc}")
    return out, lse


def rope(x, positions, theta):
    """x: [n_rows][n_heads][D] (any float dtype, taken as float64); returns the rotated rows, float64."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    pos = _i32(positions)
    assert x.ndim == 3 and pos.shape[0] == x.shape[0] and x.shape[2] % 2 == 0
    out = np.empty_like(x)
    _load().oracle_rope(_p(x), x.shape[0], x.shape[1], x.shape[2], _p(pos), float(theta), _p(out))
    return out


def round_pool(dtype, x):
    """float64 -> pool dtype with one rounding to nearest even: float32, or uint16 bf16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    code = {"f32": 0, "bf16": 1}[dtype]
    out = np.empty(x.shape, dtype=np.float32 if code == 0 else np.uint16)
    _load().oracle_round_pool(_p(x), x.size, code, _p(out))
    return out


def widen_pool(dtype, x):
    """pool dtype (float32, or uint16 bf16 bit patterns) -> float64, exact."""
    if dtype == "f32":
        return np.asarray(x, dtype=np.float32).astype(np.float64)
    return (np.asarray(x, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def partial(g: Geom, k_pool, v_pool, phys_rows, q_row, kv_head, scale):
    """(m, l, acc[D]) over a subset of physical rows for one query row (D elements)."""
    rows = np.ascontiguousarray(phys_rows, dtype=np.int64)
    q_row = np.ascontiguousarray(q_row, dtype=g.np_dtype)
    assert q_row.size == g.D
    m, l = C.c_double(), C.c_double()
    acc = np.empty(g.D, dtype=np.float64)
    rc = _load().oracle_partial(g.ref, _p(k_pool), _p(v_pool), rows.shape[0], _p(rows), _p(q_row),
                                kv_head, float(scale), C.byref(m), C.byref(l), _p(acc))
    if rc != 0:
        raise ValueError(f"oracle_partial failed: {rc}")
    return m.value, l.value, acc


def merge(m, l, acc):
    """Log-sum-exp merge of partials: returns (out[D], lse)."""
    m = np.ascontiguousarray(m, dtype=np.float64)
    l = np.ascontiguousarray(l, dtype=np.float64)
    acc = np.ascontiguousarray(acc, dtype=np.float64)
    k, D = acc.shape
    out = np.empty(D, dtype=np.float64)
    lse = C.c_double()
    rc = _load().oracle_merge(k, D, _p(m), _p(l), _p(acc), _p(out), C.byref(lse))
    if rc != 0:
        raise ValueError("merge of empty partials")
    return out, lse.value


def visible_dense(slot_stream, stream_parent, stream_spawn_tail, query_stream):
    """0/1 mask over the request's slots from the fork history alone (ancestor rule)."""
    slot_stream = _i32(slot_stream)
    stream_parent = _i32(stream_parent)
    spawn = np.ascontiguousarray(stream_spawn_tail, dtype=np.int64)
    mask = np.zeros(slot_stream.shape[0], dtype=np.uint8)
    rc = _load().oracle_visible_dense(slot_stream.shape[0], _p(slot_stream), stream_parent.shape[0],
                                      _p(stream_parent), _p(spawn), query_stream, _p(mask))
    if rc != 0:
        raise ValueError("bad fork tree")
    return mask


def visible_events(ev_stream, ev_parent, ev_new, joins, q_slot):
    """Figure 2b's reachability with synchronisation: joins[t] = thread ids whose latest tokens
    get an edge into slot t (a sync token); ev_new[t] = 1 on a thread's first token.
    Returns a 0/1 mask over the slots (q_slot itself included)."""
    ev_stream, ev_parent = _i32(ev_stream), _i32(ev_parent)
    ev_new = np.ascontiguousarray(ev_new, dtype=np.uint8)
    n = ev_stream.shape[0]
    offs = np.zeros(n + 1, np.int32)
    flat = []
    for t in range(n):
        flat += list(joins[t]) if joins is not None and t in joins else []
        offs[t + 1] = len(flat)
    flat = _i32(flat if flat else [0])
    mask = np.zeros(n, np.uint8)
    rc = _load().oracle_visible_events(n, _p(ev_stream), _p(ev_parent), _p(ev_new), _p(offs), _p(flat),
                                       int(ev_stream.max()) + 1, int(q_slot), _p(mask))
    if rc != 0:
        raise ValueError(f"oracle_visible_events failed: {rc}")
    return mask


def attention_dense(g: Geom, k_pool, v_pool, req, mask, q_row, scale):
    """Brute force over all slots with masked logits at -inf. q_row: [Hq][D]."""
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    q_row = np.ascontiguousarray(q_row, dtype=g.np_dtype)
    out = np.empty((g.Hq, g.D), dtype=np.float64)
    lse = np.empty(g.Hq, dtype=np.float64)
    rc = _load().oracle_attention_dense(g.ref, _p(k_pool), _p(v_pool), req, mask.shape[0], _p(mask),
                                        _p(q_row), float(scale), _p(out), _p(lse))
    if rc != 0:
        raise ValueError(f"oracle_attention_dense failed: {rc}")
    return out, lse
