"""Thin ctypes binding of libpasta_attn.so (include/pasta_attn.h): argument marshalling only.

Every step of the path runs in the library's HIP kernels; torch is used for device memory
and the stream.  There is no fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_CSRC = os.path.join(_HERE, "csrc")
_LIB = os.path.join(_HERE, "libpasta_attn.so")
_lib = None

OK, E_INVAL, E_CAPACITY, E_NOMEM, E_DEVICE, E_STATE = 0, -1, -2, -3, -4, -5
F32, BF16 = 0, 1
TOKEN_MAJOR, HEAD_MAJOR = 0, 1
DECODE_PLAN_ONLY, DECODE_NO_MFMA, DECODE_ROPE_Q, DECODE_NO_SHARE, DECODE_DENSE_MASK, DECODE_READ_PROBE = 1, 2, 4, 8, 16, 32
DECODE_PARTIALS_ONLY, DECODE_MERGE_ONLY, DECODE_DEVICE_LISTS, DECODE_ROW_GROUPS, DECODE_FOUR_GROUPS = 64, 128, 256, 512, 1024
APPEND_RESERVE_ONLY, APPEND_DEFER, APPEND_ROPE = 1, 2, 4
SYNC_RETIRE = 1
OP_TEXT, OP_PROMISE, OP_SYNC = 0, 1, 2
REPLAY_PLAN_ONLY, REPLAY_ROPE = 1, 2
_ERR = {E_INVAL: "E_INVAL", E_CAPACITY: "E_CAPACITY", E_NOMEM: "E_NOMEM", E_DEVICE: "E_DEVICE",
        E_STATE: "E_STATE"}

HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


class PastaError(RuntimeError):
    def __init__(self, code, where):
        super().__init__(f"{where}: {_ERR.get(code, code)}")
        self.code = code


def library_path() -> str:
    return _LIB


def build_library(verbose: bool = False) -> str:
    """Compiles csrc/pasta_attn.hip for gfx950 with hipcc (cross-compiles without a GPU)."""
    src = os.path.join(_CSRC, "pasta_attn.hip")
    cmd = ["hipcc", *HIPCC_FLAGS, src, "-o", _LIB]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + r.stderr)
    if verbose:
        print(" ".join(cmd))
    return _LIB


class Config(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32), ("dtype", C.c_int32), ("n_q_heads", C.c_int32),
        ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("n_layers", C.c_int32),
        ("max_requests", C.c_int32), ("page_tokens", C.c_int32), ("kv_layout", C.c_int32),
        ("n_phys_pages", C.c_int32), ("pages_per_request", C.c_int32), ("max_streams", C.c_int32),
        ("max_ranges", C.c_int32), ("softmax_scale", C.c_float), ("rope_theta", C.c_float),
        ("pool_tokens", C.c_int64),
        ("k_pool", C.c_void_p), ("v_pool", C.c_void_p), ("page_table", C.c_void_p),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_uint64), ("hip_stream", C.c_void_p),
    ]


class AppendArgs(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32), ("flags", C.c_uint32), ("layer", C.c_int32), ("n_rows", C.c_int32),
        ("request_id", C.c_void_p), ("stream_id", C.c_void_p), ("parent_stream", C.c_void_p),
        ("position", C.c_void_p), ("k_new", C.c_void_p), ("v_new", C.c_void_p), ("out_slot", C.c_void_p),
    ]


class SyncArgs(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32), ("flags", C.c_uint32), ("request_id", C.c_int32), ("stream_id", C.c_int32),
        ("n_join", C.c_int32), ("join_stream", C.c_void_p),
    ]


class TraceOp(C.Structure):
    _fields_ = [("kind", C.c_int32), ("a", C.c_int32), ("b", C.c_int32)]


class ReplayArgs(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32), ("flags", C.c_uint32), ("request_id", C.c_int32), ("n_ops", C.c_int32),
        ("ops", C.c_void_p), ("first_pos", C.c_int32), ("max_tokens", C.c_int32), ("k_rows", C.c_void_p),
        ("v_rows", C.c_void_p), ("q_rows", C.c_void_p), ("out", C.c_void_p), ("tok_slot", C.c_void_p),
        ("tok_stream", C.c_void_p), ("tok_pos", C.c_void_p), ("tok_pass", C.c_void_p), ("stats", C.c_void_p),
    ]


class DecodeArgs(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32), ("flags", C.c_uint32), ("layer", C.c_int32), ("n_streams", C.c_int32),
        ("request_id", C.c_void_p), ("stream_id", C.c_void_p), ("position", C.c_void_p), ("causal_skip", C.c_void_p),
        ("prefix_len", C.c_void_p), ("range_offsets", C.c_void_p), ("range_start", C.c_void_p),
        ("range_count", C.c_void_p), ("range_stride", C.c_void_p), ("q", C.c_void_p), ("out", C.c_void_p),
        ("out_lse", C.c_void_p), ("dbg_gather_offsets", C.c_void_p), ("dbg_gather_rows", C.c_void_p),
        ("dbg_plan", C.c_void_p), ("dbg_part_ml", C.c_void_p), ("dbg_part_acc", C.c_void_p),
        ("prof_event_start", C.c_void_p), ("prof_event_stop", C.c_void_p),
    ]


def load_library():
    """Loads the built library; raises if it is missing (there is no other path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            raise RuntimeError(f"{_LIB} is not built: run __graft_entry__.build() (hipcc, gfx950)")
        # torch bundles its own HIP runtime under the same SONAME as /opt/rocm's; importing it
        # first makes the loader bind this library to THAT runtime, so that torch's stream and
        # device pointers are valid in the calls below (two runtimes in one process are not).
        import torch  # noqa: F401
        L = C.CDLL(_LIB)
        L.pasta_attn_create.restype = C.c_int32
        L.pasta_attn_create.argtypes = [C.POINTER(Config), C.POINTER(C.c_void_p)]
        L.pasta_attn_append_kv.restype = C.c_int32
        L.pasta_attn_append_kv.argtypes = [C.c_void_p, C.POINTER(AppendArgs)]
        L.pasta_attn_decode_step.restype = C.c_int32
        L.pasta_attn_decode_step.argtypes = [C.c_void_p, C.POINTER(DecodeArgs)]
        L.pasta_attn_decode_step_noalloc.restype = C.c_int32
        L.pasta_attn_decode_step_noalloc.argtypes = [C.c_void_p, C.POINTER(DecodeArgs)]
        L.pasta_attn_sync.restype = C.c_int32
        L.pasta_attn_sync.argtypes = [C.c_void_p, C.POINTER(SyncArgs)]
        L.pasta_attn_stream_list.restype = C.c_int32
        L.pasta_attn_stream_list.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32,
                                             C.c_void_p, C.c_void_p, C.c_void_p]
        L.pasta_attn_replay.restype = C.c_int32
        L.pasta_attn_replay.argtypes = [C.c_void_p, C.POINTER(ReplayArgs)]
        L.pasta_attn_destroy.restype = C.c_int32
        L.pasta_attn_destroy.argtypes = [C.c_void_p]
        _lib = L
    return _lib


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _hp(a):
    return None if a is None else a.ctypes.data


def _dp(t):
    return None if t is None else (t if isinstance(t, int) else t.data_ptr())


def make_config(dtype, n_q_heads, n_kv_heads, head_dim, softmax_scale, *, n_layers=1, max_requests=1,
                page_tokens=0, kv_layout=TOKEN_MAJOR, n_phys_pages=0, pages_per_request=0,
                max_streams=2, max_ranges=1024, pool_tokens=0, rope_theta=0.0) -> Config:
    c = Config()
    c.struct_size = C.sizeof(Config)
    c.dtype = {"f32": F32, "bf16": BF16}.get(dtype, dtype)
    c.n_q_heads, c.n_kv_heads, c.head_dim = n_q_heads, n_kv_heads, head_dim
    c.n_layers, c.max_requests, c.page_tokens, c.kv_layout = n_layers, max_requests, page_tokens, kv_layout
    c.n_phys_pages, c.pages_per_request = n_phys_pages, pages_per_request
    c.max_streams, c.max_ranges, c.softmax_scale, c.pool_tokens = max_streams, max_ranges, softmax_scale, pool_tokens
    c.rope_theta = rope_theta
    return c


def query_workspace_bytes(cfg: Config) -> int:
    rc = load_library().pasta_attn_create(C.byref(cfg), None)
    if rc != OK:
        raise PastaError(rc, "pasta_attn_create(query)")
    return int(cfg.workspace_bytes)


class PastaAttn:
    """One handle.  `k_pool`, `v_pool`, `workspace` are device addresses (or torch tensors) owned
    by the caller; `stream` is a hipStream_t as an int (torch.cuda.current_stream().cuda_stream)."""

    def __init__(self, cfg: Config, k_pool, v_pool, workspace, workspace_bytes, stream=0, page_table=None):
        self._lib = load_library()
        self.cfg = cfg
        self._keep = [k_pool, v_pool, workspace]
        pt = _i32(page_table)
        cfg.k_pool, cfg.v_pool, cfg.workspace = _dp(k_pool), _dp(v_pool), _dp(workspace)
        cfg.workspace_bytes = workspace_bytes
        cfg.hip_stream = stream
        cfg.page_table = _hp(pt)
        h = C.c_void_p()
        rc = self._lib.pasta_attn_create(C.byref(cfg), C.byref(h))
        if rc != OK:
            raise PastaError(rc, "pasta_attn_create")
        self._h = h

    def append_kv(self, layer, request_id, stream_id, k_new, v_new, parent_stream=None, position=None,
                  want_slots=False, flags=0):
        rid, sid, par, pos = _i32(request_id), _i32(stream_id), _i32(parent_stream), _i32(position)
        n = 0 if rid is None else int(rid.shape[0])
        slots = np.full(n, -1, np.int32) if want_slots else None
        a = AppendArgs(C.sizeof(AppendArgs), flags, layer, n, _hp(rid), _hp(sid), _hp(par), _hp(pos), _dp(k_new),
                       _dp(v_new), _hp(slots))
        rc = self._lib.pasta_attn_append_kv(self._h, C.byref(a))
        if rc != OK:
            raise PastaError(rc, "pasta_attn_append_kv")
        return slots

    def decode_step_noalloc(self, *args, **kw):
        """The same step through the entry point that allocates nothing (partials in the library's
        static device array); same arguments as decode_step."""
        return self.decode_step(*args, _entry="pasta_attn_decode_step_noalloc", **kw)

    def decode_step(self, layer, request_id, stream_id, q, out, *, lists=None, out_lse=None, flags=0,
                    position=None, dbg_gather_offsets=None, dbg_gather_rows=None, dbg_plan=None,
                    prof_events=None, causal_skip=None, dbg_partials=None, _entry="pasta_attn_decode_step"):
        """lists = (prefix_len, range_offsets, start, count, stride) for explicit visibility;
        None uses the lists append_kv has maintained."""
        rid, sid, pos, skip = _i32(request_id), _i32(stream_id), _i32(position), _i32(causal_skip)
        n = int(rid.shape[0])
        if lists is not None:
            pl, offs, st, ct, sd = (_i32(x) for x in lists)
            if st.size == 0:  # keep valid addresses for empty arrays
                st = ct = sd = np.zeros(1, np.int32)
        else:
            pl = offs = st = ct = sd = None
        ev0, ev1 = prof_events if prof_events is not None else (None, None)
        pml, pacc = dbg_partials if dbg_partials is not None else (None, None)
        a = DecodeArgs(C.sizeof(DecodeArgs), flags, layer, n, _hp(rid), _hp(sid), _hp(pos), _hp(skip), _hp(pl), _hp(offs),
                       _hp(st), _hp(ct), _hp(sd), _dp(q), _dp(out), _dp(out_lse), _hp(dbg_gather_offsets),
                       _dp(dbg_gather_rows), _hp(dbg_plan), _dp(pml), _dp(pacc), ev0, ev1)
        rc = getattr(self._lib, _entry)(self._h, C.byref(a))
        if rc != OK:
            raise PastaError(rc, _entry)

    # ---- prepared calls: marshal once, call many times (tight serving loops) ----
    def prepare_append(self, layer, request_id, stream_id, k_new, v_new, parent_stream=None, flags=0,
                       position=None):
        """Returns f() -> status that issues this exact append; arrays are kept alive by f."""
        rid, sid, par, pos = _i32(request_id), _i32(stream_id), _i32(parent_stream), _i32(position)
        a = AppendArgs(C.sizeof(AppendArgs), flags, layer, int(rid.shape[0]), _hp(rid), _hp(sid), _hp(par),
                       _hp(pos), _dp(k_new), _dp(v_new), None)
        fn, h, ref = self._lib.pasta_attn_append_kv, self._h, C.byref(a)

        def call(_keep=(rid, sid, par, pos, a, k_new, v_new)):
            return fn(h, ref)
        return call

    def prepare_decode(self, layer, request_id, stream_id, q, out, *, lists=None, out_lse=None, flags=0,
                       prof_events=None, position=None):
        rid, sid, pos = _i32(request_id), _i32(stream_id), _i32(position)
        if lists is not None:
            pl, offs, st, ct, sd = (_i32(x) for x in lists)
            if st.size == 0:
                st = ct = sd = np.zeros(1, np.int32)
        else:
            pl = offs = st = ct = sd = None
        ev0, ev1 = prof_events if prof_events is not None else (None, None)
        a = DecodeArgs(C.sizeof(DecodeArgs), flags, layer, int(rid.shape[0]), _hp(rid), _hp(sid), _hp(pos), None, _hp(pl),
                       _hp(offs), _hp(st), _hp(ct), _hp(sd), _dp(q), _dp(out), _dp(out_lse), None, None, None,
                       None, None, ev0, ev1)
        fn, h, ref = self._lib.pasta_attn_decode_step, self._h, C.byref(a)

        def call(_keep=(rid, sid, pos, pl, offs, st, ct, sd, a, q, out, out_lse)):
            return fn(h, ref)
        return call

    def sync(self, request_id, stream_id, join_streams, retire=False):
        """stream_id (or -1: retire only) from now on also sees what join_streams see."""
        js = _i32(join_streams)
        a = SyncArgs(C.sizeof(SyncArgs), SYNC_RETIRE if retire else 0, request_id, stream_id, int(js.shape[0]), _hp(js))
        rc = self._lib.pasta_attn_sync(self._h, C.byref(a))
        if rc != OK:
            raise PastaError(rc, "pasta_attn_sync")

    def stream_list(self, request_id, stream_id):
        """(prefix_len, start[], count[], stride[]) of the maintained list of an open stream."""
        pl, nr = C.c_int32(), C.c_int32()
        rc = self._lib.pasta_attn_stream_list(self._h, request_id, stream_id, C.addressof(pl), C.addressof(nr), 0,
                                              None, None, None)
        if rc != OK:
            raise PastaError(rc, "pasta_attn_stream_list")
        n = max(nr.value, 1)
        st, ct, sd = np.zeros(n, np.int32), np.zeros(n, np.int32), np.zeros(n, np.int32)
        rc = self._lib.pasta_attn_stream_list(self._h, request_id, stream_id, C.addressof(pl), C.addressof(nr), n,
                                              _hp(st), _hp(ct), _hp(sd))
        if rc != OK:
            raise PastaError(rc, "pasta_attn_stream_list")
        return pl.value, st[:nr.value], ct[:nr.value], sd[:nr.value]

    def replay(self, request_id, ops, first_pos, max_tokens, k_rows=None, v_rows=None, q_rows=None, out=None,
               flags=0):
        """ops: sequence of (kind, a, b).  Returns dict(slot, stream, pos, pass_, stats) -- host arrays
        cut to the rows fed.  Without device buffers pass flags=REPLAY_PLAN_ONLY."""
        arr = (TraceOp * max(len(ops), 1))(*[TraceOp(int(k), int(x), int(y)) for k, x, y in ops])
        slot, stream, pos, pas = (np.full(max_tokens, -1, np.int32) for _ in range(4))
        stats = np.zeros(8, np.int64)
        a = ReplayArgs(C.sizeof(ReplayArgs), flags, request_id, len(ops), C.addressof(arr), first_pos, max_tokens,
                       _dp(k_rows), _dp(v_rows), _dp(q_rows), _dp(out), _hp(slot), _hp(stream), _hp(pos), _hp(pas),
                       _hp(stats))
        rc = self._lib.pasta_attn_replay(self._h, C.byref(a))
        if rc != OK:
            raise PastaError(rc, "pasta_attn_replay")
        n = int(stats[0])
        return dict(slot=slot[:n], stream=stream[:n], pos=pos[:n], pass_=pas[:n], stats=stats)

    def destroy(self):
        if self._h is not None:
            self._lib.pasta_attn_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass
