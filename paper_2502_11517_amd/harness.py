"""Device-memory plumbing around the C-ABI library for tests and the bench: torch allocates the
pool, the workspace, Q and the outputs and provides the stream; nothing here computes."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B
from .workloads import Workload


def _torch_dtype(dtype: str):
    return torch.float32 if dtype == "f32" else torch.bfloat16


def to_device(arr: np.ndarray, dtype: str, device) -> torch.Tensor:
    """numpy float32 / bf16-bit-pattern array -> device tensor of the pool dtype (bit exact)."""
    if dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(arr, np.float32)).to(device)
    return torch.from_numpy(np.ascontiguousarray(arr, np.uint16).view(np.int16)).to(device).view(torch.bfloat16)


def to_host_bits(t: torch.Tensor, dtype: str) -> np.ndarray:
    """device tensor -> numpy float32, or uint16 bf16 bit patterns."""
    if dtype == "f32":
        return t.detach().cpu().numpy()
    return t.detach().view(torch.int16).cpu().numpy().view(np.uint16)


class Session:
    """A handle plus the device buffers it borrows, shaped after a Workload."""

    def __init__(self, w: Workload, *, kv_layout=B.TOKEN_MAJOR, n_layers=1, device="cuda:0",
                 max_ranges=None, max_streams=None, rope_theta=0.0):
        self.w, self.device, self.n_layers, self.kv_layout = w, torch.device(device), n_layers, kv_layout
        torch.cuda.set_device(self.device)
        if max_ranges is None:
            max_ranges = min(max(1024, len(w.ev_stream) + 64), 1 << 20)  # worst case: one per token
        self.cfg = B.make_config(w.dtype, w.Hq, w.Hkv, w.D, w.scale, n_layers=n_layers,
                                 max_requests=w.max_requests, page_tokens=w.page_tokens,
                                 kv_layout=kv_layout, n_phys_pages=w.n_phys_pages,
                                 pages_per_request=w.pages_per_request,
                                 max_streams=max_streams or w.max_streams, max_ranges=max_ranges,
                                 pool_tokens=w.pool_tokens, rope_theta=rope_theta)
        ws_bytes = B.query_workspace_bytes(self.cfg)
        rows = (w.n_phys_pages * w.page_tokens) if w.page_tokens else w.max_requests * w.pool_tokens
        self.rows_per_layer = rows
        td = _torch_dtype(w.dtype)
        # uninitialised on purpose: the library must never read a row that was not appended
        self.k_pool = torch.empty(n_layers * rows * w.Hkv * w.D, dtype=td, device=self.device)
        self.v_pool = torch.empty_like(self.k_pool)
        self.workspace = torch.empty(ws_bytes + 256, dtype=torch.uint8, device=self.device)
        ws_ptr = (self.workspace.data_ptr() + 255) // 256 * 256
        self.stream = torch.cuda.current_stream(self.device)
        self.h = B.PastaAttn(self.cfg, self.k_pool, self.v_pool, ws_ptr, ws_bytes,
                             stream=self.stream.cuda_stream, page_table=w.page_table)
        self.n_done = 0

    def append_events(self, hi: int, layer: int = 0, chunk: int = 8192, lo: int | None = None, flags: int = 0,
                      positions=None):
        """Appends events [n_done, hi) of the workload's history (K/V rows from the generator);
        positions: position id per event of the history (for flags with APPEND_ROPE)."""
        w = self.w
        pos = self.n_done if lo is None else lo
        while pos < hi:
            b = min(hi, pos + chunk)
            k, v = w.kv_rows(pos, b)
            kd, vd = to_device(k, w.dtype, self.device), to_device(v, w.dtype, self.device)
            self._keep_rows = (kd, vd)  # a deferred append reads them later
            self.h.append_kv(layer, w.ev_request[pos:b], w.ev_stream[pos:b], kd, vd,
                             parent_stream=w.ev_parent[pos:b], flags=flags,
                             position=None if positions is None else positions[pos:b])
            pos = b
        if layer == 0 and lo is None:
            self.n_done = hi
        return self

    def decode(self, step: int = 0, *, layer: int = 0, explicit: bool = True, q=None, flags=0,
               want_lse=True, want_gather=False, position=None):
        w = self.w
        q = w.q(step) if q is None else q
        qd = to_device(q, w.dtype, self.device)
        out = torch.empty_like(qd)
        lse = torch.empty(w.n, w.Hq, dtype=torch.float32, device=self.device) if want_lse else None
        lists = w.lists(step) if explicit else None
        goffs = grows = None
        if want_gather:
            goffs = np.zeros(w.n + 1, np.int64)
            plan = np.zeros(8, np.int64)
            self.h.decode_step(layer, w.dec_request, w.dec_stream, qd, out, lists=lists,
                               flags=flags | B.DECODE_PLAN_ONLY, dbg_gather_offsets=goffs, dbg_plan=plan,
                               position=position)
            grows = torch.full((int(goffs[-1]),), -1, dtype=torch.int32, device=self.device)
        self.h.decode_step(layer, w.dec_request, w.dec_stream, qd, out, lists=lists, out_lse=lse, flags=flags,
                           dbg_gather_offsets=goffs, dbg_gather_rows=grows, position=position)
        return out, lse, (goffs, grows)

    def pool_bits(self, layer: int = 0):
        """(K, V) of one layer as flat numpy arrays (float32 or bf16 bit patterns)."""
        n = self.rows_per_layer * self.w.Hkv * self.w.D
        k = self.k_pool[layer * n:(layer + 1) * n]
        v = self.v_pool[layer * n:(layer + 1) * n]
        return to_host_bits(k, self.w.dtype), to_host_bits(v, self.w.dtype)

    def close(self):
        torch.cuda.synchronize(self.device)
        self.h.destroy()
