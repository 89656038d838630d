"""Helpers shared by the tests: build oracle-side pools from a workload, tolerances."""
from __future__ import annotations

import numpy as np

import oracle
from paper_2502_11517_amd import workloads as W


def geom_of(w: W.Workload, head_major: bool = False) -> oracle.Geom:
    return oracle.Geom(w.dtype, w.Hq, w.Hkv, w.D, max_requests=w.max_requests,
                       page_tokens=w.page_tokens, head_major=head_major,
                       n_phys_pages=w.n_phys_pages, pages_per_request=w.pages_per_request,
                       pool_tokens=w.pool_tokens, page_table=w.page_table)


class OraclePool:
    """One layer's K/V pool kept by the oracle, filled event by event."""

    def __init__(self, w: W.Workload, head_major: bool = False):
        self.w = w
        self.g = geom_of(w, head_major)
        self.k = self.g.new_pool()
        self.v = self.g.new_pool()
        self.tail = np.zeros(w.max_requests, np.int64)
        self.n_done = 0

    def append_events(self, hi: int, chunk: int = 8192, positions=None, theta: float = 0.0):
        """positions / theta: rotate the K rows by their position ids before they enter the pool
        (fp64 rotation, one rounding to the pool dtype)."""
        while self.n_done < hi:
            b = min(hi, self.n_done + chunk)
            k, v = self.w.kv_rows(self.n_done, b)
            if positions is not None:
                k = oracle.round_pool(self.w.dtype, oracle.rope(oracle.widen_pool(self.w.dtype, k),
                                                                positions[self.n_done:b], theta))
            rc, slots = oracle.append(self.g, self.k, self.v, self.w.ev_request[self.n_done:b], k, v,
                                      self.tail)
            assert rc == 0
            self.n_done = b
        return self

    def attention(self, step: int = 0, q=None, scale=None):
        pl, offs, st, ct, sd = self.w.lists(step)
        q = self.w.q(step) if q is None else q
        return oracle.attention(self.g, self.k, self.v, self.w.dec_request, pl, offs, st, ct, sd, q,
                                self.w.scale if scale is None else scale)


def to_f64(w_or_dtype, x: np.ndarray) -> np.ndarray:
    dtype = w_or_dtype if isinstance(w_or_dtype, str) else w_or_dtype.dtype
    if dtype == "f32":
        return np.asarray(x, np.float32).astype(np.float64)
    return W.bf16_bits_to_f32(x).astype(np.float64)


def tolerances(dtype: str):
    """(max-abs, relative L2) bounds of the parity bar: bf16 outputs 2e-2 / 1e-2, fp32 1e-5 / 1e-5."""
    return (2e-2, 1e-2) if dtype == "bf16" else (1e-5, 1e-5)


def check_close(got64: np.ndarray, ref64: np.ndarray, dtype: str, what: str = ""):
    """The parity bar, four checks that must all hold (rows = the last axis, one (stream, head) each):
    global max|d| <= atol; global relative L2 <= rtol; relative L2 of EVERY row <= rtol; and element by
    element |d| <= rtol * (max|ref_row| + |ref|) -- the absolute part scaled to the row's magnitude, since
    outputs of long softmaxes are small and a fixed 2e-2 would pass anything there."""
    atol, rtol = tolerances(dtype)
    assert got64.shape == ref64.shape, f"{what}: shape {got64.shape} != {ref64.shape}"
    assert np.all(np.isfinite(got64)), f"{what}: non-finite output"
    d = got64 - ref64
    max_abs = float(np.max(np.abs(d))) if d.size else 0.0
    rel = float(np.linalg.norm(d.ravel()) / max(np.linalg.norm(ref64.ravel()), 1e-300))
    assert max_abs <= atol, f"{what}: max|d|={max_abs:.3e} > {atol}"
    assert rel <= rtol, f"{what}: rel L2={rel:.3e} > {rtol}"
    if d.size:
        D = d.shape[-1]
        d2, r2 = d.reshape(-1, D), ref64.reshape(-1, D)
        row_ref = np.linalg.norm(r2, axis=1)
        row_rel = np.linalg.norm(d2, axis=1) / np.maximum(row_ref, 1e-300)
        row_rel = np.where((row_ref == 0) & (np.linalg.norm(d2, axis=1) == 0), 0.0, row_rel)
        worst = int(np.argmax(row_rel))
        assert row_rel[worst] <= rtol, f"{what}: row {worst} of {len(row_rel)}: rel L2={row_rel[worst]:.3e} > {rtol}"
        bound = rtol * (np.max(np.abs(r2), axis=1, keepdims=True) + np.abs(r2))
        bad = np.abs(d2) > bound
        assert not bad.any(), (f"{what}: {int(bad.sum())} elements beyond rtol*(max|ref_row|+|ref|); first at row "
                               f"{int(np.argwhere(bad)[0][0])} col {int(np.argwhere(bad)[0][1])}")
    return max_abs, rel
