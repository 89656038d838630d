"""The entry point that allocates nothing (pasta_attn_decode_step_noalloc): same results as
pasta_attn_decode_step, two calls in a row, the second with a smaller input; its refusals."""
from __future__ import annotations

import numpy as np
import pytest
import torch

from paper_2502_11517_amd import binding as B
from paper_2502_11517_amd import workloads as W
from util import OraclePool, check_close, to_f64

pytestmark = pytest.mark.gpu


def _bits(w, t):
    from paper_2502_11517_amd.harness import to_host_bits
    torch.cuda.synchronize()
    return to_host_bits(t, w.dtype)


def _both(w, s, step, lists):
    """One step through both entry points; returns (existing, noalloc) outputs and lse."""
    from paper_2502_11517_amd.harness import to_device
    qd = to_device(w.q(step), w.dtype, s.device)
    outs = []
    for fn in (s.h.decode_step, s.h.decode_step_noalloc):
        out = torch.full_like(qd, float("nan"))
        lse = torch.full((w.n, w.Hq), float("nan"), dtype=torch.float32, device=s.device)
        fn(0, w.dec_request, w.dec_stream, qd, out, lists=lists, out_lse=lse)
        outs.append((_bits(w, out), lse.cpu().numpy()))
    return outs


def test_noalloc_matches_decode_step_on_two_calls_the_second_smaller():
    from paper_2502_11517_amd.harness import Session
    big = W.config3(steps=2)                       # 8 streams, prefix 8192: 8.9k partial rows
    small = W.config3(steps=2, prefix=700, n_streams=3)
    for w in (big, small):                         # a larger step first, then a smaller one over the same scratch
        s = Session(w, kv_layout=B.HEAD_MAJOR)
        op = OraclePool(w, head_major=True)
        s.append_events(w.n_prefill)
        op.append_events(w.n_prefill)
        for step in range(2):
            hi = w.n_events(step)
            s.append_events(hi, chunk=w.n)
            op.append_events(hi)
            for lists in (None, w.lists(step)):    # maintained and explicit visibility
                (o_ref, l_ref), (o_na, l_na) = _both(w, s, step, lists)
                # same kernels, same plan: the two entry points must agree bit for bit ...
                assert np.array_equal(o_ref, o_na), f"{w.name} step {step}: outputs differ"
                assert np.array_equal(l_ref, l_na)
                # ... and with the oracle to the parity bar
                ref, ref_lse = op.attention(step)
                check_close(to_f64(w, o_na), ref, w.dtype, f"noalloc {w.name} step {step}")
                assert np.max(np.abs(l_na - ref_lse)) <= 2e-2
        s.close()


def test_noalloc_with_a_deferred_append_riding_along():
    from paper_2502_11517_amd.harness import Session, to_device
    w = W.config3(steps=3, prefix=1500, n_streams=5)
    s = Session(w, kv_layout=B.HEAD_MAJOR)
    op = OraclePool(w, head_major=True)
    s.append_events(w.n_prefill)
    op.append_events(w.n_prefill)
    keep = []
    for step in range(3):
        hi = w.n_events(step)
        s.append_events(hi, chunk=w.n, flags=B.APPEND_DEFER)
        keep.append(s._keep_rows)
        op.append_events(hi)
        qd = to_device(w.q(step), w.dtype, s.device)
        out = torch.empty_like(qd)
        s.h.decode_step_noalloc(0, w.dec_request, w.dec_stream, qd, out)
        ref, _ = op.attention(step)
        check_close(to_f64(w, _bits(w, out)), ref, w.dtype, f"noalloc deferred step {step}")
    s.close()


def test_noalloc_refusals():
    from paper_2502_11517_amd.harness import Session, to_device
    w = W.config3(steps=1, prefix=300, n_streams=2)
    s = Session(w)
    qd = to_device(w.q(0), w.dtype, s.device)
    out = torch.empty_like(qd)
    with pytest.raises(B.PastaError) as e:         # no append yet: the handle has not been set up on the device
        s.h.decode_step_noalloc(0, w.dec_request, w.dec_stream, qd, out, lists=w.lists(0))
    assert e.value.code in (B.E_STATE, B.E_INVAL)
    s.append_events(w.n_events(0))
    for flags in (B.DECODE_PLAN_ONLY, B.DECODE_DENSE_MASK):
        with pytest.raises(B.PastaError) as e:
            s.h.decode_step_noalloc(0, w.dec_request, w.dec_stream, qd, out, flags=flags)
        assert e.value.code == B.E_INVAL
    s.h.decode_step_noalloc(0, w.dec_request, w.dec_stream, qd, out)
    s.close()
    # a plan too large for the kernel arguments (config 4: 56 streams, thousands of ranges)
    w4 = W.config4()
    s = Session(w4)
    s.append_events(w4.n_prefill)
    qd = to_device(w4.q(0), w4.dtype, s.device)
    out = torch.empty_like(qd)
    with pytest.raises(B.PastaError) as e:
        s.h.decode_step_noalloc(0, w4.dec_request, w4.dec_stream, qd, out)
    assert e.value.code == B.E_CAPACITY
    s.h.decode_step(0, w4.dec_request, w4.dec_stream, qd, out)   # the existing entry point still takes it
    s.close()
