"""Maintained visibility lists read from their device-resident copy (PASTA_DECODE_DEVICE_LISTS): the
range arena and range index that the appends keep up to date, the newest range of every list riding
with the call, private work items derived by the kernels.  Same parity bar as everywhere: outputs,
lse and gather maps against the oracle, bit-exact maps."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
from paper_2502_11517_amd import binding as B
from paper_2502_11517_amd import workloads as W
from test_gpu_parity import _check_pool, _check_step, _out64, _session
from util import OraclePool, check_close

pytestmark = pytest.mark.gpu
DEV = B.DECODE_DEVICE_LISTS


def _plan(s, w, flags=0):
    plan = np.zeros(8, np.int64)
    s.h.decode_step(0, w.dec_request, w.dec_stream, None, None, flags=flags | B.DECODE_PLAN_ONLY, dbg_plan=plan)
    return plan


@pytest.mark.parametrize("cfg", ["config1", "config2", "config4", "config5"])
def test_single_step_configs_from_the_device_lists(cfg):
    """Lists rebuilt from the mirror after the prefill (bulk), then read by the kernels: the matrix-core
    kernel (configs 2, 4, 5: strided, scattered and nested-fork lists, contiguous and paged pools) and
    the vector-ALU kernel (config 1, fp32)."""
    w = getattr(W, cfg)()
    s = _session(w, kv_layout=B.HEAD_MAJOR)
    op = OraclePool(w, head_major=True).append_events(w.n_prefill)
    s.append_events(w.n_prefill)
    cache = {}
    _check_step(w, s, op, explicit=False, flags=DEV, ref_cache=cache, what=f"{cfg}, device lists")
    if w.dtype == "bf16":
        _check_step(w, s, op, explicit=False, flags=DEV | B.DECODE_NO_MFMA, ref_cache=cache, what=f"{cfg}, device lists, no mfma")
    s.close()


def test_config4_takes_the_device_lists_by_itself_and_sends_a_fixed_size_plan():
    """Config 4's plan does not fit the kernel arguments: without any flag the step reads the device
    lists, and the bytes it sends are those of the stream and request records alone."""
    w = W.config4()
    s = _session(w)
    s.append_events(w.n_prefill)
    plan = _plan(s, w)
    n_req = len(np.unique(w.dec_request))
    assert plan[6] <= 4 * (w.n * 25 + n_req * 10 + 8), plan
    lists_words = sum(len(x) for x in w.lists(0)[2:])
    assert lists_words * 4 > 4 * plan[6]       # the lists themselves are several times that
    s.close()


def test_plan_bytes_do_not_grow_with_the_lists():
    """Two requests-worth of history that differ only in how long (and how fragmented) the lists are:
    with the device lists a step sends the same number of bytes."""
    sizes = []
    for lengths in ([40, 50, 60], [400, 500, 600]):
        w = W.single_request("grow", "bf16", 8, 2, 128, 1.0, 7, 300, lengths, "random", k_std=128 ** -0.5)
        s = _session(w)
        s.append_events(w.n_prefill)
        sizes.append((int(_plan(s, w, DEV)[6]), int(_plan(s, w)[6])))
        s.close()
    assert sizes[0][0] == sizes[1][0], sizes
    assert sizes[0][1] > 4 * sizes[0][0], sizes     # the short lists sent whole (they fit the kernel arguments): several times that
    assert sizes[1][1] == sizes[1][0], sizes        # the long ones would not fit: the step takes the device lists by itself


@pytest.mark.parametrize("defer", [False, True])
def test_token_loop_keeps_the_device_lists_current(defer):
    """Config 3's append + decode loop (shortened prefix): every step's rows extend the lists -- by the
    K1 launch's patches when a range is new, by nothing at all when the newest range only grows (it
    rides with the call; a deferred append stays deferred) -- and every step decodes from the device lists."""
    w = W.config3(steps=40, prefix=1200, n_streams=6)
    s = _session(w, kv_layout=B.HEAD_MAJOR)
    op = OraclePool(w, head_major=True)
    s.append_events(w.n_prefill)
    op.append_events(w.n_prefill)
    keep = []
    for step in range(w.steps):
        hi = w.n_events(step)
        s.append_events(hi, chunk=w.n, flags=B.APPEND_DEFER if defer else 0)
        keep.append(s._keep_rows)
        if step in (0, 1, 2, 17, 38, 39):
            op.append_events(hi)
            _check_step(w, s, op, step, explicit=False, flags=DEV, what=f"loop step {step} defer {defer}")
        else:
            s.decode(step, explicit=False, want_lse=False, flags=DEV)
    _check_pool(w, s, op)
    s.close()


@pytest.mark.parametrize("seed", range(3))
def test_scattered_appends_patch_ranges_and_index(seed):
    """Rows appended a few at a time in a seeded random stream order: nearly every row opens a new
    range, so the K1 launches carry arena and index patches all the time, in calls of 1 to 7 rows and
    now and then one of 40 rows (too many to patch: that stream's copy is rebuilt instead)."""
    rng = np.random.default_rng(60 + seed)
    w = W.single_request("scatter", "bf16", 8, 2, 128, 1.0, 70 + seed, 200, [260, 300, 190, 350], "random",
                         k_std=128 ** -0.5)
    s = _session(w)
    op = OraclePool(w)
    n0 = 1 + max(int(np.nonzero(w.ev_stream == sid)[0][0]) for sid in w.dec_stream)  # every decoding stream is open
    s.append_events(n0)
    pos = n0
    while pos < w.n_prefill:
        k = 40 if rng.random() < 0.05 else int(rng.integers(1, 8))
        hi = min(w.n_prefill, pos + k)
        s.append_events(hi, chunk=64)
        pos = hi
        if rng.random() < 0.15:   # a decode from the device lists in between keeps them honest
            s.decode(0, explicit=False, want_lse=False, flags=DEV)
    op.append_events(w.n_prefill)
    _check_step(w, s, op, explicit=False, flags=DEV, what=f"scattered appends {seed}")
    _check_step(w, s, op, explicit=False, flags=DEV | B.DECODE_NO_MFMA, what=f"scattered appends {seed}, no mfma")
    s.close()


@pytest.mark.parametrize("seed", range(2))
def test_forks_joins_and_id_reuse_with_device_lists(seed):
    """The fork / sync / retire history of the maintained-list tests, decoded from the device lists at a
    few moments: a join rewrites a list (its copy is rebuilt), a retired id is opened again."""
    events = W.random_fork_sync_history(700 + seed, n_slots=420, max_ids=6, p_fork=0.08, p_sync=0.15)
    n = len(events)
    ev_s = np.array([e["stream"] for e in events], np.int32)
    ev_p = np.array([e["parent"] for e in events], np.int32)
    ev_n = np.array([1 if e["new"] else 0 for e in events], np.uint8)
    joins = {t: e["join"] for t, e in enumerate(events) if e["join"]}
    w = W.Workload(name="syncs", dtype="bf16", Hq=8, Hkv=2, D=128, scale=1.0, seed=950 + seed, max_requests=1,
                   pool_tokens=512, max_streams=6, k_std=128 ** -0.5)
    w.ev_request = np.zeros(n, np.int32)
    w.ev_stream, w.ev_parent, w.n_prefill = ev_s, np.where(ev_n == 1, ev_p, -1).astype(np.int32), n
    s = _session(w, max_ranges=4096)
    op = OraclePool(w).append_events(n)
    from paper_2502_11517_amd.harness import to_device
    checks = sorted(set([min(joins) + 1, max(joins) + 1, n // 3, n // 2, n]))
    done = 0
    for stop in checks:
        for t in range(done, stop):
            if events[t]["join"]:
                s.h.sync(0, int(ev_s[t]), events[t]["join"], retire=True)
            s.append_events(t + 1, chunk=1)
        done = stop
        live = sorted({int(x) for x in ev_s[:stop]} - {j for t, js in joins.items() if t < stop for j in js
                                                       if not any(ev_s[u] == j and ev_n[u] for u in range(t, stop))})
        rid = np.zeros(len(live), np.int32)
        q = W.f32_to_bf16_bits(np.random.default_rng([seed, stop]).standard_normal((len(live), w.Hq, w.D)).astype(np.float32))
        qd = to_device(q, w.dtype, s.device)
        out = torch.empty_like(qd)
        goffs = np.zeros(len(live) + 1, np.int64)
        s.h.decode_step(0, rid, live, qd, out, flags=DEV | B.DECODE_PLAN_ONLY, dbg_gather_offsets=goffs)
        grows = torch.full((int(goffs[-1]),), -1, dtype=torch.int32, device=s.device)
        s.h.decode_step(0, rid, live, qd, out, flags=DEV, dbg_gather_offsets=goffs, dbg_gather_rows=grows)
        got = _out64(w, out)
        grows = grows.cpu().numpy()
        for i, sid in enumerate(live):
            last = int(np.nonzero(ev_s[:stop] == sid)[0][-1])
            mask = oracle.visible_events(ev_s[:stop], ev_p[:stop], ev_n[:stop], {k: v for k, v in joins.items() if k < stop}, last)
            assert np.array_equal(grows[goffs[i]:goffs[i + 1]], np.nonzero(mask)[0]), f"stop {stop} stream {sid}"
            ref, _ = oracle.attention_dense(op.g, op.k, op.v, 0, mask, q[i], w.scale)
            check_close(got[i], ref, w.dtype, f"stop {stop} stream {sid}")
    s.close()


def test_device_lists_refusals_and_no_alloc():
    from paper_2502_11517_amd.harness import to_device
    w = W.config3(steps=2, prefix=700, n_streams=3)
    s = _session(w)
    op = OraclePool(w)
    s.append_events(w.n_events(0))
    op.append_events(w.n_events(0))
    qd = to_device(w.q(0), w.dtype, s.device)
    out = torch.empty_like(qd)
    with pytest.raises(B.PastaError) as e:       # explicit lists are the caller's: nothing on the device to read
        s.h.decode_step(0, w.dec_request, w.dec_stream, qd, out, lists=w.lists(0), flags=DEV)
    assert e.value.code == B.E_INVAL
    with pytest.raises(B.PastaError) as e:
        s.h.decode_step(0, w.dec_request, w.dec_stream, qd, out, flags=DEV | B.DECODE_DENSE_MASK)
    assert e.value.code == B.E_INVAL
    s.h.decode_step(0, w.dec_request, w.dec_stream, qd, out, flags=DEV)          # brings the copies up to date
    out2 = torch.empty_like(qd)
    s.h.decode_step_noalloc(0, w.dec_request, w.dec_stream, qd, out2, flags=DEV)  # ... which the no-alloc form may then read
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16))
    ref, _ = op.attention(0)
    check_close(_out64(w, out2), ref, w.dtype, "no-alloc, device lists")
    s.close()
