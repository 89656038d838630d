"""CPU-only tests of the C-ABI library's host side: exported symbols, argument validation,
slot assignment, the visibility lists it maintains (sizes against the oracle's dense mask),
and the launch-plan arithmetic.  No kernel is launched: appends use RESERVE_ONLY, decode steps
use PLAN_ONLY, and the pool / workspace addresses are never dereferenced."""
from __future__ import annotations

import os
import re
import subprocess

import numpy as np
import pytest

import oracle
from paper_2502_11517_amd import binding as B
from paper_2502_11517_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7000_0000_0000  # aligned, never dereferenced in these tests


@pytest.fixture(scope="module", autouse=True)
def _built():
    if not os.path.exists(B.library_path()):
        B.build_library()


def _handle(dtype="bf16", Hq=32, Hkv=8, D=128, *, n_layers=1, max_requests=1, page_tokens=0,
            n_phys_pages=0, pages_per_request=0, max_streams=12, max_ranges=4096, pool_tokens=16384,
            page_table=None, layout=B.TOKEN_MAJOR, scale=1.0):
    cfg = B.make_config(dtype, Hq, Hkv, D, scale, n_layers=n_layers, max_requests=max_requests,
                        page_tokens=page_tokens, kv_layout=layout, n_phys_pages=n_phys_pages,
                        pages_per_request=pages_per_request, max_streams=max_streams, max_ranges=max_ranges,
                        pool_tokens=pool_tokens)
    ws = B.query_workspace_bytes(cfg)
    return B.PastaAttn(cfg, FAKE, FAKE, FAKE, ws, page_table=page_table)


def _reserve(h, req, sid, par=None, layer=0):
    return h.append_kv(layer, req, sid, None, None, parent_stream=par, want_slots=True,
                       flags=B.APPEND_RESERVE_ONLY)


def _plan(h, req, sid, lists=None, flags=0):
    n = len(req)
    goffs, plan = np.zeros(n + 1, np.int64), np.zeros(8, np.int64)
    h.decode_step(0, req, sid, None, None, lists=lists, flags=flags | B.DECODE_PLAN_ONLY,
                  dbg_gather_offsets=goffs, dbg_plan=plan)
    return goffs, plan


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "pasta_attn.h")).read()
    declared = set(re.findall(r"\bint32_t\s+(pasta_attn_\w+)\s*\(", hdr))
    assert declared == {"pasta_attn_create", "pasta_attn_append_kv", "pasta_attn_decode_step", "pasta_attn_destroy",
                        "pasta_attn_sync", "pasta_attn_stream_list", "pasta_attn_replay",
                        "pasta_attn_decode_step_noalloc"}
    syms = subprocess.run(["nm", "-D", "--defined-only", B.library_path()], capture_output=True, text=True).stdout
    exported = {l.split()[-1] for l in syms.splitlines() if " T " in l}
    assert declared <= exported
    lib = B.load_library()
    for name in declared:
        assert getattr(lib, name) is not None


def test_create_validation_and_query_mode():
    ok = dict(dtype="bf16", n_q_heads=32, n_kv_heads=8, head_dim=128, softmax_scale=1.0, pool_tokens=1024)
    assert B.query_workspace_bytes(B.make_config(**ok)) > 0
    bad = [dict(n_q_heads=30), dict(head_dim=96), dict(n_kv_heads=0), dict(softmax_scale=0.0), dict(pool_tokens=0),
           dict(dtype=7), dict(n_q_heads=24, n_kv_heads=8), dict(n_layers=0), dict(max_streams=0),
           dict(page_tokens=12, n_phys_pages=4, pages_per_request=4), dict(kv_layout=5)]
    for b in bad:
        with pytest.raises(B.PastaError) as e:
            B.query_workspace_bytes(B.make_config(**{**ok, **b}))
        assert e.value.code == B.E_INVAL, b
    cfg = B.make_config(**ok)
    ws = B.query_workspace_bytes(cfg)
    with pytest.raises(B.PastaError) as e:
        B.PastaAttn(cfg, FAKE, FAKE, FAKE, ws - 1)
    assert e.value.code == B.E_CAPACITY
    with pytest.raises(B.PastaError) as e:
        B.PastaAttn(cfg, FAKE, FAKE, FAKE + 8, ws)  # misaligned workspace
    assert e.value.code == B.E_INVAL
    with pytest.raises(B.PastaError) as e:
        B.PastaAttn(B.make_config(**ok), None, FAKE, FAKE, ws)
    assert e.value.code == B.E_INVAL
    # page table entries must be inside the page pool
    pc = B.make_config(**{**ok, "page_tokens": 16, "n_phys_pages": 4, "pages_per_request": 2})
    with pytest.raises(B.PastaError) as e:
        B.PastaAttn(pc, FAKE, FAKE, FAKE, B.query_workspace_bytes(pc), page_table=[[0, 4]])
    assert e.value.code == B.E_INVAL
    # ... and distinct: a physical page named twice would alias two logical pages
    with pytest.raises(B.PastaError) as e:
        B.PastaAttn(pc, FAKE, FAKE, FAKE, B.query_workspace_bytes(pc), page_table=[[3, 3]])
    assert e.value.code == B.E_INVAL
    pc2 = B.make_config(**{**ok, "page_tokens": 16, "n_phys_pages": 4, "pages_per_request": 2, "max_requests": 2})
    with pytest.raises(B.PastaError) as e:  # across requests too
        B.PastaAttn(pc2, FAKE, FAKE, FAKE, B.query_workspace_bytes(pc2), page_table=[[0, 1], [2, 0]])
    assert e.value.code == B.E_INVAL
    B.PastaAttn(pc2, FAKE, FAKE, FAKE, B.query_workspace_bytes(pc2), page_table=[[0, 1], [2, 3]]).destroy()
    # -1 = no page assigned: only behind the assigned ones, and the request's capacity ends there
    with pytest.raises(B.PastaError) as e:
        B.PastaAttn(pc2, FAKE, FAKE, FAKE, B.query_workspace_bytes(pc2), page_table=[[-1, 1], [2, 3]])
    assert e.value.code == B.E_INVAL
    h = B.PastaAttn(pc2, FAKE, FAKE, FAKE, B.query_workspace_bytes(pc2), page_table=[[0, 1], [2, -1]])
    assert len(_reserve(h, [0] * 32, [0] * 32)) == 32
    assert len(_reserve(h, [1] * 16, [0] * 16)) == 16
    with pytest.raises(B.PastaError) as e:
        _reserve(h, [1], [0])
    assert e.value.code == B.E_CAPACITY
    h.destroy()


def test_slots_follow_call_order_per_request():
    """Single active thread: contiguous slots; two active threads: neighbouring slots that
    alternate (Section 3, Efficiency)."""
    h = _handle(max_requests=2, pool_tokens=64)
    assert _reserve(h, [0] * 5, [0] * 5).tolist() == [0, 1, 2, 3, 4]
    s = _reserve(h, [0, 0, 1, 0, 0, 1], [1, 2, 0, 1, 2, 0], par=[0, 0, -1, -1, -1, -1])
    assert s.tolist() == [5, 6, 0, 7, 8, 1]
    with pytest.raises(B.PastaError) as e:  # 64-slot pool: 56 more fit, 57 do not
        _reserve(h, [0] * 57, [1] * 57)
    assert e.value.code == B.E_CAPACITY
    assert _reserve(h, [0], [1]).tolist() == [9]  # the failed call changed nothing


def test_append_argument_errors():
    h = _handle(pool_tokens=64, max_streams=4)
    _reserve(h, [0, 0], [0, 0])
    for req, sid, par, code in [([1], [0], None, B.E_INVAL), ([0], [4], None, B.E_INVAL),
                                ([0], [1], [1], B.E_INVAL),      # parent == stream
                                ([0], [1], [2], B.E_INVAL),      # parent not open
                                ([0], [0], [0], B.E_INVAL),      # parent == itself
                                ([0, 0], [1, 1], [0, 0], B.E_INVAL)]:  # parent on an open stream
        with pytest.raises(B.PastaError) as e:
            _reserve(h, req, sid, par)
        assert e.value.code == code, (req, sid, par)
    with pytest.raises(B.PastaError) as e:
        h.append_kv(3, [0], [0], None, None, flags=B.APPEND_RESERVE_ONLY)
    assert e.value.code == B.E_STATE
    with pytest.raises(B.PastaError) as e:  # a real append needs device rows
        h.append_kv(0, [0], [0], None, None)
    assert e.value.code == B.E_INVAL
    assert _reserve(h, [0], [0]).tolist() == [2]


def test_layer_replay_reuses_the_slots():
    h = _handle(n_layers=3, pool_tokens=64)
    with pytest.raises(B.PastaError) as e:  # nothing to replay yet
        _reserve(h, [0], [0], layer=1)
    assert e.value.code == B.E_STATE
    assert _reserve(h, [0, 0, 0], [0, 0, 0], layer=0).tolist() == [0, 1, 2]
    assert _reserve(h, [0, 0, 0], [0, 0, 0], layer=1).tolist() == [0, 1, 2]
    assert _reserve(h, [0, 0, 0], [0, 0, 0], layer=2).tolist() == [0, 1, 2]
    assert _reserve(h, [0, 0], [1, 0], par=[0, -1], layer=0).tolist() == [3, 4]
    assert _reserve(h, [0, 0], [1, 0], layer=2).tolist() == [3, 4]
    with pytest.raises(B.PastaError) as e:  # more rows than layer 0 appended
        _reserve(h, [0, 0, 0], [1, 0, 0], layer=1)
    assert e.value.code == B.E_STATE


def test_paper_worked_example_through_the_maintained_lists():
    """The 28-slot scenario of Section 3 (Efficiency): sizes of what each thread sees."""
    h = _handle(pool_tokens=64, max_streams=3)
    _reserve(h, [0] * 22, [0] * 22)                       # prompt .. <promise/> #1
    _reserve(h, [0, 0, 0, 0, 0, 0], [1, 1, 0, 2, 1, 2], par=[0, -1, -1, 0, -1, -1])
    goffs, _ = _plan(h, [0, 0, 0], [1, 2, 0])
    assert np.diff(goffs).tolist() == [25, 25, 23]


@pytest.mark.parametrize("seed", range(10))
def test_maintained_list_sizes_equal_dense_mask_on_random_fork_histories(seed):
    ev_s, ev_p = W.random_fork_history(100 + seed, n_slots=80, max_streams=8)
    n_streams = int(ev_s.max()) + 1
    h = _handle(pool_tokens=128, max_streams=n_streams)
    _reserve(h, np.zeros(len(ev_s), np.int32), ev_s, ev_p)
    parent = np.full(n_streams, -1, np.int32)
    spawn = np.zeros(n_streams, np.int64)
    seen = set()
    for t, (s, p) in enumerate(zip(ev_s.tolist(), ev_p.tolist())):
        if s not in seen:
            seen.add(s)
            parent[s], spawn[s] = p, t
    sids = np.arange(n_streams, dtype=np.int32)
    goffs, _ = _plan(h, np.zeros(n_streams, np.int32), sids)
    for s in range(n_streams):
        assert goffs[s + 1] - goffs[s] == int(oracle.visible_dense(ev_s, parent, spawn, s).sum())


def test_explicit_list_validation():
    h = _handle(pool_tokens=256, max_streams=4)
    _reserve(h, [0] * 100, [0] * 100)
    ok = ([10], [0, 2], [20, 40], [3, 2], [4, 1])
    goffs, _ = _plan(h, [0], [1], ok)
    assert goffs.tolist() == [0, 15]
    bad = [
        ([10], [0, 1], [5], [1], [1]),        # range inside the prefix
        ([10], [0, 2], [20, 28], [3, 1], [4, 1]),  # second range starts at the first one's last slot
        ([10], [0, 1], [99], [2], [1]),       # runs past the tail
        ([10], [0, 1], [20], [0], [1]),       # empty range
        ([10], [0, 1], [20], [2], [0]),       # stride 0
        ([101], [0, 0], [], [], []),          # prefix beyond the tail
        ([0], [0, 0], [], [], []),            # nothing visible
        ([-1], [0, 0], [], [], []),
    ]
    for lists in bad:
        with pytest.raises(B.PastaError) as e:
            _plan(h, [0], [1], lists)
        assert e.value.code == B.E_INVAL, lists
    # the same (request, stream) twice is fine with explicit lists (several query tokens of one stream)
    goffs, _ = _plan(h, [0, 0], [1, 1], ([10, 11], [0, 0, 0], [], [], []))
    assert goffs.tolist() == [0, 10, 21]
    with pytest.raises(B.PastaError) as e:  # maintained mode, stream never opened
        _plan(h, [0], [2])
    assert e.value.code == B.E_STATE
    small = _handle(pool_tokens=256, max_streams=4, max_ranges=2)
    _reserve(small, [0] * 100, [0] * 100)
    with pytest.raises(B.PastaError) as e:
        _plan(small, [0], [1], ([10], [0, 3], [20, 30, 40], [1, 1, 1], [1, 1, 1]))
    assert e.value.code == B.E_CAPACITY


def test_plan_arithmetic_on_the_8k_prefix_8_stream_shape():
    w = W.config3(steps=2)
    h = _handle(pool_tokens=w.pool_tokens, max_streams=w.max_streams)
    ne = w.n_events(0)
    _reserve(h, w.ev_request[:ne], w.ev_stream[:ne], w.ev_parent[:ne])
    pl, offs, st, ct, sd = w.lists(0)
    for lists in (None, (pl, offs, st, ct, sd)):  # maintained and explicit agree
        goffs, plan = _plan(h, w.dec_request, w.dec_stream, lists)
        vis = [pl[i] + int(ct[offs[i]:offs[i + 1]].sum()) for i in range(w.n)]
        assert np.diff(goffs).tolist() == vis
        priv = [v - 8192 for v in vis]
        assert plan[5] == 8192 and plan[0] == 8192 // 64 * 8
        assert plan[1] == -(-8192 // plan[4]) * 8 and plan[4] % 64 == 0
        assert plan[4] == 8192 * 8 // 256  # one prefix work-group per CU
        assert plan[2] == sum(-(-p // 128) for p in priv)  # private items: 128 tokens
        assert plan[3] == plan[1] * 32 + plan[2] * 32
    # fp32 handles and NO_MFMA route everything through the private-segment kernel
    _, plan = _plan(h, w.dec_request, w.dec_stream, None, flags=B.DECODE_NO_MFMA)
    assert plan[5] == 0 and plan[1] == 0 and plan[2] == sum(-(-v // 128) for v in vis)


def test_requests_with_more_than_32_stacked_rows_choice_of_the_form():
    """One 32-row group per work-group, or four: the plan's count of shared-prefix work-groups tells which.  The
    library picks the four-group form where three of four waves compute on average and a chunk is four rounds
    (512 tokens) or more; the two flags force either form."""
    def wgs(Hq, Hkv, n, prefix, flags=0):
        w = W.single_request("form", "bf16", Hq, Hkv, 128, 1.0, 3, prefix, [2] * n, "round_robin")
        h = _handle(Hq=Hq, Hkv=Hkv, pool_tokens=w.pool_tokens, max_streams=w.max_streams)
        ne = w.n_events(0)
        _reserve(h, w.ev_request[:ne], w.ev_stream[:ne], w.ev_parent[:ne])
        _, plan = _plan(h, w.dec_request, w.dec_stream, None, flags=flags)
        R, chunks = n * (Hq // Hkv), -(-int(plan[5]) // int(plan[4]))
        assert plan[1] in (chunks * Hkv * -(-R // 32), chunks * Hkv * -(-R // 128))
        return "four" if (R > 32 and plan[1] == chunks * Hkv * -(-R // 128)) else "one"
    assert wgs(64, 8, 16, 32768) == "four"          # 128 rows over 32k tokens: chunks of 1024
    assert wgs(32, 8, 32, 32768) == "four"
    assert wgs(32, 8, 24, 32768) == "four"          # 96 rows: three of four waves
    assert wgs(32, 8, 16, 32768) == "one"           # 64 rows: two of four waves would compute
    assert wgs(32, 8, 32, 8192) == "one"            # chunks of 256 tokens: two rounds
    assert wgs(32, 8, 40, 32768) == "one"           # 160 rows: five groups over two quads
    assert wgs(32, 8, 8, 32768) == "one"            # 32 rows: nothing to choose
    assert wgs(32, 8, 16, 32768, B.DECODE_FOUR_GROUPS) == "four"
    assert wgs(32, 8, 32, 8192, B.DECODE_FOUR_GROUPS) == "four"
    assert wgs(64, 8, 16, 32768, B.DECODE_ROW_GROUPS) == "one"
    assert wgs(32, 8, 8, 32768, B.DECODE_FOUR_GROUPS) == "one"
    with pytest.raises(B.PastaError) as e:
        wgs(64, 8, 16, 32768, B.DECODE_FOUR_GROUPS | B.DECODE_ROW_GROUPS)
    assert e.value.code == B.E_INVAL


def test_nested_fork_common_prefix_is_the_minimum():
    w = W.single_request("nested", "bf16", 8, 2, 128, 1.0, 5, 300, [6, 4, 5, 3, 7], "round_robin", nested=(200, 2))
    h = _handle(Hq=8, Hkv=2, pool_tokens=w.pool_tokens, max_streams=w.max_streams)
    _reserve(h, w.ev_request, w.ev_stream, w.ev_parent)
    goffs, plan = _plan(h, w.dec_request, w.dec_stream)
    pl, offs, st, ct, sd = w.lists(0)
    assert pl.tolist() == [500, 500, 300, 300, 300]
    assert plan[5] == 300
    assert np.diff(goffs).tolist() == [pl[i] + int(ct[offs[i]:offs[i + 1]].sum()) for i in range(w.n)]


def test_destroy_and_stale_handle():
    h = _handle(pool_tokens=64)
    lib = B.load_library()
    assert lib.pasta_attn_destroy(None) == B.OK
    h.destroy()


def test_rope_flags_need_theta_and_positions():
    """PASTA_APPEND_ROPE / PASTA_DECODE_ROPE_Q are E_INVAL without rope_theta, without position
    ids, with a negative id, or together with RESERVE_ONLY; the workspace grows by the table and
    the rotated-Q buffer when rope_theta is set."""
    plain = B.make_config("bf16", 8, 2, 128, 1.0, max_streams=4, pool_tokens=256)
    roped = B.make_config("bf16", 8, 2, 128, 1.0, max_streams=4, pool_tokens=256, rope_theta=10000.0)
    assert B.query_workspace_bytes(roped) >= B.query_workspace_bytes(plain) + 64 * 8 + 4 * 8 * 128 * 2
    bad = B.make_config("bf16", 8, 2, 128, 1.0, max_streams=4, pool_tokens=256, rope_theta=-1.0)
    with pytest.raises(B.PastaError) as e:
        B.query_workspace_bytes(bad)
    assert e.value.code == B.E_INVAL
    for cfg, theta_ok in ((plain, False), (roped, True)):
        h = B.PastaAttn(cfg, FAKE, FAKE, FAKE, B.query_workspace_bytes(cfg))
        rid, sid = np.zeros(3, np.int32), np.zeros(3, np.int32)
        # RESERVE_ONLY | ROPE is refused in any case
        with pytest.raises(B.PastaError) as e:
            h.append_kv(0, rid, sid, None, None, position=[0, 1, 2], flags=B.APPEND_RESERVE_ONLY | B.APPEND_ROPE)
        assert e.value.code == B.E_INVAL
        for position in (None, [0, 1, -2]) + (() if theta_ok else ([0, 1, 2],)):
            with pytest.raises(B.PastaError) as e:
                h.append_kv(0, rid, sid, FAKE, FAKE, position=position, flags=B.APPEND_ROPE)
            assert e.value.code == B.E_INVAL
        h.append_kv(0, rid, sid, None, None, flags=B.APPEND_RESERVE_ONLY)
        for position in (None, [-1]) + (() if theta_ok else ([2],)):
            with pytest.raises(B.PastaError) as e:
                h.decode_step(0, [0], [0], FAKE, FAKE, position=position, flags=B.DECODE_ROPE_Q | B.DECODE_PLAN_ONLY)
            assert e.value.code == B.E_INVAL
        if theta_ok:
            h.decode_step(0, [0], [0], FAKE, FAKE, position=[2], flags=B.DECODE_ROPE_Q | B.DECODE_PLAN_ONLY)
        h.destroy()


def _expand(pl, st, ct, sd):
    out = list(range(pl))
    for a, c, d in zip(st.tolist(), ct.tolist(), sd.tolist()):
        out += [a + j * d for j in range(c)]
    return out


@pytest.mark.parametrize("seed", range(8))
def test_maintained_lists_through_forks_syncs_and_id_reuse_equal_reachability(seed):
    """Drive the library's bookkeeping (no device work) through a random history with nested
    forks, synchronisations and reuse of stream ids; after every event the maintained list of
    the stream that just appended must name exactly the slots reachable from its newest token
    in Figure 2b's graph (the oracle's visible_events)."""
    import oracle
    events = W.random_fork_sync_history(100 + seed, n_slots=120, max_ids=5)
    cfg = B.make_config("bf16", 8, 2, 128, 1.0, max_streams=5, pool_tokens=256, max_ranges=4096)
    h = B.PastaAttn(cfg, FAKE, FAKE, FAKE, B.query_workspace_bytes(cfg))
    ev_s = np.array([e["stream"] for e in events], np.int32)
    ev_p = np.array([e["parent"] for e in events], np.int32)
    ev_n = np.array([1 if e["new"] else 0 for e in events], np.uint8)
    joins = {t: e["join"] for t, e in enumerate(events) if e["join"]}
    assert joins
    for t, e in enumerate(events):
        if e["join"]:
            h.sync(0, e["stream"], e["join"], retire=True)
        slot = h.append_kv(0, [0], [e["stream"]], None, None, parent_stream=[e["parent"] if e["new"] else -1],
                           want_slots=True, flags=B.APPEND_RESERVE_ONLY)
        assert slot[0] == t
        got = _expand(*h.stream_list(0, e["stream"]))
        want = np.nonzero(oracle.visible_events(ev_s[: t + 1], ev_p[: t + 1], ev_n[: t + 1],
                                                {k: v for k, v in joins.items() if k <= t}, t))[0].tolist()
        assert got == want, f"event {t}: {e}"
    h.destroy()


def test_sync_argument_checks_and_retire_only():
    cfg = B.make_config("bf16", 8, 2, 128, 1.0, max_streams=4, pool_tokens=64)
    h = B.PastaAttn(cfg, FAKE, FAKE, FAKE, B.query_workspace_bytes(cfg))
    app = lambda s, par=-1: h.append_kv(0, [0], [s], None, None, parent_stream=[par], flags=B.APPEND_RESERVE_ONLY)
    for _ in range(3):
        app(0)
    app(1, 0); app(2, 0); app(1); app(2); app(0)          # slots 3..7
    for args, code in (((0, 0, [0]), B.E_INVAL), ((0, 0, [1, 1]), B.E_INVAL), ((0, 0, [3]), B.E_STATE),
                       ((0, 3, [1]), B.E_STATE), ((0, 0, [7]), B.E_INVAL), ((1, 0, [1]), B.E_INVAL),
                       ((0, 0, []), B.E_INVAL)):
        with pytest.raises(B.PastaError) as e:
            h.sync(*args)
        assert e.value.code == code, args
    with pytest.raises(B.PastaError) as e:
        h.sync(0, -1, [1])                                  # -1 needs RETIRE
    assert e.value.code == B.E_INVAL
    assert _expand(*h.stream_list(0, 0)) == [0, 1, 2, 7]
    h.sync(0, 0, [1])                                       # join without retiring: stream 1 stays open
    assert _expand(*h.stream_list(0, 0)) == [0, 1, 2, 3, 5, 7]
    assert _expand(*h.stream_list(0, 1)) == [0, 1, 2, 3, 5]
    h.sync(0, 0, [2], retire=True)
    assert h.stream_list(0, 0)[0] == 8 and len(h.stream_list(0, 0)[1]) == 0   # everything: one contiguous head
    with pytest.raises(B.PastaError) as e:
        h.stream_list(0, 2)
    assert e.value.code == B.E_STATE
    h.sync(0, -1, [1], retire=True)                         # retire only
    app(1, 0)                                               # the id opens again, as a fork of stream 0 now
    assert _expand(*h.stream_list(0, 1)) == list(range(9))
    h.destroy()


@pytest.mark.parametrize("seed", range(6))
def test_replay_plan_equals_the_oracles_interpreter(seed):
    """The library's trace replay (planning run: host bookkeeping only) against the oracle's
    independent simulation of the interpreter: same slot, stream, position id and pass for
    every token fed, same maintained list for the main thread at the end; and the planning
    run leaves the handle as it was."""
    from oracle import pasta_interp as I
    ops = W.synthetic_trace(50 + seed, n_promises=4 + seed, sync_every=2 + seed % 3)
    n_prompt = 33
    cfg = B.make_config("bf16", 8, 2, 128, 1.0, max_streams=6, pool_tokens=4096, max_ranges=8192)
    h = B.PastaAttn(cfg, FAKE, FAKE, FAKE, B.query_workspace_bytes(cfg))
    h.append_kv(0, [0] * n_prompt, [0] * n_prompt, None, None, flags=B.APPEND_RESERVE_ONLY)
    toks, passes = I.interpret(ops, n_prompt, n_prompt, 6)
    r = h.replay(0, ops, n_prompt, 4000, flags=B.REPLAY_PLAN_ONLY)
    assert r["stats"][0] == len(toks) and r["stats"][1] == passes
    assert r["stats"][2] == max(sum(1 for t in toks if t["pass_"] == p) for p in range(passes))
    for key, name in (("slot", "slot"), ("stream", "stream"), ("pos", "pos"), ("pass_", "pass_")):
        assert r[key].tolist() == [t[name] for t in toks], key
    assert h.stream_list(0, 0)[0] == n_prompt                  # unchanged by the planning run
    with pytest.raises(B.PastaError) as e:
        h.stream_list(0, 1)
    assert e.value.code == B.E_STATE
    with pytest.raises(B.PastaError) as e:                     # too few rows in the caller's arrays
        h.replay(0, ops, n_prompt, len(toks) - 1, flags=B.REPLAY_PLAN_ONLY)
    assert e.value.code == B.E_CAPACITY
    h.destroy()


def test_comparison_flags_and_causal_skip_argument_checks():
    cfg = B.make_config("bf16", 8, 2, 128, 1.0, max_streams=4, pool_tokens=1024)
    h = B.PastaAttn(cfg, FAKE, FAKE, FAKE, B.query_workspace_bytes(cfg))
    h.append_kv(0, [0] * 300, [0] * 300, None, None, flags=B.APPEND_RESERVE_ONLY)
    h.append_kv(0, [0], [1], None, None, parent_stream=[0], flags=B.APPEND_RESERVE_ONLY)
    h.append_kv(0, [0] * 4, [1] * 4, None, None, flags=B.APPEND_RESERVE_ONLY)
    plan = np.zeros(8, np.int64)
    h.decode_step(0, [0, 0], [0, 1], FAKE, FAKE, flags=B.DECODE_PLAN_ONLY, dbg_plan=plan)
    assert plan[5] == 300 and plan[1] > 0                      # a shared prefix of 300 rows
    for flag in (B.DECODE_NO_SHARE, B.DECODE_DENSE_MASK):
        h.decode_step(0, [0, 0], [0, 1], FAKE, FAKE, flags=B.DECODE_PLAN_ONLY | flag, dbg_plan=plan)
        assert plan[5] == 0 and plan[1] == 0
    goffs = np.zeros(3, np.int64)
    h.decode_step(0, [0, 0], [0, 1], FAKE, FAKE, flags=B.DECODE_PLAN_ONLY | B.DECODE_DENSE_MASK, dbg_gather_offsets=goffs)
    assert goffs.tolist() == [0, 305, 610]                     # every stream walks all 305 slots
    with pytest.raises(B.PastaError) as e:                     # dense masks are for the matrix-core kernel
        h.decode_step(0, [0], [0], FAKE, FAKE, flags=B.DECODE_PLAN_ONLY | B.DECODE_DENSE_MASK | B.DECODE_NO_MFMA)
    assert e.value.code == B.E_INVAL
    # one stream twice needs causal_skip
    with pytest.raises(B.PastaError) as e:
        h.decode_step(0, [0, 0], [1, 1], FAKE, FAKE, flags=B.DECODE_PLAN_ONLY)
    assert e.value.code == B.E_INVAL
    h.decode_step(0, [0] * 3, [1, 1, 1], FAKE, FAKE, flags=B.DECODE_PLAN_ONLY, causal_skip=[2, 1, 0], dbg_gather_offsets=(g4 := np.zeros(4, np.int64)))
    assert np.diff(g4).tolist() == [303, 304, 305]
    for skip in ([-1, 0, 0], [306, 0, 0]):                     # negative, or nothing left to see
        with pytest.raises(B.PastaError) as e:
            h.decode_step(0, [0] * 3, [1, 1, 1], FAKE, FAKE, flags=B.DECODE_PLAN_ONLY, causal_skip=skip)
        assert e.value.code == B.E_INVAL
    with pytest.raises(B.PastaError) as e:                     # not with explicit lists
        h.decode_step(0, [0], [1], FAKE, FAKE, flags=B.DECODE_PLAN_ONLY, causal_skip=[0], lists=([5], [0, 0], [], [], []))
    assert e.value.code == B.E_INVAL
    h.destroy()


def test_full_pool_and_maximum_number_of_query_rows():
    """The request's share of the pool filled to its last slot, max_requests * max_streams query
    rows in one step; one row more is E_CAPACITY and changes neither the tail nor the lists."""
    w = W.single_request("full", "bf16", 8, 2, 128, 1.0, 21, 448, [10, 9, 9, 9, 9, 9, 9], "random", slack=0)
    h = _handle(Hq=8, Hkv=2, max_streams=8, pool_tokens=w.pool_tokens)
    slots = _reserve(h, w.ev_request, w.ev_stream, w.ev_parent)
    assert slots.tolist() == list(range(512))
    rid, sid = np.zeros(8, np.int32), np.arange(1, 9, dtype=np.int32) % 8
    goffs, plan = _plan(h, rid, sid)
    pl, offs, st, ct, sd = w.lists(0)
    sizes = [int(pl[i] + ct[offs[i]:offs[i + 1]].sum()) for i in range(7)] + [448]
    assert np.diff(goffs).tolist() == sizes
    with pytest.raises(B.PastaError) as e:
        _reserve(h, [0], [3])
    assert e.value.code == B.E_CAPACITY
    goffs2, plan2 = _plan(h, rid, sid)
    assert np.array_equal(goffs, goffs2) and np.array_equal(plan, plan2)
    with pytest.raises(B.PastaError) as e:  # a ninth query row is more than the handle was sized for
        _plan(h, np.zeros(9, np.int32), np.arange(9, dtype=np.int32) % 8,
              lists=(np.full(9, 10), np.zeros(10, np.int32), [], [], []))
    assert e.value.code == B.E_INVAL
    h.destroy()


def test_device_list_plans_have_a_fixed_size_and_failed_appends_leave_the_lists_alone():
    """PLAN_ONLY with PASTA_DECODE_DEVICE_LISTS: the metadata a step sends is one record per stream,
    whatever the lists hold; without the flag a plan that would not fit the kernel arguments switches
    by itself.  An append that fails half way (capacity) restores lists, tails and token counts."""
    h = _handle(pool_tokens=4096, max_streams=4, max_ranges=4096)
    _reserve(h, [0] * 100, [0] * 100)
    _reserve(h, [0, 0], [1, 2], par=[0, 0])
    sizes = []
    for rounds in (10, 600):
        for _ in range(rounds):
            _reserve(h, [0, 0, 0], [1, 2, 1])        # 1, 2, 1 | 1, 2, 1: ranges of one and two slots
        _, plan_dev = _plan(h, [0, 0], [1, 2], flags=B.DECODE_DEVICE_LISTS)
        _, plan = _plan(h, [0, 0], [1, 2])
        sizes.append((int(plan_dev[6]), int(plan[6]), int(plan_dev[2]), int(plan[2])))
    assert sizes[0][0] == sizes[1][0] and sizes[0][1] > sizes[0][0]
    assert sizes[1][1] == sizes[1][0]                # too large for the kernel arguments: switched by itself
    before = [h.stream_list(0, s) for s in (1, 2)]
    with pytest.raises(B.PastaError) as e:           # the pool has 4096 slots: this call runs out of them
        _reserve(h, [0] * 3000, [1, 2] * 1500)
    assert e.value.code == B.E_CAPACITY
    after = [h.stream_list(0, s) for s in (1, 2)]
    for b, a_ in zip(before, after):
        assert b[0] == a_[0] and all(np.array_equal(x, y) for x, y in zip(b[1:], a_[1:]))
    assert _plan(h, [0, 0], [1, 2], flags=B.DECODE_DEVICE_LISTS)[1][2] == sizes[1][2]   # same item count: token counts restored
    h.destroy()
