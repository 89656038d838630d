"""Pins of the fp64 CPU oracle against things other than itself: a library SDPA, closed
forms, the paper's worked visibility example, brute force, invariances.  CPU only."""
from __future__ import annotations

import json
import math
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2502_11517_amd import workloads as W
from util import OraclePool, geom_of, to_f64

HERE = os.path.dirname(os.path.abspath(__file__))
LAYOUTS = [("contig", False), ("contig", True), ("paged", False), ("paged", True)]


def _tiny(dtype="f32", Hq=4, Hkv=2, D=64, prefix=40, lengths=(7, 5, 9), interleave="random", seed=7,
          paged=False, steps=1):
    w = W.single_request("tiny", dtype, Hq, Hkv, D, 0.125, seed, prefix, list(lengths), interleave,
                         steps=steps, q_std=1.0, k_std=1.0, v_std=1.0)
    if paged:
        pt = 8
        ppr = -(-w.pool_tokens // pt)
        rng = np.random.default_rng(seed + 99)
        w.page_tokens, w.pages_per_request, w.n_phys_pages = pt, ppr, ppr + 3
        w.page_table = rng.permutation(ppr + 3)[:ppr].astype(np.int32).reshape(1, ppr)
    return w


# ---------------------------------------------------------------- layout formulas vs reshape
@pytest.mark.parametrize("mode,head_major", LAYOUTS)
def test_elem_offset_matches_numpy_reshape(mode, head_major):
    """The addressing formulas, checked against numpy's own indexing of the declared shapes."""
    w = _tiny(paged=(mode == "paged"))
    g = geom_of(w, head_major)
    rows = g.rows_per_layer()
    flat = np.arange(rows * w.Hkv * w.D)
    if not head_major:
        view = flat.reshape(rows, w.Hkv, w.D)  # [row][head][d]
        at = lambda p, h: view[p, h, 0]  # noqa: E731
    elif mode == "contig":
        view = flat.reshape(w.Hkv, rows, w.D)  # [head][row][d]
        at = lambda p, h: view[h, p, 0]  # noqa: E731
    else:
        view = flat.reshape(w.n_phys_pages, w.Hkv, w.page_tokens, w.D)  # [page][head][in-page][d]
        at = lambda p, h: view[p // w.page_tokens, h, p % w.page_tokens, 0]  # noqa: E731
    for slot in (0, 1, 7, 8, 9, 33, w.pool_tokens - 1):
        p = oracle.phys_row(g, 0, slot)
        if mode == "paged":
            assert p == w.page_table[0, slot // w.page_tokens] * w.page_tokens + slot % w.page_tokens
        else:
            assert p == slot
        for h in range(w.Hkv):
            assert oracle.elem_offset(g, p, h) == at(p, h)
    assert oracle.phys_row(g, 0, w.pool_tokens + (w.page_tokens or 1) * 4) == -1
    assert oracle.phys_row(g, 1, 0) == -1


# ---------------------------------------------------------------- append
@pytest.mark.parametrize("mode,head_major", LAYOUTS)
def test_append_is_a_bitwise_copy_in_call_order(mode, head_major):
    w = _tiny("bf16", paged=(mode == "paged"))
    op = OraclePool(w, head_major).append_events(w.n_prefill)
    assert op.tail[0] == w.n_prefill
    k, v = w.kv_rows(0, w.n_prefill)
    for e in (0, 1, 39, 40, 41, w.n_prefill - 1):  # event e sits in logical slot e (one request)
        p = oracle.phys_row(op.g, 0, e)
        for h in range(w.Hkv):
            o = oracle.elem_offset(op.g, p, h)
            assert np.array_equal(op.k[o:o + w.D], k[e, h])
            assert np.array_equal(op.v[o:o + w.D], v[e, h])
    # every element of the pool is either untouched (0) or one of the appended rows
    assert np.count_nonzero(op.k) <= k.size


def test_append_single_thread_contiguous_two_threads_alternate():
    """Section 3, Efficiency: one active thread appends sequentially; two active threads land in
    neighbouring slots and alternate."""
    w = _tiny()
    g = geom_of(w)
    kp, vp, tail = g.new_pool(), g.new_pool(), np.zeros(1, np.int64)
    z = np.zeros((5, w.Hkv, w.D), np.float32)
    rc, slots = oracle.append(g, kp, vp, [0] * 5, z, z, tail)
    assert rc == 0 and slots.tolist() == [0, 1, 2, 3, 4]
    # two threads taking turns: thread A gets 5,7,9 and thread B gets 6,8,10
    rc, slots = oracle.append(g, kp, vp, [0] * 6, np.zeros((6, w.Hkv, w.D), np.float32),
                              np.zeros((6, w.Hkv, w.D), np.float32), tail)
    assert slots[0::2].tolist() == [5, 7, 9] and slots[1::2].tolist() == [6, 8, 10]


def test_append_capacity_error_changes_nothing():
    w = _tiny()
    g = geom_of(w)
    kp, vp, tail = g.new_pool(), g.new_pool(), np.zeros(1, np.int64)
    n = w.pool_tokens + 1
    ones = np.ones((n, w.Hkv, w.D), np.float32)
    rc, _ = oracle.append(g, kp, vp, [0] * n, ones, ones, tail)
    assert rc == -2 and tail[0] == 0 and not kp.any() and not vp.any()


# ---------------------------------------------------------------- visibility (A0)
def test_paper_worked_example_visibility():
    fx = json.load(open(os.path.join(HERE, "golden", "paper_sec3_visibility.json")))
    ss, par, sp = fx["slot_stream"], fx["stream_parent"], fx["stream_spawn_tail"]
    for s, exp in fx["visible"].items():
        mask = oracle.visible_dense(ss, par, sp, int(s))
        assert np.nonzero(mask)[0].tolist() == exp
    nf = fx["named_facts"]
    mask = oracle.visible_dense(ss, par, sp, nf["query_stream"])
    assert all(mask[t] for t in nf["must_see"]) and not any(mask[t] for t in nf["must_not_see"])


def _ancestors_by_graph_walk(ev_stream, ev_parent, q_slot):
    """Figure 2b read literally: every token has an edge from the token just before it in its
    thread's context; a thread's first token hangs off the spawning thread's latest token.  A
    token attends to itself and to everything reachable backwards along those edges."""
    pred = {}
    last_of = {}
    for t, (s, p) in enumerate(zip(ev_stream.tolist(), ev_parent.tolist())):
        if s in last_of:
            pred[t] = last_of[s]
        elif p >= 0:
            pred[t] = last_of[p]
        else:
            pred[t] = None
        last_of[s] = t
    vis, t = [], q_slot
    while t is not None:
        vis.append(t)
        t = pred[t]
    return sorted(vis)


@pytest.mark.parametrize("seed", range(12))
def test_visible_dense_equals_graph_walk_on_random_fork_histories(seed):
    ev_s, ev_p = W.random_fork_history(seed, n_slots=60, max_streams=7)
    n_streams = int(ev_s.max()) + 1
    parent = np.full(n_streams, -1, np.int32)
    spawn = np.zeros(n_streams, np.int64)
    seen = set()
    for t, (s, p) in enumerate(zip(ev_s.tolist(), ev_p.tolist())):
        if s not in seen:
            seen.add(s)
            parent[s], spawn[s] = p, t
    for s in range(n_streams):
        last = int(np.nonzero(ev_s == s)[0][-1])  # the stream's latest token: the query position
        mask = oracle.visible_dense(ev_s, parent, spawn, s)
        got = [t for t in np.nonzero(mask)[0].tolist() if t <= last]
        assert got == _ancestors_by_graph_walk(ev_s, ev_p, last)
        # tokens an ancestor appends AFTER the spawn must be invisible
        for t in np.nonzero(mask)[0].tolist():
            assert ev_s[t] == s or t < spawn[s]


@pytest.mark.parametrize("interleave", ["random", "round_robin"])
def test_generator_lists_equal_dense_mask(interleave):
    """The (prefix_len, ranges) lists a caller passes name exactly the ancestor-rule set."""
    w = _tiny(lengths=(7, 5, 9, 3), interleave=interleave)
    pl, offs, st, ct, sd = w.lists(0)
    ss, par, sp = w.fork_tree(0)
    g = geom_of(w)
    for i in range(w.n):
        rows = oracle.gather_map(g, 0, pl[i], st[offs[i]:offs[i + 1]], ct[offs[i]:offs[i + 1]],
                                 sd[offs[i]:offs[i + 1]])
        mask = oracle.visible_dense(ss, par, sp, int(w.dec_stream[i]))
        assert rows.tolist() == np.nonzero(mask)[0].tolist()


def test_nested_fork_lists_equal_dense_mask():
    w = W.single_request("nested", "f32", 4, 2, 64, 0.125, 5, 20, [6, 4, 5, 3, 7], "round_robin",
                         nested=(9, 2))
    pl, offs, st, ct, sd = w.lists(0)
    ss, par, sp = w.fork_tree(0)
    assert pl.tolist() == [29, 29, 20, 20, 20]
    for i in range(w.n):
        rows = oracle.gather_map(geom_of(w), 0, pl[i], st[offs[i]:offs[i + 1]], ct[offs[i]:offs[i + 1]],
                                 sd[offs[i]:offs[i + 1]])
        mask = oracle.visible_dense(ss, par, sp, int(w.dec_stream[i]))
        assert rows.tolist() == np.nonzero(mask)[0].tolist()


def test_gather_map_order_strides_and_pages():
    w = _tiny(paged=True)
    g = geom_of(w)
    rows = oracle.gather_map(g, 0, 3, [5, 20], [3, 2], [4, 1])
    slots = [0, 1, 2, 5, 9, 13, 20, 21]
    exp = [int(w.page_table[0, s // 8]) * 8 + s % 8 for s in slots]
    assert rows.tolist() == exp
    with pytest.raises(ValueError):
        oracle.gather_map(g, 0, 0, [w.pages_per_request * 8], [1], [1])


# ---------------------------------------------------------------- attention value
def _sdpa_f64(qf, Kf, Vf, G, scale):
    """Library routine: torch SDPA on CPU in fp64. qf [Hq][D]; Kf, Vf [N][Hkv][D]."""
    q = torch.from_numpy(qf)[None, :, None, :]  # [1][Hq][1][D]
    K = torch.from_numpy(Kf).permute(1, 0, 2).repeat_interleave(G, dim=0)[None]  # [1][Hq][N][D]
    V = torch.from_numpy(Vf).permute(1, 0, 2).repeat_interleave(G, dim=0)[None]
    return torch.nn.functional.scaled_dot_product_attention(q, K, V, scale=scale)[0, :, 0, :].numpy()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mode,head_major", LAYOUTS)
def test_single_stream_equals_causal_decode_sdpa(dtype, mode, head_major):
    """No fork: one stream whose list is [0, N) is ordinary decode attention of the last token."""
    w = _tiny(dtype, Hq=8, Hkv=2, prefix=50, lengths=(1,), paged=(mode == "paged"))
    op = OraclePool(w, head_major).append_events(w.n_prefill)
    N = w.n_prefill
    q = w.q(0)
    out, lse = oracle.attention(op.g, op.k, op.v, [0], [N], [0, 0], [], [], [], q, w.scale)
    k, v = w.kv_rows(0, N)
    ref = _sdpa_f64(to_f64(w, q)[0], to_f64(w, k), to_f64(w, v), w.Hq // w.Hkv, w.scale)
    assert np.max(np.abs(out[0] - ref)) < 1e-12
    # lse against scipy-free direct formula on one head
    z = w.scale * to_f64(w, k)[:, 1, :] @ to_f64(w, q)[0, 5]
    assert abs(lse[0, 5] - (np.log(np.sum(np.exp(z - z.max()))) + z.max())) < 1e-12


def test_multi_stream_equals_sdpa_per_stream_on_gathered_rows():
    """Each stream = SDPA over prefix rows + its own rows, whatever the interleave."""
    w = _tiny("bf16", Hq=8, Hkv=2, lengths=(7, 5, 9))
    op = OraclePool(w).append_events(w.n_prefill)
    out, _ = op.attention()
    k, v = w.kv_rows(0, w.n_prefill)
    q = to_f64(w, w.q(0))
    for i in range(w.n):
        own = np.nonzero(w.ev_stream == w.dec_stream[i])[0]
        idx = np.concatenate([np.arange(40), own])
        ref = _sdpa_f64(q[i], to_f64(w, k)[idx], to_f64(w, v)[idx], 4, w.scale)
        assert np.max(np.abs(out[i] - ref)) < 1e-12


def test_gqa_head_mapping_consecutive_heads_share_a_kv_head():
    w = _tiny(Hq=4, Hkv=2, prefix=9, lengths=(1,))
    op = OraclePool(w).append_events(w.n_prefill)
    N = w.n_prefill
    q = w.q(0)
    q[0, 1] = q[0, 0]  # heads 0,1 share kv head 0 -> identical outputs
    q[0, 2] = q[0, 0]  # head 2 uses kv head 1 -> differs
    out, _ = oracle.attention(op.g, op.k, op.v, [0], [N], [0, 0], [], [], [], q, w.scale)
    assert np.array_equal(out[0, 0], out[0, 1]) and not np.allclose(out[0, 0], out[0, 2])


def test_permuting_the_physical_interleave_leaves_the_output_unchanged():
    """Same logical streams, different physical orders (and page placements)."""
    outs = []
    for seed, paged, hm in ((7, False, False), (8, False, True), (9, True, False), (10, True, True)):
        w = _tiny("f32", lengths=(7, 5, 9), seed=seed, paged=paged)
        # give every stream-token fixed content, independent of where the shuffle puts it
        g = geom_of(w, hm)
        kp, vp, tail = g.new_pool(), g.new_pool(), np.zeros(1, np.int64)
        content = np.random.default_rng(1234)
        tok = {s: (content.standard_normal((60, w.Hkv, w.D)).astype(np.float32),
                   content.standard_normal((60, w.Hkv, w.D)).astype(np.float32)) for s in range(4)}
        seen = {s: 0 for s in range(4)}
        k = np.zeros((w.n_prefill, w.Hkv, w.D), np.float32)
        v = np.zeros_like(k)
        for e, s in enumerate(w.ev_stream[:w.n_prefill].tolist()):
            k[e], v[e] = tok[s][0][seen[s]], tok[s][1][seen[s]]
            seen[s] += 1
        oracle.append(g, kp, vp, w.ev_request[:w.n_prefill], k, v, tail)
        q = np.random.default_rng(99).standard_normal((w.n, w.Hq, w.D)).astype(np.float32)
        pl, offs, st, ct, sd = w.lists(0)
        outs.append(oracle.attention(g, kp, vp, w.dec_request, pl, offs, st, ct, sd, q, w.scale)[0])
    for o in outs[1:]:
        assert np.max(np.abs(o - outs[0])) < 1e-12


def test_constant_v_returns_the_constant_and_q0_returns_the_mean():
    w = _tiny("f32", lengths=(7, 5, 9))
    op = OraclePool(w).append_events(w.n_prefill)
    op_c = OraclePool(w)
    op_c.k[:] = op.k
    op_c.v[:] = 0.75
    pl, offs, st, ct, sd = w.lists(0)
    out, _ = oracle.attention(op_c.g, op_c.k, op_c.v, w.dec_request, pl, offs, st, ct, sd, w.q(0), w.scale)
    assert np.max(np.abs(out - 0.75)) < 1e-14
    out0, lse0 = oracle.attention(op.g, op.k, op.v, w.dec_request, pl, offs, st, ct, sd,
                                  np.zeros_like(w.q(0)), w.scale)
    _, v = w.kv_rows(0, w.n_prefill)
    for i in range(w.n):
        own = np.nonzero(w.ev_stream == w.dec_stream[i])[0]
        idx = np.concatenate([np.arange(40), own])
        for h in range(w.Hq):
            assert np.max(np.abs(out0[i, h] - v[idx, h // 2, :].astype(np.float64).mean(0))) < 1e-14
            assert abs(lse0[i, h] - np.log(len(idx))) < 1e-14


def test_membership_counts_with_indicator_v():
    """q = 0 and V[t] = e_(t mod D): out * |Vis| counts the visible slots in each residue class."""
    w = _tiny("f32", Hq=2, Hkv=1, lengths=(30, 41))
    g = geom_of(w)
    kp, vp, tail = g.new_pool(), g.new_pool(), np.zeros(1, np.int64)
    n = w.n_prefill
    v = np.zeros((n, 1, w.D), np.float32)
    v[np.arange(n), 0, np.arange(n) % w.D] = 1.0
    oracle.append(g, kp, vp, w.ev_request[:n], np.zeros_like(v), v, tail)
    pl, offs, st, ct, sd = w.lists(0)
    out, _ = oracle.attention(g, kp, vp, w.dec_request, pl, offs, st, ct, sd,
                              np.zeros((w.n, 2, w.D), np.float32), 1.0)
    for i in range(w.n):
        vis = np.concatenate([np.arange(40), np.nonzero(w.ev_stream == w.dec_stream[i])[0]])
        counts = np.bincount(vis % w.D, minlength=w.D)
        assert np.max(np.abs(out[i, 0] * len(vis) - counts)) < 1e-12


def test_one_and_two_visible_rows_closed_forms():
    w = _tiny("bf16", Hq=2, Hkv=1, prefix=6, lengths=(1,))
    op = OraclePool(w).append_events(w.n_prefill)
    k, v = w.kv_rows(0, w.n_prefill)
    q = w.q(0)
    out, _ = oracle.attention(op.g, op.k, op.v, [0], [0], [0, 1], [4], [1], [1], q, w.scale)
    assert np.array_equal(out[0, 0], to_f64(w, v)[4, 0])  # single row: exactly that V row
    out, _ = oracle.attention(op.g, op.k, op.v, [0], [0], [0, 2], [2, 5], [1, 1], [1, 1], q, w.scale)
    z = w.scale * to_f64(w, k)[[2, 5], 0, :] @ to_f64(w, q)[0, 1]
    p = 1.0 / (1.0 + np.exp(-(z[0] - z[1])))  # logistic of the logit difference
    ref = p * to_f64(w, v)[2, 0] + (1 - p) * to_f64(w, v)[5, 0]
    assert np.max(np.abs(out[0, 1] - ref)) < 1e-14


def test_duplicate_k_rows_get_equal_weight_and_shift_invariance():
    w = _tiny("f32", Hq=2, Hkv=1, prefix=8, lengths=(1,))
    g = geom_of(w)
    k, v = w.kv_rows(0, 9)
    k[3] = k[6]
    v[:] = 0
    v[3, 0, 0] = 1.0
    v[6, 0, 1] = 1.0
    kp, vp, tail = g.new_pool(), g.new_pool(), np.zeros(1, np.int64)
    oracle.append(g, kp, vp, [0] * 9, k, v, tail)
    q = w.q(0)
    out, lse = oracle.attention(g, kp, vp, [0], [9], [0, 0], [], [], [], q, 1.0)
    assert out[0, 0, 0] == out[0, 0, 1] and out[0, 0, 0] > 0
    # logits + 80 (q scaled so that |z| is huge): still finite, and lse moves by the shift
    big = (q.astype(np.float64) * 200).astype(np.float32)
    out2, lse2 = oracle.attention(g, kp, vp, [0], [9], [0, 0], [], [], [], big, 1.0)
    assert np.all(np.isfinite(out2)) and np.all(np.isfinite(lse2))
    zz = k[:9, 0, :].astype(np.float64) @ big[0, 0].astype(np.float64)
    assert abs(lse2[0, 0] - (zz.max() + np.log(np.sum(np.exp(zz - zz.max()))))) < 1e-9


def test_scale_enters_the_logits_linearly():
    """A dropped or misplaced softmax_scale changes this: scale s with q equals scale 1 with s*q
    (s a power of two, so the product is exact in bf16)."""
    w = _tiny("bf16", lengths=(7, 5))
    op = OraclePool(w).append_events(w.n_prefill)
    q = w.q(0)
    q_half = W.f32_to_bf16_bits(W.bf16_bits_to_f32(q) * np.float32(0.5))
    a, la = op.attention(q=q, scale=0.5)
    b, lb = op.attention(q=q_half, scale=1.0)
    c, _ = op.attention(q=q, scale=1.0)
    assert np.array_equal(a, b) and np.array_equal(la, lb) and not np.allclose(a, c)


# ---------------------------------------------------------------- split / merge (A4)
def test_split_and_merge_equals_whole():
    w = _tiny("bf16", lengths=(17, 5))
    op = OraclePool(w).append_events(w.n_prefill)
    pl, offs, st, ct, sd = w.lists(0)
    out, lse = op.attention()
    q = w.q(0)
    rng = np.random.default_rng(3)
    for i in range(w.n):
        rows = oracle.gather_map(op.g, 0, pl[i], st[offs[i]:offs[i + 1]], ct[offs[i]:offs[i + 1]],
                                 sd[offs[i]:offs[i + 1]])
        for h in (0, 3):
            cuts = np.sort(rng.choice(np.arange(1, len(rows)), size=4, replace=False))
            parts = np.split(rng.permutation(rows), cuts) + [np.zeros(0, np.int64)]  # + an empty one
            ms, ls, accs = zip(*[oracle.partial(op.g, op.k, op.v, p, q[i, h], h // 2, w.scale)
                                 for p in parts])
            assert ms[-1] == -np.inf and ls[-1] == 0.0 and not accs[-1].any()
            o, e = oracle.merge(ms, ls, np.stack(accs))
            assert np.max(np.abs(o - out[i, h])) < 1e-12 and abs(e - lse[i, h]) < 1e-12


def test_merge_against_direct_two_partial_formula():
    m = np.array([0.3, -1.2])
    l = np.array([2.0, 5.0])
    acc = np.array([[1.0, 2.0], [3.0, -4.0]])
    o, e = oracle.merge(m, l, acc)
    den = 2.0 * np.exp(0.3) + 5.0 * np.exp(-1.2)
    ref = (acc[0] * np.exp(0.3) + acc[1] * np.exp(-1.2)) / den
    assert np.max(np.abs(o - ref)) < 1e-15 and abs(e - np.log(den)) < 1e-15


# ---------------------------------------------------------------- brute force dense mask
@pytest.mark.parametrize("dtype,interleave", [("f32", "random"), ("bf16", "round_robin")])
def test_dense_mask_brute_force_equals_segment_lists(dtype, interleave):
    w = _tiny(dtype, Hq=4, Hkv=2, prefix=24, lengths=(6, 9, 4), interleave=interleave)
    op = OraclePool(w).append_events(w.n_prefill)
    out, lse = op.attention()
    ss, par, sp = w.fork_tree(0)
    q = w.q(0)
    for i in range(w.n):
        mask = oracle.visible_dense(ss, par, sp, int(w.dec_stream[i]))
        o, e = oracle.attention_dense(op.g, op.k, op.v, 0, mask, q[i], w.scale)
        assert np.max(np.abs(o - out[i])) < 1e-12 and np.max(np.abs(e - lse[i])) < 1e-12


def test_dense_brute_force_against_numpy_on_a_tiny_case():
    """attention_dense itself, against a masked softmax typed out with numpy."""
    w = _tiny("f32", Hq=2, Hkv=1, prefix=5, lengths=(3, 2))
    op = OraclePool(w).append_events(w.n_prefill)
    k, v = w.kv_rows(0, w.n_prefill)
    q = w.q(0)
    mask = np.array([1, 1, 0, 1, 1, 0, 1, 0, 1, 0], np.uint8)
    o, _ = oracle.attention_dense(op.g, op.k, op.v, 0, mask, q[1], w.scale)
    z = w.scale * k[:, 0, :].astype(np.float64) @ q[1, 1].astype(np.float64)
    z[mask == 0] = -np.inf
    p = np.exp(z - z.max())
    p /= p.sum()
    assert np.max(np.abs(o[1] - p @ v[:, 0, :].astype(np.float64))) < 1e-14


# ---------------------------------------------------------------- generators
def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7 + 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20, -3.14159], np.float32)
    b = W.f32_to_bf16_bits(x)
    assert b.tolist()[:4] == [0x3F80, 0x3F80, 0x3F82, 0x3F81]
    assert np.array_equal(b, torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))


def test_round_robin_is_right_aligned_lockstep():
    assert W._interleave_round_robin([3, 1, 2]).tolist() == [0, 0, 2, 0, 1, 2]


def test_configs_have_the_stated_shapes():
    w1, w2, w3 = W.config1(), W.config2(), W.config3()
    assert (w1.dtype, w1.Hq, w1.Hkv, w1.D, w1.n, w1.n_prefill) == ("f32", 4, 1, 64, 2, 256 + 32)
    assert (w2.Hq, w2.Hkv, w2.D, w2.n) == (32, 8, 128, 4) and 1024 + 4 * 32 <= w2.n_prefill <= 1024 + 4 * 256
    assert w3.steps == 64 and w3.n == 8 and len(w3.ev_stream) == w3.n_prefill + 64 * 8
    pl, offs, st, ct, sd = w3.lists(0)
    assert pl.min() == 8192 and np.all(sd[ct > 1] <= 8)  # the longest stream starts alone
    w4 = W.config4()
    assert w4.max_requests == 16 and w4.page_tokens == 16 and 16 <= w4.n <= 128
    used = set()
    tails = np.bincount(w4.ev_request, minlength=16)
    for r in range(16):
        pages = w4.page_table[r, :-(-int(tails[r]) // 16)].tolist()
        assert not (used & set(pages))
        used |= set(pages)


# ------------------------------------------------------------------ rotary embedding and rounding
def _rand_rows(seed, n=5, H=3, D=16):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((n, H, D)), rng.integers(0, 5000, size=n).astype(np.int32)


@pytest.mark.parametrize("D,theta", [(2, 10000.0), (16, 10000.0), (128, 10000.0), (64, 500000.0)])
def test_rope_equals_complex_multiplication(D, theta):
    """Plane f = (x[f], x[f + D/2]) read as a complex number is multiplied by
    exp(i pos theta^(-2f/D)) -- numpy's complex arithmetic as the independent statement."""
    x, pos = _rand_rows(3, D=D)
    got = oracle.rope(x, pos, theta)
    f = np.arange(D // 2)
    z = (x[..., : D // 2] + 1j * x[..., D // 2:]) * np.exp(1j * pos[:, None, None] * theta ** (-2.0 * f / D))
    assert np.allclose(got[..., : D // 2], z.real, rtol=0, atol=1e-12)
    assert np.allclose(got[..., D // 2:], z.imag, rtol=0, atol=1e-12)


def test_rope_two_dims_is_a_plane_rotation_by_pos_radians():
    x = np.array([[[1.0, 0.0]], [[0.0, 1.0]], [[2.0, -3.0]]])
    pos = np.array([1, 2, 7], np.int32)
    got = oracle.rope(x, pos, 10000.0)
    for i, p in enumerate(pos):
        c, s = math.cos(p), math.sin(p)
        a, b = x[i, 0]
        assert np.allclose(got[i, 0], [a * c - b * s, b * c + a * s], atol=1e-15)


def test_rope_invariants():
    x, pos = _rand_rows(5, n=6, H=2, D=32)
    y, _ = _rand_rows(6, n=6, H=2, D=32)
    th = 10000.0
    zero = np.zeros_like(pos)
    assert np.array_equal(oracle.rope(x, zero, th), x)  # position 0: identity
    rx = oracle.rope(x, pos, th)
    for f in range(16):  # every plane keeps its length
        assert np.allclose(rx[..., f] ** 2 + rx[..., f + 16] ** 2, x[..., f] ** 2 + x[..., f + 16] ** 2, rtol=1e-12)
    # composition: turning by a then by b = turning by a + b
    a = np.array([3, 10, 0, 77, 1000, 5], np.int32)
    assert np.allclose(oracle.rope(oracle.rope(x, a, th), pos, th), oracle.rope(x, a + pos, th), atol=1e-9)
    # relative position: <R(p) q, R(p') k> depends on p - p' only
    shift = np.full_like(pos, 123)
    d0 = (oracle.rope(x, pos, th) * oracle.rope(y, a, th)).sum(-1)
    d1 = (oracle.rope(x, pos + shift, th) * oracle.rope(y, a + shift, th)).sum(-1)
    assert np.allclose(d0, d1, atol=1e-9)
    # frequencies: at position 1 the unit vector of plane f turns by theta^(-2f/D) radians
    D = 32
    e = np.zeros((D // 2, 1, D))
    e[np.arange(D // 2), 0, np.arange(D // 2)] = 1.0
    r = oracle.rope(e, np.ones(D // 2, np.int32), th)
    ang = np.arctan2(r[np.arange(D // 2), 0, np.arange(D // 2) + D // 2], r[np.arange(D // 2), 0, np.arange(D // 2)])
    assert np.allclose(ang, np.exp(-2.0 * np.arange(D // 2) / D * math.log(th)), atol=1e-12)


def test_round_pool_is_round_to_nearest_even_once():
    # against torch's float32 -> bfloat16 conversion on float32-representable inputs
    rng = np.random.default_rng(11)
    x = np.concatenate([rng.standard_normal(4000) * 10.0 ** rng.integers(-6, 6, 4000),
                        [0.0, -0.0, 1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8), 255.5, 2.0 ** -130,
                         3.3895313892515355e38]]).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = oracle.round_pool("bf16", x.astype(np.float64))
    assert np.array_equal(got, want)
    # ties: 1 + 2^-8 lies halfway between 1 and 1 + 2^-7 -> even (1.0); 1 + 3 * 2^-8 -> 1 + 2^-6
    assert oracle.widen_pool("bf16", oracle.round_pool("bf16", np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8]))).tolist() == [1.0, 1 + 2.0 ** -6]
    # one rounding, not two: just above the tie in fp64, where a detour through fp32 would land on the tie
    y = np.array([1 + 2.0 ** -8 + 2.0 ** -40])
    assert oracle.widen_pool("bf16", oracle.round_pool("bf16", y))[0] == 1 + 2.0 ** -7
    assert np.array_equal(oracle.round_pool("f32", np.array([0.1, 1e-50, 3.0])), np.array([0.1, 1e-50, 3.0], np.float32))
    # widen is exact
    assert np.array_equal(oracle.widen_pool("bf16", want).astype(np.float32), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_attention_with_rotated_queries_and_keys_sees_relative_positions_only():
    """One stream, causal list: rotating q and every k by their positions, then shifting ALL
    positions by a constant, leaves the output unchanged; and attention_q64 on unrotated
    float64 queries equals attention() on the same queries in the pool dtype."""
    rng = np.random.default_rng(5)
    Hq, Hkv, D, N = 4, 2, 16, 40
    g = oracle.Geom("f32", Hq, Hkv, D, pool_tokens=64)
    k = rng.standard_normal((N, Hkv, D))
    v = rng.standard_normal((N, Hkv, D)).astype(np.float32)
    q = rng.standard_normal((1, Hq, D)).astype(np.float32)
    outs = []
    for shift in (0, 1000):
        pos = np.arange(N, dtype=np.int32) + shift
        kp, vp, tail = g.new_pool(), g.new_pool(), np.zeros(1, np.int64)
        kr = oracle.round_pool("f32", oracle.rope(k, pos, 10000.0))
        oracle.append(g, kp, vp, np.zeros(N, np.int32), kr, v, tail)
        qr = oracle.rope(q, np.array([N - 1 + shift], np.int32), 10000.0)
        o, _ = oracle.attention_q64(g, kp, vp, [0], [N], [0, 0], [], [], [], qr, 0.25)
        outs.append(o)
    assert np.allclose(outs[0], outs[1], atol=2e-5)  # fp32 pool rounding of the rotated keys
    o32, l32 = oracle.attention(g, kp, vp, [0], [N], [0, 0], [], [], [], q, 0.25)
    o64, l64 = oracle.attention_q64(g, kp, vp, [0], [N], [0, 0], [], [], [], q.astype(np.float64), 0.25)
    assert np.array_equal(o32, o64) and np.array_equal(l32, l64)


# ------------------------------------------------------------------ visibility with synchronisation
def _reach_by_bfs(events, q_slot):
    """Independent statement of Figure 2b with sync edges, in plain Python: predecessor sets
    built while walking the history, then a breadth-first search backwards."""
    last, preds = {}, []
    for t, e in enumerate(events):
        ps = set()
        if e["new"]:
            if e["parent"] >= 0:
                ps.add(last[e["parent"]])
        else:
            ps.add(last[e["stream"]])
        for j in e["join"]:
            ps.add(last[j])
        preds.append(ps)
        last[e["stream"]] = t
    seen, todo = {q_slot}, [q_slot]
    while todo:
        for u in preds[todo.pop()]:
            if u not in seen:
                seen.add(u)
                todo.append(u)
    return sorted(seen)


def _events_arrays(events):
    ev_s = np.array([e["stream"] for e in events], np.int32)
    ev_p = np.array([e["parent"] for e in events], np.int32)
    ev_n = np.array([1 if e["new"] else 0 for e in events], np.uint8)
    joins = {t: e["join"] for t, e in enumerate(events) if e["join"]}
    return ev_s, ev_p, ev_n, joins


def test_paper_worked_example_after_sync():
    fx = json.load(open(os.path.join(HERE, "golden", "paper_sec3_sync.json")))
    joins = {int(k): v for k, v in fx["join"].items()}
    for f in fx["facts"]:
        mask = oracle.visible_events(fx["ev_stream"], fx["ev_parent"], fx["ev_new"], joins, f["query_slot"])
        if f.get("sees_all_slots_up_to_itself"):
            assert mask[: f["query_slot"] + 1].all()
        else:
            assert all(mask[t] for t in f["must_see"]) and not any(mask[t] for t in f["must_not_see"])
    # before the sync token is in the pool the main thread sees neither fork (the first fixture's fact)
    main_before = oracle.visible_events(fx["ev_stream"], fx["ev_parent"], fx["ev_new"], joins, 24)
    assert np.nonzero(main_before)[0].tolist() == list(range(22)) + [24]


@pytest.mark.parametrize("seed", range(10))
def test_visible_events_equals_bfs_on_random_fork_sync_histories(seed):
    events = W.random_fork_sync_history(seed, n_slots=90, max_ids=5)
    ev_s, ev_p, ev_n, joins = _events_arrays(events)
    assert joins, "the generator should produce at least one synchronisation at this length"
    for q in range(0, len(events), 3):
        mask = oracle.visible_events(ev_s, ev_p, ev_n, joins, q)
        assert np.nonzero(mask)[0].tolist() == _reach_by_bfs(events, q)
    # a joined thread's tokens are visible after the sync token and not before
    t_sync = min(joins)
    child = joins[t_sync][0]
    child_tok = int(np.nonzero(ev_s[:t_sync] == child)[0][-1])
    owner_before = int(np.nonzero(ev_s[:t_sync] == ev_s[t_sync])[0][-1])
    assert oracle.visible_events(ev_s, ev_p, ev_n, joins, t_sync)[child_tok] == 1
    assert oracle.visible_events(ev_s, ev_p, ev_n, joins, owner_before)[child_tok] == 0


@pytest.mark.parametrize("seed", range(6))
def test_visible_events_without_syncs_is_the_ancestor_rule(seed):
    """No synchronisation: reachability reduces to the ancestor rule of visible_dense."""
    ev_s, ev_p = W.random_fork_history(seed, n_slots=60, max_streams=7)
    n_streams = int(ev_s.max()) + 1
    parent, spawn, ev_n = np.full(n_streams, -1, np.int32), np.zeros(n_streams, np.int64), np.zeros(len(ev_s), np.uint8)
    seen = set()
    for t, (s, p) in enumerate(zip(ev_s.tolist(), ev_p.tolist())):
        if s not in seen:
            seen.add(s)
            parent[s], spawn[s], ev_n[t] = p, t, 1
    for s in range(n_streams):
        last = int(np.nonzero(ev_s == s)[0][-1])
        dense = oracle.visible_dense(ev_s, parent, spawn, s)
        reach = oracle.visible_events(ev_s, ev_p, ev_n, None, last)
        assert np.array_equal(reach[: last + 1], dense[: last + 1]) and not reach[last + 1:].any()


# ------------------------------------------------------------------ the interpreter's control flow
def test_interpreter_reproduces_the_papers_timeline():
    from oracle import pasta_interp as I
    fx = json.load(open(os.path.join(HERE, "golden", "paper_sec3_replay.json")))
    f = fx["facts"]
    toks, passes = I.interpret([tuple(o) for o in fx["ops"]], fx["n_prompt"], fx["n_prompt"], 4)
    for p in range(3):
        assert [[t["slot"], t["stream"]] for t in toks if t["pass_"] == p] == f[f"pass{p}"]
    sync = [t for t in toks if t["join"]]
    assert len(sync) == 1 and sync[0]["slot"] == f["sync_slot"] and sync[0]["pass_"] == f["sync_pass"]
    assert sync[0]["join"] == f["sync_joins"] and sync[0]["stream"] == 0
    assert max(t["pass_"] for t in toks if t["stream"] == 2) == f["fork2_last_pass"]
    assert max(t["pass_"] for t in toks if t["stream"] == 1) == f["fork1_last_pass"]
    assert len(toks) == f["n_tokens"] and passes == f["n_passes"]
    # while it waits, the main thread feeds nothing; afterwards its tokens see every slot before them
    assert not [t for t in toks if t["stream"] == 0 and 1 < t["pass_"] < f["sync_pass"]]
    ev_s = [0] * fx["n_prompt"] + [t["stream"] for t in toks]
    ev_p = [-1] * fx["n_prompt"] + [t["parent"] for t in toks]
    ev_n = [1] + [0] * (fx["n_prompt"] - 1) + [1 if t["new"] else 0 for t in toks]
    joins = {t["slot"]: t["join"] for t in toks if t["join"]}
    last = toks[-1]["slot"]
    assert oracle.visible_events(ev_s, ev_p, ev_n, joins, last)[: last + 1].all()
    # Fork#1's token of pass 2 (the text's 'find'): sees its thread and the prompt, not the second promise / <async>
    m = oracle.visible_events(ev_s, ev_p, ev_n, joins, 26)
    assert m[20] and m[21] and m[22] and m[25] and not m[23] and not m[24] and not m[27]


@pytest.mark.parametrize("seed", range(5))
def test_interpreter_invariants_on_synthetic_traces(seed):
    from oracle import pasta_interp as I
    ops = W.synthetic_trace(seed, n_promises=5)
    toks, passes = I.interpret(ops, 100, 40, 8)
    n_text = sum(a for k, a, b in ops if k == 0)
    n_prom = sum(1 for k, a, b in ops if k == 1)
    n_sync = sum(1 for k, a, b in ops if k == 2)
    assert len(toks) == n_text + n_sync + sum(3 + b for k, a, b in ops if k == 1)  # promise, <async>, b, </async>
    assert [t["slot"] for t in toks] == list(range(40, 40 + len(toks)))
    assert sum(1 for t in toks if t["new"]) == n_prom and sum(1 for t in toks if t["join"]) <= n_sync
    # at most one token per thread and pass (two for the main thread's promise + the inserted <async>)
    for p in range(passes):
        ids = [t["stream"] for t in toks if t["pass_"] == p]
        assert len(ids) == len(set(ids)) and ids
    # the longest chain: a pass count no smaller than the main thread's own tokens, no larger than all tokens
    assert n_text + n_prom + n_sync <= passes <= len(toks)
    # estimated position ids: the main thread's ids increase; behind a promise they jump by 1 + predicted length
    main = [t for t in toks if t["stream"] == 0]
    assert all(b["pos"] > a["pos"] for a, b in zip(main, main[1:]))
    preds = [a for k, a, b in ops if k == 1]
    jumps = [b["pos"] - a["pos"] - 1 for a, b in zip(main, main[1:]) if b["pos"] - a["pos"] > 1]
    assert jumps == [x for x in preds if x > 0]
    # a fork counts on from its promise
    for t in toks:
        if t["new"]:
            prom = [m for m in main if m["slot"] == t["slot"] - 1][0]
            assert t["pos"] == prom["pos"] + 1


def test_committed_fixtures_are_what_their_script_writes():
    """tests/golden/make_fixtures.py derives the two timeline fixtures from the numbers the paper
    prints (it calls neither the library nor the oracle); the committed files must be its output."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(HERE, "golden", "make_fixtures.py"), "--check"],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
