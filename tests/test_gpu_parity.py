"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle, element by
element on the same seeded inputs.  Integer work (slots, pool bytes, gather maps) must be
bit-exact; outputs must be within max-abs 2e-2 AND relative-L2 1e-2 for bf16, 1e-5 / 1e-5
for fp32."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
from paper_2502_11517_amd import binding as B
from paper_2502_11517_amd import workloads as W
from util import OraclePool, check_close, to_f64

pytestmark = pytest.mark.gpu

LAYOUTS = [B.TOKEN_MAJOR, B.HEAD_MAJOR]


def _session(w, **kw):
    from paper_2502_11517_amd.harness import Session
    return Session(w, **kw)


def _out64(w, t):
    from paper_2502_11517_amd.harness import to_host_bits
    torch.cuda.synchronize()
    return to_f64(w, to_host_bits(t, w.dtype))


def _oracle_step(w, op, step, q, sel):
    """The oracle's outputs, lse and gather maps of the selected streams of one step."""
    pl, offs, st, ct, sd = w.lists(step)
    offs_sel, st_s, ct_s, sd_s = [0], [], [], []
    for i in sel:
        st_s += st[offs[i]:offs[i + 1]].tolist()
        ct_s += ct[offs[i]:offs[i + 1]].tolist()
        sd_s += sd[offs[i]:offs[i + 1]].tolist()
        offs_sel.append(len(st_s))
    ref, ref_lse = oracle.attention(op.g, op.k, op.v, w.dec_request[sel], pl[sel], offs_sel, st_s, ct_s, sd_s,
                                    q[sel], w.scale)
    maps = [oracle.gather_map(op.g, int(w.dec_request[i]), int(pl[i]), st[offs[i]:offs[i + 1]],
                              ct[offs[i]:offs[i + 1]], sd[offs[i]:offs[i + 1]]) for i in sel]
    return ref, ref_lse, maps


def _check_step(w, s, op, step=0, *, explicit=True, flags=0, q=None, streams=None, what="", ref_cache=None):
    """Decode on the GPU, compare outputs, lse and gather maps with the oracle.
    streams: subset of output rows to check (None: every stream).  ref_cache: a dict that keeps the
    oracle's result for (step, selection), so that several GPU modes over the same state and lists
    (explicit / maintained, kernel variants) are compared with ONE oracle evaluation."""
    out, lse, (goffs, grows) = s.decode(step, explicit=explicit, flags=flags, q=q, want_gather=True)
    got = _out64(w, out)
    lse = lse.cpu().numpy().astype(np.float64)
    grows = grows.cpu().numpy()
    sel = list(range(w.n)) if streams is None else list(streams)
    key = (step, tuple(sel), None if q is None else q.tobytes())
    if ref_cache is not None and key in ref_cache:
        ref, ref_lse, maps = ref_cache[key]
    else:
        ref, ref_lse, maps = _oracle_step(w, op, step, w.q(step) if q is None else q, sel)
        if ref_cache is not None:
            ref_cache[key] = (ref, ref_lse, maps)
    res = check_close(got[sel], ref, w.dtype, what or w.name)
    assert np.max(np.abs(lse[sel] - ref_lse)) <= (2e-2 if w.dtype == "bf16" else 1e-4), "lse"
    for i, exp in zip(sel, maps):  # gather maps: bit-exact, in list order
        assert goffs[i + 1] - goffs[i] == len(exp)
        assert np.array_equal(grows[goffs[i]:goffs[i + 1]].astype(np.int64), exp), f"gather map of stream {i}"
    return res


def _check_pool(w, s, op):
    """Every row that was appended, every kv head, K and V, bit for bit (whatever the layout); rows
    that were never appended are uninitialised device memory and are not looked at."""
    torch.cuda.synchronize()
    k, v = s.pool_bits(0)
    tails = np.bincount(w.ev_request[:op.n_done], minlength=w.max_requests)
    D, H = w.D, w.Hkv
    offs = np.fromiter((oracle.elem_offset(op.g, oracle.phys_row(op.g, r, t), h)
                        for r in range(w.max_requests) for t in range(int(tails[r])) for h in range(H)),
                       np.int64, count=int(tails.sum()) * H)
    assert len(np.unique(offs)) == len(offs)
    for lo in range(0, len(offs), 1 << 16):  # in pieces: the index array of a whole pool is large
        idx = (offs[lo:lo + (1 << 16), None] + np.arange(D)[None, :]).ravel()
        assert np.array_equal(k[idx], op.k[idx]), "K pool bytes"
        assert np.array_equal(v[idx], op.v[idx]), "V pool bytes"


# ------------------------------------------------------------------------- the five configs
@pytest.mark.parametrize("layout", LAYOUTS)
def test_config1_tiny_fp32(layout):
    w = W.config1()
    s = _session(w, kv_layout=layout)
    op = OraclePool(w, head_major=(layout == B.HEAD_MAJOR)).append_events(w.n_prefill)
    s.append_events(w.n_prefill)
    _check_pool(w, s, op)
    _check_step(w, s, op)
    _check_step(w, s, op, explicit=False)
    s.close()


@pytest.mark.parametrize("layout", LAYOUTS)
def test_config2_llama8b_prefix1k_4_streams(layout):
    w = W.config2()
    s = _session(w, kv_layout=layout)
    op = OraclePool(w, head_major=(layout == B.HEAD_MAJOR)).append_events(w.n_prefill)
    s.append_events(w.n_prefill)
    _check_pool(w, s, op)
    a = _check_step(w, s, op)
    b = _check_step(w, s, op, explicit=False)
    c = _check_step(w, s, op, flags=B.DECODE_NO_MFMA)
    print("cfg2 errors (mfma, maintained, no-mfma):", a, b, c)
    s.close()


@pytest.mark.parametrize("layout", LAYOUTS)
def test_config3_prefix8k_8_streams_64_steps(layout):
    w = W.config3()
    s = _session(w, kv_layout=layout)
    op = OraclePool(w, head_major=(layout == B.HEAD_MAJOR))
    s.append_events(w.n_prefill)
    op.append_events(w.n_prefill)
    for step in range(w.steps):
        hi = w.n_events(step)
        s.append_events(hi, chunk=w.n)  # one call of 8 rows: the step's append
        if step in (0, 1, 31, 63):
            op.append_events(hi)
            _check_step(w, s, op, step, explicit=(step != 31), what=f"cfg3 step {step}")
        else:
            s.decode(step, explicit=False, want_lse=False)
    _check_pool(w, s, op)
    s.close()


def test_config3_in_the_launch_configuration_of_the_bench():
    """Config 3 at full size exactly as bench.py runs it: head-major pool, the step's eight rows
    appended with PASTA_APPEND_DEFER (they ride with the decode launch), lists maintained by the
    library; outputs, lse and gather maps of sampled steps against the oracle, the pool at the end."""
    w = W.config3()
    s = _session(w, kv_layout=B.HEAD_MAJOR)
    op = OraclePool(w, head_major=True)
    s.append_events(w.n_prefill)
    op.append_events(w.n_prefill)
    keep = []
    for step in range(w.steps):
        hi = w.n_events(step)
        s.append_events(hi, chunk=w.n, flags=B.APPEND_DEFER)
        keep.append(s._keep_rows)
        if step in (0, 1, 2, 30, 62, 63):
            op.append_events(hi)
            _check_step(w, s, op, step, explicit=False, what=f"cfg3 as benched, step {step}")
        else:
            s.decode(step, explicit=False, want_lse=False)
    _check_pool(w, s, op)
    s.close()


def test_config4_ragged_paged_batch():
    """Every one of the 56 streams, both pool layouts, explicit and maintained lists."""
    w = W.config4()
    for layout in LAYOUTS:
        s = _session(w, kv_layout=layout)
        op = OraclePool(w, head_major=(layout == B.HEAD_MAJOR)).append_events(w.n_prefill)
        s.append_events(w.n_prefill)
        _check_pool(w, s, op)
        cache = {}
        _check_step(w, s, op, ref_cache=cache)
        _check_step(w, s, op, explicit=False, ref_cache=cache)
        s.close()


@pytest.mark.parametrize("layout", LAYOUTS)
def test_config5_long_context_nested_fork(layout):
    """Every one of the 16 streams x 64 heads (all four 32-row groups of the stacked queries), explicit
    and maintained lists; the oracle runs once per layout."""
    w = W.config5()
    s = _session(w, kv_layout=layout)
    op = OraclePool(w, head_major=(layout == B.HEAD_MAJOR)).append_events(w.n_prefill)
    s.append_events(w.n_prefill)
    _check_pool(w, s, op)
    cache = {}
    res = _check_step(w, s, op, ref_cache=cache)
    print("cfg5 errors:", res)
    _check_step(w, s, op, explicit=False, ref_cache=cache)
    s.close()


# ------------------------------------------------------------------------- shapes and edges
@pytest.mark.parametrize("dtype,Hq,Hkv,D", [("bf16", 8, 8, 128), ("bf16", 8, 4, 128), ("bf16", 16, 2, 128),
                                            ("bf16", 8, 2, 64), ("f32", 8, 2, 128), ("f32", 2, 2, 64),
                                            ("bf16", 64, 8, 128)])
def test_head_shapes(dtype, Hq, Hkv, D):
    w = W.single_request("shape", dtype, Hq, Hkv, D, D ** -0.5, 21, 700, [40, 3, 129, 77], "random")
    s = _session(w)
    op = OraclePool(w).append_events(w.n_prefill)
    s.append_events(w.n_prefill)
    _check_step(w, s, op)
    s.close()


@pytest.mark.parametrize("prefix,lengths", [(128, [1]), (127, [5, 5]), (129, [200, 1]), (1000, [1, 1, 1]),
                                            (4096 + 17, [130] * 9), (2, [300, 300]), (256, [64] * 33),
                                            (512, [20] * 40)])
def test_ragged_tiles_and_stream_counts(prefix, lengths):
    """Prefix lengths around the tile size; more stacked rows than one 32-row group (9 streams x 4:
    a full group and a ragged one; 33 streams: five groups); 40 streams x 16 heads = 640 output
    rows, which takes the narrow form of the merge."""
    w = W.single_request("ragged", "bf16", 16, 4, 128, 1.0, 33, prefix, lengths, "round_robin", k_std=128 ** -0.5)
    s = _session(w)
    op = OraclePool(w).append_events(w.n_prefill)
    s.append_events(w.n_prefill)
    _check_step(w, s, op)
    _check_step(w, s, op, explicit=False)
    s.close()


def test_single_stream_no_fork_is_causal_decode():
    w = W.single_request("nofork", "bf16", 32, 8, 128, 1.0, 5, 3000, [1], "random", k_std=128 ** -0.5)
    # the only decoding stream is the root itself: replace the fork by the root's own last token
    w.ev_stream[:] = 0
    w.ev_parent[:] = -1
    w.dec_stream[:] = 0
    w.anc_slots = [[]]
    s = _session(w)
    op = OraclePool(w).append_events(w.n_prefill)
    s.append_events(w.n_prefill)
    pl, *_ = w.lists(0)
    assert pl.tolist() == [3001]
    _check_step(w, s, op)
    _check_step(w, s, op, explicit=False)
    s.close()


def test_post_sync_stream_sees_several_forks_without_kv_movement():
    """After the sync point the main thread lists the prefix, both forks' interleaved rows and
    its own new token: one stream attending to several asynchronously decoded threads."""
    w = W.single_request("sync", "bf16", 8, 2, 128, 1.0, 8, 300, [37, 22], "random", k_std=128 ** -0.5)
    n0 = w.n_prefill
    w.ev_request = np.append(w.ev_request[:n0], 0).astype(np.int32)
    w.ev_stream = np.append(w.ev_stream[:n0], 0).astype(np.int32)   # the deferred sync token, root's
    w.ev_parent = np.append(w.ev_parent[:n0], -1).astype(np.int32)
    w.n_prefill = n0 + 1
    w.dec_stream = np.asarray([0], np.int32)
    w.dec_request = np.asarray([0], np.int32)
    w.anc_slots = [list(range(300, n0))]  # the forks' rows; the root's own slots come from the history
    s = _session(w)
    op = OraclePool(w).append_events(w.n_prefill)
    s.append_events(w.n_prefill)
    pl, offs, st, ct, sd = w.lists(0)
    assert pl.tolist() == [n0 + 1]
    _check_step(w, s, op)  # explicit lists only: the maintained list of the root has no join yet
    s.close()


def test_stream_with_no_private_rows_and_request_with_no_common_prefix():
    # (e) prefix only: a stream listing just [0, P); private only: lists that start above 0
    w = W.single_request("edge", "bf16", 8, 2, 128, 1.0, 9, 512, [30, 40], "random", k_std=128 ** -0.5)
    s = _session(w)
    op = OraclePool(w).append_events(w.n_prefill)
    s.append_events(w.n_prefill)
    from paper_2502_11517_amd.harness import to_device
    q = w.q(0)
    qd = to_device(q, w.dtype, s.device)
    out = torch.empty_like(qd)
    cases = [
        ([512, 512], [0, 0, 0], [], [], []),                        # prefix only, both streams
        ([0, 0], [0, 1, 2], [3, 100], [500, 400], [1, 1]),          # no common prefix at all
        ([512, 0], [0, 0, 1], [520], [9], [2]),                     # mixed: common prefix is 0
        ([300, 512], [0, 1, 1], [301], [70], [3]),                  # different prefix lengths
    ]
    for lists in cases:
        s.h.decode_step(0, w.dec_request, w.dec_stream, qd, out, lists=lists)
        ref, _ = oracle.attention(op.g, op.k, op.v, w.dec_request, *lists, q, w.scale)
        check_close(_out64(w, out), ref, w.dtype, f"lists {lists[0]}")
    s.close()


def test_one_visible_row_returns_that_v_row_bit_exactly():
    w = W.single_request("one", "bf16", 8, 2, 128, 1.0, 10, 200, [5], "random", k_std=128 ** -0.5)
    s = _session(w)
    s.append_events(w.n_prefill)
    from paper_2502_11517_amd.harness import to_device, to_host_bits
    qd = to_device(w.q(0), w.dtype, s.device)
    out = torch.empty_like(qd)
    s.h.decode_step(0, [0], [1], qd, out, lists=([0], [0, 1], [77], [1], [1]))
    torch.cuda.synchronize()
    _, v = w.kv_rows(0, w.n_prefill)
    got = to_host_bits(out, w.dtype)[0]
    for h in range(w.Hq):
        assert np.array_equal(got[h], v[77, h // 4])
    s.close()


# ------------------------------------------------------------------------- numerics under stress
@pytest.mark.parametrize("case", ["peaked", "planted", "large_v", "shifted", "membership"])
def test_adversarial_values(case):
    w = W.single_request("adv_" + case, "bf16", 16, 4, 128, 1.0, 44, 1500, [90, 260, 31], "random",
                         k_std=128 ** -0.5, v_std=10.0 if case == "large_v" else 1.0)
    q = w.q(0)
    s = _session(w)
    op = OraclePool(w)
    n = w.n_prefill
    k, v = w.kv_rows(0, n)
    if case == "peaked":  # q x 8: softmax close to one-hot, running max rescales
        q = W.f32_to_bf16_bits(W.bf16_bits_to_f32(q) * np.float32(8.0))
    if case == "planted":  # one K row = +c q: near one-hot on a known row
        qf = W.bf16_bits_to_f32(q)
        k = k.copy()
        k[1234, 1] = W.f32_to_bf16_bits(qf[0, 4] * np.float32(0.5))
    if case == "shifted":  # all logits moved by about +80: max subtraction must hold
        qf = W.bf16_bits_to_f32(q).astype(np.float64)
        kf = W.bf16_bits_to_f32(k).astype(np.float64)
        for g in range(w.Hkv):
            d = qf[0, g * 4] / np.dot(qf[0, g * 4], qf[0, g * 4]) * 80.0
            kf[:, g, :] += d
        k = W.f32_to_bf16_bits(kf.astype(np.float32))
    if case == "membership":  # q = 0, V[t] = e_(t mod D): out * |Vis| = class counts, exactly
        q = np.zeros_like(q)
        vf = np.zeros((n, w.Hkv, w.D), np.float32)
        vf[np.arange(n), :, np.arange(n) % w.D] = 1.0
        v = W.f32_to_bf16_bits(vf)
    from paper_2502_11517_amd.harness import to_device
    kd, vd = to_device(k, w.dtype, s.device), to_device(v, w.dtype, s.device)
    s.h.append_kv(0, w.ev_request[:n], w.ev_stream[:n], kd, vd, parent_stream=w.ev_parent[:n])
    rc, _ = oracle.append(op.g, op.k, op.v, w.ev_request[:n], k, v, op.tail)
    assert rc == 0
    op.n_done = n
    res = _check_step(w, s, op, q=q)
    print(case, res)
    if case == "membership":
        out, _, _ = s.decode(0, q=q)
        got = _out64(w, out)
        pl, offs, st, ct, sd = w.lists(0)
        for i in range(w.n):
            vis = oracle.gather_map(op.g, 0, int(pl[i]), st[offs[i]:offs[i + 1]], ct[offs[i]:offs[i + 1]],
                                    sd[offs[i]:offs[i + 1]])
            counts = np.bincount(vis % w.D, minlength=w.D)
            assert np.max(np.abs(got[i, 0] * len(vis) - counts)) < 0.06  # bf16 output rounding of ~14/1800
    s.close()


def test_multi_layer_pools_share_slots():
    w = W.single_request("layers", "bf16", 8, 2, 128, 1.0, 12, 400, [50, 60], "random", k_std=128 ** -0.5)
    s = _session(w, n_layers=3)
    from paper_2502_11517_amd.harness import to_device
    n = w.n_prefill
    k, v = w.kv_rows(0, n)
    ops = []
    for layer in range(3):  # layer l holds the rows rolled by l along the head-dim axis
        kl, vl = np.roll(k, layer, axis=2), np.roll(v, layer, axis=2)
        s.h.append_kv(layer, w.ev_request[:n], w.ev_stream[:n], to_device(kl, w.dtype, s.device),
                      to_device(vl, w.dtype, s.device), parent_stream=w.ev_parent[:n])
        op = OraclePool(w)
        oracle.append(op.g, op.k, op.v, w.ev_request[:n], kl, vl, op.tail)
        ops.append(op)
    for layer in (2, 0, 1):
        out, _, _ = s.decode(0, layer=layer, explicit=(layer != 1))
        ref, _ = ops[layer].attention()
        check_close(_out64(w, out), ref, w.dtype, f"layer {layer}")
    s.close()


def test_pool_filled_to_its_last_slot_with_every_stream_id_decoding():
    """Maximum sizes: the history fills the request's pool share exactly, and the step carries
    max_requests * max_streams query rows (all seven forks and the root).  The next append is
    refused with E_CAPACITY and leaves pool and lists as they were."""
    from paper_2502_11517_amd.harness import to_device, to_host_bits
    w = W.single_request("full", "bf16", 8, 2, 128, 1.0, 21, 448, [10, 9, 9, 9, 9, 9, 9], "random",
                         k_std=128 ** -0.5, slack=0)
    assert w.pool_tokens == w.n_prefill == 512 and w.max_streams == 8
    s = _session(w)
    op = OraclePool(w).append_events(w.n_prefill)
    s.append_events(w.n_prefill)
    pl, offs, st, ct, sd = w.lists(0)
    # the root as eighth query row: it sees its own 448 rows
    rid = np.zeros(8, np.int32)
    sid = np.arange(1, 9, dtype=np.int32) % 8  # forks 1..7, then the root
    lists = (np.append(pl, 448), np.append(offs, offs[-1]), st, ct, sd)
    rng = np.random.default_rng(21)
    q = W.f32_to_bf16_bits(rng.standard_normal((8, w.Hq, w.D), dtype=np.float32))
    qd = to_device(q, w.dtype, s.device)
    ref, _ = oracle.attention(op.g, op.k, op.v, rid, *lists, q, w.scale)
    outs = []
    for explicit in (True, False):
        out = torch.empty_like(qd)
        s.h.decode_step(0, rid, sid, qd, out, lists=lists if explicit else None)
        check_close(_out64(w, out), ref, w.dtype, f"full pool, explicit={explicit}")
        outs.append(to_host_bits(out, w.dtype).copy())
    # slot 511 (the last of the pool) is somebody's newest row and was read
    assert max(int(a + (c - 1) * d) for a, c, d in zip(st, ct, sd)) == 511
    k1, v1 = w.kv_rows(0, 1)
    with pytest.raises(B.PastaError) as e:
        s.h.append_kv(0, [0], [3], to_device(k1, w.dtype, s.device), to_device(v1, w.dtype, s.device))
    assert e.value.code == B.E_CAPACITY
    _check_pool(w, s, op)
    out = torch.empty_like(qd)
    s.h.decode_step(0, rid, sid, qd, out)
    torch.cuda.synchronize()
    assert np.array_equal(to_host_bits(out, w.dtype), outs[1])
    s.close()


@pytest.mark.parametrize("seed", range(4))
def test_maintained_lists_on_random_fork_histories_equal_dense_mask(seed):
    """Every live thread keeps decoding, forks open from any thread (nested too): the lists the
    library derives from parent_stream must name exactly the ancestor-rule set, and the
    outputs must match the brute-force dense-mask attention."""
    ev_s, ev_p = W.random_fork_history(500 + seed, n_slots=700, max_streams=9, p_fork=0.02, p_retire=0.004)
    n_streams = int(ev_s.max()) + 1
    w = W.Workload(name="forks", dtype="bf16", Hq=8, Hkv=2, D=128, scale=1.0, seed=900 + seed, max_requests=1,
                   pool_tokens=768, max_streams=n_streams, k_std=128 ** -0.5)
    w.ev_request = np.zeros(len(ev_s), np.int32)
    w.ev_stream, w.ev_parent, w.n_prefill = ev_s, ev_p, len(ev_s)
    w.dec_request = np.zeros(n_streams, np.int32)
    w.dec_stream = np.arange(n_streams, dtype=np.int32)
    s = _session(w)
    op = OraclePool(w).append_events(w.n_prefill)
    s.append_events(w.n_prefill)
    out, lse, (goffs, grows) = s.decode(0, explicit=False, want_gather=True)
    got = _out64(w, out)
    grows = grows.cpu().numpy()
    ss, par, sp = w.fork_tree(0)
    q = w.q(0)
    for i in range(n_streams):
        mask = oracle.visible_dense(ss, par, sp, i)
        assert np.array_equal(grows[goffs[i]:goffs[i + 1]], np.nonzero(mask)[0])
        ref, _ = oracle.attention_dense(op.g, op.k, op.v, 0, mask, q[i], w.scale)
        check_close(got[i], ref, w.dtype, f"stream {i}")
    s.close()


# ------------------------------------------------------------------------- random shapes
@pytest.mark.parametrize("seed", range(12))
def test_random_shapes_layouts_and_append_modes(seed):
    """Seeded random draws over what the launch plan depends on: heads per group, kv heads, prefix
    length (none, short, long enough for the long-chunk kernel variant), number and lengths of the
    streams, interleave, layout, contiguous or paged pool, eager or deferred append, two steps."""
    rng = np.random.default_rng(1000 + seed)
    G = int(rng.choice([1, 2, 4, 8]))
    Hkv = int(rng.choice([1, 2, 4, 8]))
    layout = LAYOUTS[int(rng.integers(2))]
    if seed % 3 == 2:  # paged, several requests
        w = W.config4(n_requests=int(rng.integers(1, 4)), seed=2000 + seed, pmin=int(rng.integers(1, 300)),
                      pmax=int(rng.integers(300, 5000)), page_tokens=int(rng.choice([8, 16, 32])))
        steps = 1
    else:
        n = int(rng.integers(1, 11))
        prefix = int(rng.choice([0, 1, 37, 500, 3000, 11000])) + int(rng.integers(0, 64))
        lengths = rng.integers(1, 300, size=n).tolist()
        steps = 2
        w = W.single_request("rand", "bf16", Hkv * G, Hkv, 128, 1.0, 3000 + seed, max(prefix, 1), lengths,
                             ["random", "round_robin"][int(rng.integers(2))], steps=steps, k_std=128 ** -0.5)
    s = _session(w, kv_layout=layout)
    op = OraclePool(w, head_major=(layout == B.HEAD_MAJOR))
    s.append_events(w.n_prefill)
    op.append_events(w.n_prefill)
    keep = []
    for step in range(steps):
        if w.steps > 1:
            hi = w.n_events(step)
            s.append_events(hi, chunk=w.n, flags=B.APPEND_DEFER if (seed + step) % 2 else 0)
            keep.append(getattr(s, "_keep_rows", None))
            op.append_events(hi)
        _check_step(w, s, op, step, explicit=bool((seed + step) % 2), what=f"random shape {seed}, step {step}")
    _check_pool(w, s, op)
    s.close()


# ------------------------------------------------------------------------- long prefix chunks
@pytest.mark.parametrize("layout", LAYOUTS)
def test_long_prefix_chunks_contiguous_pool_with_deferred_steps(layout):
    """A prefix long enough that every wave walks more than two 32-token blocks of its chunk (the
    kernel variant with the cheap addressing of plain blocks), of a ragged length so that full,
    ragged and deferred-row blocks meet in one launch; three append+decode steps."""
    w = W.config3(steps=3, prefix=12007, n_streams=5)
    s = _session(w, kv_layout=layout)
    op = OraclePool(w, head_major=(layout == B.HEAD_MAJOR))
    s.append_events(w.n_prefill)
    op.append_events(w.n_prefill)
    plan = np.zeros(8, np.int64)
    s.h.decode_step(0, w.dec_request, w.dec_stream, None, None, flags=B.DECODE_PLAN_ONLY, dbg_plan=plan)
    assert plan[4] > 256, "the chunk must span more than two blocks per wave"
    keep = []
    for step in range(w.steps):
        hi = w.n_events(step)
        s.append_events(hi, chunk=w.n, flags=B.APPEND_DEFER if step else 0)
        keep.append(getattr(s, "_keep_rows", None))
        op.append_events(hi)
        _check_step(w, s, op, step, explicit=(step == 1), what=f"long chunks, step {step}")
    _check_pool(w, s, op)
    s.close()


@pytest.mark.parametrize("page_tokens", [16, 64, 8])
def test_long_prefix_chunks_paged_pool(page_tokens):
    """The same variant on paged pools: pages of 16 and 64 tokens take the plain-block path
    (each half block inside one page), pages of 8 tokens must fall back to per-row addresses."""
    w = W.config4(n_requests=2, seed=77, pmin=9000, pmax=9500, page_tokens=page_tokens)
    for layout in LAYOUTS:
        s = _session(w, kv_layout=layout)
        op = OraclePool(w, head_major=(layout == B.HEAD_MAJOR)).append_events(w.n_prefill)
        s.append_events(w.n_prefill)
        plan = np.zeros(8, np.int64)
        s.h.decode_step(0, w.dec_request, w.dec_stream, None, None, flags=B.DECODE_PLAN_ONLY, dbg_plan=plan)
        assert plan[4] > 256
        cache = {}
        _check_step(w, s, op, what=f"paged {page_tokens}, layout {layout}", ref_cache=cache)
        _check_step(w, s, op, explicit=False, ref_cache=cache)
        s.close()


# ------------------------------------------------------------------------- more than 32 stacked rows
@pytest.mark.parametrize("Hq,Hkv,prefix,lengths", [
    (16, 4, 4096 + 17, [130] * 9),    # 36 rows: a full group and one of 4 rows (two waves only carry tiles)
    (16, 4, 100, [7] * 17),           # 68 rows, a prefix of less than one round
    (16, 4, 64 * 33, [3] * 33),       # 132 rows: two work-groups per (chunk, kv head), the second with 4 rows
    (64, 8, 1000, [40, 1, 300, 2, 9]),  # 8 heads per kv head, five streams: 40 rows
    (8, 1, 777, [50] * 6),            # one kv head, 48 rows
])
def test_wide_requests_four_row_groups_per_work_group(Hq, Hkv, prefix, lengths):
    """Requests with more than 32 stacked rows: the launch whose work-groups serve four 32-row groups each
    (one per wave) against the oracle, and against the row-group-per-work-group form of the same step."""
    w = W.single_request("wide", "bf16", Hq, Hkv, 128, 1.0, 41, prefix, lengths, "round_robin", k_std=128 ** -0.5)
    s = _session(w)
    op = OraclePool(w).append_events(w.n_prefill)
    s.append_events(w.n_prefill)
    plan, plan_rg = np.zeros(8, np.int64), np.zeros(8, np.int64)
    s.h.decode_step(0, w.dec_request, w.dec_stream, None, None, flags=B.DECODE_PLAN_ONLY | B.DECODE_FOUR_GROUPS, dbg_plan=plan)
    s.h.decode_step(0, w.dec_request, w.dec_stream, None, None, flags=B.DECODE_PLAN_ONLY | B.DECODE_ROW_GROUPS, dbg_plan=plan_rg)
    R = len(lengths) * (Hq // Hkv)
    n_chunks = -(-prefix // plan[4])
    assert plan[1] == n_chunks * Hkv * -(-R // 128)
    assert plan_rg[1] == -(-prefix // plan_rg[4]) * Hkv * -(-R // 32)
    cache = {}
    _check_step(w, s, op, flags=B.DECODE_FOUR_GROUPS, ref_cache=cache)
    _check_step(w, s, op, explicit=False, flags=B.DECODE_FOUR_GROUPS, ref_cache=cache)
    _check_step(w, s, op, flags=B.DECODE_ROW_GROUPS, ref_cache=cache)
    _check_step(w, s, op, ref_cache=cache)  # the form the library picks by itself
    _check_step(w, s, op, explicit=False, flags=B.DECODE_DEVICE_LISTS | B.DECODE_FOUR_GROUPS, ref_cache=cache)  # items derived by the kernels
    # the entry point that allocates nothing takes the same launch (its partial rows fit the static array here)
    from paper_2502_11517_amd.harness import to_device
    qd = to_device(w.q(0), w.dtype, s.device)
    out = torch.empty_like(qd)
    if w.n <= 24:  # (33 stream records do not fit the kernel arguments: that entry point then refuses the step)
        s.h.decode_step_noalloc(0, w.dec_request, w.dec_stream, qd, out, flags=B.DECODE_FOUR_GROUPS)
        check_close(_out64(w, out), cache[next(iter(cache))][0], w.dtype, "wide, no-alloc entry point")
    else:
        with pytest.raises(B.PastaError) as e:
            s.h.decode_step_noalloc(0, w.dec_request, w.dec_stream, qd, out, flags=B.DECODE_FOUR_GROUPS)
        assert e.value.code == B.E_CAPACITY
    s.close()


def test_wide_request_whose_prefix_ends_in_a_deferred_row():
    """Five streams fork right after the root's newest token, and that token and the forks arrive in ONE deferred
    append: the last row of the common prefix still sits in the caller's buffers when the wide work-groups
    read it."""
    w = W.single_request("fork_wide", "bf16", 64, 8, 128, 1.0, 5, 700, [1] * 5, "round_robin", k_std=128 ** -0.5)
    s = _session(w)
    op = OraclePool(w).append_events(w.n_prefill)
    s.append_events(w.n_prefill - 6)
    s.append_events(w.n_prefill, flags=B.APPEND_DEFER)
    pl, *_ = w.lists(0)
    assert min(pl.tolist()) == 700
    _check_step(w, s, op, flags=B.DECODE_FOUR_GROUPS)
    _check_pool(w, s, op)
    s.close()


@pytest.mark.parametrize("page_tokens", [16, 8])
def test_wide_requests_in_a_ragged_paged_batch(page_tokens):
    """Several requests of 5..9 streams x 8 heads per kv head, paged pools (pages of 8 tokens: one address per row)."""
    w = W.config4(n_requests=3, seed=91, pmin=200, pmax=2500, page_tokens=page_tokens, hq=64, hkv=8, smin=5, smax=9)
    s = _session(w)
    op = OraclePool(w).append_events(w.n_prefill)
    s.append_events(w.n_prefill)
    cache = {}
    _check_step(w, s, op, flags=B.DECODE_FOUR_GROUPS, ref_cache=cache)
    _check_step(w, s, op, explicit=False, flags=B.DECODE_FOUR_GROUPS, ref_cache=cache)
    s.close()


# ------------------------------------------------------------------------- deferred append
@pytest.mark.parametrize("layout", LAYOUTS)
def test_deferred_append_rides_with_the_decode_launch(layout):
    """PASTA_APPEND_DEFER: the step's rows are read from k_new / v_new by the attention launch,
    which also copies them into the pool; outputs and the final pool must be what the eager
    append gives."""
    w = W.config3(steps=6, prefix=1500, n_streams=5)
    s = _session(w, kv_layout=layout)
    op = OraclePool(w, head_major=(layout == B.HEAD_MAJOR))
    s.append_events(w.n_prefill)
    op.append_events(w.n_prefill)
    keep = []
    for step in range(w.steps):
        hi = w.n_events(step)
        s.append_events(hi, chunk=w.n, flags=B.APPEND_DEFER)
        keep.append(s._keep_rows)
        op.append_events(hi)
        _check_step(w, s, op, step, explicit=(step % 2 == 0), what=f"deferred step {step}")
    _check_pool(w, s, op)
    s.close()


def test_deferred_rows_in_the_prefix_and_in_other_streams_lists():
    from paper_2502_11517_amd.harness import to_device
    # (a) a single stream with no fork: the deferred row is the last row of its prefix
    w = W.single_request("nofork", "bf16", 8, 2, 128, 1.0, 5, 700, [1], "random", k_std=128 ** -0.5)
    w.ev_stream[:] = 0
    w.ev_parent[:] = -1
    w.dec_stream[:] = 0
    w.anc_slots = [[]]
    s = _session(w)
    op = OraclePool(w).append_events(w.n_prefill)
    s.append_events(w.n_prefill - 1)
    s.append_events(w.n_prefill, flags=B.APPEND_DEFER)
    _check_step(w, s, op)
    _check_pool(w, s, op)
    s.close()
    # (b) explicit lists that name rows another stream appended in the deferred call, paged pool
    w = W.single_request("cross", "bf16", 8, 2, 128, 1.0, 6, 300, [40, 50, 60], "random", k_std=128 ** -0.5)
    n0 = w.n_prefill
    w.page_tokens, w.pages_per_request = 16, -(-w.pool_tokens // 16)
    w.n_phys_pages = w.pages_per_request + 5
    w.page_table = np.random.default_rng(3).permutation(w.n_phys_pages)[:w.pages_per_request].astype(np.int32).reshape(1, -1)
    s = _session(w)
    op = OraclePool(w).append_events(n0)
    s.append_events(n0 - 3)
    s.append_events(n0, flags=B.APPEND_DEFER)          # the last three rows are deferred
    q = w.q(0)
    qd = to_device(q, w.dtype, s.device)
    out = torch.empty_like(qd)
    lists = ([300, 300, 0], [0, 1, 2, 4], [n0 - 3, n0 - 5, 10, n0 - 2], [3, 5, 20, 2], [1, 1, 7, 1])
    s.h.decode_step(0, w.dec_request, w.dec_stream, qd, out, lists=lists)
    ref, _ = oracle.attention(op.g, op.k, op.v, w.dec_request, *lists, q, w.scale)
    check_close(_out64(w, out), ref, w.dtype, "lists over deferred rows")
    _check_pool(w, s, op)
    s.close()


def test_deferred_append_falls_back_when_it_cannot_ride():
    """Interleaved requests in one call, a decode on another layer, a second append: K1 runs."""
    w = W.config4(n_requests=3, seed=77, pmin=100, pmax=300)
    s = _session(w)
    op = OraclePool(w).append_events(w.n_prefill)
    s.append_events(w.n_prefill - 40)
    lo = w.n_prefill - 40
    s.append_events(w.n_prefill - 20, flags=B.APPEND_DEFER)   # request 2's rows only: consecutive
    s.append_events(w.n_prefill, flags=B.APPEND_DEFER)        # flushes the first, defers the second
    _check_step(w, s, op)
    _check_pool(w, s, op)
    s.close()


def test_deferred_append_then_reserved_slots_written_by_the_caller():
    """A deferred append followed by an append that only reserves slots (the caller's own kernel
    writes those rows): the reserving call must first send the deferred rows to the pool, so that
    the next decode step reads the reserved slots from the pool and not from beyond the deferred
    call's k_new / v_new."""
    from paper_2502_11517_amd.harness import to_device
    w = W.config3(steps=3, prefix=700, n_streams=4)
    s = _session(w)  # token-major, contiguous: row `phys` of the pool viewed as [rows][Hkv][D]
    op = OraclePool(w)
    s.append_events(w.n_prefill)
    op.append_events(w.n_prefill)
    hi0, hi1 = w.n_events(0), w.n_events(1)
    s.append_events(hi0, chunk=w.n, flags=B.APPEND_DEFER)      # step 0's rows: deferred
    keep = s._keep_rows
    # step 1's rows: slots reserved by the library, rows written by the caller
    slots = s.h.append_kv(0, w.ev_request[hi0:hi1], w.ev_stream[hi0:hi1], None, None,
                          parent_stream=w.ev_parent[hi0:hi1], want_slots=True, flags=B.APPEND_RESERVE_ONLY)
    assert slots.tolist() == list(range(hi0, hi1))
    k, v = w.kv_rows(hi0, hi1)
    idx = torch.as_tensor(np.asarray(slots, np.int64), device=s.device)
    s.k_pool.view(-1, w.Hkv, w.D)[idx] = to_device(k, w.dtype, s.device)
    s.v_pool.view(-1, w.Hkv, w.D)[idx] = to_device(v, w.dtype, s.device)
    s.n_done = hi1
    op.append_events(hi1)
    _check_step(w, s, op, 1, explicit=False, what="defer, reserve, decode")
    _check_step(w, s, op, 1, explicit=True, what="defer, reserve, decode (explicit lists)")
    _check_pool(w, s, op)
    del keep
    s.close()


# ------------------------------------------------------------------------- rotary embedding
THETA = 10000.0


def _check_rope_pool(w, s, op, n_events):
    """Pool K rows after a rotating append: the oracle rotates in fp64 and rounds once; the
    kernel rotates in fp32 (angle reduced in fp64) and rounds once.  Where the fp32 result sits
    next to a rounding boundary the two may land on neighbouring values: at most 1 unit in the
    last place apart (bf16), and only on a small fraction of the elements.  V rows: bit-exact."""
    torch.cuda.synchronize()
    k, v = s.pool_bits(0)
    slots = w.event_slots(n_events)
    rows = np.array([oracle.phys_row(op.g, int(w.ev_request[e]), int(slots[e])) for e in range(n_events)])
    sample = rows[:: max(1, n_events // 600)]
    n_bad = n_all = 0
    for h in range(w.Hkv):
        offs = np.array([oracle.elem_offset(op.g, int(p), h) for p in sample])
        idx = (offs[:, None] + np.arange(w.D)[None, :]).ravel()
        assert np.array_equal(v[idx], op.v[idx])
        a, b = k[idx], op.k[idx]
        av, bv = oracle.widen_pool(w.dtype, a), oracle.widen_pool(w.dtype, b)
        # one unit in the last place of the oracle's value, plus the fp32 error of a plane whose two
        # products cancel (absolute ~1e-7 of the plane's length, many ulps of a result near zero)
        ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(bv), 1e-30))) - (7 if w.dtype == "bf16" else 23))
        assert np.all(np.abs(av - bv) <= ulp + 1e-6 * np.max(np.abs(bv))), "rotated K off by more than one ulp"
        n_bad += int((av != bv).sum())
        n_all += idx.size
    assert w.dtype == "f32" or n_bad <= 0.01 * n_all, f"{n_bad} of {n_all} rotated K elements differ"
    return n_bad, n_all


def _check_rope_step(w, s, op, step, positions, flags=0, explicit=True):
    qpos = w.q_positions(step)
    out, lse, _ = s.decode(step, explicit=explicit, flags=flags | B.DECODE_ROPE_Q, position=qpos)
    got = _out64(w, out)
    q64 = oracle.rope(oracle.widen_pool(w.dtype, w.q(step)), qpos, THETA)
    ref, ref_lse = oracle.attention_q64(op.g, op.k, op.v, w.dec_request, *w.lists(step), q64, w.scale)
    res = check_close(got, ref, w.dtype, f"{w.name} rope step {step}")
    assert np.max(np.abs(lse.cpu().numpy() - ref_lse)) <= (2e-2 if w.dtype == "bf16" else 1e-4)
    return res


@pytest.mark.parametrize("layout", LAYOUTS)
def test_rope_at_append_and_on_queries_config3_loop(layout):
    """K rotated by K1 on its way into the pool, Q rotated inside the attention kernel, position
    ids with jumps (a fork starts at its parent's next id, the parent skips ahead)."""
    w = W.config3(steps=6)
    pos = w.event_positions()
    s = _session(w, kv_layout=layout, rope_theta=THETA)
    op = OraclePool(w, head_major=(layout == B.HEAD_MAJOR))
    s.append_events(w.n_prefill, flags=B.APPEND_ROPE, positions=pos)
    op.append_events(w.n_prefill, positions=pos, theta=THETA)
    for step in range(w.steps):
        hi = w.n_events(step)
        # every other step defers the copy: the rows are then turned inside the attention launch
        s.append_events(hi, chunk=w.n, flags=B.APPEND_ROPE | (B.APPEND_DEFER if step % 2 else 0), positions=pos)
        op.append_events(hi, positions=pos, theta=THETA)
        res = _check_rope_step(w, s, op, step, pos, explicit=(step % 2 == 0))
    print("rope cfg3 errors:", res, "pool mismatches:", _check_rope_pool(w, s, op, w.n_events(w.steps - 1)))
    s.close()


@pytest.mark.parametrize("dtype,Hq,Hkv,D,flags", [("f32", 4, 1, 64, 0), ("f32", 8, 2, 128, 0),
                                                   ("bf16", 8, 2, 64, 0), ("bf16", 16, 4, 128, B.DECODE_NO_MFMA),
                                                   ("bf16", 64, 8, 128, 0)])
def test_rope_on_the_other_paths(dtype, Hq, Hkv, D, flags):
    """fp32 pools, D = 64 and the vector-ALU walker take Q from a rotated copy (k_rope_q); G = 8 on
    the matrix-core path; random interleave, so many short ranges."""
    w = W.single_request("rope", dtype, Hq, Hkv, D, D ** -0.5, 77, 300, [40, 3, 129, 77], "random")
    pos = w.event_positions()
    s = _session(w, rope_theta=THETA)
    op = OraclePool(w)
    s.append_events(w.n_prefill, flags=B.APPEND_ROPE, positions=pos)
    op.append_events(w.n_prefill, positions=pos, theta=THETA)
    _check_rope_pool(w, s, op, w.n_prefill)
    _check_rope_step(w, s, op, 0, pos, flags=flags)
    s.close()


def test_rope_large_positions_and_another_theta():
    """Position ids in the tens of thousands (angle = tens of thousands of radians at plane 0):
    the reduction of the angle has to be done in fp64 for the rotated keys to stay within one
    bf16 ulp of the oracle's."""
    w = W.single_request("rope_far", "bf16", 8, 2, 128, 128 ** -0.5, 78, 200, [30, 30], "round_robin")
    pos = w.event_positions() + 39000
    s = _session(w, rope_theta=500000.0)
    op = OraclePool(w)
    s.append_events(w.n_prefill, flags=B.APPEND_ROPE, positions=pos)
    op.append_events(w.n_prefill, positions=pos, theta=500000.0)
    _check_rope_pool(w, s, op, w.n_prefill)
    qpos = w.q_positions(0) + 39000
    out, lse, _ = s.decode(0, flags=B.DECODE_ROPE_Q, position=qpos)
    q64 = oracle.rope(oracle.widen_pool(w.dtype, w.q(0)), qpos, 500000.0)
    ref, _ = oracle.attention_q64(op.g, op.k, op.v, w.dec_request, *w.lists(0), q64, w.scale)
    check_close(_out64(w, out), ref, w.dtype, "rope far")
    s.close()


def test_rope_deferred_rows_are_turned_where_they_are_read_and_where_they_are_copied():
    """PASTA_APPEND_DEFER | PASTA_APPEND_ROPE: the attention launch reads the step's unrotated rows
    from k_new, turns them in its LDS tile, and turns them again on their way into the pool; a
    deferred rotating append that cannot ride (a second append arrives first) is flushed by K1.
    (a) no fork: the deferred row is the last row of the prefix; (b) explicit lists naming rows
    that other streams appended in the deferred call, paged pool; (c) flush."""
    from paper_2502_11517_amd.harness import to_device
    w = W.single_request("nofork", "bf16", 8, 2, 128, 1.0, 5, 700, [1], "random", k_std=128 ** -0.5)
    w.ev_stream[:] = 0
    w.ev_parent[:] = -1
    w.dec_stream[:] = 0
    w.anc_slots = [[]]
    pos = (np.arange(w.n_prefill) * 3 + 11).astype(np.int32)
    s = _session(w, rope_theta=THETA)
    op = OraclePool(w).append_events(w.n_prefill, positions=pos, theta=THETA)
    s.append_events(w.n_prefill - 1, flags=B.APPEND_ROPE, positions=pos)
    s.append_events(w.n_prefill, flags=B.APPEND_ROPE | B.APPEND_DEFER, positions=pos)
    _check_rope_step(w, s, op, 0, pos)
    _check_rope_pool(w, s, op, w.n_prefill)
    s.close()
    # (b)
    w = W.single_request("cross", "bf16", 8, 2, 128, 1.0, 6, 300, [40, 50, 60], "random", k_std=128 ** -0.5)
    n0 = w.n_prefill
    w.page_tokens, w.pages_per_request = 16, -(-w.pool_tokens // 16)
    w.n_phys_pages = w.pages_per_request + 5
    w.page_table = np.random.default_rng(3).permutation(w.n_phys_pages)[:w.pages_per_request].astype(np.int32).reshape(1, -1)
    pos = w.event_positions()
    s = _session(w, rope_theta=THETA)
    op = OraclePool(w).append_events(n0, positions=pos, theta=THETA)
    s.append_events(n0 - 3, flags=B.APPEND_ROPE, positions=pos)
    s.append_events(n0, flags=B.APPEND_ROPE | B.APPEND_DEFER, positions=pos)  # the last three rows are deferred
    q = w.q(0)
    qd = to_device(q, w.dtype, s.device)
    out = torch.empty_like(qd)
    lists = ([300, 300, 0], [0, 1, 2, 4], [n0 - 3, n0 - 5, 10, n0 - 2], [3, 5, 20, 2], [1, 1, 7, 1])
    qpos = np.array([900, 17, 3], np.int32)
    s.h.decode_step(0, w.dec_request, w.dec_stream, qd, out, lists=lists, flags=B.DECODE_ROPE_Q, position=qpos)
    q64 = oracle.rope(oracle.widen_pool(w.dtype, q), qpos, THETA)
    ref, _ = oracle.attention_q64(op.g, op.k, op.v, w.dec_request, *lists, q64, w.scale)
    check_close(_out64(w, out), ref, w.dtype, "lists over deferred rotated rows")
    _check_rope_pool(w, s, op, n0)
    s.close()
    # (c)
    w = W.config3(steps=2, prefix=200, n_streams=3)
    pos = w.event_positions()
    s = _session(w, rope_theta=THETA)
    op = OraclePool(w)
    s.append_events(w.n_prefill, flags=B.APPEND_ROPE, positions=pos)
    s.append_events(w.n_events(0), chunk=w.n, flags=B.APPEND_ROPE | B.APPEND_DEFER, positions=pos)
    s.append_events(w.n_events(1), chunk=w.n, flags=B.APPEND_ROPE | B.APPEND_DEFER, positions=pos)  # flushes the first
    op.append_events(w.n_events(1), positions=pos, theta=THETA)
    _check_rope_step(w, s, op, 1, pos)
    _check_rope_pool(w, s, op, w.n_events(1))
    s.close()


# ------------------------------------------------------------------------- synchronisation
@pytest.mark.parametrize("seed", range(3))
def test_maintained_lists_through_syncs_equal_reachability_and_dense_mask_attention(seed):
    """Forks, nested forks, synchronisations (pasta_attn_sync) and reuse of stream ids: at a few
    moments of the history every live stream decodes in maintained mode; its gather map must be
    exactly the set reachable from its newest token in Figure 2b's graph, and its output the
    brute-force attention over the whole pool with that set as mask.  No KV row is moved."""
    events = W.random_fork_sync_history(700 + seed, n_slots=420, max_ids=6, p_fork=0.08, p_sync=0.15)
    n = len(events)
    ev_s = np.array([e["stream"] for e in events], np.int32)
    ev_p = np.array([e["parent"] for e in events], np.int32)
    ev_n = np.array([1 if e["new"] else 0 for e in events], np.uint8)
    joins = {t: e["join"] for t, e in enumerate(events) if e["join"]}
    assert len(joins) >= 2
    w = W.Workload(name="syncs", dtype="bf16", Hq=8, Hkv=2, D=128, scale=1.0, seed=950 + seed, max_requests=1,
                   pool_tokens=512, max_streams=6, k_std=128 ** -0.5)
    w.ev_request = np.zeros(n, np.int32)
    w.ev_stream, w.ev_parent, w.n_prefill = ev_s, np.where(ev_n == 1, ev_p, -1).astype(np.int32), n
    s = _session(w, max_ranges=4096)
    op = OraclePool(w).append_events(n)
    from paper_2502_11517_amd.harness import to_device
    checks = sorted(set([min(joins) + 1, max(joins) + 1, n // 2, n]))
    done = 0
    for stop in checks:
        for t in range(done, stop):       # replay the history: a sync call before a sync token's row
            if events[t]["join"]:
                s.h.sync(0, int(ev_s[t]), events[t]["join"], retire=True)
            s.append_events(t + 1, chunk=1)
        done = stop
        live = sorted({int(x) for x in ev_s[:stop]} - {j for t, js in joins.items() if t < stop for j in js
                                                       if not any(ev_s[u] == j and ev_n[u] for u in range(t, stop))})
        rid = np.zeros(len(live), np.int32)
        rng = np.random.default_rng([seed, stop])
        q = W.f32_to_bf16_bits(rng.standard_normal((len(live), w.Hq, w.D)).astype(np.float32))
        qd = to_device(q, w.dtype, s.device)
        out = torch.empty_like(qd)
        goffs = np.zeros(len(live) + 1, np.int64)
        s.h.decode_step(0, rid, live, qd, out, flags=B.DECODE_PLAN_ONLY, dbg_gather_offsets=goffs)
        grows = torch.full((int(goffs[-1]),), -1, dtype=torch.int32, device=s.device)
        s.h.decode_step(0, rid, live, qd, out, dbg_gather_offsets=goffs, dbg_gather_rows=grows)
        got = _out64(w, out)
        grows = grows.cpu().numpy()
        for i, sid in enumerate(live):
            last = int(np.nonzero(ev_s[:stop] == sid)[0][-1])
            mask = oracle.visible_events(ev_s[:stop], ev_p[:stop], ev_n[:stop], {k: v for k, v in joins.items() if k < stop}, last)
            assert np.array_equal(grows[goffs[i]:goffs[i + 1]], np.nonzero(mask)[0]), f"stop {stop} stream {sid}"
            ref, _ = oracle.attention_dense(op.g, op.k, op.v, 0, mask, q[i], w.scale)
            check_close(got[i], ref, w.dtype, f"stop {stop} stream {sid}")
    s.close()


# ------------------------------------------------------------------------- trace replay
@pytest.mark.parametrize("rope", [False, True])
def test_trace_replay_matches_the_oracles_interpreter_and_dense_mask_attention(rope):
    """A whole synthetic response through pasta_attn_replay on two layer pools: every token's slot,
    stream, position id and pass equal the oracle interpreter's; every token's attention output
    equals brute-force attention over the final pool masked to what Figure 2b's graph lets that
    token reach; the pool holds exactly the fed rows (rotated by the estimated ids with rope)."""
    from oracle import pasta_interp as I
    from paper_2502_11517_amd.harness import to_device
    ops = W.synthetic_trace(7, n_promises=5, text_mean=5, block_median=14, sync_every=2, tail_text=6)
    n_prompt, L = 150, 2
    w = W.Workload(name="replay", dtype="bf16", Hq=8, Hkv=2, D=128, scale=128 ** -0.5, seed=31, max_requests=1,
                   pool_tokens=1024, max_streams=6)
    w.ev_request = np.zeros(n_prompt, np.int32)
    w.ev_stream = np.zeros(n_prompt, np.int32)
    w.ev_parent = np.full(n_prompt, -1, np.int32)
    w.n_prefill = n_prompt
    s = _session(w, n_layers=L, max_ranges=8192, rope_theta=THETA if rope else 0.0)
    toks, passes = I.interpret(ops, n_prompt, n_prompt, 6)
    n = len(toks)
    rng = np.random.default_rng(99)
    enc = W.f32_to_bf16_bits
    kp_rows = enc(rng.standard_normal((L, n_prompt, w.Hkv, w.D)).astype(np.float32))
    vp_rows = enc(rng.standard_normal((L, n_prompt, w.Hkv, w.D)).astype(np.float32))
    k_rows = enc(rng.standard_normal((L, n, w.Hkv, w.D)).astype(np.float32))
    v_rows = enc(rng.standard_normal((L, n, w.Hkv, w.D)).astype(np.float32))
    q_rows = enc(rng.standard_normal((L, n, w.Hq, w.D)).astype(np.float32))
    ppos = np.arange(n_prompt, dtype=np.int32)
    for l in range(L):  # the prompt, as stream 0
        s.h.append_kv(l, w.ev_request, w.ev_stream, to_device(kp_rows[l], w.dtype, s.device), to_device(vp_rows[l], w.dtype, s.device),
                      position=ppos, flags=B.APPEND_ROPE if rope else 0)
    plan = s.h.replay(0, ops, n_prompt, n, flags=B.REPLAY_PLAN_ONLY)  # leaves the handle as it is
    kd, vd, qd = (to_device(x, w.dtype, s.device) for x in (k_rows, v_rows, q_rows))
    out = torch.empty_like(qd)
    r = s.h.replay(0, ops, n_prompt, n, kd, vd, qd, out, flags=B.REPLAY_ROPE if rope else 0)
    got = _out64(w, out)
    for key in ("slot", "stream", "pos", "pass_"):
        assert r[key].tolist() == [t[key] for t in toks] == plan[key].tolist(), key
    assert r["stats"][1] == passes
    ev_s = [0] * n_prompt + [t["stream"] for t in toks]
    ev_p = [-1] * n_prompt + [t["parent"] for t in toks]
    ev_n = [1] + [0] * (n_prompt - 1) + [1 if t["new"] else 0 for t in toks]
    joins = {t["slot"]: t["join"] for t in toks if t["join"]}
    pos_all = np.concatenate([ppos, np.array([t["pos"] for t in toks], np.int32)])
    g = oracle.Geom(w.dtype, w.Hq, w.Hkv, w.D, pool_tokens=w.pool_tokens)
    for l in range(L):
        ka = np.concatenate([kp_rows[l], k_rows[l]])
        if rope:
            ka = oracle.round_pool(w.dtype, oracle.rope(oracle.widen_pool(w.dtype, ka), pos_all, THETA))
        okp, ovp, tail = g.new_pool(), g.new_pool(), np.zeros(1, np.int64)
        assert oracle.append(g, okp, ovp, np.zeros(n_prompt + n, np.int32), ka, np.concatenate([vp_rows[l], v_rows[l]]), tail)[0] == 0
        for i in range(0, n, 3 if l else 1):  # every token on layer 0, every third on layer 1
            mask = oracle.visible_events(ev_s, ev_p, ev_n, joins, toks[i]["slot"])
            if rope:
                q64 = oracle.rope(oracle.widen_pool(w.dtype, q_rows[l, i:i + 1]), [toks[i]["pos"]], THETA)[0]
                rows = np.nonzero(mask)[0]
                ref, _ = oracle.attention_q64(g, okp, ovp, [0], [0], [0, len(rows)], rows, np.ones(len(rows), np.int32),
                                              np.ones(len(rows), np.int32), q64[None], w.scale)
                ref = ref[0]
            else:
                ref, _ = oracle.attention_dense(g, okp, ovp, 0, mask, q_rows[l, i], w.scale)
            check_close(got[l, i], ref, w.dtype, f"layer {l} token {i}")
        kb, vb = s.pool_bits(l)
        m = (n_prompt + n) * w.Hkv * w.D
        assert np.array_equal(vb[:m], ovp[:m])
        if rope:
            d = np.abs(oracle.widen_pool(w.dtype, kb[:m]) - oracle.widen_pool(w.dtype, okp[:m]))
            assert d.max() <= 2.0 ** -7 * np.abs(oracle.widen_pool(w.dtype, okp[:m])).max() and (d != 0).mean() < 0.01
        else:
            assert np.array_equal(kb[:m], okp[:m])
    s.close()


# ------------------------------------------------------------------------- comparison modes, multi-token steps
@pytest.mark.parametrize("cfg", ["config2", "config4", "nested"])
def test_no_share_and_dense_mask_modes_give_the_same_results(cfg):
    """PASTA_DECODE_NO_SHARE (every stream reads its whole visible set itself) and
    PASTA_DECODE_DENSE_MASK (every stream walks all slots of its request under a 0/1 mask, the
    formulation the paper's own implementation uses) are other ways to the same numbers."""
    if cfg == "nested":
        ev_s, ev_p = W.random_fork_history(41, n_slots=600, max_streams=7, p_fork=0.02, p_retire=0.0)
        n_streams = int(ev_s.max()) + 1
        w = W.Workload(name="nested", dtype="bf16", Hq=16, Hkv=4, D=128, scale=1.0, seed=43, max_requests=1,
                       pool_tokens=640, max_streams=n_streams, k_std=128 ** -0.5)
        w.ev_request = np.zeros(len(ev_s), np.int32)
        w.ev_stream, w.ev_parent, w.n_prefill = ev_s, ev_p, len(ev_s)
        w.dec_request = np.zeros(n_streams, np.int32)
        w.dec_stream = np.arange(n_streams, dtype=np.int32)
        explicit = False
    else:
        w = getattr(W, cfg)() if cfg == "config2" else W.config4(n_requests=5, seed=12, pmin=100, pmax=700)
        explicit = True
    s = _session(w)
    op = OraclePool(w).append_events(w.n_prefill)
    s.append_events(w.n_prefill)
    base, _, _ = s.decode(0, explicit=explicit)
    base = _out64(w, base)
    if explicit:
        ref, _ = op.attention(0)
        check_close(base, ref, w.dtype, "lists")
    for flag, name in ((B.DECODE_NO_SHARE, "no share"), (B.DECODE_DENSE_MASK, "dense mask")):
        out, lse, _ = s.decode(0, explicit=explicit, flags=flag)
        got = _out64(w, out)
        assert np.all(np.isfinite(got))
        check_close(got, base, w.dtype, name + " vs lists")      # two roundings apart at most
        if explicit:
            check_close(got, ref, w.dtype, name + " vs oracle")
    s.close()


def test_dense_mask_mode_handles_blocks_and_items_in_which_a_stream_sees_nothing():
    """A fork that starts right after a long stretch it cannot see: whole blocks, and whole work
    items, of its dense walk are masked out (running max still -inf when they end)."""
    w = W.single_request("gap", "bf16", 8, 2, 128, 1.0, 9, 40, [700, 3], "round_robin", k_std=128 ** -0.5)
    # make stream 2's own rows come last, after ~700 rows of stream 1 that it must not see
    s = _session(w)
    op = OraclePool(w).append_events(w.n_prefill)
    s.append_events(w.n_prefill)
    ref, _ = op.attention(0)
    for flag in (0, B.DECODE_DENSE_MASK, B.DECODE_NO_SHARE):
        out, _, _ = s.decode(0, flags=flag)
        check_close(_out64(w, out), ref, w.dtype, f"flag {flag}")
    s.close()


def test_several_query_tokens_of_one_stream_in_one_step():
    """causal_skip: a stream feeds a chunk of k rows and gets k outputs in one step, query j seeing
    the chunk up to its own row; together with one-token streams of the same request."""
    from paper_2502_11517_amd.harness import to_device
    w = W.single_request("chunk", "bf16", 16, 4, 128, 1.0, 13, 300, [50, 20], "round_robin", k_std=128 ** -0.5)
    n0 = w.n_prefill
    s = _session(w, max_streams=8)  # a step holds at most max_requests * max_streams query tokens
    op = OraclePool(w).append_events(n0)
    s.append_events(n0)
    # stream 1 appends a chunk of 5 more rows (K/V rows: reuse the generator's rows [0, 5))
    k5, v5 = w.kv_rows(0, 5)
    s.h.append_kv(0, [0] * 5, [1] * 5, to_device(k5, w.dtype, s.device), to_device(v5, w.dtype, s.device))
    tail = np.zeros(1, np.int64); tail[0] = n0
    assert oracle.append(op.g, op.k, op.v, [0] * 5, k5, v5, op.tail)[0] == 0
    pl, offs, st, ct, sd = w.lists(0)
    i1 = int(np.nonzero(w.dec_stream == 1)[0][0])
    i2 = int(np.nonzero(w.dec_stream == 2)[0][0])
    rng = np.random.default_rng(3)
    q = W.f32_to_bf16_bits(rng.standard_normal((6, w.Hq, w.D)).astype(np.float32))
    qd = to_device(q, w.dtype, s.device)
    out = torch.empty_like(qd)
    s.h.decode_step(0, [0] * 6, [1, 1, 1, 1, 1, 2], qd, out, causal_skip=[4, 3, 2, 1, 0, 0])
    got = _out64(w, out)
    base1 = (int(pl[i1]), st[offs[i1]:offs[i1 + 1]].tolist(), ct[offs[i1]:offs[i1 + 1]].tolist(), sd[offs[i1]:offs[i1 + 1]].tolist())
    for j in range(5):  # query j of the chunk: the old list plus the chunk's rows n0 .. n0 + j
        lists = ([base1[0]], [0, len(base1[1]) + 1], base1[1] + [n0], base1[2] + [j + 1], base1[3] + [1])
        ref, _ = oracle.attention(op.g, op.k, op.v, [0], *lists, q[j:j + 1], w.scale)
        check_close(got[j], ref[0], w.dtype, f"chunk token {j}")
    lists2 = ([int(pl[i2])], [0, offs[i2 + 1] - offs[i2]], st[offs[i2]:offs[i2 + 1]], ct[offs[i2]:offs[i2 + 1]], sd[offs[i2]:offs[i2 + 1]])
    ref, _ = oracle.attention(op.g, op.k, op.v, [0], *lists2, q[5:6], w.scale)
    check_close(got[5], ref[0], w.dtype, "the other stream")
    s.close()
