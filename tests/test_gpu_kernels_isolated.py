"""The kernels one by one (GPU): the partial (m, l, acc) rows that the attention launch leaves
for chosen chunks and items against the oracle's partial over the same physical rows, and the
merge kernel alone on synthetic partials against the oracle's merge."""
from __future__ import annotations

import math

import numpy as np
import pytest
import torch

import oracle
from paper_2502_11517_amd import binding as B
from paper_2502_11517_amd import workloads as W
from util import OraclePool, to_f64

pytestmark = pytest.mark.gpu
LOG2E = math.log2(math.e)


def _session(w, **kw):
    from paper_2502_11517_amd.harness import Session
    return Session(w, **kw)


def _plan(s, w):
    plan = np.zeros(8, np.int64)
    s.h.decode_step(0, w.dec_request, w.dec_stream, None, None, flags=B.DECODE_PLAN_ONLY | B.DECODE_ROW_GROUPS, dbg_plan=plan)
    return plan


def _partials(s, w, rows, flags=0, ml=None, acc=None):
    """Runs one step with the partial rows in the test's own buffers; returns (ml, acc, out)."""
    from paper_2502_11517_amd.harness import to_device
    qd = to_device(w.q(0), w.dtype, s.device)
    out = torch.zeros_like(qd)
    lse = torch.zeros(w.n, w.Hq, dtype=torch.float32, device=s.device)
    if ml is None:
        ml = torch.full((rows, 2), float("nan"), dtype=torch.float32, device=s.device)
        acc = torch.full((rows, w.D), float("nan"), dtype=torch.float32, device=s.device)
    s.h.decode_step(0, w.dec_request, w.dec_stream, qd, out, out_lse=lse, flags=flags, dbg_partials=(ml, acc))
    torch.cuda.synchronize()
    return ml, acc, out, lse


@pytest.mark.parametrize("flags,wide", [(0, False), (B.DECODE_NO_MFMA, False), (0, True)])
def test_partials_of_the_attention_launch_against_the_oracle(flags, wide):
    """One request, 3 streams, a prefix of several split chunks, round-robin private rows: every
    shared-prefix partial of sampled (chunk, kv head, row) and every private partial row against
    oracle.partial over the same physical rows.  Also with the vector-ALU kernel (NO_MFMA), whose
    items are all private, and with 5 streams x 8 heads per kv head = 40 stacked rows (the work-groups
    that serve four 32-row groups each: one full group and one of 8 rows)."""
    flags |= B.DECODE_FOUR_GROUPS if wide else 0
    if wide:
        w = W.single_request("isow", "bf16", 16, 2, 128, 1.0, 92, 1500, [300, 77, 140, 20, 260], "round_robin", k_std=128 ** -0.5)
    else:
        w = W.single_request("iso", "bf16", 8, 2, 128, 1.0, 91, 1500, [300, 77, 140], "round_robin", k_std=128 ** -0.5)
    s = _session(w)
    op = OraclePool(w).append_events(w.n_prefill)
    s.append_events(w.n_prefill)
    plan = np.zeros(8, np.int64)
    s.h.decode_step(0, w.dec_request, w.dec_stream, None, None, flags=flags | B.DECODE_PLAN_ONLY, dbg_plan=plan)
    rows, chunk, pc, priv0, n_items = int(plan[3]), int(plan[4]), int(plan[5]), int(plan[7]), int(plan[2])
    ml, acc, out, _ = _partials(s, w, rows, flags=flags | B.DECODE_PARTIALS_ONLY)
    assert float(out.float().abs().max()) == 0.0, "PARTIALS_ONLY must not write the output"
    ml, acc = ml.cpu().numpy().astype(np.float64), acc.cpu().numpy().astype(np.float64)
    G, Hkv, n = w.Hq // w.Hkv, w.Hkv, w.n
    pl, offs, st, ct, sd = w.lists(0)
    q = w.q(0)
    maps = [oracle.gather_map(op.g, 0, int(pl[i]), st[offs[i]:offs[i + 1]], ct[offs[i]:offs[i + 1]], sd[offs[i]:offs[i + 1]])
            for i in range(n)]

    def check(row, phys, i, h, what):
        m, l, a = oracle.partial(op.g, op.k, op.v, phys, q[i, h], h // G, w.scale)
        assert abs(ml[row, 0] - m * LOG2E) <= 2e-3 * max(1.0, abs(m * LOG2E)), f"{what}: m {ml[row, 0]} vs {m * LOG2E}"
        assert abs(ml[row, 1] - l) <= 4e-3 * l, f"{what}: l {ml[row, 1]} vs {l}"
        assert np.linalg.norm(acc[row] - a) <= 6e-3 * np.linalg.norm(a), f"{what}: acc"

    if pc:  # shared-prefix parts: chunk c of [0, pc), all streams stacked
        assert not (flags & B.DECODE_NO_MFMA) and pc == int(pl.min())
        n_chunks, R = -(-pc // chunk), n * G
        assert n_chunks >= 3
        for c in sorted({0, 1, n_chunks - 1}):
            phys = maps[0][c * chunk:min(pc, (c + 1) * chunk)]  # the prefix head of any stream's map
            for g in range(Hkv):
                for i in range(n):
                    for gi in (0, G - 1):
                        check((g * n_chunks + c) * R + i * G + gi, phys, i, g * G + gi, f"prefix chunk {c} head {g} stream {i}")
    # private parts: consecutive pieces of each stream's list beyond the common prefix
    piece = 256 if wide else 128
    j = 0
    for i in range(n):
        rest = maps[i][pc:]
        for t0 in range(0, len(rest), piece):
            for g in range(Hkv):
                for gi in range(G):
                    check(priv0 + (j * Hkv + g) * G + gi, rest[t0:t0 + piece], i, g * G + gi, f"item {j} head {g}")
            j += 1
    assert j == n_items
    s.close()


def _merge_case(n_streams, Hq, Hkv, prefix, lengths, seed, poison):
    """MERGE_ONLY over synthetic partials: returns nothing, asserts against oracle.merge."""
    w = W.single_request("miso", "bf16", Hq, Hkv, 128, 1.0, seed, prefix, lengths, "round_robin", k_std=128 ** -0.5)
    s = _session(w)
    s.append_events(w.n_prefill)
    plan = _plan(s, w)
    rows, chunk, pc, priv0, n_items = int(plan[3]), int(plan[4]), int(plan[5]), int(plan[7]), int(plan[2])
    G, n, D = Hq // Hkv, w.n, w.D
    n_chunks, R = (-(-pc // chunk) if pc else 0), n * G
    rng = np.random.default_rng(seed)
    m = rng.normal(0.0, 3.0, size=rows)                      # log2 units
    l = rng.uniform(0.5, 40.0, size=rows)
    acc = rng.normal(size=(rows, D)) * l[:, None]
    kind = rng.integers(0, 10, size=rows)
    if poison:
        dead = kind == 0                                      # parts in which the row saw nothing
        m[dead], l[dead] = -np.inf, 0.0
        acc[dead] = rng.normal(size=(int(dead.sum()), D)) * 1e30   # must not leak into the result
        far = kind == 1
        m[far] -= 200.0                                       # weights that underflow to nothing
    # parts of each output row, in the documented layout
    pl, offs, st, ct, sd = w.lists(0)
    # (a plan sent whole cuts a stream's list beyond the common prefix into 128-token pieces; a step that reads the
    # device-resident lists cuts the visible head beyond the common prefix and the range list separately)
    piece = 128  # (the plan above asked for the row-group form)
    whole = [-(-(int(pl[i]) - pc + int(ct[offs[i]:offs[i + 1]].sum())) // piece) for i in range(n)]
    split = [-(-(int(pl[i]) - pc) // piece) + -(-int(ct[offs[i]:offs[i + 1]].sum()) // piece) for i in range(n)]
    counts = whole if sum(whole) == n_items else split
    items_of, j = [], 0
    for cnt in counts:
        items_of.append(list(range(j, j + cnt)))
        j += cnt
    assert j == n_items and priv0 + n_items * Hq == rows
    if poison:  # one row whose every part but one is dead, one stream-head with a single live part
        for c in range(1, n_chunks):
            r0 = (0 * n_chunks + c) * R + 0
            m[r0], l[r0] = -np.inf, 0.0
    ml32 = np.stack([m, l], axis=1).astype(np.float32)
    acc32 = acc.astype(np.float32)
    mld = torch.from_numpy(ml32).to(s.device)
    accd = torch.from_numpy(acc32).to(s.device)
    _, _, out, lse = _partials(s, w, rows, flags=B.DECODE_MERGE_ONLY | B.DECODE_ROW_GROUPS, ml=mld, acc=accd)
    from paper_2502_11517_amd.harness import to_host_bits
    got = to_f64(w, to_host_bits(out, w.dtype))
    lse = lse.cpu().numpy().astype(np.float64)
    ml64, acc64 = ml32.astype(np.float64), acc32.astype(np.float64)
    worst = 0.0
    for i in range(n):
        for h in range(Hq):
            g, gi = divmod(h, G)
            part_rows = [(g * n_chunks + c) * R + i * G + gi for c in range(n_chunks)]
            part_rows += [priv0 + (jj * Hkv + g) * G + gi for jj in items_of[i]]
            pr = [r for r in part_rows if ml64[r, 1] > 0]
            ref, ref_lse = oracle.merge(ml64[pr, 0] / LOG2E, ml64[pr, 1], acc64[pr])
            err = np.linalg.norm(got[i, h] - ref) / np.linalg.norm(ref)
            worst = max(worst, err)
            assert err <= 5e-3, f"stream {i} head {h}: {err}"      # bf16 output rounding
            assert abs(lse[i, h] - ref_lse) <= 1e-3 * max(1.0, abs(ref_lse))
    s.close()
    return worst, rows, n_chunks, n_items


def test_merge_alone_few_rows_wide_form():
    """< 512 output rows: the 1024-thread form; parts include dead ones (l = 0, m = -inf, garbage in
    acc), far-off maxima, a row with one live part."""
    res = _merge_case(3, 8, 2, 3000, [300, 10, 129], 5, poison=True)
    print("merge, wide form:", res)


def test_merge_alone_one_part_per_row():
    """Two interleaved streams with one private item each and no shared prefix to split: one part per
    output row."""
    res = _merge_case(2, 4, 4, 1, [90, 5], 6, poison=False)
    assert res[2] == 0 and res[3] == 2


def test_merge_alone_many_rows_narrow_forms():
    """>= 512 output rows: 40 streams x 16 heads; few parts per row (one group of D threads) and many
    (the 256-thread form)."""
    a = _merge_case(40, 16, 4, 256, [20] * 40, 7, poison=True)      # <= 8 parts per row on average
    b = _merge_case(40, 16, 4, 6000, [300] * 40, 8, poison=True)    # many parts per row
    print("merge, narrow forms:", a, b)


def test_merge_alone_about_a_thousand_parts():
    """A long prefix in several hundred split chunks and a stream with several hundred private items
    (beside a short one): about a thousand parts on each of the long stream's output rows."""
    res = _merge_case(2, 4, 1, 30000, [60000, 10], 9, poison=True)
    assert res[2] >= 400 and res[3] >= 400, res
