#!/usr/bin/env python3
"""bench.py -- multi-stream decode-attention throughput on one MI355X.

Workload: the 8-stream, 8k-prefix configuration (bf16, 32 query / 8 KV heads, D=128, prefix
8192, 8 streams of 64..512 tokens in right-aligned round-robin interleave).  One "step" is
one pass of the whole hot path on ONE layer's pool: KV-append of 8 rows (one per stream),
then the decode step (shared-prefix kernel + private-segment kernel + merge) for the 8 query
tokens.  Steps cycle through `--layers` distinct pools (default 32, Llama-8B's depth; about
1.4 GB, so every step reads a pool that is cold in the 256 MB last-level cache), and every
`layers` steps the 8 streams advance by one token -- 64 tokens x 32 layers = 2048 steps is the
configuration's full 64-step loop.

Prints ONE JSON line.  `value` = stream-tokens/s = 8 * steps / elapsed, with all inputs
resident in HBM before the timed region.  `roofline` is for the dominant kernel(s) (the
attention-partials launches), timed with HIP events on the library's stream.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published peak
MIN_SAMPLES = 8         # attention launches timed by event pairs, at least
SPINUP_S = 0.25         # seconds of untimed decode steps ahead of the warm-up (clock ramp of an idle GPU)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2048)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--layout", choices=["token", "head"], default="head")
    ap.add_argument("--event-every", type=int, default=33,
                    help="time the attention kernel of every n-th step with a HIP event pair attached to its dispatch "
                         "(a timed dispatch costs its step about 5 us: at every 8th step the run reads 0.6 us per step "
                         "slower than without events; 33 is co-prime with the 32 pools, so the samples cover all of them); "
                         "short runs sample more often, so that there are always at least 8 samples")
    ap.add_argument("--probe-launches", type=int, default=64,
                    help="after the timed region: this many launches of the read-only form of the attention launch "
                         "(same grid, same requests, no arithmetic), cycling the pools, each timed by its dispatch's events")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-mfma", action="store_true", help="route the prefix through the private-segment kernel")
    ap.add_argument("--eager-append", action="store_true",
                    help="run the KV-append as a launch of its own instead of letting it ride with the decode launch")
    ap.add_argument("--streams", type=int, default=8, help="config 3 with another number of decoding streams (side measurement)")
    ap.add_argument("--prefix", type=int, default=8192, help="config 3 with another shared-prefix length (side measurement)")
    ap.add_argument("--no-share", action="store_true",
                    help="comparison: no shared-prefix items, every stream reads its whole visible set itself")
    ap.add_argument("--row-groups", action="store_true",
                    help="comparison: requests with more than 32 stacked query rows are served one 32-row group per "
                         "work-group (PASTA_DECODE_ROW_GROUPS) instead of four groups per work-group")
    ap.add_argument("--dense-mask", action="store_true",
                    help="comparison: every stream walks the whole pool under a 0/1 mask (the paper's own formulation)")
    ap.add_argument("--rope", action="store_true",
                    help="rotary embedding by position ids inside the path: K rotated by the append (a launch of its "
                         "own, not deferred), Q rotated in the attention kernel")
    ap.add_argument("--workload", choices=["config3", "config2", "config4", "config5", "replay"], default="config3",
                    help="config3 (default) is the headline line; the others time decode steps only (their "
                         "state is a single step's) and exist to show how the kernels behave on the other shapes")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run a plain 1 GiB device copy (3x) before the loop: the known-size kernel that "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU; --gpus must be 1 "
              "(the path would shard by kv head, by request or by sequence; none of that is built)", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2502_11517_amd import binding as B
    from paper_2502_11517_amd import workloads as W
    from paper_2502_11517_amd.harness import Session, to_device, to_host_bits

    if not os.path.exists(B.library_path()):
        raise SystemExit("libpasta_attn.so is not built: run `python __graft_entry__.py` first")
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = torch.device("cuda:0")
    if args.workload == "replay":
        return replay_bench(args, dev)
    if args.workload != "config3":
        return decode_only(args, getattr(W, args.workload)(), dev)
    L = args.layers
    every = max(1, args.event_every)
    # steps beyond the timed region (same loop, untimed): as many as it takes to have MIN_SAMPLES timed launches
    n_tail = max(0, (MIN_SAMPLES + 1) * every - args.steps)
    n_all = args.steps + n_tail
    tokens = -(-n_all // L)  # token steps needed
    w = W.config3(steps=max(tokens, 2), prefix=args.prefix, n_streams=args.streams)
    layout = B.HEAD_MAJOR if args.layout == "head" else B.TOKEN_MAJOR
    theta = 10000.0
    s = Session(w, kv_layout=layout, n_layers=L, rope_theta=theta if args.rope else 0.0)
    hip = C.CDLL("libamdhip64.so.7")  # already loaded by torch: same runtime
    ev_pos = w.event_positions() if args.rope else None

    # ---- prefill every layer (layer l holds the generator's rows rolled by l along D)
    n0 = w.n_prefill
    k0, v0 = w.kv_rows(0, n0)
    kd, vd = to_device(k0, w.dtype, dev), to_device(v0, w.dtype, dev)
    for l in range(L):
        s.h.append_kv(l, w.ev_request[:n0], w.ev_stream[:n0], torch.roll(kd, l, dims=2).contiguous(),
                      torch.roll(vd, l, dims=2).contiguous(), parent_stream=w.ev_parent[:n0],
                      position=ev_pos[:n0] if args.rope else None, flags=B.APPEND_ROPE if args.rope else 0)
    torch.cuda.synchronize()

    # ---- inputs of the timed loop, all resident on the device
    ks, vs = w.kv_rows(n0, n0 + tokens * w.n)
    ks = to_device(ks, w.dtype, dev).view(tokens, w.n, w.Hkv, w.D)
    vs = to_device(vs, w.dtype, dev).view(tokens, w.n, w.Hkv, w.D)
    k_steps = [[torch.roll(ks[t], l, dims=2).contiguous() for l in range(L)] for t in range(tokens)]
    v_steps = [[torch.roll(vs[t], l, dims=2).contiguous() for l in range(L)] for t in range(tokens)]
    q_steps = [to_device(w.q(t), w.dtype, dev) for t in range(tokens)]
    out = torch.empty(L, w.n, w.Hq, w.D, dtype=torch.bfloat16, device=dev)
    flags = (B.DECODE_NO_MFMA if args.no_mfma else 0) | (B.DECODE_ROPE_Q if args.rope else 0)
    flags |= (B.DECODE_NO_SHARE if args.no_share else 0) | (B.DECODE_DENSE_MASK if args.dense_mask else 0)
    flags |= B.DECODE_ROW_GROUPS if args.row_groups else 0
    q_pos = [w.q_positions(t) if args.rope else None for t in range(tokens)]

    # HIP events around the attention-partials kernels of sampled steps (never step 0)
    n_ev = n_all // every + 1
    evs = []
    for _ in range(2 * n_ev):
        e = C.c_void_p()
        assert hip.hipEventCreate(C.byref(e)) == 0
        evs.append(e)

    ev_step = w.ev_stream[n0:n0 + w.n]
    req_step = w.ev_request[n0:n0 + w.n]
    calls = []
    for i in range(n_all):
        t, l = divmod(i, L)
        pe = (evs[2 * (i // every)], evs[2 * (i // every) + 1]) if sampled(i, every) else None
        app_flags = (0 if args.eager_append else B.APPEND_DEFER) | (B.APPEND_ROPE if args.rope else 0)
        calls.append((s.h.prepare_append(l, req_step, ev_step, k_steps[t][l], v_steps[t][l], flags=app_flags,
                                         position=ev_pos[n0 + t * w.n:n0 + (t + 1) * w.n] if args.rope else None),
                      s.h.prepare_decode(l, w.dec_request, w.dec_stream, q_steps[t], out[l], flags=flags,
                                         prof_events=pe, position=q_pos[t])))

    if args.calibrate:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- warm-up: decode only (no state change).  Every pool is touched once whatever --warmup says (first
    # touches of a pool cost page-table walks that are no part of a steady-state step), then `warmup` more steps.
    warm = [s.h.prepare_decode(l, w.dec_request, w.dec_stream, q_steps[0], out[l], flags=flags, position=q_pos[0])
            for l in range(L)]
    # Then the device is kept busy for SPINUP_S with the same decode steps: an idle GPU starts a run at low
    # clocks and takes milliseconds to ramp, far longer than a short timed region lasts.
    t_spin = time.perf_counter()
    n_spin = 0
    while n_spin < L or time.perf_counter() - t_spin < SPINUP_S:
        for i in range(64):
            assert warm[(n_spin + i) % L]() == 0
        n_spin += 64
        torch.cuda.synchronize()
    for i in range(args.warmup):
        assert warm[i % L]() == 0
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` append+decode passes
    t0 = time.perf_counter()
    for app, dec in calls[:args.steps]:
        ra = app()
        rd = dec()
        if ra or rd:
            raise SystemExit(f"library error in timed loop: append {ra} decode {rd}")
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    # ---- the same loop goes on, untimed, until enough launches have been timed by their events
    for app, dec in calls[args.steps:]:
        if app() or dec():
            raise SystemExit("library error after the timed loop")
    torch.cuda.synchronize()

    # ---- kernel time from the events
    ms = C.c_float()
    durs, n_in_region = [], 0
    for j in range(n_all):
        if sampled(j, every):
            a, b = evs[2 * (j // every)], evs[2 * (j // every) + 1]
            assert hip.hipEventElapsedTime(C.byref(ms), a, b) == 0
            durs.append(ms.value * 1e-3)
            n_in_region += j < args.steps
    kern_s = float(np.mean(durs))

    # ---- what a plain read of the same bytes costs at this launch's shape: the read-only form of the
    # attention launch (same grid, same requests by the same waves, no arithmetic), on the final state
    probe_s = None
    if args.probe_launches > 0 and not (args.no_mfma or args.dense_mask):
        pflags = (flags | B.DECODE_READ_PROBE) & ~B.DECODE_ROPE_Q
        scratch_out = torch.empty(w.n, w.Hq, w.D, dtype=torch.bfloat16, device=dev)
        pev = []
        for _ in range(2 * args.probe_launches):
            e = C.c_void_p()
            assert hip.hipEventCreate(C.byref(e)) == 0
            pev.append(e)
        pcalls = [s.h.prepare_decode(i % L, w.dec_request, w.dec_stream, q_steps[-1], scratch_out, flags=pflags,
                                     prof_events=(pev[2 * i], pev[2 * i + 1])) for i in range(args.probe_launches)]
        for c_ in pcalls:
            assert c_() == 0
        torch.cuda.synchronize()
        pd = []
        for i in range(args.probe_launches):
            assert hip.hipEventElapsedTime(C.byref(ms), pev[2 * i], pev[2 * i + 1]) == 0
            pd.append(ms.value * 1e-3)
        probe_s = float(np.median(pd[len(pd) // 4:]))  # the first quarter warms the variant's code

    # algorithmic bytes of the attention-partials kernels per launch: every visible K and V row
    # once (prefix rows once for all streams) + Q read; averaged over the timed steps
    row_bytes = 2 * w.Hkv * w.D * 2
    alg = []
    for t in range(tokens):
        pl, offs, st, ct, sd = w.lists(t)
        pc = int(pl.min())
        priv = int(sum(int(pl[i]) - pc + int(ct[offs[i]:offs[i + 1]].sum()) for i in range(w.n)))
        alg.append((pc + priv) * row_bytes + w.n * w.Hq * w.D * 2)
    alg_bytes = float(np.mean([alg[j // L] for j in range(n_all) if sampled(j, every)]))  # of the timed launches
    alg_step = float(np.mean([alg[i // L] for i in range(args.steps)]))                   # of the timed region's steps
    achieved = alg_bytes / kern_s / 1e9

    # ---- CPU baseline: the fp64 oracle as it stands, on the host cores, for a bounded sample
    # of the same workload (decode steps of the final state on layer 0), plus a parity spot check
    result_extra = {}
    cpu = None
    if not args.no_cpu_baseline:
        import oracle

        last = tokens - 1
        ne = w.n_events(last)
        g = oracle.Geom(w.dtype, w.Hq, w.Hkv, w.D, head_major=(layout == B.HEAD_MAJOR), pool_tokens=w.pool_tokens)
        kp, vp, tail = g.new_pool(), g.new_pool(), np.zeros(1, np.int64)
        ka, va = w.kv_rows(0, ne)
        if args.rope:  # the oracle's pool holds keys rotated in fp64 and rounded once
            ka = oracle.round_pool(w.dtype, oracle.rope(oracle.widen_pool(w.dtype, ka), ev_pos[:ne], theta))
        assert oracle.append(g, kp, vp, w.ev_request[:ne], ka, va, tail)[0] == 0
        lists = w.lists(last)
        q = w.q(last)
        reps, t_cpu = 0, 0.0
        while reps < 3 or (t_cpu < 10.0 and reps < 512):
            c0 = time.perf_counter()
            if args.rope:
                q64 = oracle.rope(oracle.widen_pool(w.dtype, q), q_pos[last], theta)
                ref, _ = oracle.attention_q64(g, kp, vp, w.dec_request, *lists, q64, w.scale)
            else:
                ref, _ = oracle.attention(g, kp, vp, w.dec_request, *lists, q, w.scale)
            t_cpu += time.perf_counter() - c0
            reps += 1
        cpu = {"value": w.n * reps / t_cpu, "unit": "stream-tokens/s", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": f"{reps} decode steps ({w.n} streams x 32 heads, {ne} pool rows) of one layer, fp64, "
                         f"{t_cpu:.1f} s; append not included (a {w.n * 4} KiB copy)"}
        chk = torch.empty(w.n, w.Hq, w.D, dtype=torch.bfloat16, device=dev)
        s.h.decode_step(0, w.dec_request, w.dec_stream, q_steps[last], chk, lists=lists, flags=flags,
                        position=q_pos[last])
        torch.cuda.synchronize()
        got = W.bf16_bits_to_f32(to_host_bits(chk, w.dtype)).astype(np.float64)
        result_extra["parity_vs_oracle"] = {"max_abs": float(np.max(np.abs(got - ref))),
                                            "rel_l2": float(np.linalg.norm(got - ref) / np.linalg.norm(ref))}
    # HBM traffic of the dominant kernel: NOT measured in this run -- read from the committed rocprofv3 --pmc
    # summary (FETCH_SIZE + WRITE_SIZE per launch, scaled by a copy of known size), and labelled as such
    traffic, traffic_src = None, None
    prof = os.path.join(ROOT, "profiles", "k_attn_config3.txt")
    if os.path.exists(prof) and not args.no_mfma:
        for line in open(prof):
            if line.startswith("TRAFFIC_BYTES_PER_LAUNCH="):
                traffic = float(line.split("=")[1])
                traffic_src = "profiles/k_attn_config3.txt (rocprofv3 --pmc, a separate run of this command)"
    res = {
        "metric": "multi-stream decode-attention stream-tokens/s (append + decode step, per layer)",
        "value": w.n * args.steps / elapsed,
        "unit": "stream-tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"config 3: bf16 32q/8kv heads D=128, prefix {args.prefix}, {args.streams} streams L~U[64,512] "
                               "right-aligned round-robin, append+decode per step",
                   "n_layers_cycled": L, "kv_layout": args.layout, "visibility": "maintained lists",
                   "before_the_timed_region": f"every pool touched once, {SPINUP_S} s of decode steps to bring the clocks up, "
                                              f"then the {args.warmup} warm-up steps",
                   "after_the_timed_region": f"{n_tail} more steps of the same loop, untimed, so that {len(durs)} launches "
                                             f"carry event pairs (every {every}th step)",
                   "append": "eager (own launch)" if (args.eager_append or args.rope) else "deferred (rides with the decode launch)",
                   "visibility_mode": "dense mask over the whole pool" if args.dense_mask else
                                      ("lists, prefix not shared" if args.no_share else "lists, shared prefix"),
                   "rope": "K rotated at append, Q in the attention kernel, theta 1e4" if args.rope else "off (Q, K arrive rotated)",
                   "model_tokens_per_s": w.n * args.steps / elapsed / L},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_src,
                     "kernel": "k_attn (shared-prefix + private-segment partials, one launch)",
                     "kernel_us": kern_s * 1e6, "kernel_us_median": float(np.median(durs)) * 1e6,
                     "kernel_us_min": float(np.min(durs)) * 1e6, "kernel_samples": len(durs),
                     "kernel_samples_in_timed_region": n_in_region,
                     "algorithmic_bytes": alg_bytes,
                     "measured_read_us": None if probe_s is None else probe_s * 1e6,
                     "measured_read_GBps": None if probe_s is None else alg_bytes / probe_s / 1e9,
                     "frac_of_measured_read": None if probe_s is None else probe_s / kern_s},
        "whole_step": {"algorithmic_GBps": alg_step / (elapsed / args.steps) / 1e9},
        "cpu_baseline": cpu,
    }
    res.update(result_extra)
    print(json.dumps(res))
    s.close()


def event_period(steps, asked):
    """Sampling period of the timed launches: the asked one, but short runs sample more often (at least 8
    samples when the run has that many steps after step 0)."""
    return max(1, min(asked, (steps - 1) // 8)) if steps > 1 else 1


def sampled(i, every):
    """Step i carries an event pair: every `every`-th step, never step 0 (the first launch after the warm-up's
    synchronisation finds an empty queue)."""
    return i > 0 and i % every == 0


def decode_only(args, w, dev):
    """Decode steps of a single-step configuration, cycling `--layers` pools that hold the same
    rows (only the decode is timed: these configurations define no token loop)."""
    import torch

    from paper_2502_11517_amd import binding as B
    from paper_2502_11517_amd.harness import Session, to_device

    row_bytes = 2 * w.Hkv * w.D * (2 if w.dtype == "bf16" else 4)
    pool_rows = (w.n_phys_pages * w.page_tokens) if w.page_tokens else w.max_requests * w.pool_tokens
    L = max(1, min(args.layers, int(6e9 // (pool_rows * row_bytes))))
    layout = B.HEAD_MAJOR if args.layout == "head" else B.TOKEN_MAJOR
    s = Session(w, kv_layout=layout, n_layers=L)
    hip = C.CDLL("libamdhip64.so.7")
    ne = w.n_events(0)
    for lo in range(0, ne, 65536):
        hi = min(ne, lo + 65536)
        k, v = w.kv_rows(lo, hi)
        kd, vd = to_device(k, w.dtype, dev), to_device(v, w.dtype, dev)
        for l in range(L):
            s.h.append_kv(l, w.ev_request[lo:hi], w.ev_stream[lo:hi], kd, vd, parent_stream=w.ev_parent[lo:hi])
        torch.cuda.synchronize()
    q = to_device(w.q(0), w.dtype, dev)
    out = torch.empty(L, w.n, w.Hq, w.D, dtype=q.dtype, device=dev)
    flags = (B.DECODE_NO_MFMA if args.no_mfma else 0) | (B.DECODE_ROW_GROUPS if args.row_groups else 0)
    every = event_period(args.steps, args.event_every)
    n_ev = args.steps // every + 1
    evs = []
    for _ in range(2 * n_ev):
        e = C.c_void_p()
        assert hip.hipEventCreate(C.byref(e)) == 0
        evs.append(e)
    calls = []
    for i in range(args.steps):
        j = i // every
        pe = (evs[2 * j], evs[2 * j + 1]) if sampled(i, every) else None
        calls.append(s.h.prepare_decode(i % L, w.dec_request, w.dec_stream, q, out[i % L], flags=flags, prof_events=pe))
    warm = [s.h.prepare_decode(l, w.dec_request, w.dec_stream, q, out[l], flags=flags) for l in range(L)]
    t_spin, n_spin = time.perf_counter(), 0
    while n_spin < L or time.perf_counter() - t_spin < SPINUP_S:  # every pool once, and the clocks up
        for i in range(16):
            assert warm[(n_spin + i) % L]() == 0
        n_spin += 16
        torch.cuda.synchronize()
    for i in range(args.warmup):
        assert warm[i % L]() == 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for c in calls:
        if c():
            raise SystemExit("library error in timed loop")
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms = C.c_float()
    durs = []
    for j in range(args.steps):
        if sampled(j, every):
            assert hip.hipEventElapsedTime(C.byref(ms), evs[2 * (j // every)], evs[2 * (j // every) + 1]) == 0
            durs.append(ms.value * 1e-3)
    kern_s = float(np.mean(durs))
    probe_s = None
    if args.probe_launches > 0 and not args.no_mfma and w.dtype == "bf16":
        pev = []
        for _ in range(2 * args.probe_launches):
            e = C.c_void_p()
            assert hip.hipEventCreate(C.byref(e)) == 0
            pev.append(e)
        pcalls = [s.h.prepare_decode(i % L, w.dec_request, w.dec_stream, q, out[i % L], flags=flags | B.DECODE_READ_PROBE,
                                     prof_events=(pev[2 * i], pev[2 * i + 1])) for i in range(args.probe_launches)]
        for c in pcalls:
            assert c() == 0
        torch.cuda.synchronize()
        pd = []
        for i in range(args.probe_launches):
            assert hip.hipEventElapsedTime(C.byref(ms), pev[2 * i], pev[2 * i + 1]) == 0
            pd.append(ms.value * 1e-3)
        probe_s = float(np.median(pd[len(pd) // 4:]))
    # algorithmic bytes: per request the common prefix once, everything else once per stream
    pl, offs, st, ct, sd = w.lists(0)
    rows = 0
    for r in np.unique(w.dec_request):
        idx = np.nonzero(w.dec_request == r)[0]
        pc = int(pl[idx].min())
        rows += pc + sum(int(pl[i]) - pc + int(ct[offs[i]:offs[i + 1]].sum()) for i in idx)
    alg_bytes = rows * row_bytes + w.n * w.Hq * w.D * (2 if w.dtype == "bf16" else 4)
    achieved = alg_bytes / kern_s / 1e9
    # the contraction side of the same launch: every visible row meets the query rows that see it, 2 D
    # multiply-adds for the logit and 2 D for the weighted sum per (row, query row) pair
    G = w.Hq // w.Hkv
    pairs = 0
    for r in np.unique(w.dec_request):
        idx = np.nonzero(w.dec_request == r)[0]
        pc = int(pl[idx].min())
        pairs += pc * len(idx) + sum(int(pl[i]) - pc + int(ct[offs[i]:offs[i + 1]].sum()) for i in idx)
    flops = 4.0 * w.D * pairs * w.Hq
    print(json.dumps({
        "metric": "multi-stream decode-attention stream-tokens/s (decode step only, per layer)",
        "value": w.n * args.steps / elapsed, "unit": "stream-tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{args.workload} ({w.name}): {w.n} streams, {rows} distinct visible rows, decode only",
                   "n_layers_cycled": L, "kv_layout": args.layout},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "kernel": "attention-partials launch", "kernel_us": kern_s * 1e6,
                     "kernel_us_median": float(np.median(durs)) * 1e6, "kernel_us_min": float(np.min(durs)) * 1e6,
                     "kernel_samples": len(durs), "algorithmic_bytes": alg_bytes,
                     "measured_read_us": None if probe_s is None else probe_s * 1e6,
                     "measured_read_GBps": None if probe_s is None else alg_bytes / probe_s / 1e9,
                     "frac_of_measured_read": None if probe_s is None else probe_s / kern_s},
        "roofline_mfma": {"bound": "mfma", "achieved": flops / kern_s / 1e12, "peak": 2500.0, "unit": "TFLOP/s",
                          "frac": flops / kern_s / 1e12 / 2500.0, "algorithmic_flops": flops,
                          "note": "same launch priced as a bf16 contraction (stacked query rows x visible rows); "
                                  "the larger of the two fractions says which roofline is nearer"},
        "cpu_baseline": None}))
    s.close()


def replay_bench(args, dev):
    """A whole synthetic response through the interpreter's control flow (pasta_attn_replay) on
    `--layers` pools, against the same number of tokens decoded as ONE sequential thread: what the
    asynchronous decoding buys at the attention path.  Trace: blocks of median ~38 tokens (the
    paper's statistic), predicted lengths in multiples of ten, a sync every third promise."""
    import torch

    from paper_2502_11517_amd import binding as B
    from paper_2502_11517_amd import workloads as W
    from paper_2502_11517_amd.harness import Session

    L, P = args.layers, 1024
    ops = W.synthetic_trace(2025, n_promises=9, text_mean=12, block_median=38, sync_every=3, tail_text=24)
    w = W.Workload(name="replay", dtype="bf16", Hq=32, Hkv=8, D=128, scale=1.0, seed=1, max_requests=1,
                   pool_tokens=4096, max_streams=8, k_std=128 ** -0.5)
    w.ev_request = np.zeros(P, np.int32)
    w.ev_stream = np.zeros(P, np.int32)
    w.ev_parent = np.full(P, -1, np.int32)
    w.n_prefill = P
    results, host_s = {}, {}
    n_tok = None
    for mode in ("pasta", "sequential"):
        s = Session(w, kv_layout=B.HEAD_MAJOR, n_layers=L, max_ranges=16384, rope_theta=10000.0 if args.rope else 0.0)
        g = torch.Generator(device=dev).manual_seed(7)
        kp = torch.randn(P, w.Hkv, w.D, device=dev, generator=g).to(torch.bfloat16) * 0.088
        vp = torch.randn(P, w.Hkv, w.D, device=dev, generator=g).to(torch.bfloat16)
        for l in range(L):
            s.h.append_kv(l, w.ev_request, w.ev_stream, kp, vp, position=np.arange(P, dtype=np.int32),
                          flags=B.APPEND_ROPE if args.rope else 0)
        plan = s.h.replay(0, ops, P, 4096 - P, flags=B.REPLAY_PLAN_ONLY)
        if n_tok is None:
            n_tok = int(plan["stats"][0])
            pasta_stats = plan["stats"].copy()
        run_ops = ops if mode == "pasta" else [(B.OP_TEXT, n_tok, 0)]
        kd = torch.randn(L, n_tok, w.Hkv, w.D, device=dev, generator=g).to(torch.bfloat16) * 0.088
        vd = torch.randn(L, n_tok, w.Hkv, w.D, device=dev, generator=g).to(torch.bfloat16)
        qd = torch.randn(L, n_tok, w.Hq, w.D, device=dev, generator=g).to(torch.bfloat16)
        out = torch.empty_like(qd)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        r = s.h.replay(0, run_ops, P, n_tok, kd, vd, qd, out, flags=B.REPLAY_ROPE if args.rope else 0)
        t_host = time.perf_counter() - t0  # all launches enqueued
        torch.cuda.synchronize()
        results[mode] = (time.perf_counter() - t0, int(r["stats"][1]))
        host_s[mode] = t_host
        assert int(r["stats"][0]) == n_tok and bool(torch.isfinite(out.float()).all())
        s.close()
        del s, kd, vd, qd, out
    t_p, passes_p = results["pasta"]
    t_s, passes_s = results["sequential"]
    n_content = sum(a for k, a, b in ops if k == 0) + sum(b for k, a, b in ops if k == 1)
    print(json.dumps({
        "metric": "trace replay: tokens/s through the attention path (append + decode on every layer, whole response)",
        "value": n_tok / t_p, "unit": "tokens/s", "n_gpus": 1, "steps": passes_p * L, "warmup": 0,
        "ms_per_step": t_p / (passes_p * L) * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"replay: prompt {P}, synthetic trace of 9 promises (block median ~38 tokens, predicted "
                               f"lengths in tens, sync every 3), bf16 32q/8kv heads D=128, {L} layers",
                   "rope": bool(args.rope)},
        "trace": {"tokens": n_tok, "passes": passes_p, "most_rows_in_a_pass": int(pasta_stats[2]),
                  "forks": int(pasta_stats[3]), "syncs": int(pasta_stats[4]),
                  "theoretical_parallelism": n_content / passes_p,
                  "rows_per_pass": n_tok / passes_p},
        "sequential": {"passes": passes_s, "seconds": t_s, "tokens_per_s": n_tok / t_s,
                       "host_enqueue_seconds": host_s["sequential"]},
        "pasta": {"passes": passes_p, "seconds": t_p, "host_enqueue_seconds": host_s["pasta"]},
        "speedup_at_the_attention_path": t_s / t_p,
        "roofline": None, "cpu_baseline": None}))


if __name__ == "__main__":
    main()
