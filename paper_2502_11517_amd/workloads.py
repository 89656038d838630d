"""Seeded synthetic workloads for the multi-stream decode-attention step.

This module only GENERATES inputs (fork histories, interleave orders, K/V/Q values, page
tables, the callers' visibility lists).  It holds none of the method's arithmetic and is the
one module both the HIP path's tests and the CPU oracle's tests draw inputs from.

The paper (arxiv 2502.11517) evaluates on AlpacaEval prompts run through finetuned
Gemma-7B models; neither is needed here, because the attention step depends only on shapes
and on the fork structure.  The five configurations below stand in for that workload.  The
statistics the paper does print (Section 3: batch 1, pool of 2048 slots, three concurrent
threads in the worked example; Section 5.3: median asynchronous block just under 40 tokens)
are far smaller than these; the shapes here are Llama-style stress sizes.

Conventions (where the configuration text leaves a choice open):
  * stream 0 of every request is the root (main thread); it owns the shared prefix and is
    paused (waiting at its sync point) while the forks decode, as in the paper's example.
  * "random interleave": a uniform shuffle of the multiset {s repeated L_s times}; the j-th
    occurrence of s is the j-th token of s.
  * "round-robin": right-aligned lock-step -- at time tau in [0, L_max) every stream with
    L_s >= L_max - tau appends one token, in stream-id order (all streams are live at the
    end and started at different times, the situation of Figure 2c).
  * log-normal lengths (config 4): exp(N(ln 96, 1)) rounded, clamped to [1, 1024].
  * seeds: 1000 + configuration number.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

ROOT = 0


# ----------------------------------------------------------------------------- number formats
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 bit patterns (uint16). Inputs are finite."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


# ----------------------------------------------------------------------------- list encoding
def slots_to_ranges(slots):
    """Encodes an ascending slot list as (start, count, stride) arithmetic runs, greedily."""
    out = []
    i, n = 0, len(slots)
    while i < n:
        if i + 1 >= n:
            out.append((int(slots[i]), 1, 1))
            break
        st = int(slots[i + 1]) - int(slots[i])
        j = i + 1
        while j + 1 < n and int(slots[j + 1]) - int(slots[j]) == st:
            j += 1
        out.append((int(slots[i]), j - i + 1, st))
        i = j + 1
    return out


@dataclass
class Workload:
    name: str
    dtype: str  # "f32" | "bf16"
    Hq: int
    Hkv: int
    D: int
    scale: float
    seed: int
    max_requests: int = 1
    page_tokens: int = 0
    pool_tokens: int = 0
    n_phys_pages: int = 0
    pages_per_request: int = 0
    page_table: np.ndarray | None = None
    max_streams: int = 2
    q_std: float = 1.0
    k_std: float = 1.0
    v_std: float = 1.0
    # fork history: one entry per pool row in call (= physical) order
    ev_request: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int32))
    ev_stream: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int32))
    ev_parent: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int32))
    n_prefill: int = 0  # events [0, n_prefill) are the state before the first decode step
    # the streams that decode, in output-row order
    dec_request: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int32))
    dec_stream: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int32))
    steps: int = 1  # decode steps; steps > 1: every step appends one row per decoding stream first
    # scenario statement: what each decoding stream sees of OTHER streams (its ancestors):
    # anc_slots[i] = ascending logical slots of ancestors visible to decoding stream i
    anc_slots: list = field(default_factory=list)

    # ---- derived
    @property
    def n(self) -> int:
        return int(self.dec_request.shape[0])

    @property
    def np_dtype(self):
        return np.float32 if self.dtype == "f32" else np.uint16

    def n_events(self, step: int = 0) -> int:
        """Pool rows that exist when decode step `step` runs (step 0 = after the prefill)."""
        if self.steps == 1:
            return self.n_prefill
        return self.n_prefill + (step + 1) * self.n

    def _encode(self, x: np.ndarray) -> np.ndarray:
        return x.astype(np.float32) if self.dtype == "f32" else f32_to_bf16_bits(x)

    def kv_rows(self, lo: int, hi: int):
        """K and V rows [hi-lo][Hkv][D] of events [lo, hi), deterministic per event block."""
        B = 2048
        ks, vs = [], []
        b0 = lo // B
        while b0 * B < hi:
            rng = np.random.default_rng([self.seed, 1, b0])
            k = rng.standard_normal((B, self.Hkv, self.D), dtype=np.float32) * np.float32(self.k_std)
            v = rng.standard_normal((B, self.Hkv, self.D), dtype=np.float32) * np.float32(self.v_std)
            a, b = max(lo, b0 * B) - b0 * B, min(hi, (b0 + 1) * B) - b0 * B
            ks.append(self._encode(k[a:b]))
            vs.append(self._encode(v[a:b]))
            b0 += 1
        if not ks:
            z = np.zeros((0, self.Hkv, self.D), self.np_dtype)
            return z, z.copy()
        return np.concatenate(ks), np.concatenate(vs)

    def q(self, step: int = 0) -> np.ndarray:
        rng = np.random.default_rng([self.seed, 2, step])
        x = rng.standard_normal((self.n, self.Hq, self.D), dtype=np.float32) * np.float32(self.q_std)
        return self._encode(x)

    def event_positions(self, n_events: int | None = None) -> np.ndarray:
        """A position id for every event, as inputs for the rotary option: a stream counts up from
        where it starts; a fork starts at its parent's next id, and the parent then jumps ahead by
        a seeded multiple of ten (the stand-in for a predicted block length)."""
        n_events = len(self.ev_request) if n_events is None else n_events
        rng = np.random.default_rng([self.seed, 3])
        nxt: dict = {}
        pos = np.empty(n_events, np.int32)
        for e in range(n_events):
            key = (int(self.ev_request[e]), int(self.ev_stream[e]))
            if key not in nxt:
                par = (key[0], int(self.ev_parent[e]))
                if par in nxt:
                    nxt[key] = nxt[par]
                    nxt[par] += 10 * int(rng.integers(1, 30))
                else:
                    nxt[key] = 0
            pos[e] = nxt[key]
            nxt[key] += 1
        return pos

    def q_positions(self, step: int = 0) -> np.ndarray:
        """Position id of each decoding stream's newest token at decode step `step`."""
        ne = self.n_events(step)
        pos = self.event_positions(ne)
        out = np.zeros(self.n, np.int32)
        for i in range(self.n):
            m = np.nonzero((self.ev_request[:ne] == self.dec_request[i]) & (self.ev_stream[:ne] == self.dec_stream[i]))[0]
            out[i] = pos[m[-1]] if m.size else 0
        return out

    def event_slots(self, n_events: int | None = None) -> np.ndarray:
        """Logical slot of every event: its rank among the events of its request."""
        n_events = len(self.ev_request) if n_events is None else n_events
        req = self.ev_request[:n_events]
        order = np.argsort(req, kind="stable")
        sorted_req = req[order]
        first = np.searchsorted(sorted_req, sorted_req, side="left")
        slots = np.empty(n_events, np.int32)
        slots[order] = (np.arange(n_events) - first).astype(np.int32)
        return slots

    def lists(self, step: int = 0):
        """The caller's visibility lists at decode step `step`:
        (prefix_len[n], range_offsets[n+1], start, count, stride).  Each decoding stream sees
        the ancestor slots the scenario states (anc_slots) plus the slots it owns."""
        ne = self.n_events(step)
        slots = self.event_slots(ne)
        pl, offs, st, ct, sd = [], [0], [], [], []
        for i in range(self.n):
            own = slots[(self.ev_request[:ne] == self.dec_request[i])
                        & (self.ev_stream[:ne] == self.dec_stream[i])]
            vis = np.sort(np.concatenate([np.asarray(self.anc_slots[i], np.int64), own.astype(np.int64)]))
            assert np.all(np.diff(vis) > 0)
            neq = np.nonzero(vis != np.arange(len(vis)))[0]
            p = int(neq[0]) if len(neq) else len(vis)
            pl.append(p)
            for (a, c, s) in slots_to_ranges(vis[p:]):
                st.append(a), ct.append(c), sd.append(s)
            offs.append(len(st))
        i32 = lambda a: np.asarray(a, dtype=np.int32)  # noqa: E731
        return i32(pl), i32(offs), i32(st), i32(ct), i32(sd)

    def fork_tree(self, req: int, n_events: int | None = None):
        """Fork history of one request for a dense-mask check:
        (slot_stream[tail], stream_parent[max_streams], stream_spawn_tail[max_streams])."""
        n_events = len(self.ev_request) if n_events is None else n_events
        sel = np.nonzero(self.ev_request[:n_events] == req)[0]
        slot_stream = self.ev_stream[sel].astype(np.int32)
        parent = np.full(self.max_streams, -1, np.int32)
        spawn = np.zeros(self.max_streams, np.int64)
        seen = set()
        for t, e in enumerate(sel):
            s = int(self.ev_stream[e])
            if s not in seen:
                seen.add(s)
                parent[s] = self.ev_parent[e]
                spawn[s] = t
        return slot_stream, parent, spawn


# ----------------------------------------------------------------------------- interleaves
def _interleave_random(rng, lengths):
    order = np.repeat(np.arange(len(lengths)), lengths)
    rng.shuffle(order)
    return order


def _interleave_round_robin(lengths):
    lmax = int(max(lengths)) if len(lengths) else 0
    order = []
    for tau in range(lmax):
        for s, L in enumerate(lengths):
            if L >= lmax - tau:
                order.append(s)
    return np.asarray(order, dtype=np.int64)


def _fork_events(order, first_id, parents):
    """Events for interleaved fork tokens: stream ids first_id + order; the first token of a
    stream carries its parent."""
    seen = set()
    ev_s, ev_p = [], []
    for o in order:
        s = first_id + int(o)
        ev_s.append(s)
        ev_p.append(-1 if s in seen else parents[int(o)])
        seen.add(s)
    return ev_s, ev_p


def _finish(w: Workload, ev_r, ev_s, ev_p, n_prefill):
    w.ev_request = np.asarray(ev_r, np.int32)
    w.ev_stream = np.asarray(ev_s, np.int32)
    w.ev_parent = np.asarray(ev_p, np.int32)
    w.n_prefill = n_prefill
    return w


def single_request(name, dtype, Hq, Hkv, D, scale, seed, prefix, lengths, interleave, steps=1,
                   q_std=1.0, k_std=1.0, v_std=1.0, nested=None, slack=64):
    """One request: root prefix, then forks with the given lengths.
    nested = (sub_prefix_tokens, n_children): a fork that decodes sub_prefix_tokens alone and
    then spawns the first n_children of the streams (the rest fork from the root)."""
    rng = np.random.default_rng(seed)
    n = len(lengths)
    ev_s = [ROOT] * prefix
    ev_p = [-1] * prefix
    first = 1
    parents = [ROOT] * n
    anc = [list(range(prefix)) for _ in range(n)]
    if nested is not None:
        sub, nch = nested
        ev_s += [1] * sub
        ev_p += [ROOT] + [-1] * (sub - 1)
        first = 2
        for c in range(nch):
            parents[c] = 1
            anc[c] = list(range(prefix + sub))
    order = _interleave_random(rng, lengths) if interleave == "random" else _interleave_round_robin(lengths)
    fs, fp = _fork_events(order, first, parents)
    ev_s += fs
    ev_p += fp
    n_prefill = len(ev_s)
    if steps > 1:  # every further step appends one row per decoding stream, in stream order
        for _ in range(steps):
            ev_s += [first + i for i in range(n)]
            ev_p += [-1] * n
    w = Workload(name=name, dtype=dtype, Hq=Hq, Hkv=Hkv, D=D, scale=scale, seed=seed,
                 max_requests=1, pool_tokens=-(-(len(ev_s) + slack) // 64) * 64,
                 max_streams=first + n, q_std=q_std, k_std=k_std, v_std=v_std, steps=steps)
    w.dec_request = np.zeros(n, np.int32)
    w.dec_stream = np.arange(first, first + n, dtype=np.int32)
    w.anc_slots = anc
    return _finish(w, [0] * len(ev_s), ev_s, ev_p, n_prefill)


def config1():
    """Tiny fp32: 4 query heads, 1 KV head, D=64; prefix 256; 2 streams x 16 tokens, random
    interleave; Q, K, V ~ N(0,1)/sqrt(64); textbook scale 1/sqrt(64)."""
    return single_request("cfg1_tiny_f32", "f32", 4, 1, 64, 0.125, 1001, 256, [16, 16], "random",
                          q_std=0.125, k_std=0.125, v_std=0.125)


def config2():
    """bf16 32/8/128; prefix 1024; 4 streams, lengths uniform in [32,256], random interleave;
    Q, V ~ N(0,1), K ~ N(0,1)/sqrt(128) (scale folded into K, so softmax_scale = 1)."""
    rng = np.random.default_rng(1002)
    L = rng.integers(32, 257, size=4).tolist()
    return single_request("cfg2_llama8b_p1k_s4", "bf16", 32, 8, 128, 1.0, 1002, 1024, L, "random",
                          k_std=128 ** -0.5)


def config3(steps: int = 64, prefix: int = 8192, n_streams: int = 8):
    """bf16 32/8/128; prefix 8192; 8 streams, lengths uniform in [64,512], right-aligned
    round-robin interleave; 64 consecutive decode steps, each preceded by the append of one
    row per stream."""
    rng = np.random.default_rng(1003)
    L = rng.integers(64, 513, size=n_streams).tolist()
    return single_request("cfg3_llama8b_p8k_s8", "bf16", 32, 8, 128, 1.0, 1003, prefix, L,
                          "round_robin", steps=steps, k_std=128 ** -0.5)


def config5():
    """bf16 64/8/128; prefix 32768; 16 streams of 256..2048 tokens; streams 0-3 are children of
    a fork that first decoded a 512-token sub-prefix alone (nested fork); round-robin."""
    rng = np.random.default_rng(1005)
    L = rng.integers(256, 2049, size=16).tolist()
    return single_request("cfg5_long_p32k_s16_nested", "bf16", 64, 8, 128, 1.0, 1005, 32768, L,
                          "round_robin", k_std=128 ** -0.5, nested=(512, 4))


def config4(n_requests: int = 16, seed: int = 1004, pmin: int = 256, pmax: int = 4096,
            page_tokens: int = 16, hq: int = 32, hkv: int = 8, smin: int = 1, smax: int = 8):
    """Ragged paged batch: 16 independent requests, bf16 32/8/128; per request a prefix uniform
    in [256,4096] and 1..8 streams with log-normal lengths (median 96, cap 1024), random
    interleave; 16-token pages placed by a seeded permutation of the page pool."""
    rng = np.random.default_rng(seed)
    ev_r, ev_s, ev_p = [], [], []
    dec_r, dec_s, anc = [], [], []
    tails = []
    max_streams = 2
    per_req = []
    for r in range(n_requests):
        P = int(rng.integers(pmin, pmax + 1))
        ns = int(rng.integers(smin, smax + 1))
        L = np.clip(np.rint(np.exp(rng.normal(np.log(96.0), 1.0, size=ns))), 1, 1024).astype(int).tolist()
        order = _interleave_random(rng, L)
        fs, fp = _fork_events(order, 1, [ROOT] * ns)
        per_req.append(([ROOT] * P + fs, [-1] * P + fp))
        for i in range(ns):
            dec_r.append(r), dec_s.append(1 + i), anc.append(list(range(P)))
        tails.append(P + len(fs))
        max_streams = max(max_streams, ns + 1)
    # requests are prefilled one after the other (their pools are independent)
    for r, (s_list, p_list) in enumerate(per_req):
        ev_r += [r] * len(s_list)
        ev_s += s_list
        ev_p += p_list
    ppr = max(-(-(t + 1) // page_tokens) for t in tails)
    need = [-(-(t + 1) // page_tokens) for t in tails]
    n_phys = sum(need) + 8
    perm = rng.permutation(n_phys).astype(np.int32)
    table = np.zeros((n_requests, ppr), np.int32)
    pos = 0
    for r in range(n_requests):
        table[r, :need[r]] = perm[pos:pos + need[r]]
        table[r, need[r]:] = -1  # no page assigned: beyond the request's tail
        pos += need[r]
    w = Workload(name="cfg4_ragged_paged16", dtype="bf16", Hq=hq, Hkv=hkv, D=128, scale=1.0, seed=seed,
                 max_requests=n_requests, page_tokens=page_tokens, n_phys_pages=n_phys,
                 pages_per_request=ppr, page_table=table, max_streams=max_streams,
                 k_std=128 ** -0.5)
    w.dec_request = np.asarray(dec_r, np.int32)
    w.dec_stream = np.asarray(dec_s, np.int32)
    w.anc_slots = anc
    return _finish(w, ev_r, ev_s, ev_p, len(ev_r))


def random_fork_history(seed: int, n_slots: int = 48, max_streams: int = 6, p_fork: float = 0.15,
                        p_retire: float = 0.05):
    """A random fork history for one request in which EVERY live stream (the root included)
    keeps decoding, forks open at random times from random live streams (nested forks
    included) and streams retire at random -- the general situation of Figure 2b.
    Returns (ev_stream[n_slots], ev_parent[n_slots]); slot t is event t."""
    rng = np.random.default_rng(seed)
    live = [ROOT]
    next_id = 1
    ev_s, ev_p = [ROOT], [-1]
    while len(ev_s) < n_slots:
        if next_id < max_streams and rng.random() < p_fork:
            par = int(rng.choice(live))
            ev_s.append(next_id), ev_p.append(par)
            live.append(next_id)
            next_id += 1
            continue
        if len(live) > 1 and rng.random() < p_retire:
            live.pop(int(rng.integers(0, len(live))))
        for s in list(live):  # one lock-step round: every live stream appends one token
            if len(ev_s) < n_slots:
                ev_s.append(s), ev_p.append(-1)
    return np.asarray(ev_s, np.int32), np.asarray(ev_p, np.int32)


def random_fork_sync_history(seed: int, n_slots: int = 80, max_ids: int = 5, p_fork: float = 0.2,
                             p_sync: float = 0.12):
    """A random history for one request with forks, synchronisations and reuse of thread ids:
    every live thread appends one token per lock-step round; now and then a live thread spawns a
    child (nested forks included); now and then a thread whose children have no live children of
    their own waits for them: the children end, the thread's next token is its sync token, and
    the children's ids become free for later forks.
    Returns a list of events in pool order, each a dict
      {"stream": id, "parent": id or -1, "new": first token of a thread, "join": [ids joined by this token]}."""
    rng = np.random.default_rng(seed)
    live, children, free_ids = [ROOT], {ROOT: []}, list(range(1, max_ids))
    events = [dict(stream=ROOT, parent=-1, new=True, join=[])]
    pending_join: dict = {}
    while len(events) < n_slots:
        r = rng.random()
        if free_ids and r < p_fork:
            par = int(rng.choice(live))
            cid = free_ids.pop(0)
            events.append(dict(stream=cid, parent=par, new=True, join=[]))
            live.append(cid)
            children[par].append(cid)
            children[cid] = []
            continue
        if r > 1.0 - p_sync:
            cands = [x for x in live if children[x] and x not in pending_join
                     and all(not children[c] and c not in pending_join for c in children[x])]
            if cands:
                x = int(rng.choice(cands))
                pending_join[x] = list(children[x])
                for c in children[x]:
                    live.remove(c)
                children[x] = []
        for sid in list(live):  # one lock-step round
            if len(events) >= n_slots:
                break
            j = pending_join.pop(sid, [])
            events.append(dict(stream=sid, parent=-1, new=False, join=j))
            for c in j:  # the joined ids are free again once the sync token is in the pool
                del children[c]
                free_ids.append(c)
    return events


def synthetic_trace(seed: int, n_promises: int = 6, text_mean: int = 12, block_median: int = 38,
                    sync_every: int = 3, tail_text: int = 20):
    """A synthetic annotation trace for the replay: what the main thread would emit.  Blocks have a
    log-normal length around `block_median` tokens (the paper reports a median asynchronous block
    just under 40 tokens); the predicted length is the true length rounded to a multiple of ten,
    now and then off by ten (the predictions are not exact); a sync follows every `sync_every`
    promises.  Returns a list of (kind, a, b) with kind 0 = TEXT, 1 = PROMISE, 2 = SYNC."""
    rng = np.random.default_rng([seed, 4])
    ops = []
    for i in range(n_promises):
        ops.append((0, int(rng.integers(1, 2 * text_mean)), 0))
        true_len = int(np.clip(np.rint(rng.lognormal(np.log(block_median), 0.6)), 1, 400))
        pred = max(0, 10 * int(np.rint(true_len / 10.0)) + 10 * int(rng.integers(-1, 2)))
        ops.append((1, pred, true_len))
        if (i + 1) % sync_every == 0:
            ops.append((0, int(rng.integers(1, text_mean)), 0))
            ops.append((2, 0, 0))
    if ops[-1][0] != 2:
        ops.append((0, int(rng.integers(1, text_mean)), 0))
        ops.append((2, 0, 0))
    ops.append((0, tail_text, 0))
    return ops
