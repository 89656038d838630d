// Trace replay: the PASTA-LANG interpreter's control flow (arxiv 2502.11517, Section 3,
// "Interpreter" and "Efficiency"; Figure 2) driven by a SYNTHETIC annotation trace instead of a
// model's samples.  The trace says what the main thread would emit -- runs of ordinary tokens,
// promise tags (with the predicted and the actual length of their asynchronous block), sync
// tags -- and the replay does what the interpreter does with them, one forward pass after the
// other, through this library's own entry points:
//   * every active thread feeds one token per pass; the rows enter the pool in the order
//     main thread, (a fork born in this pass), older forks by age -- so concurrently active
//     threads interleave (Figure 2c);
//   * a promise token spawns a thread at once: the interpreter-inserted <async> token is the
//     next row of the same pass and the fork's first query; the fork then feeds its content
//     tokens and its </async> token, one per pass, and ends;
//   * a sync token is held back: the main thread pauses until every thread it spawned has
//     ended; the next pass joins them (pasta_attn_sync, ids retired), feeds the sync token and
//     the main thread goes on, now seeing the forks' rows where they are;
//   * position ids (Section 4, "Training a PASTA-SFT model": the predicted block length gives
//     estimated ids; appendix "Positional Embedding", the multiples-of-ten variant): the fork
//     counts on from the promise, the main thread skips the PREDICTED length.
// Everything here is host bookkeeping plus calls of append_kv / sync / decode_step.
#pragma once
#include <vector>

namespace {

struct ReplayFork {
  int32_t stream;     // library stream id
  int32_t next_pos;   // position id of its next token
  int32_t remaining;  // tokens still to feed (content + </async>)
};

}  // namespace

extern "C" int32_t pasta_attn_replay(pasta_attn* h, const pasta_replay_args* a) {
  if (!h || h->magic != kMagic) return PASTA_E_STATE;
  if (!a || a->struct_size != sizeof(pasta_replay_args)) return PASTA_E_INVAL;
  const pasta_attn_config& c = h->cfg;
  if (a->request_id < 0 || a->request_id >= c.max_requests) return PASTA_E_INVAL;
  if (a->n_ops < 0 || (a->n_ops > 0 && !a->ops) || a->first_pos < 0 || a->max_tokens < 0) return PASTA_E_INVAL;
  const bool plan_only = a->flags & PASTA_REPLAY_PLAN_ONLY;
  const bool rope = a->flags & PASTA_REPLAY_ROPE;
  if (!plan_only && (!a->k_rows || !a->v_rows || !a->q_rows || !a->out)) return PASTA_E_INVAL;
  if (rope && !(c.rope_theta > 0.f)) return PASTA_E_INVAL;
  for (int i = 0; i < a->n_ops; ++i) {
    const pasta_trace_op& op = a->ops[i];
    if (op.kind < PASTA_OP_TEXT || op.kind > PASTA_OP_SYNC) return PASTA_E_INVAL;
    if (op.kind == PASTA_OP_TEXT && op.a < 1) return PASTA_E_INVAL;
    if (op.kind == PASTA_OP_PROMISE && (op.a < 0 || op.b < 0)) return PASTA_E_INVAL;
  }
  if (!sstate(h, a->request_id, 0).open) return PASTA_E_STATE;  // the prompt must be in the pool as stream 0

  // a planning run leaves the handle as it found it
  std::vector<int64_t> saved_tail, saved_tail_before;
  std::vector<StreamState> saved_streams;
  auto restore = [&]() {
    if (!plan_only) return;
    h->tail.swap(saved_tail);
    h->tail_before.swap(saved_tail_before);
    const size_t base = (size_t)a->request_id * c.max_streams;
    for (int s = 0; s < c.max_streams; ++s) h->streams[base + s] = std::move(saved_streams[s]);
  };
  try {
    if (plan_only) {
      saved_tail = h->tail;
      saved_tail_before = h->tail_before;
      const size_t base = (size_t)a->request_id * c.max_streams;
      saved_streams.assign(h->streams.begin() + base, h->streams.begin() + base + c.max_streams);
    }
    const size_t row_bytes = (size_t)c.n_kv_heads * c.head_dim * h->elem, q_bytes = (size_t)c.n_q_heads * c.head_dim * h->elem;
    std::vector<ReplayFork> forks;          // by age; ended forks stay until the sync that joins them
    std::vector<char> id_used(c.max_streams, 0);
    for (int s = 0; s < c.max_streams; ++s) id_used[s] = sstate(h, a->request_id, s).open ? 1 : 0;
    std::vector<int32_t> spawned;           // stream ids spawned since the last sync
    int32_t main_pos = a->first_pos;
    int op_i = 0, text_left = 0;
    bool waiting = false;                   // a sync token has been produced and is held back
    int64_t n_tok = 0, n_pass = 0, max_active = 0, n_sync = 0, n_fork = 0;
    std::vector<int32_t> rid, sid, par, pos, slots;
    int rc = PASTA_OK;

    for (;;) {
      size_t alive = 0;
      for (const ReplayFork& f : forks) alive += f.remaining > 0;
      const bool main_done = op_i >= a->n_ops;
      if (main_done && alive == 0) break;
      rid.clear(); sid.clear(); par.clear(); pos.clear();
      auto push = [&](int32_t stream, int32_t parent, int32_t p) {
        rid.push_back(a->request_id); sid.push_back(stream); par.push_back(parent); pos.push_back(p);
      };
      const size_t n_old = forks.size();  // a fork born in this pass has fed its <async> already
      if (!main_done) {
        const pasta_trace_op& op = a->ops[op_i];
        if (op.kind == PASTA_OP_SYNC) waiting = true;
        if (waiting) {
          if (alive == 0) {  // nothing (left) to wait for: join, then the sync token goes in
            if (!spawned.empty()) {
              pasta_sync_args sa{sizeof(pasta_sync_args), PASTA_SYNC_RETIRE, a->request_id, 0, (int32_t)spawned.size(),
                                 spawned.data()};
              rc = pasta_attn_sync(h, &sa);
              if (rc != PASTA_OK) break;
              for (int32_t s : spawned) id_used[s] = 0;
              spawned.clear();
            }
            forks.clear();
            push(0, -1, main_pos++);
            waiting = false;
            n_sync++;
            op_i++;
          }  // else: the main thread sits this pass out
        } else if (op.kind == PASTA_OP_TEXT) {
          if (text_left == 0) text_left = op.a;
          push(0, -1, main_pos++);
          if (--text_left == 0) op_i++;
        } else {  // PASTA_OP_PROMISE
          int32_t fid = -1;
          for (int s = 1; s < c.max_streams; ++s)
            if (!id_used[s]) { fid = s; break; }
          if (fid < 0) { rc = PASTA_E_CAPACITY; break; }
          id_used[fid] = 1;
          push(0, -1, main_pos);                       // the promise token
          push(fid, 0, main_pos + 1);                  // the inserted <async> token: the fork's first row
          forks.push_back({fid, main_pos + 2, op.b + 1});  // content and </async> still to come
          main_pos += 1 + op.a;                        // the main thread skips the PREDICTED block length
          spawned.push_back(fid);
          n_fork++;
          op_i++;
        }
      }
      for (size_t t = 0; t < (forks.empty() ? 0 : std::min(n_old, forks.size())); ++t) {
        ReplayFork& f = forks[t];
        if (f.remaining <= 0) continue;
        push(f.stream, -1, f.next_pos++);
        f.remaining--;
      }
      const int n = (int)rid.size();
      if (n_tok + n > a->max_tokens) { rc = PASTA_E_CAPACITY; break; }

      // ---- the pass on every layer: rows into the pool (the copy rides with the decode launch), one query per row
      slots.assign(n, -1);
      for (int layer = 0; layer < (plan_only ? 1 : c.n_layers) && rc == PASTA_OK; ++layer) {
        const size_t tok_off = (size_t)layer * a->max_tokens + n_tok;
        pasta_append_args aa{};
        aa.struct_size = sizeof(aa);
        aa.layer = layer;
        aa.n_rows = n;
        aa.request_id = rid.data();
        aa.stream_id = sid.data();
        aa.parent_stream = par.data();
        aa.position = pos.data();
        aa.out_slot = layer == 0 ? slots.data() : nullptr;
        if (plan_only) {
          aa.flags = PASTA_APPEND_RESERVE_ONLY;
        } else {
          aa.flags = PASTA_APPEND_DEFER | (rope ? PASTA_APPEND_ROPE : 0u);
          aa.k_new = (const char*)a->k_rows + tok_off * row_bytes;
          aa.v_new = (const char*)a->v_rows + tok_off * row_bytes;
        }
        rc = pasta_attn_append_kv(h, &aa);
        if (rc != PASTA_OK || plan_only) break;
        pasta_decode_args da{};
        da.struct_size = sizeof(da);
        da.flags = rope ? PASTA_DECODE_ROPE_Q : 0u;
        da.layer = layer;
        da.n_streams = n;
        da.request_id = rid.data();
        da.stream_id = sid.data();
        da.position = pos.data();
        da.q = (const char*)a->q_rows + tok_off * q_bytes;
        da.out = (char*)a->out + tok_off * q_bytes;
        rc = pasta_attn_decode_step(h, &da);
      }
      if (rc != PASTA_OK) break;
      for (int i = 0; i < n; ++i) {
        if (a->tok_slot) a->tok_slot[n_tok + i] = slots[i];
        if (a->tok_stream) a->tok_stream[n_tok + i] = sid[i];
        if (a->tok_pos) a->tok_pos[n_tok + i] = pos[i];
        if (a->tok_pass) a->tok_pass[n_tok + i] = (int32_t)n_pass;
      }
      n_tok += n;
      n_pass++;
      max_active = std::max<int64_t>(max_active, n);
    }
    if (rc == PASTA_OK && a->stats) {
      a->stats[0] = n_tok;        // rows fed = queries answered
      a->stats[1] = n_pass;       // forward passes = the longest chain that had to be sequential
      a->stats[2] = max_active;   // most rows in one pass
      a->stats[3] = n_fork;
      a->stats[4] = n_sync;
      a->stats[5] = main_pos;     // the main thread's next position id
      a->stats[6] = a->stats[7] = 0;
    }
    restore();
    return rc;
  } catch (const std::bad_alloc&) {
    restore();
    return PASTA_E_NOMEM;
  }
}
