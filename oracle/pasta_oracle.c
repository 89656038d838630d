/*
 * pasta_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, fp64 CPU statement of what the multi-stream decode-attention
 * step of PASTA's interpreter computes (arxiv 2502.11517, Section 3, paragraph
 * "Efficiency"; Figure 2b for the visibility rule, Figure 2c for the pool).
 * Only tests, the smoke check and the bench's cpu_baseline leg may call it.
 * It shares no code, header, table or helper with the HIP library: the pool
 * addressing formulas below are written out again here on purpose.
 *
 * What is an exact definition here and what is a convention:
 *   - attention value: textbook softmax attention over the gathered rows, in
 *     fp64 (exact definition; the GPU reaches the same value up to rounding).
 *   - visibility: the paper's ancestor rule (a token of an asynchronous thread
 *     sees its own thread and the tokens of the spawning thread that existed
 *     before the spawn), applied transitively for nested forks.
 *   - pool layout (token-major / head-major, pages): this build's convention;
 *     the paper only says "single contiguous pre-allocated pool".
 *
 * Pins (tests/test_oracle_*.py): library SDPA in fp64 for the single-stream
 * case, closed forms (constant V, q = 0, one / two visible rows), the paper's
 * worked visibility example, brute-force dense mask on tiny shapes,
 * permutation invariance, split/merge identity.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC pasta_oracle.c -o libpasta_oracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  int32_t dtype; /* 0 = fp32, 1 = bf16 (stored as uint16) */
  int32_t n_q_heads, n_kv_heads, head_dim;
  int32_t max_requests;
  int32_t page_tokens; /* 0 = contiguous */
  int32_t head_major;  /* 0 = token-major, 1 = head-major */
  int32_t n_phys_pages;
  int32_t pages_per_request;
  int32_t pad_;
  int64_t pool_tokens;
  const int32_t *page_table; /* [max_requests][pages_per_request] */
} oracle_geom;

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ---------- element widening (exact) ---------- */
static double widen(const void *base, int dtype, int64_t idx) {
  if (dtype == 2) return ((const double *)base)[idx]; /* fp64: rotated queries only */
  if (dtype == 0) return (double)((const float *)base)[idx];
  uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16; /* bf16 = top half of fp32 */
  float f;
  memcpy(&f, &bits, 4);
  return (double)f;
}
static int elem_bytes(int dtype) { return dtype == 0 ? 4 : 2; }

/* ---------- pool addressing (this build's layout convention) ---------- */
int64_t oracle_rows_per_layer(const oracle_geom *g) {
  if (g->page_tokens == 0) return (int64_t)g->max_requests * g->pool_tokens;
  return (int64_t)g->n_phys_pages * g->page_tokens;
}

/* logical slot of a request -> physical row of the layer's pool; -1 if out of range */
int64_t oracle_phys_row(const oracle_geom *g, int32_t req, int64_t slot) {
  if (req < 0 || req >= g->max_requests || slot < 0) return -1;
  if (g->page_tokens == 0) {
    if (slot >= g->pool_tokens) return -1;
    return (int64_t)req * g->pool_tokens + slot;
  }
  int64_t lp = slot / g->page_tokens;
  if (lp >= g->pages_per_request) return -1;
  int64_t pp = g->page_table[(int64_t)req * g->pages_per_request + lp];
  if (pp < 0 || pp >= g->n_phys_pages) return -1;
  return pp * g->page_tokens + slot % g->page_tokens;
}

/* element offset of (physical row, kv head) inside one layer's K or V pool */
int64_t oracle_elem_offset(const oracle_geom *g, int64_t phys, int32_t head) {
  const int64_t D = g->head_dim, H = g->n_kv_heads;
  if (!g->head_major) return (phys * H + head) * D;
  if (g->page_tokens == 0) return ((int64_t)head * oracle_rows_per_layer(g) + phys) * D;
  int64_t page = phys / g->page_tokens, in_page = phys % g->page_tokens;
  return ((page * H + head) * g->page_tokens + in_page) * D;
}

/* ---------- A1: append (Section 3, Efficiency: rows go to the pool tail in
 * the order the active threads produce them) ---------- */
int oracle_append(const oracle_geom *g, void *k_pool, void *v_pool, int32_t n_rows,
                  const int32_t *request_id, const void *k_new, const void *v_new,
                  int64_t *tail /* [max_requests], in/out */, int32_t *out_slot) {
  const int64_t D = g->head_dim, H = g->n_kv_heads;
  const int eb = elem_bytes(g->dtype);
  /* first pass: capacity, so that a failing call changes nothing */
  int64_t *t2 = (int64_t *)malloc(sizeof(int64_t) * (size_t)g->max_requests);
  if (!t2) return -3;
  memcpy(t2, tail, sizeof(int64_t) * (size_t)g->max_requests);
  for (int32_t i = 0; i < n_rows; ++i) {
    int32_t r = request_id[i];
    if (r < 0 || r >= g->max_requests) { free(t2); return -1; }
    if (oracle_phys_row(g, r, t2[r]) < 0) { free(t2); return -2; }
    t2[r]++;
  }
  free(t2);
  for (int32_t i = 0; i < n_rows; ++i) {
    int32_t r = request_id[i];
    int64_t slot = tail[r]++;
    int64_t phys = oracle_phys_row(g, r, slot);
    for (int32_t h = 0; h < H; ++h) {
      int64_t dst = oracle_elem_offset(g, phys, h);
      int64_t src = ((int64_t)i * H + h) * D;
      memcpy((char *)k_pool + dst * eb, (const char *)k_new + src * eb, (size_t)(D * eb));
      memcpy((char *)v_pool + dst * eb, (const char *)v_new + src * eb, (size_t)(D * eb));
    }
    if (out_slot) out_slot[i] = (int32_t)slot;
  }
  return 0;
}

/* ---------- gather map: the visible list of one stream, in list order, as
 * physical rows.  out_rows may be NULL (count only).  Returns the count, or
 * -1 if a slot falls outside the request's pool. ---------- */
int64_t oracle_gather_map(const oracle_geom *g, int32_t req, int32_t prefix_len, int32_t n_ranges,
                          const int32_t *start, const int32_t *count, const int32_t *stride,
                          int64_t *out_rows) {
  int64_t n = 0;
  for (int64_t t = 0; t < prefix_len; ++t) {
    int64_t p = oracle_phys_row(g, req, t);
    if (p < 0) return -1;
    if (out_rows) out_rows[n] = p;
    n++;
  }
  for (int32_t k = 0; k < n_ranges; ++k)
    for (int64_t j = 0; j < count[k]; ++j) {
      int64_t p = oracle_phys_row(g, req, (int64_t)start[k] + j * stride[k]);
      if (p < 0) return -1;
      if (out_rows) out_rows[n] = p;
      n++;
    }
  return n;
}

/* ---------- textbook attention of one query head over a list of physical
 * rows: copy the rows to contiguous fp64 buffers, logits, max-subtracted
 * softmax, weighted sum.  Also usable as the "partial" (m, l, acc) of a
 * subset when normalise == 0. ---------- */
static int attend_rows_q(const oracle_geom *g, const void *k_pool, const void *v_pool, int64_t n,
                         const int64_t *rows, const void *q, int q_dtype, int64_t q_off, int32_t kv_head,
                         double scale, int normalise, double *out /* [D] */, double *m_out,
                         double *l_out) {
  const int64_t D = g->head_dim;
  double *Kc = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1) * (size_t)D);
  double *Vc = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1) * (size_t)D);
  double *z = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
  if (!Kc || !Vc || !z) { free(Kc); free(Vc); free(z); return -3; }
  for (int64_t t = 0; t < n; ++t) {
    int64_t off = oracle_elem_offset(g, rows[t], kv_head);
    for (int64_t d = 0; d < D; ++d) {
      Kc[t * D + d] = widen(k_pool, g->dtype, off + d);
      Vc[t * D + d] = widen(v_pool, g->dtype, off + d);
    }
  }
  double m = -INFINITY;
  for (int64_t t = 0; t < n; ++t) {
    double s = 0.0;
    for (int64_t d = 0; d < D; ++d) s += widen(q, q_dtype, q_off + d) * Kc[t * D + d];
    z[t] = scale * s;
    if (z[t] > m) m = z[t];
  }
  double l = 0.0;
  for (int64_t d = 0; d < D; ++d) out[d] = 0.0;
  for (int64_t t = 0; t < n; ++t) {
    double p = exp(z[t] - m);
    l += p;
    for (int64_t d = 0; d < D; ++d) out[d] += p * Vc[t * D + d];
  }
  if (normalise && n > 0)
    for (int64_t d = 0; d < D; ++d) out[d] /= l;
  *m_out = m;
  *l_out = l;
  free(Kc); free(Vc); free(z);
  return 0;
}

static int attend_rows(const oracle_geom *g, const void *k_pool, const void *v_pool, int64_t n,
                       const int64_t *rows, const void *q, int64_t q_off, int32_t kv_head,
                       double scale, int normalise, double *out, double *m_out, double *l_out) {
  return attend_rows_q(g, k_pool, v_pool, n, rows, q, g->dtype, q_off, kv_head, scale, normalise, out,
                       m_out, l_out);
}

/* ---------- A2+A3+A4 as one definition: for each stream gather its visible
 * rows and run textbook attention per query head.
 * q: [n][Hq][D] pool dtype.  out: [n][Hq][D] fp64.  lse: [n][Hq] fp64 or NULL. */
static int attention_core(const oracle_geom *g, const void *k_pool, const void *v_pool, int32_t n_streams,
                          const int32_t *request_id, const int32_t *prefix_len,
                          const int32_t *range_offsets, const int32_t *range_start,
                          const int32_t *range_count, const int32_t *range_stride, const void *q,
                          int q_dtype, double scale, double *out, double *lse) {
  const int64_t D = g->head_dim, Hq = g->n_q_heads;
  const int32_t G = g->n_q_heads / g->n_kv_heads;
  int64_t **maps = (int64_t **)calloc((size_t)n_streams, sizeof(int64_t *));
  int64_t *cnt = (int64_t *)calloc((size_t)n_streams, sizeof(int64_t));
  if (!maps || !cnt) { free(maps); free(cnt); return -3; }
  int rc = 0;
  for (int32_t s = 0; s < n_streams; ++s) {
    int32_t r0 = range_offsets[s], r1 = range_offsets[s + 1];
    int64_t n = oracle_gather_map(g, request_id[s], prefix_len[s], r1 - r0, range_start + r0,
                                  range_count + r0, range_stride + r0, NULL);
    if (n <= 0) { rc = -1; break; }
    maps[s] = (int64_t *)malloc(sizeof(int64_t) * (size_t)n);
    if (!maps[s]) { rc = -3; break; }
    cnt[s] = oracle_gather_map(g, request_id[s], prefix_len[s], r1 - r0, range_start + r0,
                               range_count + r0, range_stride + r0, maps[s]);
  }
  if (rc == 0) {
    int64_t total = (int64_t)n_streams * Hq;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t w = 0; w < total; ++w) {
      int32_t s = (int32_t)(w / Hq), h = (int32_t)(w % Hq);
      double m, l;
      int r = attend_rows_q(g, k_pool, v_pool, cnt[s], maps[s], q, q_dtype, ((int64_t)s * Hq + h) * D,
                            h / G, scale, 1, out + ((int64_t)s * Hq + h) * D, &m, &l);
      if (r != 0) {
#pragma omp atomic write
        rc = r;
      }
      if (lse) lse[(int64_t)s * Hq + h] = m + log(l);
    }
  }
  for (int32_t s = 0; s < n_streams; ++s) free(maps[s]);
  free(maps); free(cnt);
  return rc;
}

int oracle_attention(const oracle_geom *g, const void *k_pool, const void *v_pool, int32_t n_streams,
                     const int32_t *request_id, const int32_t *prefix_len,
                     const int32_t *range_offsets, const int32_t *range_start,
                     const int32_t *range_count, const int32_t *range_stride, const void *q,
                     double scale, double *out, double *lse) {
  return attention_core(g, k_pool, v_pool, n_streams, request_id, prefix_len, range_offsets, range_start,
                        range_count, range_stride, q, g->dtype, scale, out, lse);
}

/* The same with queries given in fp64 (queries rotated by oracle_rope are not
 * rounded back to the pool dtype: the rotation is part of the definition, the
 * rounding of a rotated query would be an implementation's choice). */
int oracle_attention_q64(const oracle_geom *g, const void *k_pool, const void *v_pool, int32_t n_streams,
                         const int32_t *request_id, const int32_t *prefix_len,
                         const int32_t *range_offsets, const int32_t *range_start,
                         const int32_t *range_count, const int32_t *range_stride, const double *q,
                         double scale, double *out, double *lse) {
  return attention_core(g, k_pool, v_pool, n_streams, request_id, prefix_len, range_offsets, range_start,
                        range_count, range_stride, q, 2, scale, out, lse);
}

/* ---------- rotary position embedding with given (estimated) position ids.
 * The paper assigns position ids to tokens after a promise from the predicted
 * length of the asynchronous block (Section 4, "Training a PASTA-SFT model";
 * appendix "Positional Embedding") and leaves the embedding to the base model.
 * Rotary embedding (RoFormer) in the half-split pairing that Gemma / Llama
 * implementations use: the head dim is D/2 planes (x[f], x[f + D/2]); plane f is
 * turned by the angle pos * theta^(-2 f / D).
 * x, out: [n_rows][n_heads][D] fp64; pos: [n_rows]. ---------- */
void oracle_rope(const double *x, int64_t n_rows, int32_t n_heads, int32_t D, const int32_t *pos,
                 double theta, double *out) {
  const int32_t half = D / 2;
  for (int64_t r = 0; r < n_rows; ++r)
    for (int32_t h = 0; h < n_heads; ++h) {
      const double *xi = x + (r * n_heads + h) * (int64_t)D;
      double *oi = out + (r * n_heads + h) * (int64_t)D;
      for (int32_t f = 0; f < half; ++f) {
        double angle = (double)pos[r] * pow(theta, -2.0 * (double)f / (double)D);
        double c = cos(angle), sn = sin(angle);
        oi[f] = xi[f] * c - xi[f + half] * sn;
        oi[f + half] = xi[f + half] * c + xi[f] * sn;
      }
    }
}

/* ---------- fp64 -> pool dtype, one rounding to nearest even (what "the pool
 * holds rotated keys in bf16 / fp32" means).  out: float[n] or uint16[n]. */
void oracle_round_pool(const double *x, int64_t n, int32_t dtype, void *out) {
  for (int64_t i = 0; i < n; ++i) {
    if (dtype == 0) { ((float *)out)[i] = (float)x[i]; continue; }
    double v = x[i];
    float f;
    if (v == 0.0 || !isfinite(v)) {
      f = (float)v;
    } else {
      int e;
      (void)frexp(v, &e);          /* |v| = m 2^e, m in [0.5, 1) */
      int ulp_exp = (e - 1) - 7;   /* bf16 keeps 8 significant bits */
      if (ulp_exp < -133) ulp_exp = -133; /* subnormal range of bf16 */
      double q = nearbyint(ldexp(v, -ulp_exp)); /* ties to even in the default rounding mode */
      f = (float)ldexp(q, ulp_exp);             /* exact: at most 9 significant bits */
    }
    uint32_t bits;
    memcpy(&bits, &f, 4);
    ((uint16_t *)out)[i] = (uint16_t)(bits >> 16);
  }
}

/* ---------- partial over an arbitrary subset of physical rows (for testing
 * the split kernels and the merge in isolation): m = max z, l = sum e^{z-m},
 * acc = sum e^{z-m} v.  An empty subset gives (-inf, 0, 0). ---------- */
int oracle_partial(const oracle_geom *g, const void *k_pool, const void *v_pool, int64_t n,
                   const int64_t *phys_rows, const void *q_row /* [D] pool dtype */, int32_t kv_head,
                   double scale, double *m, double *l, double *acc /* [D] */) {
  return attend_rows(g, k_pool, v_pool, n, phys_rows, q_row, 0, kv_head, scale, 0, acc, m, l);
}

/* ---------- A4: log-sum-exp merge of k partials, written from the identity
 * sum_t e^{z_t} v_t = sum_i e^{m_i} acc_i. ---------- */
int oracle_merge(int32_t k, int32_t D, const double *m, const double *l, const double *acc /* [k][D] */,
                 double *out /* [D] */, double *lse) {
  double M = -INFINITY;
  for (int32_t i = 0; i < k; ++i)
    if (l[i] > 0.0 && m[i] > M) M = m[i];
  double L = 0.0;
  for (int32_t d = 0; d < D; ++d) out[d] = 0.0;
  if (M == -INFINITY) { if (lse) *lse = -INFINITY; return -1; }
  for (int32_t i = 0; i < k; ++i) {
    if (!(l[i] > 0.0)) continue; /* empty partial contributes nothing */
    double w = exp(m[i] - M);
    L += l[i] * w;
    for (int32_t d = 0; d < D; ++d) out[d] += acc[(int64_t)i * D + d] * w;
  }
  for (int32_t d = 0; d < D; ++d) out[d] /= L;
  if (lse) *lse = M + log(L);
  return 0;
}

/* ---------- A0, dense form: the paper's rule from the fork history alone.
 * slot_stream[t]      owner of pool slot t (one request)
 * stream_parent[s]    spawning stream, -1 for the root
 * stream_spawn_tail[s] number of pool slots that existed when s was spawned
 * A query of stream qs sees slot t iff t belongs to qs, or t belongs to an
 * ancestor a of qs and existed before the child of a on the path to qs was
 * spawned (and before every later spawn on that path).
 * mask_out: [n_slots] bytes, 1 = visible. ---------- */
int oracle_visible_dense(int64_t n_slots, const int32_t *slot_stream, int32_t n_streams,
                         const int32_t *stream_parent, const int64_t *stream_spawn_tail, int32_t qs,
                         uint8_t *mask_out) {
  if (qs < 0 || qs >= n_streams) return -1;
  for (int64_t t = 0; t < n_slots; ++t) {
    int32_t a = qs;
    int64_t bound = INT64_MAX;
    int vis = 0, hops = 0;
    for (;;) {
      if (slot_stream[t] == a && t < bound) { vis = 1; break; }
      if (stream_parent[a] < 0) break;
      if (stream_spawn_tail[a] < bound) bound = stream_spawn_tail[a];
      a = stream_parent[a];
      if (++hops > n_streams) return -1; /* cycle in the fork tree */
    }
    mask_out[t] = (uint8_t)vis;
  }
  return 0;
}

/* ---------- A0 with synchronisation, as the paper draws it (Figure 2b): "each
 * directed edge connects a token to the very next token that may attend to it;
 * a token can attend to any ancestor token reachable by following these edges
 * backward".  Edges into pool slot t, from the history alone:
 *   - the previous token of t's own thread;
 *   - if t is the first token of a forked thread: the spawning thread's latest
 *     token at that moment (ev_parent[t] >= 0 on that slot);
 *   - if t is a token with which its thread synchronises (the sync token that
 *     enters the pool once the awaited forks are complete): the latest token of
 *     every joined thread (join_streams[join_offsets[t] .. join_offsets[t+1])).
 * A thread id may be used again after its thread has ended: the slot that
 * carries ev_parent >= 0 (or the very first use) starts a NEW thread.
 * ev_new[t] = 1 marks such first tokens.  mask_out[u] = 1 iff slot u is q_slot
 * or reachable backwards from q_slot.  One request. ---------- */
int oracle_visible_events(int64_t n_slots, const int32_t *ev_stream, const int32_t *ev_parent,
                          const uint8_t *ev_new, const int32_t *join_offsets,
                          const int32_t *join_streams, int32_t n_stream_ids, int64_t q_slot,
                          uint8_t *mask_out) {
  if (q_slot < 0 || q_slot >= n_slots) return -1;
  int64_t *last_of = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n_stream_ids > 0 ? n_stream_ids : 1));
  int64_t *pred_off = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n_slots + 1));
  int64_t n_join_total = join_offsets ? join_offsets[n_slots] : 0;
  int64_t *pred = (int64_t *)malloc(sizeof(int64_t) * (size_t)(2 * n_slots + n_join_total + 1));
  int64_t *stack = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n_slots + 1));
  if (!last_of || !pred_off || !pred || !stack) { free(last_of); free(pred_off); free(pred); free(stack); return -3; }
  for (int32_t s = 0; s < n_stream_ids; ++s) last_of[s] = -1;
  int64_t np = 0;
  int rc = 0;
  for (int64_t t = 0; t < n_slots && rc == 0; ++t) {
    int32_t s = ev_stream[t];
    pred_off[t] = np;
    if (s < 0 || s >= n_stream_ids) { rc = -1; break; }
    if (ev_new[t]) {
      if (ev_parent[t] >= 0) {
        if (ev_parent[t] >= n_stream_ids || last_of[ev_parent[t]] < 0) { rc = -1; break; }
        pred[np++] = last_of[ev_parent[t]];
      }
    } else {
      if (last_of[s] < 0) { rc = -1; break; }
      pred[np++] = last_of[s];
    }
    if (join_offsets)
      for (int32_t k = join_offsets[t]; k < join_offsets[t + 1]; ++k) {
        int32_t j = join_streams[k];
        if (j < 0 || j >= n_stream_ids || last_of[j] < 0) { rc = -1; break; }
        pred[np++] = last_of[j];
      }
    last_of[s] = t;
  }
  if (rc == 0) {
    pred_off[n_slots] = np;
    memset(mask_out, 0, (size_t)n_slots);
    int64_t top = 0;
    stack[top++] = q_slot;
    mask_out[q_slot] = 1;
    while (top > 0) {
      int64_t t = stack[--top];
      for (int64_t k = pred_off[t]; k < pred_off[t + 1]; ++k)
        if (!mask_out[pred[k]]) { mask_out[pred[k]] = 1; stack[top++] = pred[k]; }
    }
  }
  free(last_of); free(pred_off); free(pred); free(stack);
  return rc;
}

/* ---------- brute force: attention of one stream over ALL slots [0, n_slots)
 * of its request with masked logits set to -inf (the paper's dense-mask form).
 * q_row: [Hq][D]; out: [Hq][D] fp64; lse: [Hq] or NULL. ---------- */
int oracle_attention_dense(const oracle_geom *g, const void *k_pool, const void *v_pool, int32_t req,
                           int64_t n_slots, const uint8_t *mask, const void *q_row, double scale,
                           double *out, double *lse) {
  const int64_t D = g->head_dim;
  const int32_t G = g->n_q_heads / g->n_kv_heads;
  double *z = (double *)malloc(sizeof(double) * (size_t)(n_slots > 0 ? n_slots : 1));
  if (!z) return -3;
  for (int32_t h = 0; h < g->n_q_heads; ++h) {
    int32_t kh = h / G;
    double m = -INFINITY;
    for (int64_t t = 0; t < n_slots; ++t) {
      if (!mask[t]) { z[t] = -INFINITY; continue; }
      int64_t off = oracle_elem_offset(g, oracle_phys_row(g, req, t), kh);
      double s = 0.0;
      for (int64_t d = 0; d < D; ++d)
        s += widen(q_row, g->dtype, (int64_t)h * D + d) * widen(k_pool, g->dtype, off + d);
      z[t] = scale * s;
      if (z[t] > m) m = z[t];
    }
    double l = 0.0;
    for (int64_t t = 0; t < n_slots; ++t)
      if (mask[t]) l += exp(z[t] - m);
    for (int64_t d = 0; d < D; ++d) {
      double o = 0.0;
      for (int64_t t = 0; t < n_slots; ++t) {
        if (!mask[t]) continue;
        int64_t off = oracle_elem_offset(g, oracle_phys_row(g, req, t), kh);
        o += exp(z[t] - m) / l * widen(v_pool, g->dtype, off + d);
      }
      out[(int64_t)h * D + d] = o;
    }
    if (lse) lse[h] = m + log(l);
  }
  free(z);
  return 0;
}
