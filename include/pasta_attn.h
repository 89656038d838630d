/*
 * pasta_attn.h -- C ABI of the multi-stream decode-attention step of PASTA's
 * asynchronous decoding (arxiv 2502.11517, Section 3 "Language and Interpreter
 * Design", paragraph "Efficiency", and Figure 2b/2c).
 *
 * The operation.  Several decoding threads ("streams") of one response each
 * decode their next token in the same forward pass against ONE pre-allocated
 * KV pool.  Streams append their K/V rows to the pool tail as they decode, so
 * rows of concurrently active streams are physically interleaved (Section 3,
 * Efficiency: single contiguous pre-allocated pool with an interleaved layout;
 * Figure 2c).  A query row of stream s attends only to the tokens reachable
 * from it in the fork graph: its own tokens plus the tokens of its ancestors
 * that existed before the fork (Section 3, Efficiency, the attention-mask
 * paragraph; Figure 2b).  In this library that visible set is a list
 *
 *     Vis(s) = [0, prefix_len_s)  U  { start_k + j*stride_k : j < count_k }_k
 *
 * of logical slots of the request's pool, and one decode step computes, for
 * every active stream s and query head h (KV head g = h / (Hq/Hkv)),
 *
 *     z_t = softmax_scale * <q[s,h,:], K[t,g,:]>          t in Vis(s)
 *     out[s,h,:] = sum_t softmax(z)_t * V[t,g,:]
 *     lse[s,h]   = log sum_t exp(z_t)
 *
 * No KV row is ever moved or copied after it has been appended (Section 3,
 * Efficiency, last paragraphs; contrast with the appendix "Naive Interpreter
 * Implementation").
 *
 * Everything runs on one GPU (gfx950).  The library exports eight symbols:
 * the four calls of the hot path (pasta_attn_create, pasta_attn_append_kv,
 * pasta_attn_decode_step, pasta_attn_destroy), three calls of host control
 * flow around it (pasta_attn_sync, pasta_attn_stream_list: the fork / sync
 * lifecycle of the maintained lists; pasta_attn_replay: a whole response
 * through the interpreter's control flow) and pasta_attn_decode_step_noalloc
 * (the decode step for callers that may not allocate).  All entry points
 * return a status code; none throws or aborts.  "HOST" / "DEVICE" below say
 * where a pointer must point.  The library allocates NO device memory: pool,
 * workspace, Q and outputs are the caller's (the one piece of device memory
 * of its own is the fixed-size static array of the no-alloc entry point).
 * The page table alone is a HOST array: it is written once, create copies it
 * into the workspace, and the host-side planner reads it too.
 */
#ifndef PASTA_ATTN_H
#define PASTA_ATTN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pasta_attn pasta_attn; /* opaque; one per (shape, pool) */

enum {
  PASTA_OK = 0,
  PASTA_E_INVAL = -1,    /* bad argument; nothing enqueued, no state changed */
  PASTA_E_CAPACITY = -2, /* pool / page table / stream table / workspace full */
  PASTA_E_NOMEM = -3,    /* host allocation failed */
  PASTA_E_DEVICE = -4,   /* a HIP call failed (or no GPU is present) */
  PASTA_E_STATE = -5     /* unknown stream, destroyed handle, layer order */
};

enum { PASTA_F32 = 0, PASTA_BF16 = 1 };

/* Placement of one token's rows inside a layer's pool.  The paper fixes only
 * "one contiguous pool, rows appended at the tail"; the order of the head and
 * token axes is this library's choice and a create-time fact.
 *
 * Physical row of (request r, logical slot t):
 *   contiguous mode (page_tokens == 0):  phys = r * pool_tokens + t
 *   paged mode      (page_tokens  > 0):  phys = page_table[r][t / page_tokens]
 *                                               * page_tokens + t % page_tokens
 * With rows_per_layer = max_requests * pool_tokens (contiguous) or
 * n_phys_pages * page_tokens (paged), the ELEMENT offset of (phys, kv head g)
 * inside a layer's K (or V) pool is
 *   TOKEN_MAJOR:              (phys * Hkv + g) * D
 *   HEAD_MAJOR, contiguous:   (g * rows_per_layer + phys) * D
 *   HEAD_MAJOR, paged:        ((page * Hkv + g) * page_tokens + phys % page_tokens) * D,
 *                             page = phys / page_tokens
 * and layer l starts at element l * rows_per_layer * Hkv * D.               */
enum { PASTA_LAYOUT_TOKEN_MAJOR = 0, PASTA_LAYOUT_HEAD_MAJOR = 1 };

typedef struct {
  uint32_t struct_size;   /* sizeof(pasta_attn_config); ABI check */
  int32_t dtype;          /* PASTA_F32 | PASTA_BF16: pool, Q and out element type */
  int32_t n_q_heads;      /* Hq */
  int32_t n_kv_heads;     /* Hkv; Hq % Hkv == 0, Hq/Hkv in {1,2,4,8} */
  int32_t head_dim;       /* D in {64, 128} */
  int32_t n_layers;       /* >= 1 pools that share one slot assignment */
  int32_t max_requests;   /* 1 = the paper's batch-1 setting */
  int32_t page_tokens;    /* 0 = contiguous; else a power of two (e.g. 16) */
  int32_t kv_layout;      /* PASTA_LAYOUT_* */
  int32_t n_phys_pages;   /* paged mode: physical pages per layer */
  int32_t pages_per_request; /* paged mode: columns of page_table */
  int32_t max_streams;    /* stream ids per request are 0 .. max_streams-1 */
  int32_t max_ranges;     /* most range descriptors one decode_step may carry
                             (sum over its streams) */
  float softmax_scale;    /* applied to q.k; explicit, never implied */
  float rope_theta;       /* base of the rotary position embedding, e.g. 10000; 0 = the
                             library never rotates (PASTA_APPEND_ROPE / PASTA_DECODE_ROPE_Q
                             are then E_INVAL).  See "Rotary embedding" below. */
  int64_t pool_tokens;    /* contiguous mode: slots per request per layer (the
                             paper's fixed maximum sequence length) */
  void *k_pool;           /* DEVICE, borrowed for the handle's lifetime:
                             n_layers * rows_per_layer * Hkv * D elements */
  void *v_pool;           /* DEVICE, same shape */
  const int32_t *page_table; /* HOST [max_requests][pages_per_request], copied at
                             create (paged mode; NULL otherwise).  A request's assigned
                             pages come first, each in [0, n_phys_pages) and distinct over
                             the whole table; -1 = no page assigned (only after the
                             assigned ones): the request's capacity ends there. */
  void *workspace;        /* DEVICE, borrowed, 256-byte aligned */
  uint64_t workspace_bytes; /* in: bytes provided; query mode writes bytes needed */
  void *hip_stream;       /* hipStream_t of the caller; all work is enqueued here */
} pasta_attn_config;

/* Rotary embedding (optional).  Tokens decoded after a promise get ESTIMATED
 * position ids, because the length of the asynchronous block before them is
 * only predicted (Section 4, "Training a PASTA-SFT model": the model predicts each
 * block's length in the promise tag's tokens attribute; appendix "Positional
 * Embedding": lengths in multiples of ten).  Where the rotation is applied is not
 * stated; here the caller passes the ids and the library can apply the base
 * model's rotary embedding while it touches the data anyway: to K in append_kv
 * (PASTA_APPEND_ROPE) and to Q in decode_step (PASTA_DECODE_ROPE_Q).  Convention:
 * half-split pairs over the whole head dim -- with f = i mod D/2 and
 * angle = position * rope_theta^(-2 f / D),
 *   out[i]       = x[i] cos(angle) - x[i + D/2] sin(angle)        (i <  D/2)
 *   out[i + D/2] = x[i + D/2] cos(angle) + x[i] sin(angle)
 * computed in fp32 (angle reduced in fp64) and rounded once to the pool dtype.
 * V is never rotated.                                                        */

/* Creates a handle.  With out == NULL ("query mode") only validates cfg and
 * writes the required size into cfg->workspace_bytes; pointers in cfg may be
 * NULL then.  Otherwise cfg->workspace_bytes must be at least that size.
 * Makes no HIP call that needs a device except one synchronous copy of the
 * page table into the workspace (paged mode).
 * Errors: E_INVAL (shape / NULL / misaligned / bad page table), E_CAPACITY
 * (workspace too small), E_NOMEM, E_DEVICE.                                  */
int32_t pasta_attn_create(pasta_attn_config *cfg, pasta_attn **out);

/* KV append (Section 3, Efficiency: every active thread appends its new
 * KV-cache row to the pool tail, so rows of concurrently active threads land
 * in neighbouring slots and alternate; Figure 2c).
 * Row i takes logical slot tail[request_id[i]]++ in CALL ORDER -- call order
 * IS the physical interleave.  The same slots are used for every layer: the
 * call with layer == 0 comes first, assigns the slots and advances the
 * bookkeeping (tails, visibility lists), so that a decode_step on layer 0 may
 * follow at once; the identical call for each of the layers 1 .. n_layers-1
 * (before the next layer-0 append) writes those layers' rows to the same slots
 * and changes no state.  A token the interpreter defers (the paper's <sync/>
 * row) is simply not passed until it is to enter the pool.                   */
enum {
  PASTA_APPEND_RESERVE_ONLY = 1u, /* assign slots and advance the bookkeeping, copy nothing:
                                    the caller's own kernel writes the rows (out_slot says
                                    where); k_new / v_new may be NULL */
  PASTA_APPEND_DEFER = 2u,       /* bookkeeping now, copy later: the rows are copied into the
                                    pool by the attention launch of the next decode_step on
                                    the same layer (which reads them from k_new / v_new
                                    wherever its lists name them), or by a small launch of
                                    their own at the next call on the handle that cannot
                                    take them along.  k_new / v_new must stay valid and
                                    unchanged until that work has run.  Saves one launch
                                    per append + decode step; ignored for more than 32 rows. */
  PASTA_APPEND_ROPE = 4u         /* rotate every K row by position[i] on its way into the
                                    pool (needs position != NULL and rope_theta > 0; not
                                    with RESERVE_ONLY).  Combines with DEFER: the rows are then
                                    turned by the small launch that a decode_step with
                                    rotations puts ahead of its attention launch. */
};

typedef struct {
  uint32_t struct_size;
  uint32_t flags;               /* PASTA_APPEND_* */
  int32_t layer;
  int32_t n_rows;               /* >= 0; 0 is a no-op */
  const int32_t *request_id;    /* HOST [n_rows], each in [0, max_requests) */
  const int32_t *stream_id;     /* HOST [n_rows], each in [0, max_streams) */
  const int32_t *parent_stream; /* HOST [n_rows] or NULL.  >= 0 only on a row that
                                   OPENS stream_id: the new stream inherits the
                                   parent's visible set as of this row (ancestor
                                   rule).  -1 otherwise; a row with -1 whose stream
                                   is unknown opens a root stream (empty visible
                                   set). */
  const int32_t *position;      /* HOST [n_rows] or NULL: position ids >= 0 (the paper's
                                   length-predicted ids).  Used only with
                                   PASTA_APPEND_ROPE; otherwise K arrives already
                                   rotated and the ids are ignored */
  const void *k_new;            /* DEVICE [n_rows][Hkv][D], pool dtype */
  const void *v_new;            /* DEVICE [n_rows][Hkv][D] */
  int32_t *out_slot;            /* HOST [n_rows] or NULL: logical slot given to row i */
} pasta_append_args;

/* Errors: E_INVAL (NULL, ids out of range, parent unknown or equal to the
 * stream, parent given for a stream that is already open), E_CAPACITY (pool or
 * page table full; max_ranges exceeded), E_STATE (layer out of range; a
 * layer > 0 call that does not replay the latest layer-0 call), E_DEVICE.  A failing call enqueues nothing and changes no state.           */
int32_t pasta_attn_append_kv(pasta_attn *h, const pasta_append_args *a);

/* One decode step: one query token per active stream, all in one pass over
 * the shared pool (Section 1, Interpreter: several non-contiguous chunks are
 * decoded simultaneously; Section 3, Efficiency: masked attention over the
 * interleaved pool).  The step attends to exactly the listed rows and nothing
 * implicit: the caller appends the current token's K/V first if the token is
 * to see itself.
 *
 * Visibility comes in one of two modes:
 *   explicit   (range_offsets != NULL): prefix_len[n] and a CSR of
 *              (start, count, stride) descriptors per stream, all HOST.  Within
 *              a stream every range must start after the last slot of the one
 *              before it, the first must start at or after prefix_len, all slots
 *              must be < tail of the request, count >= 1, stride >= 1, and the
 *              visible set must not be empty.
 *   maintained (range_offsets == NULL): the lists that append_kv has been
 *              keeping for (request_id[i], stream_id[i]).
 * Output row i belongs to stream i of the call.                              */
enum {
  PASTA_DECODE_PLAN_ONLY = 1u, /* validate + plan + fill HOST debug outputs, enqueue nothing */
  PASTA_DECODE_NO_MFMA = 2u,   /* route the shared prefix through the private-segment
                                  kernel too (the path F32 always takes) */
  PASTA_DECODE_ROPE_Q = 4u,    /* rotate query row i by position[i] before use (q itself is
                                  not modified; needs position != NULL, rope_theta > 0) */
  /* Two comparison modes, same results, more bytes -- what the segment lists and the shared
   * prefix save (the appendix on the naive interpreter; Section 5.1: the paper's own
   * implementation runs attention over its whole static pool under a mask): */
  PASTA_DECODE_NO_SHARE = 8u,  /* no shared-prefix items: every stream reads its whole
                                  visible set by itself (the prefix once per stream) */
  PASTA_DECODE_DENSE_MASK = 16u, /* every stream walks ALL slots [0, tail) of its request and
                                  masks what it may not see: the lists are turned into a 0/1
                                  byte mask per stream on the host, copied to the device, and
                                  applied to the logits.  BF16, head_dim 128 only. */
  PASTA_DECODE_DEVICE_LISTS = 256u, /* maintained mode: take the lists from their device-resident copy even when the
                                       step's plan would fit the kernel arguments (see "Maintained lists on the
                                       device" below); E_INVAL with explicit lists, causal_skip or DENSE_MASK,
                                       E_CAPACITY when the copy has no room */
  /* A request with more than 32 stacked query rows (streams x heads per kv head) is served in groups of 32 rows:
   * one group per work-group, or -- when every request of the step with a shared prefix is that wide -- four
   * groups per work-group.  The library picks by the step's shape; these two flags force either form (both:
   * E_INVAL; FOUR_GROUPS has no effect on a step with a request of 32 rows or fewer): */
  PASTA_DECODE_ROW_GROUPS = 512u,
  PASTA_DECODE_FOUR_GROUPS = 1024u,
  /* Two flags for testing the kernels one by one (with dbg_part_ml / dbg_part_acc below): */
  PASTA_DECODE_PARTIALS_ONLY = 64u, /* the attention launch(es) only, no merge: `out` is NOT written */
  PASTA_DECODE_MERGE_ONLY = 128u,   /* the merge launch only, over the partial rows as the buffers hold them
                                       (no attention launch, a deferred append is copied by a launch of its own) */
  PASTA_DECODE_READ_PROBE = 32u /* measurement aid: in place of the attention launch, its read-only
                                  form -- the same grid, the same requests for K and V by the same
                                  waves, no arithmetic -- and no merge: `out` is NOT written.  What a
                                  plain read of the step's bytes costs with this split of the work
                                  (the prof events then time that launch).  A deferred append is
                                  copied by a launch of its own first.  BF16, head_dim 128 only. */
};

/* Maintained lists on the device.  The lists that append_kv keeps per (request, stream) have a copy in the
 * workspace: every range with the running token count, and an index from token number to range.  Appends of up
 * to 32 rows bring the entries they change up to date in their own K1 launch; larger appends, forks and joins
 * mark a stream's copy for a rebuild, done (one stream-ordered copy) by the next decode step that reads it.  A
 * decode step in maintained mode whose plan would not fit the kernel arguments then sends one fixed-size record
 * per stream -- with the stream's newest range, which changes at every append, inline -- and the kernels find
 * ranges and derive the private work items themselves: the bytes a step sends do not grow with the lists, no
 * KV row and no list entry moves at a join (Section 3, "Efficiency").  Small plans ride in the kernel arguments
 * as before (no dependent loads on the way to the first K/V request).                                      */
typedef struct {
  uint32_t struct_size;
  uint32_t flags;               /* PASTA_DECODE_* */
  int32_t layer;
  int32_t n_streams;            /* n >= 1 query tokens, at most max_requests * max_streams
                                   (and at most 65535 per call: E_CAPACITY beyond) */
  const int32_t *request_id;    /* HOST [n] */
  const int32_t *stream_id;     /* HOST [n]; (request, stream) pairs distinct */
  const int32_t *position;      /* HOST [n] or NULL: position id >= 0 of each query token;
                                   used only with PASTA_DECODE_ROPE_Q */
  const int32_t *causal_skip;   /* HOST [n] or NULL.  Several query tokens of ONE stream in one
                                   step (the inserted <async> token together with the fork's
                                   first token; a prompt fed in chunks): maintained mode, the
                                   stream's rows appended first, then one entry per token with
                                   causal_skip[i] = how many of the stream's NEWEST own rows
                                   query i does not see (k-1, ..., 1, 0 for a chunk of k).  With
                                   it, and in explicit mode, (request, stream) pairs may repeat. */
  const int32_t *prefix_len;    /* HOST [n]   (explicit mode) */
  const int32_t *range_offsets; /* HOST [n+1] (explicit mode) or NULL */
  const int32_t *range_start;   /* HOST [range_offsets[n]] */
  const int32_t *range_count;
  const int32_t *range_stride;
  const void *q;                /* DEVICE [n][Hq][D], pool dtype */
  void *out;                    /* DEVICE [n][Hq][D], pool dtype (BF16: round to
                                   nearest even from fp32 accumulators) */
  float *out_lse;               /* DEVICE [n][Hq] or NULL: natural-log sum-exp */
  int64_t *dbg_gather_offsets;  /* HOST [n+1] or NULL: out, CSR over the visited rows */
  int32_t *dbg_gather_rows;     /* DEVICE [sum |Vis(s)|] or NULL: out, the PHYSICAL
                                   row of every visited K row in list order, as
                                   written by the kernels that read them (kv head 0) */
  int64_t *dbg_plan;            /* HOST [8] or NULL: out, launch plan: {prefix tiles,
                                   prefix work-groups, private items, partial rows,
                                   tokens per prefix chunk, common-prefix tokens
                                   summed over requests, metadata bytes, first private
                                   partial row} */
  float *dbg_part_ml;           /* DEVICE [rows][2] fp32 or NULL (both or neither) */
  float *dbg_part_acc;          /* DEVICE [rows][head_dim] fp32 or NULL: when given, the step's split partials live
                                   here instead of in the workspace; rows = dbg_plan[3] of the same call planned with
                                   PASTA_DECODE_PLAN_ONLY.  One row per (split part, query row): m = the part's largest
                                   logit times log2(e) (softmax_scale applied; -inf and l = 0 for a part in which the
                                   row sees nothing), l = sum of 2^(logit log2 e - m), acc = the same weights times V,
                                   not normalised.  Rows of a step over ONE request: the shared-prefix part of (kv head
                                   g, chunk c, stacked query row r = stream index * G + head in group) is row
                                   (g * n_chunks + c) * R + r, with R = n_streams * G and n_chunks = ceil(dbg_plan[5] /
                                   dbg_plan[4]); the private part of (item j, kv head g, head in group i) is row
                                   dbg_plan[7] + (j * Hkv + g) * G + i, the items of a stream being consecutive
                                   128-token pieces of its list beyond the common prefix, stream after stream
                                   (256-token pieces when the step takes the four-groups-per-work-group form,
                                   see PASTA_DECODE_FOUR_GROUPS; a step that reads the device-resident lists cuts the
                                   visible head beyond the common prefix and the range list into pieces separately). */
  void *prof_event_start;       /* hipEvent_t or NULL (both or neither): they receive the start and the */
  void *prof_event_stop;        /* end of the attention-partials kernel's execution (attached to its
                                   dispatch; with PASTA_DECODE_NO_MFMA or F32: recorded on the stream
                                   before and after that launch) */
} pasta_decode_args;

/* Errors: E_INVAL (see above), E_STATE (unknown stream in maintained mode,
 * layer out of range), E_CAPACITY (more ranges than max_ranges, workspace),
 * E_DEVICE.  Validation is complete before anything is enqueued.  Device work
 * is asynchronous on cfg.hip_stream; the call returns without synchronising. */
int32_t pasta_attn_decode_step(pasta_attn *h, const pasta_decode_args *a);

/* The same decode step for callers that cannot allocate: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Identical arguments and results; what differs:
 *   - the split partials (one (m, l, acc[head_dim]) fp32 row per split chunk and query row) go to
 *     a static device array inside the library, PASTA_NOALLOC_SCRATCH_BYTES (16 MiB) per GPU the
 *     library runs on, held until the process ends, instead of the workspace.  A step whose
 *     private items alone need more rows than fit returns E_CAPACITY; shared-prefix chunks are
 *     made longer until the rows fit.  The array keeps the last call's contents, nothing in it
 *     has to start at zero, and ALL handles on one GPU share it: calls that overlap on one GPU
 *     (different streams, different handles) race;
 *   - the call makes no device or pinned-host allocation and grows no host buffer: the handle must
 *     have been set up by an earlier append_kv on the device (else E_STATE), and the step's plan
 *     must be small enough to ride in the kernel arguments (about 3 KB of stream / range / item
 *     records: else E_CAPACITY);
 *   - PASTA_DECODE_PLAN_ONLY and PASTA_DECODE_DENSE_MASK (host staging) are E_INVAL.
 * Other errors as decode_step.                                                 */
#define PASTA_NOALLOC_SCRATCH_BYTES (16u << 20)
int32_t pasta_attn_decode_step_noalloc(pasta_attn *h, const pasta_decode_args *a);

/* Synchronisation (Section 3, Efficiency: a thread that has decoded its sync
 * token waits for its forks; when they are complete the sync token enters the
 * pool and the thread resumes "conditioning on both forks' generations";
 * Figure 2b: the joined threads' last tokens get edges into the sync token).
 * From this call on, stream `stream_id` of `request_id` also sees everything
 * that the streams join_stream[0 .. n_join) see at this moment (their own rows,
 * what they inherited, what they joined earlier).  Host bookkeeping of the
 * maintained lists only: no KV row moves, nothing is enqueued; the caller then
 * appends the sync token's row to `stream_id` as any other row.
 * PASTA_SYNC_RETIRE closes the joined streams afterwards: their ids may be
 * opened again by a later append, their rows stay where they are.  With
 * stream_id == -1 and PASTA_SYNC_RETIRE the listed streams are only closed.
 * Errors: E_INVAL (ids out of range, stream_id among join_stream, duplicates,
 * stream_id == -1 without RETIRE), E_STATE (a stream is not open), E_CAPACITY
 * (max_ranges exceeded), E_NOMEM.  A failing call changes no state.          */
enum { PASTA_SYNC_RETIRE = 1u };

typedef struct {
  uint32_t struct_size;
  uint32_t flags;               /* PASTA_SYNC_* */
  int32_t request_id;
  int32_t stream_id;            /* the stream that waited, or -1 (retire only) */
  int32_t n_join;               /* >= 1 */
  const int32_t *join_stream;   /* HOST [n_join], distinct, open streams */
} pasta_sync_args;

int32_t pasta_attn_sync(pasta_attn *h, const pasta_sync_args *a);

/* Reads the maintained visibility list of one open stream (HOST outputs): what
 * decode_step would use for it in maintained mode.  *prefix_len and *n_ranges
 * are always written; at most `cap` descriptors go to start / count / stride
 * (which may be NULL when cap == 0).
 * Errors: E_INVAL, E_STATE (stream not open).                                */
int32_t pasta_attn_stream_list(pasta_attn *h, int32_t request_id, int32_t stream_id, int32_t *prefix_len,
                               int32_t *n_ranges, int32_t cap, int32_t *start, int32_t *count,
                               int32_t *stride);

/* Trace replay (Section 3, "Interpreter" and "Efficiency"; Figure 2): runs a whole
 * response through append_kv / sync / decode_step the way the interpreter would,
 * from a SYNTHETIC trace of what the main thread emits.  One forward pass feeds one
 * token of every active thread:
 *   TEXT a          a ordinary tokens of the main thread, one per pass.
 *   PROMISE a, b    a promise token; a = the block length the tag predicts (a
 *                   multiple of ten in the paper), b = content tokens the forked
 *                   thread really decodes.  The same pass carries the
 *                   interpreter-inserted <async> token as the fork's first row;
 *                   the fork then feeds its b content tokens and its </async>
 *                   token, one per pass, and ends.
 *   SYNC            the sync token is held back while any spawned thread is alive;
 *                   then the threads are joined (ids retired), the token is fed
 *                   and the main thread goes on.
 * Rows of a pass enter the pool in the order main thread, fork born in this pass,
 * older forks by age.  Forks take the lowest free stream id >= 1; the prompt must be
 * in the pool already as stream 0 of the request.  Position ids: the main thread
 * counts from first_pos; a fork counts on from its promise; the main thread skips
 * the PREDICTED length a after a promise (estimated ids: Section 4, "Training a
 * PASTA-SFT model"; appendix "Positional Embedding").
 * Data is indexed by the order in which rows are fed ("token index" t, the order
 * of the pool slots): k_rows / v_rows [n_layers][max_tokens][Hkv][D], q_rows / out
 * [n_layers][max_tokens][Hq][D], all DEVICE; every pass runs on all n_layers pools.
 * A planning run (PASTA_REPLAY_PLAN_ONLY: no device pointers needed) fills the HOST
 * outputs and leaves the handle unchanged, so that a caller can lay its data out.
 * Errors: as append_kv / sync / decode_step; E_CAPACITY also when the trace feeds
 * more than max_tokens rows or needs more than max_streams threads at once.  A
 * failing real run may have executed some passes.                              */
enum { PASTA_OP_TEXT = 0, PASTA_OP_PROMISE = 1, PASTA_OP_SYNC = 2 };
enum {
  PASTA_REPLAY_PLAN_ONLY = 1u, /* host outputs only; handle state restored */
  PASTA_REPLAY_ROPE = 2u       /* PASTA_APPEND_ROPE / PASTA_DECODE_ROPE_Q with the ids above */
};

typedef struct { int32_t kind, a, b; } pasta_trace_op;

typedef struct {
  uint32_t struct_size;
  uint32_t flags;               /* PASTA_REPLAY_* */
  int32_t request_id;
  int32_t n_ops;
  const pasta_trace_op *ops;    /* HOST [n_ops] */
  int32_t first_pos;            /* position id of the main thread's first fed token */
  int32_t max_tokens;           /* rows the data arrays hold per layer */
  const void *k_rows, *v_rows;  /* DEVICE, see above */
  const void *q_rows;
  void *out;
  int32_t *tok_slot;            /* HOST [max_tokens] or NULL: logical slot of token t */
  int32_t *tok_stream;          /* HOST or NULL: stream id that fed it */
  int32_t *tok_pos;             /* HOST or NULL: its position id */
  int32_t *tok_pass;            /* HOST or NULL: the pass that fed it */
  int64_t *stats;               /* HOST [8] or NULL: {rows fed, passes, most rows in a pass,
                                   forks, syncs, next main position id, 0, 0} */
} pasta_replay_args;

int32_t pasta_attn_replay(pasta_attn *h, const pasta_replay_args *a);

/* Frees host state only; does not synchronise (the caller synchronises before
 * freeing pool / workspace).  NULL is a no-op.                               */
int32_t pasta_attn_destroy(pasta_attn *h);

#ifdef __cplusplus
}
#endif
#endif /* PASTA_ATTN_H */
