// C-ABI library of the multi-stream decode-attention step (include/pasta_attn.h).
// Host side: argument validation, the visibility lists kept per (request, stream)
// (arxiv 2502.11517, Section 3 "Efficiency": ancestor rule of Figure 2b), slot assignment
// at the pool tail (Figure 2c), and the launch plan.  Every step of the arithmetic runs in
// the gfx950 kernels included below.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <unordered_map>
#include <vector>

#include "../../include/pasta_attn.h"
#include "k_append.hpp"
#include "k_attn.hpp"
#include "k_merge.hpp"
#include "k_private.hpp"

using namespace pasta;

namespace {

constexpr uint32_t kMagic = 0x50415354u;  // "PAST"
constexpr int kRing = 8;                  // metadata staging buffers in flight
constexpr int kRelayMaxWords = 2 * kRelayWords;  // largest plan that travels to the device inside kernel arguments
constexpr int kNumCUs = 256;              // MI355X; planning default until the device has been asked
constexpr int kTargetPrefixWgs = 768;     // most shared-prefix work-groups budgeted for

struct Range { int32_t start, count, stride; };

struct StreamState {
  bool open = false;
  int32_t prefix_len = 0;        // visible head [0, prefix_len)
  std::vector<Range> ranges;     // then these, span-ascending
  int64_t range_tokens = 0;      // tokens in `ranges`
  // The copy of the range list that lives on the device (workspace): ranges with running token counts in
  // the arena, and an index "range that holds range token 32 j".  Small appends patch it through the K1
  // launch, everything else (prefill, fork, join, relocation) marks it dirty and it is rebuilt from this
  // mirror at the next decode step that wants it.  The newest range is never relied on: it grows with
  // every append and rides with each call instead.
  int32_t seg_off = -1, seg_cap = 0;    // arena segment (DevRange entries)
  int32_t cseg_off = -1, cseg_cap = 0;  // index segment (int32 entries)
  int32_t dev_ranges = 0;        // arena entries [0, dev_ranges) are exact
  int32_t dev_cidx = 0;          // index entries [0, dev_cidx) are on the device; all later ones lie in the newest range
  bool dirty = true;
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct ListView {  // one stream's visible list for this call
  int32_t prefix_len;
  const Range* ranges;   // maintained mode
  int32_t n_ranges;
  const int32_t *start, *count, *stride;  // explicit mode (ranges == nullptr)
  Range at(int k) const { return ranges ? ranges[k] : Range{start[k], count[k], stride[k]}; }
};



// Host buffers of one decode_step's plan.  They live in the handle and keep their capacity from
// call to call, so that a step in a serving loop touches no allocator; create reserves what a
// plan small enough to ride in the kernel arguments can need.
struct PlanBuf {
  std::vector<ListView> lv;
  std::vector<Range> trim;               // the lists that causal_skip shortens (never grown past its reserve: views point into it)
  std::vector<uint8_t> seen, mask;
  std::vector<int32_t> mask_base, req_idx_of, stream_req_idx, stream_local, req_streams, blob;
  std::vector<DevReq> reqs;
  std::vector<DevStream> streams;
  std::vector<DevRange> ranges;
  std::vector<DevItem> items;
};

}  // namespace

struct pasta_attn {
  uint32_t magic = kMagic;
  pasta_attn_config cfg{};
  int G = 1, elem = 2, page_shift = 31;
  int64_t rows_per_layer = 0, layer_elems = 0, req_capacity = 0;
  Layout lay{};
  std::vector<int32_t> page_table;
  std::vector<int32_t> req_pages;        // paged mode: pages assigned to each request (its capacity)
  std::vector<int64_t> tail;             // per request
  std::vector<int64_t> tail_before;      // tails before the latest layer-0 append
  std::vector<StreamState> streams;      // [max_requests * max_streams]
  // workspace carve-up (byte offsets)
  size_t off_page_table = 0, off_meta = 0, meta_bytes = 0, off_ml = 0, off_acc = 0;
  size_t off_rope = 0, off_qrot = 0, off_krot = 0;  // rope_theta > 0: rotary table (fp64, D/2 entries), rotated Q,
                                                   // rotated K rows of a deferred append
  size_t off_mask = 0, mask_bytes = 0;  // dense-mask comparison mode: one byte per (stream, slot)
  uint8_t* mask_pinned = nullptr;       // its host staging, allocated at first use
  hipEvent_t mask_ev{};
  bool mask_ev_used = false;
  int64_t part_rows_cap = 0;
  // a deferred append (PASTA_APPEND_DEFER): its copy is done by the next decode_step's launch
  struct Pending {
    bool active = false;
    int layer = 0, n_rows = 0;
    const void *k_new = nullptr, *v_new = nullptr;
    int32_t dst_rows[kAppendInline]{};
    bool rope = false;                 // PASTA_APPEND_ROPE: K still to be rotated by pos
    int32_t pos[kAppendInline]{};
    std::vector<int32_t> req_pend0, req_src0;  // per request: first deferred slot, its row in k_new
    std::vector<int32_t> stage_p0, stage_s0, stage_last;  // (their buffers while a call is looked at)
  } pending;
  PlanBuf pb;
  // device-resident lists: carve-up and bump allocation (entries)
  size_t off_arena = 0, off_cidx = 0;
  int64_t arena_cap = 0, cidx_cap = 0, arena_top = 0, cidx_top = 0;
  bool tables_reset = false;             // the segments ran out: start over at the next call (all streams dirty)
  bool lists_in_use = false;             // a decode step has read the device copy: appends keep it current from then on
                                         // (before that they only mark what changed, and may be deferred freely)
  std::vector<DevRange> stage_r;         // staging of one stream's lists for a rebuild
  std::vector<int32_t> stage_c;
  struct Undo { int64_t key; bool open; int32_t prefix_len; int32_t n_ranges; Range last; int64_t range_tokens;
                int32_t dev_ranges, dev_cidx; bool dirty; bool replaced; std::vector<Range> saved; };
  std::vector<Undo> undo;                // append_kv: what to restore if a later row of the call fails
  std::vector<int64_t> t2;
  std::vector<int32_t> dst_rows, slots;
  int tune_prefix_chunk = 0, tune_priv_chunk = 0;  // forced chunk sizes (tokens; 0 = heuristic): set only by -DPASTA_TUNING builds
  // device-side readiness (deferred so that the host logic works without a GPU)
  bool device_ready = false;
  char* pinned = nullptr;                // kRing * meta_bytes
  hipEvent_t ring_ev[kRing]{};
  int ring_ev_made = 0;                  // events created so far (all kRing once the device is ready)
  int device = 0, n_cus = kNumCUs;       // the device current at first use and its compute-unit count
  bool ring_used[kRing]{};
  int ring_next = 0, relay_next = 0;
};

namespace {

int64_t meta_words_cap(const pasta_attn_config& c) {
  // streams + reqs + req_streams + ranges (+1 per stream for the uncommon prefix tail) + items
  const int64_t ns = (int64_t)c.max_requests * c.max_streams;
  const int64_t ranges = (int64_t)c.max_ranges + ns;
  const int64_t cap_tokens = c.page_tokens ? (int64_t)c.pages_per_request * c.page_tokens : c.pool_tokens;
  // items: every stream can split its private list into chunks; bounded by total tokens/chunk + streams
  const int64_t items = ns * ((cap_tokens + kPrivChunk - 1) / kPrivChunk + 1);
  return ns * (int64_t)(sizeof(DevStream) / 4) + (int64_t)c.max_requests * (sizeof(DevReq) / 4) + ns +
         ranges * 4 + std::min<int64_t>(items, (int64_t)1 << 22) * (int64_t)(sizeof(DevItem) / 4) + 64;
}

int validate_cfg(const pasta_attn_config* c) {
  if (!c || c->struct_size != sizeof(pasta_attn_config)) return PASTA_E_INVAL;
  if (c->dtype != PASTA_F32 && c->dtype != PASTA_BF16) return PASTA_E_INVAL;
  if (c->n_q_heads < 1 || c->n_kv_heads < 1 || c->n_q_heads % c->n_kv_heads) return PASTA_E_INVAL;
  const int G = c->n_q_heads / c->n_kv_heads;
  if (G != 1 && G != 2 && G != 4 && G != 8) return PASTA_E_INVAL;
  if (c->head_dim != 64 && c->head_dim != 128) return PASTA_E_INVAL;
  if (c->n_layers < 1 || c->max_requests < 1 || c->max_streams < 1 || c->max_ranges < 1) return PASTA_E_INVAL;
  if (c->kv_layout != PASTA_LAYOUT_TOKEN_MAJOR && c->kv_layout != PASTA_LAYOUT_HEAD_MAJOR) return PASTA_E_INVAL;
  if (!(c->softmax_scale > 0.f) || !std::isfinite(c->softmax_scale)) return PASTA_E_INVAL;
  if (!(c->rope_theta >= 0.f) || !std::isfinite(c->rope_theta) || (c->rope_theta > 0.f && c->rope_theta < 1.f))
    return PASTA_E_INVAL;
  if (c->page_tokens == 0) {
    if (c->pool_tokens < 1) return PASTA_E_INVAL;
    if ((int64_t)c->max_requests * c->pool_tokens >= ((int64_t)1 << 31)) return PASTA_E_INVAL;
  } else {
    if (c->page_tokens < 1 || (c->page_tokens & (c->page_tokens - 1))) return PASTA_E_INVAL;
    if (c->n_phys_pages < 1 || c->pages_per_request < 1) return PASTA_E_INVAL;
    if ((int64_t)c->n_phys_pages * c->page_tokens >= ((int64_t)1 << 31)) return PASTA_E_INVAL;
  }
  return PASTA_OK;
}

// Partial-row budget: enough for the split-K parallelism aimed for at the largest stacked
// row count, plus one row per (private item, query head).
int64_t part_rows_budget(const pasta_attn_config& c) {
  const int64_t ns = (int64_t)c.max_requests * c.max_streams;
  const int64_t cap_tokens = c.page_tokens ? (int64_t)c.pages_per_request * c.page_tokens : c.pool_tokens;
  const int64_t prefix = (int64_t)(kTargetPrefixWgs + c.n_kv_heads * c.max_requests) * c.max_streams *
                         (c.n_q_heads / c.n_kv_heads) * 2;
  const int64_t items = std::min<int64_t>(ns * ((cap_tokens + kPrivChunk - 1) / kPrivChunk + 1),
                                          (int64_t)c.max_requests * cap_tokens / 16 + ns * 2);
  return prefix + items * c.n_q_heads;
}

void carve(pasta_attn* h) {
  const pasta_attn_config& c = h->cfg;
  size_t off = 0;
  h->off_page_table = off;
  off += align_up((size_t)c.max_requests * (c.page_tokens ? c.pages_per_request : 0) * 4 + 4, 256);
  h->meta_bytes = align_up((size_t)meta_words_cap(c) * 4, 256);
  h->off_meta = off;
  off += h->meta_bytes * kRing;
  h->part_rows_cap = part_rows_budget(c);
  h->off_ml = off;
  off += align_up((size_t)h->part_rows_cap * sizeof(float2), 256);
  h->off_acc = off;
  off += align_up((size_t)h->part_rows_cap * c.head_dim * sizeof(float), 256);
  {
    const int64_t cap_tokens = c.page_tokens ? (int64_t)c.pages_per_request * c.page_tokens : c.pool_tokens;
    h->mask_bytes = align_up((size_t)c.max_requests * c.max_streams * (size_t)cap_tokens + 256, 256);
    h->off_mask = off;
    off += h->mask_bytes;
  }
  {  // device-resident lists: room for every range twice over (segments grow by doubling) and for the index
    const int64_t ns = (int64_t)c.max_requests * c.max_streams;
    const int64_t cap_tokens = c.page_tokens ? (int64_t)c.pages_per_request * c.page_tokens : c.pool_tokens;
    h->arena_cap = std::min<int64_t>(4 * ((int64_t)c.max_ranges + ns * 16), (int64_t)1 << 26);
    h->cidx_cap = std::min<int64_t>(2 * (ns * (cap_tokens / kCidxTokens + 16)), (int64_t)1 << 26);
    h->off_arena = off;
    off += align_up((size_t)h->arena_cap * sizeof(DevRange), 256);
    h->off_cidx = off;
    off += align_up((size_t)h->cidx_cap * 4, 256);
  }
  if (c.rope_theta > 0.f) {
    h->off_rope = off;
    off += align_up((size_t)(c.head_dim / 2) * sizeof(double), 256);
    h->off_qrot = off;
    off += align_up((size_t)c.max_requests * c.max_streams * c.n_q_heads * c.head_dim * h->elem, 256);
    h->off_krot = off;
    off += align_up((size_t)kAppendInline * c.n_kv_heads * c.head_dim * h->elem, 256);
  }
  h->cfg.workspace_bytes = off;
}

int ensure_device(pasta_attn* h) {
  if (h->device_ready) return PASTA_OK;
  // every step is skipped on re-entry once it has succeeded, so a failure leaks nothing
  if (!h->pinned && hipHostMalloc((void**)&h->pinned, h->meta_bytes * kRing, hipHostMallocDefault) != hipSuccess) {
    (void)hipGetLastError();
    h->pinned = nullptr;
    return PASTA_E_DEVICE;
  }
  for (; h->ring_ev_made < kRing; ++h->ring_ev_made)
    if (hipEventCreateWithFlags(&h->ring_ev[h->ring_ev_made], hipEventDisableTiming) != hipSuccess) {
      (void)hipGetLastError();
      return PASTA_E_DEVICE;
    }
  int n_cu = 0;
  if (hipGetDevice(&h->device) != hipSuccess ||
      hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, h->device) != hipSuccess || n_cu < 1) {
    (void)hipGetLastError();
    return PASTA_E_DEVICE;
  }
  h->n_cus = n_cu;
  if (h->cfg.page_tokens) {
    if (hipMemcpy((char*)h->cfg.workspace + h->off_page_table, h->page_table.data(),
                  h->page_table.size() * 4, hipMemcpyHostToDevice) != hipSuccess) {
      (void)hipGetLastError();
      return PASTA_E_DEVICE;
    }
  }
  if (h->cfg.rope_theta > 0.f) {  // theta^(-2f/D) / (2 pi) in fp64: angles are taken in revolutions
    const int D = h->cfg.head_dim;
    std::vector<double> tab(D / 2);
    for (int f = 0; f < D / 2; ++f)
      tab[f] = std::pow((double)h->cfg.rope_theta, -2.0 * f / D) / 6.283185307179586476925286766559;
    if (hipMemcpy((char*)h->cfg.workspace + h->off_rope, tab.data(), tab.size() * sizeof(double),
                  hipMemcpyHostToDevice) != hipSuccess) {
      (void)hipGetLastError();
      return PASTA_E_DEVICE;
    }
  }
  h->device_ready = true;
  return PASTA_OK;
}

// Copies `bytes` of host metadata to the next device staging slot, asynchronously on the
// caller's stream; returns the device address.  A slot is reused only after the copy that
// last read its pinned half has completed.
int upload_meta(pasta_attn* h, const void* src, size_t bytes, const int32_t** dev_out) {
  if (bytes > h->meta_bytes) return PASTA_E_CAPACITY;
  const int s = h->ring_next;
  h->ring_next = (s + 1) % kRing;
  if (h->ring_used[s] && hipEventSynchronize(h->ring_ev[s]) != hipSuccess) return PASTA_E_DEVICE;
  char* host = h->pinned + (size_t)s * h->meta_bytes;
  std::memcpy(host, src, bytes);
  char* dev = (char*)h->cfg.workspace + h->off_meta + (size_t)s * h->meta_bytes;
  hipStream_t st = (hipStream_t)h->cfg.hip_stream;
  if (hipMemcpyAsync(dev, host, bytes, hipMemcpyHostToDevice, st) != hipSuccess) return PASTA_E_DEVICE;
  if (hipEventRecord(h->ring_ev[s], st) != hipSuccess) return PASTA_E_DEVICE;
  h->ring_used[s] = true;
  *dev_out = (const int32_t*)dev;
  return PASTA_OK;
}

// Copies host data to a device address in the workspace, asynchronously on the caller's stream, through
// the pinned ring (in pieces of one staging slot).
int upload_to(pasta_attn* h, void* dev_dst, const void* src, size_t bytes) {
  hipStream_t st = (hipStream_t)h->cfg.hip_stream;
  for (size_t lo = 0; lo < bytes; lo += h->meta_bytes) {
    const size_t n = std::min(h->meta_bytes, bytes - lo);
    const int sl = h->ring_next;
    h->ring_next = (sl + 1) % kRing;
    if (h->ring_used[sl] && hipEventSynchronize(h->ring_ev[sl]) != hipSuccess) return PASTA_E_DEVICE;
    char* host = h->pinned + (size_t)sl * h->meta_bytes;
    std::memcpy(host, (const char*)src + lo, n);
    if (hipMemcpyAsync((char*)dev_dst + lo, host, n, hipMemcpyHostToDevice, st) != hipSuccess) return PASTA_E_DEVICE;
    if (hipEventRecord(h->ring_ev[sl], st) != hipSuccess) return PASTA_E_DEVICE;
    h->ring_used[sl] = true;
  }
  return PASTA_OK;
}

constexpr int kNoRoom = 1;  // rebuild_tables: the segments ran out (not an error: the call plans from the host lists)

// Rebuilds the device copy of one stream's range list and range index from the mirror.
int rebuild_tables(pasta_attn* h, StreamState& st) {
  const int64_t n = (int64_t)st.ranges.size();
  const int64_t n_c = (st.range_tokens + kCidxTokens - 1) / kCidxTokens;
  if (n > st.seg_cap) {
    const int64_t cap = std::max<int64_t>(16, 2 * n);
    if (h->arena_top + cap > h->arena_cap) { h->tables_reset = true; return kNoRoom; }
    st.seg_off = (int32_t)h->arena_top;
    st.seg_cap = (int32_t)cap;
    h->arena_top += cap;
  }
  if (n_c > st.cseg_cap) {
    const int64_t cap = std::max<int64_t>(16, 2 * n_c);
    if (h->cidx_top + cap > h->cidx_cap) { h->tables_reset = true; return kNoRoom; }
    st.cseg_off = (int32_t)h->cidx_top;
    st.cseg_cap = (int32_t)cap;
    h->cidx_top += cap;
  }
  std::vector<DevRange>& sr = h->stage_r;
  std::vector<int32_t>& sc = h->stage_c;
  sr.resize((size_t)n);
  sc.resize((size_t)n_c);
  int64_t cum = 0, tok = 0;
  for (int64_t k = 0; k < n; ++k) {
    const Range& g = st.ranges[(size_t)k];
    sr[(size_t)k] = DevRange{g.start, g.count, g.stride, (int32_t)cum};
    for (; tok < cum + g.count; tok += kCidxTokens) sc[(size_t)(tok / kCidxTokens)] = (int32_t)k;
    cum += g.count;
  }
  int rc = PASTA_OK;
  if (n) rc = upload_to(h, (char*)h->cfg.workspace + h->off_arena + (size_t)st.seg_off * sizeof(DevRange), sr.data(), (size_t)n * sizeof(DevRange));
  if (rc == PASTA_OK && n_c) rc = upload_to(h, (char*)h->cfg.workspace + h->off_cidx + (size_t)st.cseg_off * 4, sc.data(), (size_t)n_c * 4);
  if (rc != PASTA_OK) return rc;
  st.dev_ranges = (int32_t)n;
  st.dev_cidx = (int32_t)n_c;
  st.dirty = false;
  return PASTA_OK;
}

inline StreamState& sstate(pasta_attn* h, int req, int sid) {
  return h->streams[(size_t)req * h->cfg.max_streams + sid];
}

// logical slot -> physical row on the host (same formula as the header states)
inline int64_t host_phys(const pasta_attn* h, int req, int64_t slot) {
  if (!h->cfg.page_tokens) return (int64_t)req * h->cfg.pool_tokens + slot;
  const int64_t pp = h->page_table[(size_t)req * h->cfg.pages_per_request + (slot >> h->page_shift)];
  return (pp << h->page_shift) | (slot & (h->cfg.page_tokens - 1));
}

// Adds an owned slot to a stream's list (slots arrive in increasing order).
void add_slot(StreamState& s, int32_t slot) {
  if (s.ranges.empty() && slot == s.prefix_len) { s.prefix_len++; return; }
  s.range_tokens++;
  if (!s.ranges.empty()) {
    Range& r = s.ranges.back();
    if (r.count == 1 && slot > r.start) { r.stride = slot - r.start; r.count = 2; return; }
    if (slot == r.start + (int64_t)r.count * r.stride) { r.count++; return; }
  }
  s.ranges.push_back({slot, 1, 1});
}

template <typename T, int D>
int launch_private_g(int G, dim3 grid, hipStream_t st, const DecodeParams& p) {
  switch (G) {
    case 1: k_private<T, D, 1><<<grid, 256, 0, st>>>(p); break;
    case 2: k_private<T, D, 2><<<grid, 256, 0, st>>>(p); break;
    case 4: k_private<T, D, 4><<<grid, 256, 0, st>>>(p); break;
    case 8: k_private<T, D, 8><<<grid, 256, 0, st>>>(p); break;
    default: return PASTA_E_INVAL;
  }
  return PASTA_OK;
}
template <typename T, int D, int NT>
int launch_merge_nt(int G, dim3 grid, hipStream_t st, const DecodeParams& p) {
  switch (G) {
    case 1: k_merge<T, D, 1, NT><<<grid, NT, 0, st>>>(p); break;
    case 2: k_merge<T, D, 2, NT><<<grid, NT, 0, st>>>(p); break;
    case 4: k_merge<T, D, 4, NT><<<grid, NT, 0, st>>>(p); break;
    case 8: k_merge<T, D, 8, NT><<<grid, NT, 0, st>>>(p); break;
    default: return PASTA_E_INVAL;
  }
  return PASTA_OK;
}
// Width of the merge work-groups: wide for steps with few output rows (a chain of latencies);
// with many rows the launch is bound by the rate at which wavefronts start, so it gets as few
// as the rows' parts can feed: one group of D threads when a row has about a batch of parts.
template <typename T, int D>
int launch_merge_g(int G, dim3 grid, hipStream_t st, const DecodeParams& p, int64_t total_parts) {
  const int64_t rows = (int64_t)grid.x * grid.y * grid.z;
  if (rows < kMergeManyRows) return launch_merge_nt<T, D, kMergeThreads>(G, grid, st, p);
  if (total_parts <= 8 * rows) return launch_merge_nt<T, D, D>(G, grid, st, p);
  return launch_merge_nt<T, D, kMergeThreadsSmall>(G, grid, st, p);
}

int launch_private(const pasta_attn* h, dim3 grid, hipStream_t st, const DecodeParams& p) {
  const int D = h->cfg.head_dim;
  if (h->cfg.dtype == PASTA_F32)
    return D == 64 ? launch_private_g<float, 64>(h->G, grid, st, p) : launch_private_g<float, 128>(h->G, grid, st, p);
  return D == 64 ? launch_private_g<uint16_t, 64>(h->G, grid, st, p)
                 : launch_private_g<uint16_t, 128>(h->G, grid, st, p);
}
// grid = (Hkv, G, n); total_parts = partial rows that the launch reads, over all its output rows
int launch_merge(const pasta_attn* h, dim3 grid, hipStream_t st, const DecodeParams& p, int64_t total_parts) {
  const int D = h->cfg.head_dim;
  if (h->cfg.dtype == PASTA_F32)
    return D == 64 ? launch_merge_g<float, 64>(h->G, grid, st, p, total_parts)
                   : launch_merge_g<float, 128>(h->G, grid, st, p, total_parts);
  return D == 64 ? launch_merge_g<uint16_t, 64>(h->G, grid, st, p, total_parts)
                 : launch_merge_g<uint16_t, 128>(h->G, grid, st, p, total_parts);
}

struct ListPatches {  // entries of the device-resident lists that an append brings up to date
  int n_r = 0, n_c = 0;
  int32_t r_idx[kPatchMax];
  DevRange r_val[kPatchMax];
  int32_t c_idx[kPatchMax];
  int32_t c_val[kPatchMax];
};

int launch_append(pasta_attn* h, int layer, int n_rows, const void* k_new, const void* v_new,
                  const int32_t* dst_rows, const int32_t* positions = nullptr,  // positions: rotate K
                  const ListPatches* patches = nullptr) {
  const pasta_attn_config& c = h->cfg;
  hipStream_t st = (hipStream_t)c.hip_stream;
  AppendParams p{};
  p.arena = (DevRange*)((char*)c.workspace + h->off_arena);
  p.cidx = (int32_t*)((char*)c.workspace + h->off_cidx);
  if (patches) {  // (only with rows that travel in the kernel arguments: one launch)
    p.n_rpatch = patches->n_r;
    p.n_cpatch = patches->n_c;
    std::memcpy(p.rp_idx, patches->r_idx, sizeof(int32_t) * patches->n_r);
    std::memcpy(p.rp_val, patches->r_val, sizeof(DevRange) * patches->n_r);
    std::memcpy(p.cp_idx, patches->c_idx, sizeof(int32_t) * patches->n_c);
    std::memcpy(p.cp_val, patches->c_val, sizeof(int32_t) * patches->n_c);
  }
  p.k = (char*)c.k_pool + (size_t)layer * h->layer_elems * h->elem;
  p.v = (char*)c.v_pool + (size_t)layer * h->layer_elems * h->elem;
  p.lay = h->lay;
  p.Hkv = c.n_kv_heads;
  p.pieces_per_head = c.head_dim * h->elem / 16;
  p.elem_shift = h->elem == 4 ? 2 : 1;
  const size_t row_bytes = (size_t)c.n_kv_heads * c.head_dim * h->elem;
  p.rope_tab = positions ? (const double*)((const char*)c.workspace + h->off_rope) : nullptr;
  p.pos_rows = nullptr;
  if (n_rows <= kAppendInline) {
    p.k_new = (const uint4*)k_new;
    p.v_new = (const uint4*)v_new;
    p.n_rows = n_rows;
    p.dst_rows = nullptr;
    std::memcpy(p.inline_rows, dst_rows, (size_t)n_rows * 4);
    if (positions) std::memcpy(p.inline_pos, positions, (size_t)n_rows * 4);
    const long long total = 2ll * n_rows * c.n_kv_heads * p.pieces_per_head;
    k_append<<<dim3((unsigned)((total + 255) / 256)), 256, 0, st>>>(p);
    return hipGetLastError() == hipSuccess ? PASTA_OK : PASTA_E_DEVICE;
  }
  // large appends (prefill) go in pieces that fit one staging slot
  const size_t per = h->meta_bytes / 4;
  for (size_t lo = 0; lo < (size_t)n_rows; lo += per) {
    const size_t n = std::min(per, (size_t)n_rows - lo);
    const int32_t* dev = nullptr;
    int rc = upload_meta(h, dst_rows + lo, n * 4, &dev);
    if (rc != PASTA_OK) return rc;
    p.dst_rows = dev;
    if (positions) {
      rc = upload_meta(h, positions + lo, n * 4, &dev);
      if (rc != PASTA_OK) return rc;
      p.pos_rows = dev;
    }
    p.n_rows = (int)n;
    p.k_new = (const uint4*)((const char*)k_new + lo * row_bytes);
    p.v_new = (const uint4*)((const char*)v_new + lo * row_bytes);
    const long long total = 2ll * (long long)n * c.n_kv_heads * p.pieces_per_head;
    k_append<<<dim3((unsigned)((total + 255) / 256)), 256, 0, st>>>(p);
    if (hipGetLastError() != hipSuccess) return PASTA_E_DEVICE;
  }
  return PASTA_OK;
}

// Performs a deferred append's copy with K1 (when no decode_step took it along).
int flush_pending(pasta_attn* h) {
  if (!h->pending.active) return PASTA_OK;
  h->pending.active = false;
  return launch_append(h, h->pending.layer, h->pending.n_rows, h->pending.k_new, h->pending.v_new,
                       h->pending.dst_rows, h->pending.rope ? h->pending.pos : nullptr);
}

}  // namespace

// =============================================================================== create
extern "C" int32_t pasta_attn_create(pasta_attn_config* cfg, pasta_attn** out) {
  int rc = validate_cfg(cfg);
  if (rc != PASTA_OK) return rc;
  pasta_attn* h = new (std::nothrow) pasta_attn();
  if (!h) return PASTA_E_NOMEM;
  h->cfg = *cfg;
  h->G = cfg->n_q_heads / cfg->n_kv_heads;
  h->elem = cfg->dtype == PASTA_F32 ? 4 : 2;
  const int64_t D = cfg->head_dim, H = cfg->n_kv_heads;
  if (cfg->page_tokens) {
    h->page_shift = 0;
    while ((1 << h->page_shift) < cfg->page_tokens) h->page_shift++;
    h->rows_per_layer = (int64_t)cfg->n_phys_pages * cfg->page_tokens;
    h->req_capacity = (int64_t)cfg->pages_per_request * cfg->page_tokens;
  } else {
    h->rows_per_layer = (int64_t)cfg->max_requests * cfg->pool_tokens;
    h->req_capacity = cfg->pool_tokens;
  }
  h->layer_elems = h->rows_per_layer * H * D;
  Layout& L = h->lay;
  L.paged = cfg->page_tokens ? 1 : 0;
  L.pages_per_request = cfg->pages_per_request;
  L.pool_tokens = (int)cfg->pool_tokens;
  L.page_shift = cfg->page_tokens ? h->page_shift : 31;
  L.page_mask = cfg->page_tokens ? cfg->page_tokens - 1 : 0x7fffffff;
  if (cfg->kv_layout == PASTA_LAYOUT_TOKEN_MAJOR) {
    L.slot_stride = (int)(H * D);
    L.head_stride = D;
    L.page_stride = cfg->page_tokens ? (int64_t)cfg->page_tokens * H * D : 0;
  } else if (!cfg->page_tokens) {
    L.slot_stride = (int)D;
    L.head_stride = h->rows_per_layer * D;
    L.page_stride = 0;
  } else {
    L.slot_stride = (int)D;
    L.head_stride = (int64_t)cfg->page_tokens * D;
    L.page_stride = (int64_t)cfg->page_tokens * H * D;
  }
  const uint64_t given = cfg->workspace_bytes;
  carve(h);
  if (!out) {  // query mode
    cfg->workspace_bytes = h->cfg.workspace_bytes;
    delete h;
    return PASTA_OK;
  }
  auto fail = [&](int code) { delete h; return code; };
  if (!cfg->k_pool || !cfg->v_pool || !cfg->workspace) return fail(PASTA_E_INVAL);
  if (((uintptr_t)cfg->workspace & 255) || ((uintptr_t)cfg->k_pool & 15) || ((uintptr_t)cfg->v_pool & 15))
    return fail(PASTA_E_INVAL);
  if (given < h->cfg.workspace_bytes) return fail(PASTA_E_CAPACITY);
  h->cfg.workspace_bytes = given;
  if (cfg->page_tokens) {
    if (!cfg->page_table) return fail(PASTA_E_INVAL);
    const size_t n = (size_t)cfg->max_requests * cfg->pages_per_request;
    try {
      h->page_table.assign(cfg->page_table, cfg->page_table + n);
      // a request's assigned pages come first, -1 ("no page") after them; assigned pages must be
      // distinct over the whole table: a page named twice would alias two logical pages
      std::vector<uint8_t> taken((size_t)cfg->n_phys_pages, 0);
      h->req_pages.assign(cfg->max_requests, 0);
      for (int r = 0; r < cfg->max_requests; ++r) {
        bool ended = false;
        for (int k = 0; k < cfg->pages_per_request; ++k) {
          const int32_t pp = h->page_table[(size_t)r * cfg->pages_per_request + k];
          if (pp == -1) { ended = true; continue; }
          if (ended || pp < 0 || pp >= cfg->n_phys_pages || taken[pp]) return fail(PASTA_E_INVAL);
          taken[pp] = 1;
          h->req_pages[r] = k + 1;
        }
      }
    } catch (const std::bad_alloc&) { return fail(PASTA_E_NOMEM); }
    h->cfg.page_table = nullptr;  // the caller's array is not kept
  }
#ifdef PASTA_TUNING  // tuning builds only: forced chunk sizes from the environment
  if (const char* e = std::getenv("PASTA_PREFIX_CHUNK")) h->tune_prefix_chunk = std::atoi(e);
  if (const char* e = std::getenv("PASTA_PRIV_CHUNK")) h->tune_priv_chunk = std::atoi(e);
#endif
  try {
    h->tail.assign(cfg->max_requests, 0);
    h->tail_before.assign(cfg->max_requests, 0);
    h->streams.resize((size_t)cfg->max_requests * cfg->max_streams);
    // plan buffers: what a plan that rides in the kernel arguments can need (larger plans grow them on demand)
    const size_t ns = (size_t)cfg->max_requests * cfg->max_streams, nsc = std::min<size_t>(ns, 65535);
    PlanBuf& pb = h->pb;
    pb.lv.reserve(nsc); pb.mask_base.reserve(nsc); pb.stream_req_idx.reserve(nsc); pb.stream_local.reserve(nsc);
    pb.req_streams.reserve(nsc); pb.streams.reserve(nsc);
    pb.seen.reserve(ns);
    pb.req_idx_of.reserve(cfg->max_requests); pb.reqs.reserve(cfg->max_requests);
    pb.ranges.reserve(std::min<size_t>((size_t)cfg->max_ranges + nsc, kInlineMetaWords));
    pb.items.reserve(kInlineMetaWords / (sizeof(DevItem) / 4));
    pb.blob.reserve(kInlineMetaWords + 16);
  } catch (...) { return fail(PASTA_E_NOMEM); }
#if defined(PASTA_TUNING) && PASTA_TUNING >= 2
  std::fprintf(stderr, "PASTA_CLOCKS byte offset in workspace: %zu\n", h->off_ml + (size_t)(h->part_rows_cap - 16 * PASTA_CLK_WGS) * 8);
#endif
  *out = h;
  return PASTA_OK;
}

extern "C" int32_t pasta_attn_destroy(pasta_attn* h) {
  if (!h) return PASTA_OK;
  if (h->magic != kMagic) return PASTA_E_STATE;
  if (h->device_ready) (void)flush_pending(h);  // a deferred append still owes its copy
  h->magic = 0;
  for (int i = 0; i < h->ring_ev_made; ++i) (void)hipEventDestroy(h->ring_ev[i]);
  if (h->pinned) (void)hipHostFree(h->pinned);
  if (h->mask_pinned) { (void)hipHostFree(h->mask_pinned); (void)hipEventDestroy(h->mask_ev); }
  delete h;
  return PASTA_OK;
}

// =============================================================================== append
extern "C" int32_t pasta_attn_append_kv(pasta_attn* h, const pasta_append_args* a) {
  if (!h || h->magic != kMagic) return PASTA_E_STATE;
  if (!a || a->struct_size != sizeof(pasta_append_args)) return PASTA_E_INVAL;
  const pasta_attn_config& c = h->cfg;
  if (a->layer < 0 || a->layer >= c.n_layers) return PASTA_E_STATE;
  if (a->n_rows < 0) return PASTA_E_INVAL;
  if (a->n_rows == 0) return PASTA_OK;
  const bool reserve_only = a->flags & PASTA_APPEND_RESERVE_ONLY;
  if (!a->request_id || !a->stream_id) return PASTA_E_INVAL;
  if (!reserve_only && (!a->k_new || !a->v_new)) return PASTA_E_INVAL;
  if (!reserve_only && (((uintptr_t)a->k_new & 15) || ((uintptr_t)a->v_new & 15))) return PASTA_E_INVAL;
  const bool rope = a->flags & PASTA_APPEND_ROPE;
  if (rope) {
    if (reserve_only || !a->position || !(c.rope_theta > 0.f)) return PASTA_E_INVAL;
    for (int i = 0; i < a->n_rows; ++i)
      if (a->position[i] < 0) return PASTA_E_INVAL;
  }
  const bool commit = a->layer == 0;  // layer 0 assigns the slots; other layers replay them

  // ---- the rows, one by one, on the live state; what a failing call has to put back is logged
  // (per touched stream: its state at first touch -- an append only ever changes a list's newest range
  // or adds ranges behind it)
  std::vector<int64_t>& t2 = h->t2;
  std::vector<int32_t>&dst_rows = h->dst_rows, &slots = h->slots;
  std::vector<pasta_attn::Undo>& undo = h->undo;
  auto roll_back = [&]() {
    for (size_t u = undo.size(); u-- > 0;) {
      pasta_attn::Undo& e = undo[u];
      StreamState& st = h->streams[(size_t)e.key];
      if (e.replaced) st.ranges = std::move(e.saved);
      st.ranges.resize((size_t)e.n_ranges);
      if (e.n_ranges) st.ranges.back() = e.last;
      st.open = e.open; st.prefix_len = e.prefix_len; st.range_tokens = e.range_tokens;
      st.dev_ranges = e.dev_ranges; st.dev_cidx = e.dev_cidx; st.dirty = e.dirty;
    }
    undo.clear();
  };
  try {
    t2 = commit ? h->tail : h->tail_before;
    dst_rows.resize(a->n_rows);
    slots.resize(a->n_rows);
    undo.clear();
    auto touch = [&](int req, int sid) -> StreamState& {  // logs the stream's state the first time it is touched
      const int64_t key = (int64_t)req * c.max_streams + sid;
      StreamState& st = h->streams[(size_t)key];
      for (const auto& e : undo)
        if (e.key == key) return st;
      pasta_attn::Undo e{};
      e.key = key; e.open = st.open; e.prefix_len = st.prefix_len; e.n_ranges = (int32_t)st.ranges.size();
      if (e.n_ranges) e.last = st.ranges.back();
      e.range_tokens = st.range_tokens; e.dev_ranges = st.dev_ranges; e.dev_cidx = st.dev_cidx; e.dirty = st.dirty;
      undo.push_back(std::move(e));
      return st;
    };
    auto fail = [&](int code) { roll_back(); return code; };
    for (int i = 0; i < a->n_rows; ++i) {
      const int r = a->request_id[i], s = a->stream_id[i];
      const int par = a->parent_stream ? a->parent_stream[i] : -1;
      if (r < 0 || r >= c.max_requests || s < 0 || s >= c.max_streams) return fail(PASTA_E_INVAL);
      if (par < -1 || par >= c.max_streams || par == s) return fail(PASTA_E_INVAL);
      const int64_t slot = t2[r];
      if (slot >= (c.page_tokens ? (int64_t)h->req_pages[r] << h->page_shift : h->req_capacity)) return fail(PASTA_E_CAPACITY);
      if (!commit) {  // replay: same slots as the layer-0 call, lists untouched
        if (slot >= h->tail[r]) return fail(PASTA_E_STATE);
        slots[i] = (int32_t)slot;
        dst_rows[i] = (int32_t)host_phys(h, r, slot);
        t2[r] = slot + 1;
        continue;
      }
      StreamState& st = touch(r, s);
      if (par >= 0 || !st.open) {  // the row opens the stream: as a fork of `par`, or as a root (empty visible set)
        if (par >= 0 && st.open) return fail(PASTA_E_INVAL);  // parent only on the row that opens the stream
        const StreamState* ps = nullptr;
        if (par >= 0) {
          ps = &sstate(h, r, par);
          if (!ps->open) return fail(PASTA_E_INVAL);
        }
        pasta_attn::Undo* ue = nullptr;
        for (auto& e : undo)
          if (e.key == (int64_t)r * c.max_streams + s) ue = &e;
        if (!ue->replaced) { ue->replaced = true; ue->saved = std::move(st.ranges); st.ranges.clear(); }
        if (ps) {  // ancestor rule: inherit what the parent sees now
          st.prefix_len = ps->prefix_len;
          st.ranges = ps->ranges;
          st.range_tokens = ps->range_tokens;
        } else {
          st.prefix_len = 0;
          st.ranges.clear();
          st.range_tokens = 0;
        }
        st.open = true;
        st.dirty = true;  // the device copy is rebuilt from the mirror when a decode step wants it
        st.dev_ranges = st.dev_cidx = 0;
      }
      add_slot(st, (int32_t)slot);
      if ((int64_t)st.ranges.size() > c.max_ranges) return fail(PASTA_E_CAPACITY);
      slots[i] = (int32_t)slot;
      dst_rows[i] = (int32_t)host_phys(h, r, slot);
      t2[r] = slot + 1;
    }
  } catch (...) { roll_back(); return PASTA_E_NOMEM; }

  // ---- what the call changes in the device-resident lists.  A stream whose ranges only GREW needs
  // nothing (its newest range rides with every decode call, and index entries that are not on the device
  // mean "the newest range").  A stream that got NEW ranges has its arena and index entries brought up to
  // date by this call's K1 launch when they are few and the launch exists; otherwise its copy is marked
  // for a rebuild.
  ListPatches patches;
  bool need_k1 = false;  // patches exist: the copy cannot be left to a later decode launch
  if (commit) {
    const bool k1_possible = !reserve_only && a->n_rows <= kAppendInline;
    for (auto& e : undo) {
      StreamState& st = h->streams[(size_t)e.key];
      const int32_t nb = e.n_ranges, na = (int32_t)st.ranges.size();
      if (st.dirty) continue;
      if (!h->lists_in_use) {  // no step has read the device copy so far: nothing to keep current
        if (na != nb) st.dirty = true;
        continue;
      }
      if (na == nb) {  // growth only
        st.dev_ranges = std::min(st.dev_ranges, std::max(na - 1, 0));
        continue;
      }
      const int64_t n_cidx = (st.range_tokens + kCidxTokens - 1) / kCidxTokens;
      const int32_t k0 = std::min(st.dev_ranges, std::max(nb - 1, 0));  // first arena entry to (re)write
      const int64_t want_r = na - k0, want_c = n_cidx - st.dev_cidx;
      if (!k1_possible || na > st.seg_cap || n_cidx > st.cseg_cap || patches.n_r + want_r > kPatchMax ||
          patches.n_c + want_c > kPatchMax) {
        st.dirty = true;
        continue;
      }
      int64_t cum = st.range_tokens;  // tokens before range k, walking down from the end
      for (int32_t k = na - 1; k >= k0; --k) cum -= st.ranges[k].count;
      int64_t tok = (int64_t)st.dev_cidx * kCidxTokens;  // next index entry's token (lies at or behind range k0's start)
      for (int32_t k = k0; k < na; ++k) {
        const Range& g = st.ranges[k];
        patches.r_idx[patches.n_r] = st.seg_off + k;
        patches.r_val[patches.n_r++] = DevRange{g.start, g.count, g.stride, (int32_t)cum};
        for (; tok < cum + g.count && tok < st.range_tokens; tok += kCidxTokens) {
          patches.c_idx[patches.n_c] = st.cseg_off + (int32_t)(tok / kCidxTokens);
          patches.c_val[patches.n_c++] = k;
        }
        cum += g.count;
      }
      st.dev_ranges = na;
      st.dev_cidx = (int32_t)n_cidx;
      need_k1 = true;
    }
  }

  // ---- enqueue K1, or leave the copy to the next decode_step (PASTA_APPEND_DEFER)
  int rc = PASTA_OK;
  auto fail_dev = [&](int code) { if (commit) roll_back(); return code; };
  // At most one deferred append is outstanding, and the slots it covers are the newest of their
  // requests: any later append -- also one that only reserves slots for the caller's own kernel --
  // first sends the deferred rows to the pool (a deferred append exists only on a ready device).
  rc = flush_pending(h);
  if (rc != PASTA_OK) return fail_dev(rc);
  if (!reserve_only) {
    rc = ensure_device(h);
    if (rc != PASTA_OK) return fail_dev(rc);
    bool defer = (a->flags & PASTA_APPEND_DEFER) && a->n_rows <= kAppendInline && !need_k1;
    std::vector<int32_t>&p0 = h->pending.stage_p0, &s0 = h->pending.stage_s0;
    if (defer) {  // rows of one request must be consecutive in the call: slot t <-> row src0 + (t - pend0)
      p0.assign(c.max_requests, INT32_MAX);
      s0.assign(c.max_requests, 0);
      std::vector<int32_t>& last = h->pending.stage_last;
      last.assign(c.max_requests, -2);
      for (int i = 0; i < a->n_rows && defer; ++i) {
        const int r = a->request_id[i];
        if (p0[r] == INT32_MAX) { p0[r] = slots[i]; s0[r] = i; }
        else if (last[r] != i - 1) defer = false;
        last[r] = i;
      }
    }
    if (defer) {
      pasta_attn::Pending& pd = h->pending;
      pd.active = true;
      pd.layer = a->layer;
      pd.n_rows = a->n_rows;
      pd.k_new = a->k_new;
      pd.v_new = a->v_new;
      std::memcpy(pd.dst_rows, dst_rows.data(), (size_t)a->n_rows * 4);
      pd.rope = rope;
      if (rope) std::memcpy(pd.pos, a->position, (size_t)a->n_rows * 4);
      pd.req_pend0.swap(p0);
      pd.req_src0.swap(s0);
    } else {
      rc = launch_append(h, a->layer, a->n_rows, a->k_new, a->v_new, dst_rows.data(), rope ? a->position : nullptr,
                         need_k1 ? &patches : nullptr);
      if (rc != PASTA_OK) return fail_dev(rc);
    }
  }

  // ---- commit
  if (a->out_slot) std::memcpy(a->out_slot, slots.data(), (size_t)a->n_rows * 4);
  if (commit) {
    h->tail_before = h->tail;
    h->tail.swap(t2);
    undo.clear();
  }
  return PASTA_OK;
}

// =============================================================================== sync
// Union of visible sets, rebuilt slot by slot in ascending order so that the result is in the
// same canonical form as a list grown by appends (contiguous head in prefix_len, then strided
// descriptors).  Host work proportional to the number of visible slots; a sync is rare.
extern "C" int32_t pasta_attn_sync(pasta_attn* h, const pasta_sync_args* a) {
  if (!h || h->magic != kMagic) return PASTA_E_STATE;
  if (!a || a->struct_size != sizeof(pasta_sync_args)) return PASTA_E_INVAL;
  const pasta_attn_config& c = h->cfg;
  const bool retire = a->flags & PASTA_SYNC_RETIRE;
  if (a->request_id < 0 || a->request_id >= c.max_requests) return PASTA_E_INVAL;
  if (a->n_join < 1 || !a->join_stream) return PASTA_E_INVAL;
  if (a->stream_id < -1 || a->stream_id >= c.max_streams || (a->stream_id == -1 && !retire)) return PASTA_E_INVAL;
  for (int i = 0; i < a->n_join; ++i) {
    const int j = a->join_stream[i];
    if (j < 0 || j >= c.max_streams || j == a->stream_id) return PASTA_E_INVAL;
    for (int k = 0; k < i; ++k)
      if (a->join_stream[k] == j) return PASTA_E_INVAL;
    if (!sstate(h, a->request_id, j).open) return PASTA_E_STATE;
  }
  try {
    if (a->stream_id >= 0) {
      StreamState& dst = sstate(h, a->request_id, a->stream_id);
      if (!dst.open) return PASTA_E_STATE;
      // k-way merge of the lists' slots (each list ascending), duplicates dropped
      struct Cursor { const StreamState* s; int64_t next; size_t ri; int32_t k; };  // next < prefix_len: in the head
      std::vector<Cursor> cur;
      cur.push_back({&dst, 0, 0, 0});
      for (int i = 0; i < a->n_join; ++i) cur.push_back({&sstate(h, a->request_id, a->join_stream[i]), 0, 0, 0});
      auto peek = [](const Cursor& q) -> int64_t {
        if (q.next < q.s->prefix_len) return q.next;
        if (q.ri < q.s->ranges.size()) return (int64_t)q.s->ranges[q.ri].start + (int64_t)q.k * q.s->ranges[q.ri].stride;
        return INT64_MAX;
      };
      auto advance = [](Cursor& q) {
        if (q.next < q.s->prefix_len) { q.next++; return; }
        if (++q.k >= q.s->ranges[q.ri].count) { q.k = 0; q.ri++; }
      };
      // the common head [0, min prefix_len) needs no merging
      int64_t head = INT64_MAX;
      for (auto& q : cur) head = std::min<int64_t>(head, q.s->prefix_len);
      StreamState merged;
      merged.open = true;
      merged.prefix_len = (int32_t)head;
      for (auto& q : cur) q.next = head;
      for (;;) {
        int64_t lo = INT64_MAX;
        for (auto& q : cur) lo = std::min(lo, peek(q));
        if (lo == INT64_MAX) break;
        add_slot(merged, (int32_t)lo);
        for (auto& q : cur)
          if (peek(q) == lo) advance(q);
        if ((int64_t)merged.ranges.size() > c.max_ranges) return PASTA_E_CAPACITY;
      }
      merged.range_tokens = 0;
      for (const Range& g : merged.ranges) merged.range_tokens += g.count;
      merged.seg_off = dst.seg_off; merged.seg_cap = dst.seg_cap;      // the device copy keeps its segments
      merged.cseg_off = dst.cseg_off; merged.cseg_cap = dst.cseg_cap;  // and is rebuilt from the joined list
      dst = std::move(merged);                                         // when a decode step next wants it
    }
    if (retire)
      for (int i = 0; i < a->n_join; ++i) {
        StreamState& js = sstate(h, a->request_id, a->join_stream[i]);
        js.open = false;
        js.prefix_len = 0;
        js.ranges.clear();
        js.range_tokens = 0;
        js.dirty = true;
        js.dev_ranges = js.dev_cidx = 0;
      }
  } catch (const std::bad_alloc&) {
    return PASTA_E_NOMEM;
  }
  return PASTA_OK;
}

extern "C" int32_t pasta_attn_stream_list(pasta_attn* h, int32_t request_id, int32_t stream_id, int32_t* prefix_len,
                                          int32_t* n_ranges, int32_t cap, int32_t* start, int32_t* count,
                                          int32_t* stride) {
  if (!h || h->magic != kMagic) return PASTA_E_STATE;
  const pasta_attn_config& c = h->cfg;
  if (request_id < 0 || request_id >= c.max_requests || stream_id < 0 || stream_id >= c.max_streams) return PASTA_E_INVAL;
  if (!prefix_len || !n_ranges || cap < 0 || (cap > 0 && (!start || !count || !stride))) return PASTA_E_INVAL;
  const StreamState& s = sstate(h, request_id, stream_id);
  if (!s.open) return PASTA_E_STATE;
  *prefix_len = s.prefix_len;
  *n_ranges = (int32_t)s.ranges.size();
  for (int32_t k = 0; k < cap && k < (int32_t)s.ranges.size(); ++k) {
    start[k] = s.ranges[k].start;
    count[k] = s.ranges[k].count;
    stride[k] = s.ranges[k].stride;
  }
  return PASTA_OK;
}

// =============================================================================== decode
namespace {

// The scratch of the entry point that allocates nothing: partial (m, l) and accumulator rows of one
// decode step.  One array per GPU that the library runs on, held until the process ends; host code
// reaches it only through the address that hipGetSymbolAddress returns for the current device.
constexpr size_t kScratchBytes = (size_t)16 << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
void* g_scratch_ptr[kMaxDevices] = {};

// `no_alloc`: the partials go to the static scratch array instead of the workspace, and the call
// must get by without any allocation, device or host (see pasta_attn_decode_step_noalloc).
int32_t decode_impl(pasta_attn* h, const pasta_decode_args* a, const bool no_alloc) {
  if (!h || h->magic != kMagic) return PASTA_E_STATE;
  if (!a || a->struct_size != sizeof(pasta_decode_args)) return PASTA_E_INVAL;
  const pasta_attn_config& c = h->cfg;
  if (a->layer < 0 || a->layer >= c.n_layers) return PASTA_E_STATE;
  const int n = a->n_streams;
  if (n < 1 || n > c.max_requests * c.max_streams) return PASTA_E_INVAL;
  if (n > 65535) return PASTA_E_CAPACITY;  // one grid dimension of the merge launch counts the query rows
  if (!a->request_id || !a->stream_id) return PASTA_E_INVAL;
  const bool plan_only = a->flags & PASTA_DECODE_PLAN_ONLY;
  if (!plan_only && (!a->q || !a->out)) return PASTA_E_INVAL;
  if (!plan_only && (((uintptr_t)a->q & 15) || ((uintptr_t)a->out & 3))) return PASTA_E_INVAL;
  const bool rope_q = a->flags & PASTA_DECODE_ROPE_Q;
  if (rope_q) {
    if (!a->position || !(c.rope_theta > 0.f)) return PASTA_E_INVAL;
    for (int i = 0; i < n; ++i)
      if (a->position[i] < 0) return PASTA_E_INVAL;
  }
  const bool explicit_mode = a->range_offsets != nullptr;
  if (explicit_mode && !a->prefix_len) return PASTA_E_INVAL;
  if (explicit_mode && a->causal_skip) return PASTA_E_INVAL;  // the lists say it all there
  const bool no_share = a->flags & (PASTA_DECODE_NO_SHARE | PASTA_DECODE_DENSE_MASK);
  const bool dense = a->flags & PASTA_DECODE_DENSE_MASK;
  const bool probe = a->flags & PASTA_DECODE_READ_PROBE;
  const bool partials_only = a->flags & PASTA_DECODE_PARTIALS_ONLY, merge_only = a->flags & PASTA_DECODE_MERGE_ONLY;
  if ((partials_only && merge_only) || ((partials_only || merge_only) && probe)) return PASTA_E_INVAL;
  if ((a->dbg_part_ml == nullptr) != (a->dbg_part_acc == nullptr)) return PASTA_E_INVAL;
  if (a->dbg_part_ml && (no_alloc || ((uintptr_t)a->dbg_part_ml & 7) || ((uintptr_t)a->dbg_part_acc & 15))) return PASTA_E_INVAL;
  if (probe && (dense || no_alloc || (a->flags & PASTA_DECODE_NO_MFMA))) return PASTA_E_INVAL;
  if (dense && (c.dtype != PASTA_BF16 || c.head_dim != 128 || (a->flags & PASTA_DECODE_NO_MFMA))) return PASTA_E_INVAL;
  const int G = h->G, D = c.head_dim, Hkv = c.n_kv_heads;
  float2* part_ml = nullptr;   // where this call's partials go
  float* part_acc = nullptr;
  int64_t part_rows_cap = h->part_rows_cap;
  if (no_alloc) {
    // nothing here may allocate: the handle must have been through its set-up (any append_kv does
    // that), the plan must fit the kernel arguments, and the comparison mode with its host staging is out
    if (plan_only || dense) return PASTA_E_INVAL;
    if (!h->device_ready) return PASTA_E_STATE;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { (void)hipGetLastError(); return PASTA_E_DEVICE; }
    if (!g_scratch_ptr[dev]) {  // once per device, with that device current
      void* ptr = nullptr;
      if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) { (void)hipGetLastError(); return PASTA_E_DEVICE; }
      g_scratch_ptr[dev] = ptr;
    }
    part_rows_cap = (int64_t)(kScratchBytes / (sizeof(float2) + (size_t)D * sizeof(float)));
    part_ml = (float2*)g_scratch_ptr[dev];
    part_acc = (float*)((char*)g_scratch_ptr[dev] + align_up((size_t)part_rows_cap * sizeof(float2), 256));
    part_rows_cap -= 64;  // (the alignment gap between the two arrays)
  } else if (!plan_only) {  // before planning: the plan is sized to the device's compute-unit count
    const int rc0 = ensure_device(h);
    if (rc0 != PASTA_OK) return rc0;
    part_ml = (float2*)((char*)c.workspace + h->off_ml);
    part_acc = (float*)((char*)c.workspace + h->off_acc);
    if (a->dbg_part_ml) { part_ml = (float2*)a->dbg_part_ml; part_acc = a->dbg_part_acc; }
  }
  // a buffer of the plan may grow only where allocation is allowed
  auto room = [&](const auto& v, size_t want) { return !no_alloc || want <= v.capacity(); };

  try {
    // ---- lists + validation
    PlanBuf& pb = h->pb;
    if (!room(pb.lv, n) || !room(pb.mask_base, n) || !room(pb.stream_req_idx, n) || !room(pb.streams, n)) return PASTA_E_CAPACITY;
    std::vector<ListView>& lv = pb.lv;
    lv.resize(n);
    std::vector<Range>& trim = pb.trim;    // storage of the views that causal_skip shortens (stable: never past its reserve)
    trim.clear();
    if (a->causal_skip && trim.capacity() < (size_t)c.max_ranges) {
      if (no_alloc) return PASTA_E_CAPACITY;
      trim.reserve((size_t)c.max_ranges);
    }
    std::vector<uint8_t>& seen = pb.seen;
    seen.assign((size_t)c.max_requests * c.max_streams, 0);  // (reserved at create)
    int64_t total_ranges = 0;
    for (int i = 0; i < n; ++i) {
      const int r = a->request_id[i], s = a->stream_id[i];
      if (r < 0 || r >= c.max_requests || s < 0 || s >= c.max_streams) return PASTA_E_INVAL;
      uint8_t& sn = seen[(size_t)r * c.max_streams + s];
      if (sn && !explicit_mode && !a->causal_skip) return PASTA_E_INVAL;  // one query token per stream, unless said otherwise
      sn = 1;
      ListView& v = lv[i];
      if (explicit_mode) {
        const int32_t r0 = a->range_offsets[i], r1 = a->range_offsets[i + 1];
        if (r0 < 0 || r1 < r0 || (i == 0 && r0 != 0)) return PASTA_E_INVAL;
        if (r1 > r0 && (!a->range_start || !a->range_count || !a->range_stride)) return PASTA_E_INVAL;
        v = ListView{a->prefix_len[i], nullptr, r1 - r0, a->range_start + r0, a->range_count + r0,
                     a->range_stride + r0};
        const int64_t tail = h->tail[r];
        if (v.prefix_len < 0 || v.prefix_len > tail) return PASTA_E_INVAL;
        int64_t last = (int64_t)v.prefix_len - 1;
        for (int k = 0; k < v.n_ranges; ++k) {
          const Range g = v.at(k);
          if (g.count < 1 || g.stride < 1 || g.start <= last) return PASTA_E_INVAL;
          last = (int64_t)g.start + (int64_t)(g.count - 1) * g.stride;
          if (last >= tail) return PASTA_E_INVAL;
        }
        if (v.prefix_len == 0 && v.n_ranges == 0) return PASTA_E_INVAL;
      } else {
        const StreamState& ss = sstate(h, r, s);
        if (!ss.open) return PASTA_E_STATE;
        v = ListView{ss.prefix_len, ss.ranges.data(), (int32_t)ss.ranges.size(), nullptr, nullptr, nullptr};
        const int skip = a->causal_skip ? a->causal_skip[i] : 0;
        if (skip < 0) return PASTA_E_INVAL;
        if (skip > 0) {  // a view without the stream's `skip` newest rows: they are the largest slots of its list
          if (trim.size() + ss.ranges.size() > (size_t)c.max_ranges) return PASTA_E_CAPACITY;
          const size_t t0 = trim.size();
          trim.insert(trim.end(), ss.ranges.begin(), ss.ranges.end());
          int left = skip;
          while (left > 0 && trim.size() > t0) {
            const int take = std::min(left, trim.back().count);
            trim.back().count -= take;
            left -= take;
            if (trim.back().count == 0) trim.pop_back();
          }
          if (left > ss.prefix_len) return PASTA_E_INVAL;
          v = ListView{ss.prefix_len - left, trim.data() + t0, (int32_t)(trim.size() - t0), nullptr, nullptr, nullptr};
        }
        if (v.prefix_len == 0 && v.n_ranges == 0) return PASTA_E_INVAL;
      }
      total_ranges += v.n_ranges;
    }
    if (total_ranges > c.max_ranges) return PASTA_E_CAPACITY;

    // ---- dense-mask comparison mode: the lists become one 0/1 byte per (stream, slot), and every
    // stream's list becomes "all slots of its request"
    std::vector<uint8_t>& mask = pb.mask;
    std::vector<int32_t>& mask_base = pb.mask_base;
    mask_base.assign(n, 0);
    if (dense) {
      size_t total = 0;
      for (int i = 0; i < n; ++i) {
        mask_base[i] = (int32_t)total;
        total += (size_t)h->tail[a->request_id[i]];
      }
      if (total + 256 > h->mask_bytes) return PASTA_E_CAPACITY;
      mask.assign(total + 256, 0);
      for (int i = 0; i < n; ++i) {
        uint8_t* m = mask.data() + mask_base[i];
        std::memset(m, 1, (size_t)lv[i].prefix_len);
        for (int k = 0; k < lv[i].n_ranges; ++k) {
          const Range g = lv[i].at(k);
          for (int j = 0; j < g.count; ++j) m[(int64_t)g.start + (int64_t)j * g.stride] = 1;
        }
        lv[i] = ListView{(int32_t)h->tail[a->request_id[i]], nullptr, 0, nullptr, nullptr, nullptr};
      }
      total_ranges = 0;
    }

    // ---- group by request (order of first appearance)
    std::vector<int32_t>& req_idx_of = pb.req_idx_of;
    req_idx_of.assign(c.max_requests, -1);  // (reserved at create, as is reqs)
    std::vector<DevReq>& reqs = pb.reqs;
    reqs.clear();
    std::vector<int32_t>&stream_req_idx = pb.stream_req_idx, &stream_local = pb.stream_local;
    stream_req_idx.resize(n);
    stream_local.resize(n);
    for (int i = 0; i < n; ++i) {
      const int r = a->request_id[i];
      if (req_idx_of[r] < 0) {
        req_idx_of[r] = (int32_t)reqs.size();
        DevReq q{};
        q.req = r;
        q.pc = INT32_MAX;
        q.pend0 = INT32_MAX;
        reqs.push_back(q);
      }
      DevReq& q = reqs[req_idx_of[r]];
      stream_req_idx[i] = req_idx_of[r];
      stream_local[i] = q.n_streams++;
      q.pc = std::min(q.pc, lv[i].prefix_len);
    }
    std::vector<int32_t>& req_streams = pb.req_streams;
    req_streams.resize(n);
    {
      int32_t pos = 0;
      for (auto& q : reqs) { q.stream0 = pos; pos += q.n_streams; }
      for (int i = 0; i < n; ++i) req_streams[reqs[stream_req_idx[i]].stream0 + stream_local[i]] = i;
    }

    // ---- shared-prefix plan: only what the matrix-core kernel takes; the rest is private
    // (the matrix-core kernel addresses a layer's pool and the query rows with 32-bit byte offsets)
    const bool mfma = c.dtype == PASTA_BF16 && !(a->flags & PASTA_DECODE_NO_MFMA) && attn_kernel_supports(D, G) &&
                      h->layer_elems * h->elem < ((int64_t)1 << 32) - 65536 &&
                      (int64_t)n * c.n_q_heads * D * h->elem < ((int64_t)1 << 31);
    if ((dense || probe) && !mfma) return PASTA_E_INVAL;  // the mask and the read-only form belong to the matrix-core kernel
    int64_t pc_total = 0, pc_weighted = 0;  // the second counts a prefix once per work-group that reads it
    for (auto& q : reqs) {
      if (!mfma || q.pc < kTile || no_share) q.pc = 0;
      pc_total += q.pc;
    }
    // More than 32 stacked rows per request: the rows go in groups of 32.  When EVERY request with a
    // shared prefix is that wide, the launch may take the form whose work-groups serve four row groups
    // each (one per wave, over shared tiles); otherwise each row group is a work-group of its own.
    // The wide form pays where its waves are busy and its pipeline gets going -- every such request
    // keeps three of four waves computing on average, and a chunk is four rounds or more -- and loses
    // a few per cent elsewhere (measured on 12 to 32 streams over prefixes of 8k and 32k tokens); the
    // caller may force either form.
    bool wide = mfma && !dense && pc_total > 0 && !(a->flags & PASTA_DECODE_ROW_GROUPS);
    const bool force_wide = a->flags & PASTA_DECODE_FOUR_GROUPS;
    if ((a->flags & PASTA_DECODE_ROW_GROUPS) && force_wide) return PASTA_E_INVAL;
    for (auto& q : reqs) {
      if (q.pc <= 0) continue;
      const int R_all = q.n_streams * G;
      if (R_all <= 32) wide = false;
      const int n_rg = (R_all + 31) / 32, n_quads = (n_rg + 3) / 4;
      if (!force_wide && n_rg < 3 * n_quads) wide = false;  // on average fewer than three of a work-group's four waves would compute
    }
    auto row_units = [&](const DevReq& q) -> int64_t {  // shared-prefix work-groups per (chunk, kv head)
      const int64_t n_rg = (q.n_streams * G + 31) / 32;
      return wide ? (n_rg + 3) / 4 : n_rg;
    };
    if (wide && !force_wide) {  // the chunk the wide form would get: at least four rounds of four 32-token blocks?
      int64_t pw = 0;
      for (auto& q : reqs) pw += (int64_t)q.pc * row_units(q);
      if (pw * Hkv / h->n_cus < 4 * 4 * 32) wide = false;
    }
    for (auto& q : reqs) pc_weighted += (int64_t)q.pc * row_units(q);
    // Chunking.  Every chunk costs one partial row per stacked query row (written here, read
    // by the merge), so chunks should be long; but the step wants at least one shared-prefix
    // work-group per CU to keep enough loads in flight.  Tokens per chunk = the largest
    // multiple of the 64-token tile that still gives kNumCUs prefix work-groups.  Private
    // items stay at 128 tokens: they are few and their rows are scattered.
    int64_t priv_chunk = kPrivChunk, chunk_tokens = kTile;
    if (mfma) {
      chunk_tokens = std::max<int64_t>(kTile, pc_weighted * Hkv / h->n_cus / kTile * kTile);
      priv_chunk = wide ? 256 : 128;  // (beside the long wide work-groups the private items get one slot per CU: longer items keep more in flight there)
      if (h->tune_prefix_chunk >= kTile) chunk_tokens = h->tune_prefix_chunk / kTile * kTile;
      if (h->tune_priv_chunk >= 32) priv_chunk = std::min<int64_t>(h->tune_priv_chunk / 32 * 32, kGatherMax);  // whole 32-token blocks
    }
    // ---- where the lists come from.  Maintained lists have a copy on the device (range arena + range
    // index, kept up to date by the appends): a step may then send a fixed-size record per stream and let
    // the kernels derive the private work items, instead of sending every range and item.  A plan small
    // enough to ride in the kernel arguments is sent whole all the same -- its items then cost the
    // kernels no dependent loads -- unless the caller asks for the device lists.
    bool dev_lists = false;
    if (!explicit_mode && !a->causal_skip && !dense) {
      int64_t words = (int64_t)n * (sizeof(DevStream) / 4 + 1) + (int64_t)reqs.size() * (sizeof(DevReq) / 4) + 8;
      for (int i = 0; i < n; ++i) {
        const StreamState& ss = sstate(h, a->request_id[i], a->stream_id[i]);
        const int64_t priv = (int64_t)lv[i].prefix_len - reqs[stream_req_idx[i]].pc + ss.range_tokens;
        words += ((int64_t)lv[i].n_ranges + 1) * 4 + (priv + priv_chunk - 1) / priv_chunk * (sizeof(DevItem) / 4);
      }
      dev_lists = (a->flags & PASTA_DECODE_DEVICE_LISTS) || words > kInlineMetaWords;
    } else if (a->flags & PASTA_DECODE_DEVICE_LISTS) {
      return PASTA_E_INVAL;
    }
    if (dev_lists && !plan_only) {  // the copies this step reads must be current (all but each list's newest range)
      if (h->tables_reset) {        // the segments ran out earlier: start over
        h->tables_reset = false;
        h->arena_top = h->cidx_top = 0;
        for (StreamState& ss : h->streams) { ss.seg_off = ss.cseg_off = -1; ss.seg_cap = ss.cseg_cap = 0; ss.dirty = true; }
      }
      for (int i = 0; i < n && dev_lists; ++i) {
        StreamState& ss = sstate(h, a->request_id[i], a->stream_id[i]);
        if (!ss.dirty && ss.dev_ranges >= (int32_t)ss.ranges.size() - 1) continue;
        if (no_alloc) { dev_lists = false; break; }  // (a rebuild stages through buffers that may have to grow)
        const int rb = rebuild_tables(h, ss);
        if (rb == kNoRoom) dev_lists = false;
        else if (rb != PASTA_OK) return rb;
      }
      if (!dev_lists && (a->flags & PASTA_DECODE_DEVICE_LISTS)) return PASTA_E_CAPACITY;
      if (dev_lists) h->lists_in_use = true;
    }
    // private items
    std::vector<DevStream>& streams = pb.streams;
    std::vector<DevRange>& ranges = pb.ranges;
    std::vector<DevItem>& items = pb.items;
    streams.assign(n, DevStream{});
    ranges.clear();
    items.clear();
    if (!dev_lists) {
      if (!room(ranges, (size_t)total_ranges + n)) return PASTA_E_CAPACITY;
      ranges.reserve((size_t)total_ranges + n);
    }
    int64_t gather_total = 0, n_items_total = 0;
    for (int i = 0; i < n; ++i) {
      DevStream& ds = streams[i];
      const DevReq& q = reqs[stream_req_idx[i]];
      ds.req = q.req;
      ds.req_idx = stream_req_idx[i];
      ds.local = stream_local[i];
      ds.pos = rope_q ? a->position[i] : 0;
      ds.mask_base = mask_base[i];
      ds.pc = q.pc;
      if (dev_lists) {
        const StreamState& ss = sstate(h, a->request_id[i], a->stream_id[i]);
        const int64_t extra = (int64_t)lv[i].prefix_len - q.pc, T = ss.range_tokens;
        if (gather_total + q.pc + extra + T > INT32_MAX) return PASTA_E_CAPACITY;
        ds.extra = (int32_t)extra;
        ds.n_ranges = (int32_t)ss.ranges.size();
        ds.seg_off = ss.seg_off;
        ds.range_tokens = (int32_t)T;
        ds.cseg_off = ss.cseg_off;
        ds.n_cidx = ss.dev_cidx;
        if (ds.n_ranges) {
          const Range& g = ss.ranges.back();
          ds.last[0] = g.start; ds.last[1] = g.count; ds.last[2] = g.stride; ds.last[3] = (int32_t)(T - g.count);
        }
        ds.item_begin = (int32_t)n_items_total;
        n_items_total += (extra + priv_chunk - 1) / priv_chunk + (T + priv_chunk - 1) / priv_chunk;
        ds.item_end = (int32_t)n_items_total;
        ds.gather_base = (int32_t)gather_total;
        if (a->dbg_gather_offsets) a->dbg_gather_offsets[i] = gather_total;
        gather_total += (int64_t)q.pc + extra + T;
        continue;
      }
      ds.range_begin = (int32_t)ranges.size();
      int32_t cum = 0;
      if (lv[i].prefix_len > q.pc) {
        ranges.push_back({q.pc, lv[i].prefix_len - q.pc, 1, 0});
        cum = lv[i].prefix_len - q.pc;
      }
      for (int k = 0; k < lv[i].n_ranges; ++k) {
        const Range g = lv[i].at(k);
        ranges.push_back({g.start, g.count, g.stride, cum});
        cum += g.count;
      }
      ds.range_end = (int32_t)ranges.size();
      ds.item_begin = (int32_t)items.size();
      int32_t rcur = ds.range_begin;
      for (int32_t t = 0; t < cum; t += (int32_t)priv_chunk) {
        while (rcur + 1 < ds.range_end && ranges[rcur + 1].cum <= t) rcur++;
        DevItem it{};
        it.stream = i;
        it.tok_begin = t;
        it.tok_count = std::min<int32_t>((int32_t)priv_chunk, cum - t);
        it.range_first = rcur;
        int32_t rlast = rcur;
        while (rlast + 1 < ds.range_end && ranges[rlast + 1].cum < t + it.tok_count) rlast++;
        it.n_ranges = rlast - rcur + 1;
        it.gather_pos = (int32_t)(gather_total + q.pc + t);
        it.slot0 = ranges[rcur].start + (t - ranges[rcur].cum) * ranges[rcur].stride;
        it.stride = it.n_ranges == 1 ? ranges[rcur].stride : 0;  // 0: rows come from the expanded list
        if (!room(items, items.size() + 1)) return PASTA_E_CAPACITY;
        items.push_back(it);
      }
      ds.item_end = (int32_t)items.size();
      n_items_total = (int64_t)items.size();
      if (gather_total + q.pc + cum > INT32_MAX) return PASTA_E_CAPACITY;
      ds.gather_base = (int32_t)gather_total;
      if (a->dbg_gather_offsets) a->dbg_gather_offsets[i] = gather_total;
      gather_total += (int64_t)q.pc + cum;
    }
    if (a->dbg_gather_offsets) a->dbg_gather_offsets[n] = gather_total;

    // split-K chunks of the common prefixes; grow the chunk until the partial rows fit
    const int64_t priv_rows = n_items_total * c.n_q_heads;
    int64_t n_prefix_wgs = 0, prefix_rows = 0;
    if (pc_total > 0) {
      for (;; chunk_tokens += kTile) {
        n_prefix_wgs = 0;
        prefix_rows = 0;
        for (auto& q : reqs) {
          q.n_chunks = q.pc ? (int32_t)((q.pc + chunk_tokens - 1) / chunk_tokens) : 0;
          q.chunk_tokens = (int32_t)chunk_tokens;
          q.wg_begin = (int32_t)n_prefix_wgs;
          q.part_base = (int32_t)prefix_rows;
          n_prefix_wgs += (int64_t)q.n_chunks * Hkv * row_units(q);
          prefix_rows += (int64_t)q.n_chunks * Hkv * q.n_streams * G;
        }
        if (prefix_rows + priv_rows <= part_rows_cap) break;
        if (chunk_tokens > (int64_t)1 << 30) return PASTA_E_CAPACITY;
      }
    } else {
      for (auto& q : reqs) { q.n_chunks = 0; q.chunk_tokens = kTile; q.wg_begin = 0; q.part_base = 0; }
      if (priv_rows > part_rows_cap) return PASTA_E_CAPACITY;
    }

    for (int i = 0; i < n; ++i) {  // the merge's view of each stream's request (known now that the chunks are)
      const DevReq& q = reqs[stream_req_idx[i]];
      streams[i].m_pre0 = q.part_base + streams[i].local * G;
      streams[i].m_n_pre = q.n_chunks;
      streams[i].m_R = q.n_streams * G;
    }
    // ---- metadata blob
    std::vector<int32_t>& blob = pb.blob;
    blob.clear();
    {
      const size_t words = (streams.size() * sizeof(DevStream) + reqs.size() * sizeof(DevReq) + req_streams.size() * 4 +
                            ranges.size() * sizeof(DevRange) + items.size() * sizeof(DevItem)) / 4 + 8;
      if (no_alloc && words > (size_t)kInlineMetaWords) return PASTA_E_CAPACITY;  // larger plans need the pinned staging
      if (!room(blob, words)) return PASTA_E_CAPACITY;
      blob.reserve(words);
    }
    DecodeParams p{};
    auto put = [&](const void* src, size_t bytes) -> int {
      const int off = (int)blob.size();
      blob.resize(blob.size() + (bytes + 3) / 4);
      if (bytes) std::memcpy(blob.data() + off, src, bytes);
      return off;
    };
    p.off_streams = put(streams.data(), streams.size() * sizeof(DevStream));
    p.off_reqs = put(reqs.data(), reqs.size() * sizeof(DevReq));
    p.off_req_streams = put(req_streams.data(), req_streams.size() * 4);
    p.off_ranges = put(ranges.data(), ranges.size() * sizeof(DevRange));
    p.off_items = put(items.data(), items.size() * sizeof(DevItem));
    if (blob.size() * 4 > h->meta_bytes) return PASTA_E_CAPACITY;

    if (a->dbg_plan) {
      int64_t tiles = 0;
      for (auto& q : reqs) tiles += (int64_t)(q.pc + kTile - 1) / kTile * Hkv;
      a->dbg_plan[0] = tiles;
      a->dbg_plan[1] = n_prefix_wgs;
      a->dbg_plan[2] = n_items_total;
      a->dbg_plan[3] = prefix_rows + priv_rows;
      a->dbg_plan[4] = pc_total ? chunk_tokens : 0;
      a->dbg_plan[5] = pc_total;
      a->dbg_plan[6] = (int64_t)blob.size() * 4;
      a->dbg_plan[7] = prefix_rows;
    }
    if (plan_only) return PASTA_OK;

    // ---- enqueue
    int rc = PASTA_OK;
    hipStream_t st = (hipStream_t)c.hip_stream;
    int meta_slot = -1;  // pinned staging slot that this call's kernels read, if any
    // a deferred append rides along with the matrix-core launch of its layer; otherwise K1 runs now
    const bool take_pending = h->pending.active && mfma && h->pending.layer == a->layer && !probe && !merge_only;
    if (h->pending.active && !take_pending) {
      rc = flush_pending(h);
      if (rc != PASTA_OK) return rc;
    }
    if (take_pending) {
      const pasta_attn::Pending& pd = h->pending;
      for (auto& q : reqs) { q.pend0 = pd.req_pend0[q.req]; q.pend_src0 = pd.req_src0[q.req]; }
      p.k_pend = pd.k_new;
      p.v_pend = pd.v_new;
      p.pend_n = pd.n_rows;
      std::memcpy(p.pend_dst, pd.dst_rows, sizeof(p.pend_dst));
      if (pd.rope) {  // turned by the small launch below, before the attention launch reads them
        p.pend_rope = 1;
        std::memcpy(p.pend_pos, pd.pos, sizeof(p.pend_pos));
      }
      // the blob was built before these fields were known: patch the table in place
      std::memcpy(blob.data() + p.off_reqs, reqs.data(), reqs.size() * sizeof(DevReq));
    }
    if (dense) {  // the masks travel like the paper's mask tensors: host -> device, every step
      if (!h->mask_pinned) {
        if (hipHostMalloc((void**)&h->mask_pinned, h->mask_bytes, hipHostMallocDefault) != hipSuccess) {
          (void)hipGetLastError();
          h->mask_pinned = nullptr;
          return PASTA_E_DEVICE;
        }
        if (hipEventCreateWithFlags(&h->mask_ev, hipEventDisableTiming) != hipSuccess) return PASTA_E_DEVICE;
      }
      if (h->mask_ev_used && hipEventSynchronize(h->mask_ev) != hipSuccess) return PASTA_E_DEVICE;
      std::memcpy(h->mask_pinned, mask.data(), mask.size());
      uint8_t* dev_mask = (uint8_t*)c.workspace + h->off_mask;
      if (hipMemcpyAsync(dev_mask, h->mask_pinned, mask.size(), hipMemcpyHostToDevice, st) != hipSuccess) return PASTA_E_DEVICE;
      if (hipEventRecord(h->mask_ev, st) != hipSuccess) return PASTA_E_DEVICE;
      h->mask_ev_used = true;
      p.dense_mask = dev_mask;
    }
    if (blob.size() <= (size_t)kInlineMetaWords) {  // small plan: rides in the kernel arguments
      p.meta = nullptr;
      std::memcpy(p.inline_meta, blob.data(), blob.size() * 4);
    } else {
      // large plan: it stays in pinned host memory and the kernels read it in place -- each
      // work-group touches a few dozen bytes of it, and a copy-engine transfer ahead of the
      // attention launch costs tens of microseconds on the stream (config 4: 97 -> 61 us per
      // step).  The slot is reused only after the launches that read it have completed.
      if (blob.size() * 4 > h->meta_bytes) return PASTA_E_CAPACITY;
      if (blob.size() <= (size_t)kRelayMaxWords) {
        // ... unless it is only a few KB (device-resident lists: one record per stream): then it travels to a
        // device staging slot inside the kernel arguments of one or two tiny launches
        const int sl = h->relay_next;
        h->relay_next = (sl + 1) % kRing;
        int32_t* dev = (int32_t*)((char*)c.workspace + h->off_meta + (size_t)sl * h->meta_bytes);
        for (size_t lo = 0; lo < blob.size(); lo += kRelayWords) {
          RelayParams rp;
          rp.dst = dev + lo;
          rp.n_words = (int)std::min<size_t>(kRelayWords, blob.size() - lo);
          std::memcpy(rp.words, blob.data() + lo, (size_t)rp.n_words * 4);
          k_meta_relay<<<dim3(1), 256, 0, st>>>(rp);
        }
        p.meta = dev;
      } else {
        meta_slot = h->ring_next;
        h->ring_next = (meta_slot + 1) % kRing;
        if (h->ring_used[meta_slot] && hipEventSynchronize(h->ring_ev[meta_slot]) != hipSuccess) return PASTA_E_DEVICE;
        char* host = h->pinned + (size_t)meta_slot * h->meta_bytes;
        std::memcpy(host, blob.data(), blob.size() * 4);
        p.meta = (const int32_t*)host;
      }
    }
    p.k = (const char*)c.k_pool + (size_t)a->layer * h->layer_elems * h->elem;
    p.v = (const char*)c.v_pool + (size_t)a->layer * h->layer_elems * h->elem;
    p.q = a->q;
    p.out = a->out;
    p.lse = a->out_lse;
    p.dbg_rows = a->dbg_gather_rows;
    p.page_table = (const int32_t*)((const char*)c.workspace + h->off_page_table);
    p.part_acc = part_acc;
    p.part_ml = part_ml;
    p.lay = h->lay;
    p.n_streams = n;
    p.n_reqs = (int)reqs.size();
    p.n_items = (int)n_items_total;
    p.n_mfma_items = mfma ? (int)n_items_total : 0;
    p.arena = (const DevRange*)((const char*)c.workspace + h->off_arena);
    p.cidx = (const int32_t*)((const char*)c.workspace + h->off_cidx);
    p.dev_tables = dev_lists ? 1 : 0;
    p.priv_chunk = (int)priv_chunk;
    p.n_prefix_wgs = (int)n_prefix_wgs;
    p.priv_part_base = (int)prefix_rows;
    p.Hq = c.n_q_heads;
    p.Hkv = Hkv;
    p.scale_log2e = c.softmax_scale * kLog2e;
#if defined(PASTA_TUNING) && PASTA_TUNING >= 2
    p.clock_row0 = h->part_rows_cap - 16 * PASTA_CLK_WGS + (a->layer & 1) * 8 * PASTA_CLK_WGS;  // the tail of the (m, l) array, two halves
#endif
    p.single_req = reqs.size() == 1 ? 1 : 0;
    if (p.single_req && n <= 16) {  // item ranges of the streams as kernel-argument scalars
      p.single_req = 2;
      for (int i = 0; i < n; ++i) {
        p.s_items[2 * i] = streams[i].item_begin;
        p.s_items[2 * i + 1] = streams[i].item_end - streams[i].item_begin;
      }
    }
    p.req0 = reqs[0];

    if (rope_q || p.pend_rope) {
      // one small launch turns what has to be turned: Q into its buffer, the deferred K rows into theirs
      p.rope_tab = (const double*)((const char*)c.workspace + h->off_rope);
      p.rope_q = rope_q ? 1 : 0;
      uint4* q_rot = (uint4*)((char*)c.workspace + h->off_qrot);
      uint4* k_rot = (uint4*)((char*)c.workspace + h->off_krot);
      const int pph = D * h->elem / 16;
      const long long nq = rope_q ? (long long)n * c.n_q_heads * pph : 0;
      const long long nk = p.pend_rope ? (long long)p.pend_n * Hkv * pph : 0;
      k_rope_prep<<<dim3((unsigned)((nq + nk + 255) / 256)), 256, 0, st>>>(p, q_rot, k_rot, pph, h->elem == 4, nq);
      if (rope_q) p.q = q_rot;
      if (p.pend_rope) { p.k_pend = k_rot; p.pend_rope = 0; }
    }
    // Profiling events: the matrix-core launch hands them to the dispatch itself, so they carry the
    // start and the end of that kernel's execution (what a kernel trace reports) and put no packet of
    // their own on the stream; around the vector-ALU form they are recorded on the stream.
    const hipEvent_t ev0 = (hipEvent_t)a->prof_event_start, ev1 = (hipEvent_t)a->prof_event_stop;
    const bool ev_in_dispatch = mfma && ev0 && ev1;
    if (ev0 && !ev_in_dispatch && hipEventRecord(ev0, st) != hipSuccess) return PASTA_E_DEVICE;
    if (merge_only) {
      // (kernel-isolated test of the merge: the partial buffers are taken as they are)
    } else if (mfma) {
      const unsigned grid = (unsigned)(n_items_total * Hkv + n_prefix_wgs);
      auto launch = [&](auto kernel) {
        if (ev_in_dispatch) hipExtLaunchKernelGGL(kernel, dim3(grid), dim3(kAttnThreads), 0, st, ev0, ev1, 0, p);
        else kernel<<<dim3(grid), kAttnThreads, 0, st>>>(p);
      };
      if (dense) {  // the variant that carries the dense-mask mode
        if (h->lay.paged) launch(k_attn<true, true>);
        else launch(k_attn<false, true>);
      } else {
        // prefix chunks of more than two 32-token blocks per wave: the variant whose loop has the
        // cheap addressing of plain blocks
        const bool long_items = n_prefix_wgs > 0 && chunk_tokens > 2 * 4 * 32;
        if (probe && !wide) {
          if (h->lay.paged) { if (long_items) launch(k_attn<true, false, true, true>); else launch(k_attn<true, false, false, true>); }
          else { if (long_items) launch(k_attn<false, false, true, true>); else launch(k_attn<false, false, false, true>); }
        } else if (!wide) {
          if (h->lay.paged) { if (long_items) launch(k_attn<true, false, true>); else launch(k_attn<true, false>); }
          else { if (long_items) launch(k_attn<false, false, true>); else launch(k_attn<false, false>); }
        } else if (probe) {
          if (h->lay.paged) launch(k_attn<true, false, false, true, true>);
          else launch(k_attn<false, false, false, true, true>);
        } else {
          if (h->lay.paged) launch(k_attn<true, false, false, false, true>);
          else launch(k_attn<false, false, false, false, true>);
        }
      }
      if (take_pending) h->pending.active = false;
    } else if (n_items_total > 0) {
      const unsigned waves = (unsigned)n_items_total * Hkv;
      rc = launch_private(h, dim3((waves + 3) / 4), st, p);
      if (rc != PASTA_OK) return rc;
    }
    if (ev1 && !ev_in_dispatch && hipEventRecord(ev1, st) != hipSuccess) return PASTA_E_DEVICE;
    int64_t merge_parts = 0;  // every output row reads its request's prefix chunks and its stream's items
    for (int i = 0; i < n; ++i)
      merge_parts += (int64_t)(reqs[stream_req_idx[i]].n_chunks + streams[i].item_end - streams[i].item_begin) * c.n_q_heads;
    if (!probe && !partials_only) {
      rc = launch_merge(h, dim3((unsigned)Hkv, (unsigned)G, (unsigned)n), st, p, merge_parts);
      if (rc != PASTA_OK) return rc;
    }
    if (meta_slot >= 0) {
      if (hipEventRecord(h->ring_ev[meta_slot], st) != hipSuccess) return PASTA_E_DEVICE;
      h->ring_used[meta_slot] = true;
    }
    if (hipGetLastError() != hipSuccess) return PASTA_E_DEVICE;
    return PASTA_OK;
  } catch (const std::bad_alloc&) {
    return PASTA_E_NOMEM;
  }
}

}  // namespace

extern "C" int32_t pasta_attn_decode_step(pasta_attn* h, const pasta_decode_args* a) { return decode_impl(h, a, false); }

extern "C" int32_t pasta_attn_decode_step_noalloc(pasta_attn* h, const pasta_decode_args* a) {
  return decode_impl(h, a, true);
}

#include "replay.hpp"
