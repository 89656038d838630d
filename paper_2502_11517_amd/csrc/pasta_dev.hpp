// Device-side structures and small helpers shared by the gfx950 kernels of the
// multi-stream decode-attention step (arxiv 2502.11517, Section 3, "Efficiency").
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pasta {

constexpr int kWave = 64;            // CDNA wavefront
constexpr int kPrivChunk = 128;      // tokens one work item of the vector-ALU private kernel walks
constexpr int kInlineMetaWords = 768; // per-call metadata up to this size rides in the kernel arguments
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Pool addressing, the formulas of include/pasta_attn.h folded into shifts and strides:
//   element offset(phys, g) = (phys >> page_shift) * page_stride
//                           + (phys & page_mask) * slot_stride + g * head_stride
// Contiguous pools use page_shift = 31 (one page holds everything).
struct Layout {
  long long page_stride;  // elements
  long long head_stride;  // elements
  int slot_stride;        // elements
  int page_shift;
  int page_mask;
  // logical slot -> physical row
  int paged;              // 0: phys = req * pool_tokens + slot
  int pages_per_request;  // 1: phys = page_table[req][slot >> shift] << shift | slot & mask
  int pool_tokens;
};

__device__ __forceinline__ long long elem_off(const Layout& L, int phys, int g) {
  return (long long)(phys >> L.page_shift) * L.page_stride +
         (long long)(phys & L.page_mask) * L.slot_stride + (long long)g * L.head_stride;
}

__device__ __forceinline__ int phys_row(const Layout& L, const int32_t* __restrict__ page_table,
                                        int req, int slot) {
  if (!L.paged) return req * L.pool_tokens + slot;
  int pp = page_table[req * L.pages_per_request + (slot >> L.page_shift)];
  return (pp << L.page_shift) | (slot & L.page_mask);
}

// ---- per-call metadata (int32 words in one blob; offsets travel in DecodeParams) ----
struct DevStream {      // one per decoding stream, call order
  int32_t req;          // request id
  int32_t req_idx;      // index into DevReq[]
  int32_t local;        // rank among the request's streams in this call: stacked-Q row block
  int32_t pc;           // tokens of the list handled by the shared-prefix kernel
  int32_t range_begin;  // private list = ranges [range_begin, range_end)
  int32_t range_end;
  int32_t item_begin;   // private work items [item_begin, item_end)
  int32_t item_end;
  int32_t gather_base;  // first entry of this stream in dbg_gather_rows
  int32_t pos;          // position id of the stream's query token (rotary embedding of Q)
  int32_t mask_base;    // dense-mask mode: this stream's mask bytes start here (one per slot of its request)
  // what the merge needs of the stream's request, copied here so that it is one record away:
  int32_t m_pre0;       // part_base + local * G: first shared-prefix partial row of the stream (kv head 0, chunk 0, head 0)
  int32_t m_n_pre;      // split-K chunks of the request's common prefix
  int32_t m_R;          // stacked rows of the request: shared-prefix part i of kv head g is row m_pre0 + (g * m_n_pre + i) * m_R + gi
  // ---- device-resident lists (DecodeParams::dev_tables): the stream's ranges are not in the blob but in the
  // arena that the appends keep up to date, and its private work items are derived by the kernels
  int32_t extra;        // prefix_len - pc: visible head beyond the common prefix (private, contiguous slots pc ..)
  int32_t n_ranges;     // ranges of the list: k < n_ranges - 1 at arena[seg_off + k], the newest one in `last`
  int32_t seg_off;
  int32_t range_tokens; // tokens in the ranges
  int32_t cseg_off;     // cidx[cseg_off + j] = index of the range that holds range token 32 j ...
  int32_t n_cidx;       // ... for j < n_cidx; later ones lie in the newest range
  int32_t last[4];      // the newest range (start, count, stride, cum): it grows with every append, so it rides
                        // with the call instead of being written to the arena each time
};                      // 24 words
struct DevRange {       // slots start + j*stride, j < count; cum = private tokens before it (device-resident
  int32_t start, count, stride, cum;  // lists: tokens of the stream's RANGES before it)
};
constexpr int kCidxTokens = 32;  // granularity of the range index over a stream's range tokens
struct DevItem {        // a chunk of one stream's private token list
  int32_t stream, tok_begin, tok_count;
  int32_t range_first;  // the range that holds token tok_begin
  int32_t n_ranges;     // ranges the chunk overlaps
  int32_t gather_pos;   // first entry of this chunk in dbg_gather_rows
  int32_t slot0;        // n_ranges == 1: token j of the chunk is logical slot slot0 + j*stride
  int32_t stride;
};                      // (8 words: the request and its deferred rows are found through the stream's DevReq)
struct DevReq {         // one per request present in the call
  int32_t req;
  int32_t pc;           // common prefix handled by the shared-prefix kernel
  int32_t n_streams;    // R = n_streams * G stacked query rows
  int32_t stream0;      // first entry in req_streams[]
  int32_t wg_begin;     // first prefix work-group of this request
  int32_t n_chunks;     // split-K chunks of [0, pc)
  int32_t chunk_tokens; // tokens per chunk (multiple of the LDS tile)
  int32_t part_base;    // first partial row: row = part_base + ((g*n_chunks + c)*R + r)
  int32_t pend0;        // deferred append, as in DevItem
  int32_t pend_src0;
};

struct DecodeParams {
  const void* k;        // layer base of the K pool
  const void* v;
  const void* q;        // [n][Hq][D]
  void* out;            // [n][Hq][D]
  float* lse;           // [n][Hq] or null
  int32_t* dbg_rows;    // or null
  const int32_t* meta;  // blob
  const int32_t* page_table;
  float* part_acc;      // [rows][D]
  float2* part_ml;      // [rows] (m in log2 units, l)
  Layout lay;
  int off_streams, off_reqs, off_req_streams, off_ranges, off_items;
  int n_streams, n_reqs, n_items, n_prefix_wgs;
  int n_mfma_items;     // private items taken by the matrix-core kernel (all or none)
  int priv_part_base;   // private partial row = priv_part_base + ((item*Hkv + g)*G + i)
  int Hq, Hkv;
  float scale_log2e;    // softmax_scale * log2(e): logits are kept in log2 units
#if defined(PASTA_TUNING) && PASTA_TUNING >= 2
  long long clock_row0; // first float2 slot of the phase-clock area (tuning builds only)
#endif
  // A deferred append (PASTA_APPEND_DEFER) rides along: its rows are read from k_pend / v_pend
  // ([row][Hkv][D]) wherever a list names them, and copied to the pool by the first work-groups.
  const void* k_pend;
  const void* v_pend;
  int pend_n;           // rows of the deferred append (0: none)
  int32_t pend_dst[32]; // their physical rows
  int32_t pend_pos[32]; // their position ids, when pend_rope
  // Rotary embedding: both flags are for the small launch ahead of the attention launch (k_rope_prep),
  // which writes rotated copies; the attention launch then gets q / k_pend pointing at those.
  int rope_q;           // 1: Q rows are to be turned by their streams' position ids
  int pend_rope;        // 1: the deferred K rows are still unrotated (PASTA_APPEND_ROPE), to be turned by pend_pos
  int32_t s_items[32];  // single_req with <= 16 streams: stream i's private items are
                        //   [s_items[2i], s_items[2i] + s_items[2i+1]) -- spares the merge a table look-up
  const uint8_t* dense_mask;  // comparison mode: 0/1 per (stream, slot); null otherwise
  const DevRange* arena;      // device-resident lists: range arena and range index (see DevStream)
  const int32_t* cidx;
  int dev_tables;             // 1: the blob holds no ranges and no items
  int priv_chunk;             // tokens per private work item
  const double* rope_tab;  // theta^(-2f/D) / (2 pi), f < D/2 (device), for k_rope_prep
  int single_req;       // 1: the call holds one request; its DevReq is req0 and stream i of
  DevReq req0;          //    the call is stacked-row block i (no table look-ups on the way
                        //    to the first K/V load)
  int32_t inline_meta[kInlineMetaWords];  // the blob itself when meta == nullptr (small plans:
                                          // no host-to-device copy on the step's critical path)
};

static_assert(sizeof(DecodeParams) <= 4096, "kernel arguments are limited to 4 KB");

// The metadata blob: device memory, or the copy inside the kernel arguments.  The inline copy
// is addressed through the kernarg segment pointer (DecodeParams is always the first kernel
// parameter, at offset 0), never through the address of the by-value parameter: taking that
// address makes the compiler copy all of it to scratch memory.
__device__ __forceinline__ const int32_t* meta_of(const DecodeParams& p) {
  if (p.meta) return p.meta;
  typedef const char __attribute__((address_space(4))) * kernarg_ptr;
  kernarg_ptr ka = (kernarg_ptr)__builtin_amdgcn_kernarg_segment_ptr();
  return (const int32_t*)(ka + __builtin_offsetof(DecodeParams, inline_meta));
}

// One 32-bit word of the blob, loaded through a pointer of known address space (global or
// kernel-argument memory, chosen by a uniform branch).  meta_of()'s merged pointer makes FLAT
// loads, whose completion is not ordered with other loads: fine before anything else is in
// flight, costly (a wait for everything) once the K/V loads are.
__device__ __forceinline__ int32_t meta_word(const DecodeParams& p, int word) {
  if (p.meta) return p.meta[word];
  typedef const char __attribute__((address_space(4))) * kernarg_ptr;
  kernarg_ptr ka = (kernarg_ptr)__builtin_amdgcn_kernarg_segment_ptr();
  return *(const int32_t __attribute__((address_space(4)))*)(ka + __builtin_offsetof(DecodeParams, inline_meta) + 4 * word);
}

__device__ __forceinline__ const int32_t* s_items_of(const DecodeParams& p) {
  (void)p;
  typedef const char __attribute__((address_space(4))) * kernarg_ptr;
  kernarg_ptr ka = (kernarg_ptr)__builtin_amdgcn_kernarg_segment_ptr();
  return (const int32_t*)(ka + __builtin_offsetof(DecodeParams, s_items));
}

__device__ __forceinline__ const int32_t* pend_dst_of(const DecodeParams& p) {
  (void)p;
  typedef const char __attribute__((address_space(4))) * kernarg_ptr;
  kernarg_ptr ka = (kernarg_ptr)__builtin_amdgcn_kernarg_segment_ptr();
  return (const int32_t*)(ka + __builtin_offsetof(DecodeParams, pend_dst));
}

__device__ __forceinline__ const int32_t* pend_pos_of(const DecodeParams& p) {
  (void)p;
  typedef const char __attribute__((address_space(4))) * kernarg_ptr;
  kernarg_ptr ka = (kernarg_ptr)__builtin_amdgcn_kernarg_segment_ptr();
  return (const int32_t*)(ka + __builtin_offsetof(DecodeParams, pend_pos));
}

// ---- device-resident lists: the pieces the kernels share
__device__ __forceinline__ DevRange dev_range_at(const DecodeParams& p, const DevStream& st, int k) {
  if (k >= st.n_ranges - 1) return DevRange{st.last[0], st.last[1], st.last[2], st.last[3]};
  return p.arena[st.seg_off + k];
}
__device__ __forceinline__ int dev_cidx_at(const DecodeParams& p, const DevStream& st, int j) {
  return j < st.n_cidx ? p.cidx[st.cseg_off + j] : st.n_ranges - 1;
}
// The call's stream whose private items include work item `item` (item_begin is ascending over the
// streams of a call; streams without items have item_begin == item_end).  Every lane searches.
__device__ __forceinline__ int dev_stream_of_item(const DecodeParams& p, const int32_t* meta, int item) {
  const DevStream* streams = reinterpret_cast<const DevStream*>(meta + p.off_streams);
  int lo = 0, hi = p.n_streams - 1;  // last stream with item_begin <= item
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (streams[mid].item_begin <= item) lo = mid; else hi = mid - 1;
  }
  return lo;  // (a stream without items shares its item_begin with the NEXT stream, which the search prefers)
}
// Work item `item` of stream i, derived: first the pieces of the visible head beyond the common prefix
// (contiguous slots), then the pieces of the range list, both in steps of priv_chunk tokens.  For a piece
// of the range list only tok_begin / tok_count / gather_pos are filled in here (tok_begin in range tokens):
// its ranges are looked up by the caller (dev_item_candidates).
__device__ __forceinline__ DevItem dev_item(const DecodeParams& p, const DevStream& st, int i, int item, bool& in_ranges) {
  const int C = p.priv_chunk;
  const int ci = item - st.item_begin;
  const int n_extra = (st.extra + C - 1) / C;
  DevItem it;
  it.stream = i;
  it.range_first = 0;
  it.n_ranges = 1;
  in_ranges = ci >= n_extra;
  if (!in_ranges) {
    it.tok_begin = ci * C;
    it.tok_count = min(C, st.extra - ci * C);
    it.gather_pos = st.gather_base + st.pc + ci * C;
    it.slot0 = st.pc + ci * C;
    it.stride = 1;
  } else {
    const int t0 = (ci - n_extra) * C;
    it.tok_begin = t0;
    it.tok_count = min(C, st.range_tokens - t0);
    it.gather_pos = st.gather_base + st.pc + st.extra + t0;
    it.slot0 = 0;
    it.stride = 0;
  }
  return it;
}
// The ranges that can hold tokens [t0, t0 + n) of the stream's range list: all of them when they fit
// `cap` entries, else the stretch that the range index points at.  Returns the first candidate's index.
__device__ __forceinline__ int dev_item_candidates(const DecodeParams& p, const DevStream& st, int t0, int n, int cap, int& count) {
  if (st.n_ranges <= cap) { count = st.n_ranges; return 0; }
  const int first = dev_cidx_at(p, st, t0 / kCidxTokens);
  const int j_hi = (t0 + n - 1) / kCidxTokens + 1;
  const int hi = j_hi * kCidxTokens < st.range_tokens ? dev_cidx_at(p, st, j_hi) : st.n_ranges - 1;
  count = min(hi - first + 1, cap);  // (n tokens overlap at most n ranges; cap >= n)
  return first;
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// fp32 -> bf16, round to nearest even (finite inputs; NaN stays NaN)
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

}  // namespace pasta
