// K2 + K3 on the matrix cores, one launch.
//
// K2, shared prefix.  Every stream forked from the same thread sees the same prefix rows of the
// pool (arxiv 2502.11517, Section 3, "Efficiency": a forked thread attends to the spawning
// thread's tokens that existed before the fork; the appendix on the naive interpreter names
// the cost of duplicating that prefix per thread).  Here the prefix K/V rows of one kv head
// are read from HBM ONCE per step and used for all R = n_streams * G query rows stacked
// together, so  S = Q_stack K^T  and  O = P V  are small dense contractions.  Work item =
// (request, kv head, split-K chunk of the common prefix, group of up to 32 stacked rows).
//
// K3, private segments.  A stream's own rows are interleaved with the other streams' rows in
// the pool (Section 3, "Efficiency"; Figure 2c).  Work item = (stream, kv head, chunk of the
// stream's private list).  A chunk that lies inside one (start, count, stride) range is
// addressed arithmetically; otherwise its ranges are expanded to physical rows in LDS.  Only
// the G query rows of that stream are live.
//
// A decode step is a chain of latencies more than a stream of bytes: what bounds it is how
// many bytes are in flight and how long a block takes from "data arrived" to "accumulated".
// So every WAVEFRONT of the four in a work-group is its own pipeline, and there is no
// work-group barrier in the loop:
//   * a wave owns the 32-token blocks w, w+4, ... of the item.  Its first block is loaded
//     straight into its LDS tile (global_load_lds, 16 B per lane), its second block into
//     registers, both requested before anything is waited for; later blocks follow through the
//     registers, one block ahead of the computation;
//   * the wave's LDS tile holds K and V of one block, each with the 16-byte XOR swizzle that
//     makes its kind of read free of bank conflicts;
//     S^T[32 tok x 32 rows] = K Q^T with v_mfma_f32_32x32x16_bf16 (A = K rows, B = Q rows);
//   * online softmax in registers: a lane holds 16 tokens of one row, its partner lane
//     (lane ^ 32) the other 16 -- one lane exchange per block for the row max;
//   * P = 2^(scale S - m) goes to bf16 IN REGISTERS: the S^T accumulator layout is already the
//     B-operand layout of the next MFMA for a suitable token order inside the contraction
//     (slot (ks, half, e) <-> token 16 ks + 8 (e / 4) + 4 half + e % 4), and V^T is fetched
//     from LDS with the transposing read in exactly that order;
//   * O^T[128 x 32 rows] += V^T P^T, four 32-row M-tiles per wave.
// The four waves' (m, l, O) are combined once, at the end, through LDS, and leave as coalesced
// 512-byte stores: one partial (m, l, acc[D]) per live row for the merge kernel (they stay in
// this XCD's L2, where the merge of the same kv head looks for them).  Logits are kept in
// log2 units.
#pragma once
#include <type_traits>

#include "mfma_util.hpp"

namespace pasta {

constexpr int kBlock = 32;  // tokens per wave block
constexpr int kRawBuffer = 0x00020000;  // buffer descriptor word 3: raw buffer of 32-bit data, no swizzle

struct AttnTile {             // one wave's 16 KB: K and V block, later its O^T on the way out
  u32x4 kt[kBlock * 16];      // K block [row][16 pieces], piece p of row r at p ^ (r & 15)
  u32x4 vt[kBlock * 16];      // V block [row][16 pieces], piece p of row r at p ^ v_swizzle(r)
};

// The two operands are read differently, so they are swizzled differently.  K (and Q): 16 lanes
// read one 16-byte piece each of 16 consecutive rows -- p ^ (r & 15) spreads them over all 64
// banks.  V: a transposing read takes 64 contiguous bytes of each of FOUR consecutive rows per
// bank cycle; rows are 256 bytes = one trip round the banks apart, so the four rows must land in
// four different quarters of the row (with K's swizzle they would share one: a 4-way conflict,
// 8 instead of 2 cycles per read -- measured).
__device__ __forceinline__ int v_swizzle(int r) { return (r & 3) << 2; }

struct AttnLds {
  AttnTile tile[4];           // first member: wave w's area starts at byte w * 16 KB
  u32x4 q[32 * 16];            // stacked Q rows, same swizzle (rows >= R are zero)
  float mw[4][32], lw[4][32];  // per-wave row max / row sum at the end of the item
  uint8_t mask[kGatherMax];    // dense-mask comparison mode: the item's slice of its stream's mask
  int sel[2];                  // device-resident lists: which candidate ranges hold an item's first and last token
  int rows[kGatherMax];        // listed gather items: row code of every token
  DevRange ranges[kGatherMax]; // listed gather items: the ranges the item overlaps
};

struct BlockRegs { u32x4 k[8], v[8]; };  // one lane's share of a 32-token block

// (FORM only keeps the instantiations of different kernels apart: the host pass of the compiler cannot
// check this body -- it has no device builtins -- and refuses a specialization it has already tried)
template <bool PAGED, bool GATHER, bool DENSE, bool LONG, bool PROBE, int FORM = 0>
__device__ __forceinline__ void attn_item(const DecodeParams& p, AttnLds& lds, const int32_t* meta, int wi) {
  constexpr int D = 128;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave index, known uniform: scalar branches below
  const int l32 = lane & 31, hh = lane >> 5;
  const int G = p.Hq / p.Hkv;
  PASTA_CLK(0);

  // ---- decode the work item
  int req, g, R, n_tok, slot0, stride, gather_pos, pend0, pend_src0;
  int row0 = 0;  // first stacked row of this item's row group (shared-prefix items)
  long long part_row0;
  const int32_t* req_streams = nullptr;
  int q_stream = 0, n_req_streams = 0;
  bool listed = false;
  if constexpr (!GATHER) {
    DevReq rq;
    if (p.single_req) {  // scalar loads from the kernel arguments
      rq.req = p.req0.req; rq.pc = p.req0.pc; rq.n_streams = p.req0.n_streams; rq.stream0 = 0;
      rq.wg_begin = p.req0.wg_begin; rq.n_chunks = p.req0.n_chunks;
      rq.chunk_tokens = p.req0.chunk_tokens; rq.part_base = p.req0.part_base;
      rq.pend0 = p.req0.pend0; rq.pend_src0 = p.req0.pend_src0;
    } else {
      const DevReq* reqs = reinterpret_cast<const DevReq*>(meta + p.off_reqs);
      int qi = 0;
      for (; qi < p.n_reqs - 1; ++qi) {
        const int b = reqs[qi].wg_begin;
        if (wi >= b && wi < b + reqs[qi].n_chunks * p.Hkv * ((reqs[qi].n_streams * G + 31) >> 5)) break;
      }
      rq = reqs[qi];
      req_streams = meta + p.off_req_streams + rq.stream0;
    }
    // kv head = work-group index mod Hkv: with 8 kv heads every work-group of head g (private
    // items included, their index is item * Hkv + g) lands on XCD g, whose L2 then holds all of
    // that head's partials for the merge.  A request with more than 32 stacked rows is served
    // in row groups of 32: the groups of one (chunk, kv head) are neighbours in launch order on
    // the same XCD, so the chunk comes from HBM once and from that XCD's L2 for the others.
    const int R_all = rq.n_streams * G;
    const int n_rg = (R_all + 31) >> 5;
    const int wl = wi - rq.wg_begin;
    const int t = wl / p.Hkv;
    const int c = t / n_rg;
    row0 = (t % n_rg) * 32;
    g = wl % p.Hkv;
    req = rq.req;
    R = min(32, R_all - row0);
    n_req_streams = rq.n_streams;
    slot0 = c * rq.chunk_tokens;
    stride = 1;
    n_tok = min(rq.chunk_tokens, rq.pc - slot0);
    part_row0 = rq.part_base + (long long)(g * rq.n_chunks + c) * R_all + row0;
    gather_pos = slot0;
    pend0 = rq.pend0;
    pend_src0 = rq.pend_src0;
  } else {
    const int item = wi / p.Hkv;
    g = wi % p.Hkv;
    // the work item: from the blob, or -- device-resident lists -- derived from the stream's record;
    // a piece of a device-resident range list then finds its ranges among the candidates below
    DevItem it;
    int nr = 0, range0 = 0;      // ranges to bring into LDS: [range0, range0 + nr) of the blob or of the stream's arena
    bool in_ranges = false;
    DevStream dst{};
    if (!p.dev_tables) {
      it = reinterpret_cast<const DevItem*>(meta + p.off_items)[item];
      nr = it.n_ranges > 1 ? it.n_ranges : 0;
      range0 = it.range_first;
    } else {
      const int si = dev_stream_of_item(p, meta, item);
      dst = reinterpret_cast<const DevStream*>(meta + p.off_streams)[si];
      it = dev_item(p, dst, si, item, in_ranges);
      if (in_ranges) range0 = dev_item_candidates(p, dst, it.tok_begin, it.tok_count, kGatherMax, nr);
    }
    if (p.single_req) {  // scalars from the kernel arguments
      req = p.req0.req; pend0 = p.req0.pend0; pend_src0 = p.req0.pend_src0;
    } else {
      const int qi = reinterpret_cast<const DevStream*>(meta + p.off_streams)[it.stream].req_idx;
      const DevReq rq = reinterpret_cast<const DevReq*>(meta + p.off_reqs)[qi];
      req = rq.req; pend0 = rq.pend0; pend_src0 = rq.pend_src0;
    }
    R = G;
    q_stream = it.stream;
    n_tok = it.tok_count;
    slot0 = it.slot0;
    stride = it.stride;
    part_row0 = p.priv_part_base + (long long)(item * p.Hkv + g) * G;
    gather_pos = it.gather_pos;
    listed = it.n_ranges > 1;
    if (DENSE && p.dense_mask) {  // comparison mode: the list is [0, tail), what may be seen is in the mask
      const int mb = meta_word(p, p.off_streams + it.stream * (int)(sizeof(DevStream) / 4) +
                                      (int)(__builtin_offsetof(DevStream, mask_base) / 4));
      for (int j = tid; j < kGatherMax; j += kAttnThreads)
        lds.mask[j] = j < n_tok ? p.dense_mask[mb + slot0 + j] : 0;  // published by the Q barrier
    }
    if (p.dev_tables && in_ranges) {
      // candidates -> LDS; the two that hold the piece's first and last token are found on the way
      const int t_lo = it.tok_begin, t_hi = it.tok_begin + it.tok_count - 1;
      for (int r = tid; r < nr; r += kAttnThreads) {
        const DevRange rg = dev_range_at(p, dst, range0 + r);
        lds.ranges[r] = rg;
        if (rg.cum <= t_lo && t_lo < rg.cum + rg.count) lds.sel[0] = r;
        if (rg.cum <= t_hi && t_hi < rg.cum + rg.count) lds.sel[1] = r;
      }
      __syncthreads();
      const int ra = lds.sel[0], rb = lds.sel[1];
      const DevRange r0 = lds.ranges[ra];
      it.slot0 = r0.start + (t_lo - r0.cum) * r0.stride;
      it.stride = r0.stride;
      it.n_ranges = rb - ra + 1;
      slot0 = it.slot0;
      stride = it.stride;
      listed = it.n_ranges > 1;
      range0 = ra;                 // from here on: index into lds.ranges
      nr = it.n_ranges;
    }
    if (listed) {  // ranges the item overlaps -> LDS, then every token of the item -> row code
      const DevRange* lr = lds.ranges;
      if (!p.dev_tables) {
        const DevRange* ranges = reinterpret_cast<const DevRange*>(meta + p.off_ranges);
        for (int r = tid; r < nr; r += kAttnThreads) lds.ranges[r] = ranges[range0 + r];
        __syncthreads();
      } else {
        lr = lds.ranges + range0;
      }
      for (int j = tid; j < n_tok; j += kAttnThreads) {
        const int tok = it.tok_begin + j;
        int lo = 0, hi = nr - 1;  // last range with cum <= tok
        while (lo < hi) {
          const int mid = (lo + hi + 1) >> 1;
          if (lr[mid].cum <= tok) lo = mid; else hi = mid - 1;
        }
        const DevRange rg = lr[lo];
        const int slot = rg.start + (tok - rg.cum) * rg.stride;
        const int phys = phys_row(p.lay, p.page_table, req, slot);
        lds.rows[j] = slot >= pend0 ? -1 - (pend_src0 + (slot - pend0)) : phys;  // deferred rows: -(1 + row)
        if (p.dbg_rows && g == 0) p.dbg_rows[gather_pos + j] = phys;
      }
      __syncthreads();
    }
  }
  // (work-group-uniform values, but loaded per lane: tell the compiler, so that the branches on
  // them are scalar and its wait-count bookkeeping sees an exhaustive if / else)
  n_tok = __builtin_amdgcn_readfirstlane(n_tok);
  const int n_blocks = (n_tok + kBlock - 1) / kBlock;
  req = __builtin_amdgcn_readfirstlane(req);
  R = __builtin_amdgcn_readfirstlane(R);
  g = __builtin_amdgcn_readfirstlane(g);
  slot0 = __builtin_amdgcn_readfirstlane(slot0);
  stride = __builtin_amdgcn_readfirstlane(stride);
  pend0 = __builtin_amdgcn_readfirstlane(pend0);
  pend_src0 = __builtin_amdgcn_readfirstlane(pend_src0);
  listed = __builtin_amdgcn_readfirstlane((int)listed) != 0;

  // ---- block loads: lane -> piece (lane & 15) of rows (lane >> 4) + 4 i, i < 8
  const char* kb = reinterpret_cast<const char*>(p.k);
  const char* vb = reinterpret_cast<const char*>(p.v);
  const char* kpend = reinterpret_cast<const char*>(p.k_pend);
  const char* vpend = reinterpret_cast<const char*>(p.v_pend);
  const int piece = lane & 15, rbase = lane >> 4;  // rbase 0..3
  auto phys_of = [&](int j) -> int {  // physical pool row of token j (not for listed items)
    const int t = slot0 + j * stride;
    if constexpr (PAGED) {
      const int pp = p.page_table[req * p.lay.pages_per_request + (t >> p.lay.page_shift)];
      return (pp << p.lay.page_shift) | (t & p.lay.page_mask);
    } else {
      return req * p.lay.pool_tokens + t;
    }
  };
  auto src_of = [&](int j, bool& is_pend) -> long long {  // byte offset of token j's row of head g; branch-free
    const int t = slot0 + j * stride;
    int phys = phys_of(j);
    int pidx = pend_src0 + (t - pend0);
    is_pend = t >= pend0;
    if constexpr (GATHER) {
      const int code = lds.rows[j];  // j < kGatherMax; meaningful only for listed items
      if (listed) { is_pend = code < 0; pidx = -1 - code; phys = code; }
    }
    const long long off_pool = elem_off(p.lay, is_pend ? 0 : phys, g) * 2;
    const long long off_pend = ((long long)pidx * p.Hkv + g) * D * 2;
    return is_pend ? off_pend : off_pool;
  };
  // A PLAIN block: 32 existing tokens whose rows are an arithmetic progression in memory (a
  // contiguous pool: any stride; a paged pool: consecutive slots starting at a multiple of 32,
  // pages of 16 tokens or more, so each half of the block lies inside one page), none of them a
  // deferred row.  Its addresses are a wave-uniform base per half block (scalar arithmetic, the
  // page-table entries through scalar loads) plus a 32-bit lane part that is the same for every
  // block of the item; all other blocks (listed, ragged, with deferred rows) compute one address
  // per row, which costs about 12 vector instructions per row.  Only the LONG instantiation has
  // this path, and only in its steady-state loop: launches whose waves have at most two blocks
  // never get there, and merely carrying the code made them slower (measured: +0.9 us on a
  // 13 us launch).
  const long long row_bytes = (long long)stride * p.lay.slot_stride * 2;
  const bool arith = LONG && !listed && row_bytes < (1ll << 26) &&  // 31 row steps fit 32 bits
                     (!PAGED || (stride == 1 && (slot0 & 31) == 0 && p.lay.page_shift >= 4));
  const uint32_t lane_row = (uint32_t)rbase * (uint32_t)row_bytes;
  auto plain = [&](int b) -> bool {
    return arith && b * kBlock + kBlock <= n_tok && slot0 + (b * kBlock + kBlock - 1) * stride < pend0;
  };
  auto load_block = [&](BlockRegs& br, int b, auto try_plain) {  // block b -> registers, natural piece order
    if (try_plain.value && plain(b)) {
      // buffer loads: descriptor base = the first row of each half block (scalar), lane part in
      // the offset register, row step in the scalar offset -- no vector arithmetic per load
      const uint32_t lo = lane_row + piece * 16, step = 4u * (uint32_t)row_bytes;
      long long off2[2];
      int pp[2] = {0, 0};
      if constexpr (PAGED) {  // both page look-ups first (scalar loads)
#pragma unroll
        for (int hb = 0; hb < 2; ++hb)
          pp[hb] = scalar_load_i32(p.page_table, req * p.lay.pages_per_request + ((slot0 + b * kBlock + 16 * hb) >> p.lay.page_shift));
      }
#pragma unroll
      for (int hb = 0; hb < 2; ++hb) {
        const int t = slot0 + (b * kBlock + 16 * hb) * stride;  // uniform
        const int phys = PAGED ? ((pp[hb] << p.lay.page_shift) | (t & p.lay.page_mask)) : req * p.lay.pool_tokens + t;
        off2[hb] = elem_off(p.lay, phys, g) * 2;
      }
#pragma unroll
      for (int hb = 0; hb < 2; ++hb) {
        const long long off = off2[hb];
        const __amdgpu_buffer_rsrc_t kr = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(kb + off), 0, 0x7fffffff, kRawBuffer);
        const __amdgpu_buffer_rsrc_t vr = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(vb + off), 0, 0x7fffffff, kRawBuffer);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          br.k[4 * hb + i] = __builtin_amdgcn_raw_buffer_load_b128(kr, lo, i * step, 0);
          br.v[4 * hb + i] = __builtin_amdgcn_raw_buffer_load_b128(vr, lo, i * step, 0);
        }
      }
      return;
    }
    long long off[8];
    bool pnd[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int j = min(b * kBlock + rbase + 4 * i, n_tok - 1);  // rows past the end repeat the last one
      off[i] = src_of(j, pnd[i]) + piece * 16;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      br.k[i] = *reinterpret_cast<const u32x4*>((pnd[i] ? kpend : kb) + off[i]);
      br.v[i] = *reinterpret_cast<const u32x4*>((pnd[i] ? vpend : vb) + off[i]);
    }
  };
  u32x4* ktw = lds.tile[w].kt;
  u32x4* vtw = lds.tile[w].vt;
  // Loads that go straight into this wave's LDS tile, no registers in between: one such load writes
  // 64 consecutive 16-byte pieces (lane l at piece l of the destination), so instruction i fills
  // rows 4 i .. 4 i + 3 and the swizzle moves to the global side -- the lane whose LDS place is
  // position (lane & 15) of row r fetches piece (lane & 15) ^ (r & 15) of that row.  They are
  // BUFFER loads (32-bit offsets from the layer's base: the host sends no pool of 4 GiB or more per
  // layer this way): the compiler counts a buffer load into LDS like any vector-memory load, whereas
  // with the flat-encoded form in flight it turns every wait it inserts itself -- in front of the
  // transposing LDS reads, in front of the first use of a register load -- into a wait for ALL loads,
  // which would hold the first block's P V until the second block has arrived.  A block that holds
  // rows of a deferred append (they live in the caller's k_new / v_new, anywhere in memory) goes
  // through registers instead.
  const __amdgpu_buffer_rsrc_t k_rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(kb), 0, -1, kRawBuffer);
  const __amdgpu_buffer_rsrc_t v_rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(vb), 0, -1, kRawBuffer);
  typedef __attribute__((address_space(3))) void* lds_ptr;
  // A PLAIN block -- 32 existing tokens of an item in a contiguous pool that is not a listed one, none
  // of them a deferred row -- has rows in arithmetic progression: its addresses are a wave-uniform
  // byte offset (scalar arithmetic, riding in the load's scalar offset) plus a lane part that is the
  // same for every block of the item (computed once: four variants for K's swizzle, one for V's, one
  // for loads into registers).  Every other block computes one address per row, about a dozen vector
  // instructions each -- which, at 32 rows per wave, is what stands between the start of a work-group
  // and its first request.
  const uint32_t row_bytes32 = (uint32_t)__builtin_amdgcn_readfirstlane(stride * p.lay.slot_stride * 2);
  const bool arith_item = !PAGED && !listed;
  uint32_t lane_k[4], lane_v, lane_n;
#pragma unroll
  for (int c4 = 0; c4 < 4; ++c4) lane_k[c4] = (uint32_t)rbase * row_bytes32 + (uint32_t)((piece ^ rbase ^ (4 * c4)) * 16);
  lane_v = (uint32_t)rbase * row_bytes32 + (uint32_t)((piece ^ (rbase << 2)) * 16);
  lane_n = (uint32_t)rbase * row_bytes32 + (uint32_t)(piece * 16);
  auto plain_block = [&](int b) -> bool {
    return arith_item && b * kBlock + kBlock <= n_tok && slot0 + (b * kBlock + kBlock - 1) * stride < pend0;
  };
  auto block_base = [&](int b) -> uint32_t {  // byte offset of a plain block's first row of this kv head
    const long long e = elem_off(p.lay, req * p.lay.pool_tokens + slot0 + b * kBlock * stride, g) * 2;
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)e);
  };
  // Rows of a deferred append are the newest slots of their request, so in a list (ascending slots) they
  // come LAST: a block holds them as a run at its end.  Up to four of them behind at least one pool row
  // are PATCHED: the block is fetched from the pool as if nothing were deferred (in their places, and in
  // the places past the item's end, the block's last pool row once more), the deferred rows themselves
  // come through one register per lane, requested ahead of everything, and are written over their places
  // when the block has landed.  (Fetching them into LDS under lane masks costs a loop per row group; on a
  // step of a few streams that was 1.9 us of 11.)  Other mixes take that masked path.
  struct DmaRows { uint32_t off[8]; bool any_pend; bool plain; uint32_t base; bool patch; int first_pend, n_pend; };
  auto is_pend = [&](int j) -> bool {  // j < n_tok
    if constexpr (GATHER) {
      if (listed) return lds.rows[j] < 0;
    }
    return slot0 + j * stride >= pend0;
  };
  auto dma_rows = [&](int b) -> DmaRows {  // K-side offsets of block b's rows for this lane's LDS places
    DmaRows d;
    d.plain = plain_block(b);
    d.any_pend = false;
    d.patch = false;
    d.first_pend = kBlock;
    d.n_pend = 0;
    d.base = 0;
    if (d.plain) {
      d.base = block_base(b);
      return d;
    }
    {
      const int jl = b * kBlock + l32;
      const uint32_t m = (uint32_t)__builtin_amdgcn_ballot_w64(jl < n_tok && is_pend(jl));  // both halves of the wave agree
      if (m) {
        d.first_pend = __builtin_ctz(m);
        d.n_pend = min(kBlock, n_tok - b * kBlock) - d.first_pend;
        d.patch = d.first_pend > 0 && d.n_pend <= 4;
        d.any_pend = !d.patch;
      }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = rbase + 4 * i;
      int j = min(b * kBlock + r, n_tok - 1);  // rows past the end repeat the last one
      if (d.patch && r >= d.first_pend) j = b * kBlock + d.first_pend - 1;  // ... the last one in the pool
      bool pn;
      const long long o = src_of(j, pn);
      d.off[i] = (uint32_t)o + (uint32_t)((piece ^ (r & 15)) * 16);
    }
    return d;
  };
  auto dma_half = [&](int b, const DmaRows& d, auto is_v) {  // K (or V) of block b -> kt (vt)
    u32x4* dst = is_v.value ? vtw : ktw;
    if (d.plain) {
#pragma unroll
      for (int i = 0; i < 8; ++i)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(is_v.value ? v_rs : k_rs, (lds_ptr)(dst + 64 * i), 16,
                                                 is_v.value ? lane_v : lane_k[i & 3], d.base + (uint32_t)(4 * i) * row_bytes32, 0, 0);
    } else if (!d.any_pend) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {  // the row offset is a multiple of 256: bits 4..7 hold the piece alone
        const int r = rbase + 4 * i;
        const uint32_t o = is_v.value ? d.off[i] ^ (uint32_t)(((r & 15) ^ v_swizzle(r)) << 4) : d.off[i];
        __builtin_amdgcn_raw_ptr_buffer_load_lds(is_v.value ? v_rs : k_rs, (lds_ptr)(dst + 64 * i), 16, o, 0, 0, 0);
      }
    } else {
      // some row of the block is a deferred one (the newest rows of a list sit in its last block): those
      // lanes fetch from the caller's rows through a descriptor of their own, the others from the pool --
      // two loads into LDS under complementary lane masks (a lane that is switched off neither reads nor
      // writes its LDS place), nothing waited for here.  The explicit waits further down count one load
      // per row group; where a group needed two, they wait for a little more than they have to, never
      // for less (loads return in issue order).
      const __amdgpu_buffer_rsrc_t p_rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(is_v.value ? vpend : kpend), 0, -1, kRawBuffer);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int r = rbase + 4 * i;
        const int j = min(b * kBlock + r, n_tok - 1);
        bool pn;
        uint32_t o = (uint32_t)src_of(j, pn) + (uint32_t)((piece ^ (r & 15)) * 16);  // deferred rows: offset in k_new / v_new
        if (is_v.value) o ^= (uint32_t)(((r & 15) ^ v_swizzle(r)) << 4);
        if (pn) __builtin_amdgcn_raw_ptr_buffer_load_lds(p_rs, (lds_ptr)(dst + 64 * i), 16, o, 0, 0, 0);
        else __builtin_amdgcn_raw_ptr_buffer_load_lds(is_v.value ? v_rs : k_rs, (lds_ptr)(dst + 64 * i), 16, o, 0, 0, 0);
      }
    }
  };
  auto load_half = [&](u32x4 (&dst)[8], int b, auto is_v) {  // K (or V) of block b -> registers, natural piece order
    if (plain_block(b)) {
      const uint32_t base = block_base(b);
#pragma unroll
      for (int i = 0; i < 8; ++i)
        dst[i] = __builtin_amdgcn_raw_buffer_load_b128(is_v.value ? v_rs : k_rs, lane_n, base + (uint32_t)(4 * i) * row_bytes32, 0);
      return;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int j = min(b * kBlock + rbase + 4 * i, n_tok - 1);
      bool pn;
      const long long o = src_of(j, pn) + piece * 16;
      dst[i] = *reinterpret_cast<const u32x4*>((pn ? (is_v.value ? vpend : kpend) : (is_v.value ? vb : kb)) + o);
    }
  };
  // ---- everything this wave needs first is requested here, before anything is waited for: its
  // share of the stacked Q rows (2 loads), then -- in the order in which they are needed, because
  // loads return in issue order -- K of its first block (into LDS), K of its second block (into
  // registers), V of the first (LDS), V of the second (registers).
  {
    const __amdgpu_buffer_rsrc_t q_rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.q), 0, -1, kRawBuffer);
#pragma unroll
    for (int i = 0; i < 2; ++i) {  // wave w fills pieces [128 w + 64 i, + 64) of lds.q: rows 8 w + 4 i + rbase
      const int r = 8 * w + 4 * i + rbase;
      u32x4* dst = lds.q + 128 * w + 64 * i;
      const int gp = piece ^ (r & 15);  // the global piece that lives at this lane's LDS place
      if (r < R) {
        const int ra = row0 + r;  // row of the request's stack
        const int s = GATHER ? q_stream : (req_streams ? req_streams[ra / G] : ra / G);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(q_rs, (lds_ptr)dst, 16, (uint32_t)((s * p.Hq + (g * G + ra % G)) * 256 + gp * 16), 0, 0, 0);
      } else {
        dst[lane] = u32x4{0u, 0u, 0u, 0u};  // rows past R are zero
      }
    }
  }
  BlockRegs br;
  const bool has1 = w < n_blocks, has2 = w + 4 < n_blocks;

  auto report_rows = [&]() {
    if (p.dbg_rows && g == 0 && row0 == 0 && !listed) {  // listed items reported their rows while expanding
      const DevStream* streams = reinterpret_cast<const DevStream*>(meta + p.off_streams);
      for (int j = tid; j < n_tok; j += kAttnThreads) {
        const int phys = phys_of(j);
        if constexpr (GATHER) {
          p.dbg_rows[gather_pos + j] = phys;
        } else {
          for (int k = 0; k < n_req_streams; ++k)
            p.dbg_rows[streams[req_streams ? req_streams[k] : k].gather_base + gather_pos + j] = phys;
        }
      }
    }
  };

  f32x16 O[4];  // O^T M-tile mt: d = 32 mt + 8 (i / 4) + 4 hh + i % 4, row l32
  float m_run = -INFINITY, l_run = 0.f;  // row l32; l_run covers this lane's 16 tokens of every block
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int i = 0; i < 16; ++i) O[mt][i] = 0.f;

  // V^T reads: token row 16 ks + 8 e4 + 4 hh + r2 (r2 = bits 2..3 of the lane), columns
  // 32 mt + 16 cblk + 4 (lane & 3) ...: with V's swizzle the lane's byte address is a per-M-tile
  // lane part (the 64-byte quarter is mt ^ r2) plus a constant that fits the instruction's offset.
  const char* vrd[4];
  {
    const int bl = lane & 15, cblk = (lane >> 4) & 1, r2 = bl >> 2;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
      vrd[mt] = reinterpret_cast<const char*>(vtw) + (4 * hh + r2) * 256 + (mt ^ r2) * 64 +
                (2 * cblk + ((bl >> 1) & 1)) * 16 + (bl & 1) * 8;
  }
  auto tile_sync = [&]() {  // orders this wave's own LDS writes (or landed loads) before its reads
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  };
  auto regs_to_tile = [&](const u32x4 (&src)[8], auto is_v) {  // rows rbase + 4 i of the block
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = rbase + 4 * i;
      if constexpr (is_v.value) vtw[r * 16 + (piece ^ v_swizzle(r))] = src[i];
      else ktw[r * 16 + (piece ^ (r & 15))] = src[i];
    }
  };
  // ---- S^T = K Q^T of the block in the tile: lane (token l32 | row l32, half hh); then the tokens
  // that do not exist (a block that reaches past the item's end) or may not be seen (dense-mask mode)
  // are hidden.  Register i of lane (row, hh) is token 8 (i / 4) + 4 hh + i % 4 of the block.
  auto s_block = [&](int b) -> f32x16 {
    f32x16 S;
#pragma unroll
    for (int i = 0; i < 16; ++i) S[i] = 0.f;
    {  // operands of step kk + 1 are requested before step kk is issued: LDS latency once, not 8 times
      u32x4 a[2], qv[2];
      const int pc0 = hh ^ (l32 & 15);
      a[0] = ktw[l32 * 16 + pc0];
      qv[0] = lds.q[l32 * 16 + pc0];
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        if (kk + 1 < 8) {
          const int pc = (2 * kk + 2 + hh) ^ (l32 & 15);
          a[(kk + 1) & 1] = ktw[l32 * 16 + pc];
          qv[(kk + 1) & 1] = lds.q[l32 * 16 + pc];
        }
        S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(&a[kk & 1]),
                                                    *reinterpret_cast<const bf16x8*>(&qv[kk & 1]), S, 0, 0, 0);
      }
      // (left alone, the scheduler pulls each pair of reads back behind the MFMA before it)
      __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);  // 4 LDS reads
#pragma unroll
      for (int kk = 0; kk < 6; ++kk) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // 1 MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);  // 2 LDS reads
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
    }
    const int tok0 = b * kBlock + 4 * hh;
    bool hide = b * kBlock + kBlock > n_tok;
    if constexpr (GATHER && DENSE) hide = hide || p.dense_mask != nullptr;
    if (hide) {
      asm volatile("" ::: "memory");  // keeps this a branch: the common case has nothing to hide
      const int left = n_tok - tok0;  // this lane's tokens 8 (i / 4) + i % 4 below `left` exist
      uint32_t mk[4] = {~0u, ~0u, ~0u, ~0u};  // one byte per token: tokens tok0 + 8 k .. + 3 in mk[k]
      if constexpr (GATHER && DENSE) {
        if (p.dense_mask) {
#pragma unroll
          for (int k = 0; k < 4; ++k) mk[k] = *reinterpret_cast<const uint32_t*>(&lds.mask[(tok0 + 8 * k) & (kGatherMax - 1)]);
        }
      }
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const bool seen = (8 * (i >> 2) + (i & 3)) < left && ((mk[i >> 2] >> (8 * (i & 3))) & 0xffu);
        S[i] = seen ? S[i] : -INFINITY;
      }
    }
    return S;
  };
  auto row_max = [&](const f32x16& S) -> float {  // of this lane's 16 tokens
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < 16; ++i) mx = fmaxf(mx, S[i]);
    return mx;
  };
  struct PBlock { bf16x8 ks[2]; };  // P^T as B operand: contraction step ks holds registers 8 ks .. 8 ks + 7
  // 2^(scale S - mref), summed into ps, rounded to bf16 in registers
  auto exp_pack = [&](f32x16& S, float mref, float& ps) -> PBlock {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      S[i] = fast_exp2(fmaf(S[i], p.scale_log2e, -mref));
      ps += S[i];
    }
    PBlock P;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      u32x4 pk;
      pk[0] = pack_bf16x2(S[8 * ks + 0], S[8 * ks + 1]);
      pk[1] = pack_bf16x2(S[8 * ks + 2], S[8 * ks + 3]);
      pk[2] = pack_bf16x2(S[8 * ks + 4], S[8 * ks + 5]);
      pk[3] = pack_bf16x2(S[8 * ks + 6], S[8 * ks + 7]);
      P.ks[ks] = *reinterpret_cast<const bf16x8*>(&pk);
    }
    return P;
  };
  // ---- O^T += V^T P^T for the V block in the tile.  Slot (ks, hh, e) is token
  // 16 ks + 8 (e / 4) + 4 hh + e % 4: per transposing read, 4 consecutive token rows x 16 columns
  // per 16-lane block.
  auto pv_block = [&](const PBlock& P) {
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) {
        s16x4 part[2];
#pragma unroll
        for (int e4 = 0; e4 < 2; ++e4)
          part[e4] = lds_read_tr16(reinterpret_cast<const uint16_t*>(vrd[mt] + (16 * ks + 8 * e4) * 256));
        u32x4 a4;
        a4[0] = reinterpret_cast<const uint32_t*>(&part[0])[0];
        a4[1] = reinterpret_cast<const uint32_t*>(&part[0])[1];
        a4[2] = reinterpret_cast<const uint32_t*>(&part[1])[0];
        a4[3] = reinterpret_cast<const uint32_t*>(&part[1])[1];
        O[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(&a4), P.ks[ks], O[mt], 0, 0, 0);
      }
    }
  };

  // ---- the wave's first block and, if it has one, its second: S of both, ONE softmax over the 64
  // tokens (nothing to rescale), then P V of the first as soon as its V is there and P V of the
  // second when the very last load has arrived -- all that is left to do at that point.  Written
  // once per (has1, has2) case, as straight-line code of its own: how many loads stand behind the
  // one that is waited for is a constant only inside one case.
  u32x4 probe_acc = u32x4{0u, 0u, 0u, 0u};
  auto first_blocks = [&](auto h1, auto h2) {
    DmaRows d{};
    u32x4 patch_k = u32x4{0u, 0u, 0u, 0u}, patch_v = u32x4{0u, 0u, 0u, 0u};  // deferred rows of the first block (lane: row lane / 16 of the run)
    int patch_row = -1;                                        // this lane's row of the block, -1: none
    if constexpr (h1.value) {
      d = dma_rows(w);
      if (d.patch) {
        if ((lane >> 4) < d.n_pend) {
          patch_row = d.first_pend + (lane >> 4);
          bool pn;
          const long long o = src_of(w * kBlock + patch_row, pn) + piece * 16;  // in k_new / v_new
          patch_k = *reinterpret_cast<const u32x4*>(kpend + o);
          patch_v = *reinterpret_cast<const u32x4*>(vpend + o);
        }
        __builtin_amdgcn_sched_barrier(0);                     // ahead of the block: loads return in issue order
      }
      dma_half(w, d, std::false_type{});                       // K1 -> tile
      __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (h2.value) {
      load_half(br.k, w + 4, std::false_type{});               // K2 -> registers
      __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (h1.value) {
      dma_half(w, d, std::true_type{});                        // V1 -> tile
      __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (h2.value) {
      load_half(br.v, w + 4, std::true_type{});                // V2 -> registers
      __builtin_amdgcn_sched_barrier(0);
    }
    PASTA_CLK(1);
    // Q has landed once at most the block loads issued behind it are outstanding
    wait_vmcnt<h2.value ? 32 : (h1.value ? 16 : 0)>();
    report_rows();
    lds_barrier();  // Q visible to every wave; the only barrier before the end of the item, and it
                    // does not wait for the block loads still in flight
    PASTA_CLK(2);
    if constexpr (PROBE) {  // read-only form: the same requests, nothing computed
      wait_vmcnt<0>();
      tile_sync();
      if constexpr (h1.value) probe_acc = probe_acc ^ ktw[lane] ^ vtw[lane];
      if constexpr (h2.value) {
#pragma unroll
        for (int i = 0; i < 8; ++i) probe_acc = probe_acc ^ br.k[i] ^ br.v[i];
      }
    } else if constexpr (h1.value) {
      wait_vmcnt<h2.value ? 24 : 8>();                          // K1 is in the tile
      tile_sync();
      if (d.patch) {
        if (patch_row >= 0) ktw[patch_row * 16 + (piece ^ (patch_row & 15))] = patch_k;
        tile_sync();
      }
      PASTA_CLK(3);
      f32x16 S1 = s_block(w);
      float mx = row_max(S1);
      f32x16 S2;
      if constexpr (h2.value) {
        tile_sync();
        regs_to_tile(br.k, std::false_type{});                  // K2 over K1 (LDS operations of a wave stay in order)
        tile_sync();
        S2 = s_block(w + 4);
        mx = fmaxf(mx, row_max(S2));
      }
      mx = fmaxf(mx, __shfl_xor(mx, 32, kWave)) * p.scale_log2e;
      m_run = mx;                                               // -inf: the row sees nothing here (dense-mask mode)
      const float mref = mx == -INFINITY ? 0.f : mx;
      float ps = 0.f;
      const PBlock P1 = exp_pack(S1, mref, ps);
      PBlock P2;
      if constexpr (h2.value) P2 = exp_pack(S2, mref, ps);
      l_run = ps;
      PASTA_CLK(5);
      wait_vmcnt<h2.value ? 8 : 0>();                           // V1 is in the tile
      tile_sync();
      if (d.patch) {
        if (patch_row >= 0) vtw[patch_row * 16 + (piece ^ v_swizzle(patch_row))] = patch_v;
        tile_sync();
      }
      pv_block(P1);
      PASTA_CLK(4);
      if constexpr (h2.value) {
        tile_sync();
        regs_to_tile(br.v, std::true_type{});                   // V2 over V1
        tile_sync();
        if (LONG && w + 8 < n_blocks) load_block(br, w + 8, std::true_type{});
        pv_block(P2);
      }
      tile_sync();
    }
  };
  // a later block (long chunks only): registers -> tile, the block after it requested, online softmax
  auto later_block = [&](int b) {
    regs_to_tile(br.k, std::false_type{});
    regs_to_tile(br.v, std::true_type{});
    tile_sync();
    if (b + 4 < n_blocks) load_block(br, b + 4, std::true_type{});  // in flight while this block is computed
    f32x16 S = s_block(b);
    // online softmax in log2 units; the scale (> 0) is applied inside the exponent: 2^(s z - m)
    float mx = row_max(S);
    mx = fmaxf(mx, __shfl_xor(mx, 32, kWave)) * p.scale_log2e;
    const float mn = fmaxf(m_run, mx);            // -inf while the row has seen nothing (dense-mask mode)
    const float mref = mn == -INFINITY ? 0.f : mn;
    const float corr = fast_exp2(m_run - mref);
    m_run = mn;
    float ps = 0.f;
    const PBlock P = exp_pack(S, mref, ps);
    l_run = l_run * corr + ps;
    if (!__all(corr == 1.f)) {  // the running max moves rarely once a few blocks are in
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) O[mt][i] *= corr;
    }
    pv_block(P);
    tile_sync();  // the tile may be overwritten by the next block
  };

  // this wave's blocks w, w + 4, ...
  if (has2) first_blocks(std::true_type{}, std::true_type{});
  else if (has1) first_blocks(std::true_type{}, std::false_type{});
  else first_blocks(std::false_type{}, std::false_type{});
  if constexpr (PROBE) {
    // What a plain read of this launch's bytes costs at this launch's shape (a measurement aid): every
    // wave has requested its blocks exactly as above and now only folds them together; later blocks of
    // long items follow through the registers.  The store below never happens for real data.
    if constexpr (LONG) {
      for (int b = w + 8; b < n_blocks; b += 4) {
        load_block(br, b, std::true_type{});
#pragma unroll
        for (int i = 0; i < 8; ++i) probe_acc = probe_acc ^ br.k[i] ^ br.v[i];
      }
    }
    if ((probe_acc[0] ^ probe_acc[1] ^ probe_acc[2] ^ probe_acc[3]) == 0x9E3779B9u && n_tok < 0)
      p.part_ml[part_row0] = make_float2(0.f, 0.f);
    PASTA_CLK(7);
    return;
  }
  if constexpr (LONG) {  // no other launch has items of more than eight blocks
    for (int b = w + 8; b < n_blocks; b += 4) later_block(b);
  }
  PASTA_CLK(6);

  // ---- combine the four waves.  Each wave parks its (unscaled) O^T in its OWN tile area as soon
  // as it is done -- [32 rows][32 pieces of 4 floats], piece c of row r at c ^ r -- so only one
  // barrier stands between the slowest wave and the output; the scales 2^(m_w - m) are applied
  // while adding.
  f32x4* otile = reinterpret_cast<f32x4*>(&lds.tile[w]);  // 1024 pieces = 16 KB
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int b4 = 0; b4 < 4; ++b4) {
      const int c = 8 * mt + 2 * b4 + hh;  // floats 32 mt + 8 b4 + 4 hh .. + 3 of row l32
      if (l32 < R) otile[l32 * 32 + (c ^ l32)] = f32x4{O[mt][4 * b4], O[mt][4 * b4 + 1], O[mt][4 * b4 + 2], O[mt][4 * b4 + 3]};
    }
  {
    const float lw = l_run + __shfl_xor(l_run, 32, kWave);
    if (hh == 0) { lds.mw[w][l32] = m_run; lds.lw[w][l32] = lw; }
  }
  __syncthreads();
  // Thread (rr = 8 pass + tid / 32, c = tid % 32) adds the four waves' 16-byte piece c of row rr.
  // Everything is read from LDS first, for all four passes and without a branch in between (rows
  // past R hold stale tile bytes: read, never stored), so the LDS latency is paid once.
  {
    const int r0 = tid >> 5, c = tid & 31;
    float mw4[4][4], lw4[4][4];
    f32x4 pc[4][4];
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) {
      if (pass * 8 >= R) break;  // (R is the same for the whole work-group: private items stop after one pass)
      const int rr = pass * 8 + r0;
      const f32x4* src = reinterpret_cast<const f32x4*>(&lds.tile[0]) + rr * 32 + (c ^ rr);  // + 1024 per wave
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        mw4[pass][k] = lds.mw[k][rr];
        lw4[pass][k] = lds.lw[k][rr];
        pc[pass][k] = src[1024 * k];
      }
    }
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) {
      if (pass * 8 >= R) break;
      const int rr = pass * 8 + r0;
      const float ma = fmaxf(fmaxf(mw4[pass][0], mw4[pass][1]), fmaxf(mw4[pass][2], mw4[pass][3]));
      const float mr = ma == -INFINITY ? 0.f : ma;  // -inf: the row saw nothing in this item (dense-mask mode)
      float sc[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) sc[k] = fast_exp2(mw4[pass][k] - mr);
      const f32x4 acc = pc[pass][0] * sc[0] + pc[pass][1] * sc[1] + pc[pass][2] * sc[2] + pc[pass][3] * sc[3];
      if (rr < R) {
        *reinterpret_cast<f32x4*>(p.part_acc + (part_row0 + rr) * D + 4 * c) = acc;
        if (c == 0) {  // one lane per row also writes (m, l)
          const float l_all = lw4[pass][0] * sc[0] + lw4[pass][1] * sc[1] + lw4[pass][2] * sc[2] + lw4[pass][3] * sc[3];
          p.part_ml[part_row0 + rr] = make_float2(ma, l_all);
        }
      }
    }
  }
  PASTA_CLK(7);
}

template <bool PAGED, bool PROBE>
__device__ __forceinline__ void attn_item_wide(const DecodeParams& p, AttnLds& lds, const int32_t* meta, int wi);

// One launch for all partials of a decode step; the shared-prefix items' work-groups come
// first, the private (gather) items' after them.
// DENSE = the variant that also carries the dense-mask comparison mode (p.dense_mask); the plain
// variant has none of that code.  LONG = the variant for launches with long items: its
// steady-state loop addresses plain blocks through buffer loads.  PROBE = the read-only form of the
// same launch (every request of the real one, no arithmetic, no output): what a plain read of these
// bytes costs with this split of the work.  WIDE = every request with a shared prefix has more than
// 32 stacked rows: the shared-prefix work-groups take four row groups each (attn_item_wide).
template <bool PAGED, bool DENSE, bool LONG = false, bool PROBE = false, bool WIDE = false>
__global__ __launch_bounds__(kAttnThreads, 2) void k_attn(DecodeParams p) {
  static_assert(!LONG || !DENSE, "the long-item variant exists for the list mode");
  static_assert(!WIDE || (!DENSE && !LONG), "the wide form replaces the shared-prefix items of the list mode");
  __shared__ AttnLds lds;
  const int32_t* meta = meta_of(p);
  // The deferred append's copy into the pool (K1's job).  No work-group of this launch reads those
  // pool rows -- lists that name them are served from k_pend / v_pend -- so the copy needs no
  // ordering against the rest of the launch.  Normally it is spread thin: work-group b moves
  // the 16 pieces of one (row, kv head) of K or V with its first 16 threads, which fetch them
  // here, carry them through their item, and store them at the very end -- nobody waits for it.
  u32x4 pend_val = u32x4{0u, 0u, 0u, 0u};
  int pend_u = -1;  // this thread's piece of the copy, -1: none
  const int pend_pieces = p.Hkv * 16;  // 16-byte pieces per row
  const int pend_total = 2 * p.pend_n * pend_pieces;
  auto pend_store = [&](int t, u32x4 val) {
    const bool is_v = t >= pend_total / 2;
    const int u = is_v ? t - pend_total / 2 : t;
    const int row = u / pend_pieces, gh = (u % pend_pieces) >> 4, pc16 = u & 15;
    char* base = reinterpret_cast<char*>(const_cast<void*>(is_v ? p.v : p.k));
    *reinterpret_cast<u32x4*>(base + (elem_off(p.lay, pend_dst_of(p)[row], gh) + pc16 * 8) * 2) = val;
  };
  auto pend_load = [&](int t) -> u32x4 {
    const bool is_v = t >= pend_total / 2;
    const int u = is_v ? t - pend_total / 2 : t;
    return reinterpret_cast<const u32x4*>(is_v ? p.v_pend : p.k_pend)[u];
  };
  if (p.pend_n > 0) {
    if (pend_total <= (int)gridDim.x * 16) {
      if (threadIdx.x < 16 && (int)blockIdx.x * 16 < pend_total) {
        pend_u = blockIdx.x * 16 + threadIdx.x;
        pend_val = pend_load(pend_u);
      }
    } else {  // few work-groups, many rows: all of it here and now
      for (int t = blockIdx.x * kAttnThreads + threadIdx.x; t < pend_total; t += gridDim.x * kAttnThreads) {
        pend_store(t, pend_load(t));
      }
    }
  }
  if constexpr (WIDE) {  // (the wide work-groups have no register to spare for carrying it, and are long enough not to care)
    if (pend_u >= 0) { pend_store(pend_u, pend_val); pend_u = -1; }
  }
  // shared-prefix items first: they are the longer ones (up to two blocks per wave against one)
  const int n_prefix_wgs = (int)gridDim.x - p.n_mfma_items * p.Hkv;  // a multiple of Hkv
  // (a raised wave priority for the shared-prefix items, so that the longer items issue their loads
  // first where a SIMD holds a wave of each kind, paid while the private items' compute was heavier;
  // with the present kernel it costs 0.25 us per launch and is gone)
  if ((int)blockIdx.x < n_prefix_wgs) {
    if constexpr (WIDE) attn_item_wide<PAGED, PROBE>(p, lds, meta, blockIdx.x);
    else attn_item<PAGED, false, DENSE, LONG, PROBE>(p, lds, meta, blockIdx.x);
  } else attn_item<PAGED, true, DENSE, LONG, PROBE, WIDE ? 1 : 0>(p, lds, meta, blockIdx.x - n_prefix_wgs);
  if (pend_u >= 0) pend_store(pend_u, pend_val);
}

// K2 for a request with MORE than 32 stacked rows (many streams, or a wide GQA group): the rows are
// served in groups of 32, and here the four waves of a work-group take one row group EACH over the
// same tokens.  Work item = (request, kv head, split-K chunk, four row groups).  A round is four
// 32-token blocks: wave w brings block 4 r + w into tile w (through its registers, requested one
// round ahead), a barrier publishes the four tiles, every wave computes all four blocks for its own
// 32 rows, a second barrier frees the tiles.  So the chunk crosses the memory system once per FOUR
// row groups (the row-group form of attn_item reads it once per group -- from L2, but the L2-to-CU
// traffic is what that form is bound by), and there is nothing to combine at the end: each wave
// owns its rows' (m, l, O) for the whole chunk.  Q stays in registers (the B operands of S^T = K Q^T,
// fetched once per item).
template <bool PAGED, bool PROBE>
__device__ __forceinline__ void attn_item_wide(const DecodeParams& p, AttnLds& lds, const int32_t* meta, int wi) {
  constexpr int D = 128;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hh = lane >> 5;
  const int G = p.Hq / p.Hkv;
  PASTA_CLK(0);

  // ---- decode the work item
  DevReq rq;
  const int32_t* req_streams = nullptr;
  if (p.single_req) {
    rq.req = p.req0.req; rq.pc = p.req0.pc; rq.n_streams = p.req0.n_streams; rq.stream0 = 0;
    rq.wg_begin = p.req0.wg_begin; rq.n_chunks = p.req0.n_chunks;
    rq.chunk_tokens = p.req0.chunk_tokens; rq.part_base = p.req0.part_base;
    rq.pend0 = p.req0.pend0; rq.pend_src0 = p.req0.pend_src0;
  } else {
    const DevReq* reqs = reinterpret_cast<const DevReq*>(meta + p.off_reqs);
    int qi = 0;
    for (; qi < p.n_reqs - 1; ++qi) {
      const int b = reqs[qi].wg_begin;
      if (wi >= b && wi < b + reqs[qi].n_chunks * p.Hkv * ((reqs[qi].n_streams * G + 127) >> 7)) break;
    }
    rq = reqs[qi];
    req_streams = meta + p.off_req_streams + rq.stream0;
  }
  const int R_all = rq.n_streams * G;
  const int n_quads = (R_all + 127) >> 7;
  const int wl = wi - rq.wg_begin;
  const int tq = wl / p.Hkv;
  const int c = __builtin_amdgcn_readfirstlane(tq / n_quads);
  const int quad = tq % n_quads;
  const int g = __builtin_amdgcn_readfirstlane(wl % p.Hkv);
  const int req = __builtin_amdgcn_readfirstlane(rq.req);
  const int row0 = __builtin_amdgcn_readfirstlane((quad * 4 + w) * 32);   // this WAVE's first stacked row
  const int R = __builtin_amdgcn_readfirstlane(max(0, min(32, R_all - row0)));  // 0: a wave that only carries tiles
  const int slot0 = __builtin_amdgcn_readfirstlane(c * rq.chunk_tokens);  // a multiple of 64
  const int n_tok = __builtin_amdgcn_readfirstlane(min(rq.chunk_tokens, rq.pc - slot0));
  const int n_blocks = (n_tok + kBlock - 1) / kBlock;
  const long long part_row0 = rq.part_base + (long long)(g * rq.n_chunks + c) * R_all + row0;
  const int pend0 = __builtin_amdgcn_readfirstlane(rq.pend0);  // slots from here on are rows of a deferred append
  const int pend_src0 = __builtin_amdgcn_readfirstlane(rq.pend_src0);

  const char* kb = reinterpret_cast<const char*>(p.k);
  const char* vb = reinterpret_cast<const char*>(p.v);
  const char* kpend = reinterpret_cast<const char*>(p.k_pend);
  const char* vpend = reinterpret_cast<const char*>(p.v_pend);
  const int piece = lane & 15, rbase = lane >> 4;

  // ---- Q: lane (row l32, half hh) holds pieces 2 kk + hh of its row, the B operand of step kk
  u32x4 qreg[8];
  {
    const int ra = row0 + l32;
    const bool live = l32 < R;
    const int s = live ? (req_streams ? req_streams[ra / G] : ra / G) : 0;
    const char* qrow = reinterpret_cast<const char*>(p.q) + (long long)(s * p.Hq + (g * G + (live ? ra % G : 0))) * (D * 2);
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      qreg[kk] = *reinterpret_cast<const u32x4*>(qrow + (2 * kk + hh) * 16);
      if (!live) qreg[kk] = u32x4{0u, 0u, 0u, 0u};  // rows past R are zero
    }
  }
  if (p.dbg_rows && g == 0 && quad == 0) {
    const DevStream* streams = reinterpret_cast<const DevStream*>(meta + p.off_streams);
    for (int j = tid; j < n_tok; j += kAttnThreads) {
      const int phys = phys_row(p.lay, p.page_table, req, slot0 + j);
      for (int k = 0; k < rq.n_streams; ++k)
        p.dbg_rows[streams[req_streams ? req_streams[k] : k].gather_base + slot0 + j] = phys;
    }
  }

  // ---- block loads: lane -> piece (lane & 15) of rows (lane >> 4) + 4 i.  A full block inside the
  // chunk is two runs of 16 consecutive slots, each inside one page (pages of 16 tokens or more):
  // wave-uniform base per run (page-table entries through scalar loads), lane part in the offset
  // register, row step in the scalar offset.  The chunk's ragged last block takes one address per row.
  const uint32_t row_bytes = (uint32_t)p.lay.slot_stride * 2u;
  const uint32_t lane_n = (uint32_t)rbase * row_bytes + (uint32_t)(piece * 16);
  const bool runs_ok = !PAGED || p.lay.page_shift >= 4;
  auto load_block = [&](BlockRegs& br, int b) {
    if (runs_ok && b * kBlock + kBlock <= n_tok && slot0 + b * kBlock + kBlock <= pend0) {
      int pp[2] = {0, 0};
      if constexpr (PAGED) {
#pragma unroll
        for (int hb = 0; hb < 2; ++hb)
          pp[hb] = scalar_load_i32(p.page_table, req * p.lay.pages_per_request + ((slot0 + b * kBlock + 16 * hb) >> p.lay.page_shift));
      }
#pragma unroll
      for (int hb = 0; hb < 2; ++hb) {
        const int t = slot0 + b * kBlock + 16 * hb;
        const int phys = PAGED ? ((pp[hb] << p.lay.page_shift) | (t & p.lay.page_mask)) : req * p.lay.pool_tokens + t;
        const long long off = elem_off(p.lay, phys, g) * 2;
        const __amdgpu_buffer_rsrc_t kr = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(kb + off), 0, 0x7fffffff, kRawBuffer);
        const __amdgpu_buffer_rsrc_t vr = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(vb + off), 0, 0x7fffffff, kRawBuffer);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          br.k[4 * hb + i] = __builtin_amdgcn_raw_buffer_load_b128(kr, lane_n, (uint32_t)(4 * i) * row_bytes, 0);
          br.v[4 * hb + i] = __builtin_amdgcn_raw_buffer_load_b128(vr, lane_n, (uint32_t)(4 * i) * row_bytes, 0);
        }
      }
      return;
    }
    long long off[8];
    bool pnd[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int t = slot0 + min(b * kBlock + rbase + 4 * i, n_tok - 1);  // rows past the end repeat the last one
      pnd[i] = t >= pend0;  // (a single stream that has not forked: its newest row is part of its prefix)
      const long long off_pool = elem_off(p.lay, pnd[i] ? 0 : phys_row(p.lay, p.page_table, req, t), g) * 2;
      const long long off_pend = ((long long)(pend_src0 + (t - pend0)) * p.Hkv + g) * D * 2;
      off[i] = (pnd[i] ? off_pend : off_pool) + piece * 16;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      br.k[i] = *reinterpret_cast<const u32x4*>((pnd[i] ? kpend : kb) + off[i]);
      br.v[i] = *reinterpret_cast<const u32x4*>((pnd[i] ? vpend : vb) + off[i]);
    }
  };
  BlockRegs br;
  const int n_rounds = (n_blocks + 3) >> 2;
  if (w < n_blocks) load_block(br, w);

  if constexpr (PROBE) {  // read-only form: the same requests, nothing computed
    u32x4 acc = u32x4{0u, 0u, 0u, 0u};
    for (int b = w; b < n_blocks; b += 4) {
      if (b != w) load_block(br, b);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc = acc ^ br.k[i] ^ br.v[i] ^ qreg[i];
    }
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9E3779B9u && n_tok < 0) p.part_ml[part_row0] = make_float2(0.f, 0.f);
    return;
  }

  f32x16 O[4];  // O^T M-tile mt: d = 32 mt + 8 (i / 4) + 4 hh + i % 4, row l32
  float m_run = -INFINITY, l_run = 0.f;
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int i = 0; i < 16; ++i) O[mt][i] = 0.f;

  u32x4* ktw = lds.tile[w].kt;
  u32x4* vtw = lds.tile[w].vt;
  // V^T reads (see attn_item): byte offset inside a tile's V half, per M-tile
  int vrd[4];
  {
    const int bl = lane & 15, cblk = (lane >> 4) & 1, r2 = bl >> 2;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
      vrd[mt] = (4 * hh + r2) * 256 + (mt ^ r2) * 64 + (2 * cblk + ((bl >> 1) & 1)) * 16 + (bl & 1) * 8;
  }
  // One block after the other, online softmax in log2 units.  (Two blocks per softmax step, their S^T chains
  // interleaved, took the same time: the launch is bound by what it has in flight, not by this chain.)
  auto block_compute = [&](int t, int b) {  // block b, in tile t, for this wave's rows
    const u32x4* kt = lds.tile[t].kt;
    const char* vt = reinterpret_cast<const char*>(lds.tile[t].vt);
    f32x16 S;
#pragma unroll
    for (int i = 0; i < 16; ++i) S[i] = 0.f;
    {
      u32x4 a[2];
      a[0] = kt[l32 * 16 + (hh ^ (l32 & 15))];
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        if (kk + 1 < 8) a[(kk + 1) & 1] = kt[l32 * 16 + ((2 * kk + 2 + hh) ^ (l32 & 15))];
        S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(&a[kk & 1]),
                                                    *reinterpret_cast<const bf16x8*>(&qreg[kk]), S, 0, 0, 0);
      }
    }
    if (b * kBlock + kBlock > n_tok) {  // the chunk's ragged last block: tokens past its end are hidden
      asm volatile("" ::: "memory");
      const int left = n_tok - (b * kBlock + 4 * hh);
#pragma unroll
      for (int i = 0; i < 16; ++i) S[i] = (8 * (i >> 2) + (i & 3)) < left ? S[i] : -INFINITY;
    }
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < 16; ++i) mx = fmaxf(mx, S[i]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, kWave)) * p.scale_log2e;  // finite: every block holds at least one token
    const float mn = fmaxf(m_run, mx);
    const float corr = fast_exp2(m_run - mn);
    m_run = mn;
    float ps = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      S[i] = fast_exp2(fmaf(S[i], p.scale_log2e, -mn));
      ps += S[i];
    }
    l_run = l_run * corr + ps;
    bf16x8 P[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      u32x4 pk;
      pk[0] = pack_bf16x2(S[8 * ks + 0], S[8 * ks + 1]);
      pk[1] = pack_bf16x2(S[8 * ks + 2], S[8 * ks + 3]);
      pk[2] = pack_bf16x2(S[8 * ks + 4], S[8 * ks + 5]);
      pk[3] = pack_bf16x2(S[8 * ks + 6], S[8 * ks + 7]);
      P[ks] = *reinterpret_cast<const bf16x8*>(&pk);
    }
    if (!__all(corr == 1.f)) {  // the running max moves rarely once a few blocks are in
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) O[mt][i] *= corr;
    }
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) {
        s16x4 part[2];
#pragma unroll
        for (int e4 = 0; e4 < 2; ++e4)
          part[e4] = lds_read_tr16(reinterpret_cast<const uint16_t*>(vt + vrd[mt] + (16 * ks + 8 * e4) * 256));
        u32x4 a4;
        a4[0] = reinterpret_cast<const uint32_t*>(&part[0])[0];
        a4[1] = reinterpret_cast<const uint32_t*>(&part[0])[1];
        a4[2] = reinterpret_cast<const uint32_t*>(&part[1])[0];
        a4[3] = reinterpret_cast<const uint32_t*>(&part[1])[1];
        O[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(&a4), P[ks], O[mt], 0, 0, 0);
      }
    }
  };

  for (int r = 0; r < n_rounds; ++r) {
    if (4 * r + w < n_blocks) {  // this wave's block of the round: registers -> its tile
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int rr = rbase + 4 * i;
        ktw[rr * 16 + (piece ^ (rr & 15))] = br.k[i];
        vtw[rr * 16 + (piece ^ v_swizzle(rr))] = br.v[i];
      }
    }
    if (4 * (r + 1) + w < n_blocks) load_block(br, 4 * (r + 1) + w);  // in flight while this round is computed
    lds_barrier();  // the round's tiles are complete (it does not wait for the loads just requested)
    if (r == 0) PASTA_CLK(1);
    if (r == 1) PASTA_CLK(2);
    if (R > 0) {
#pragma unroll
      for (int t = 0; t < 4; ++t)
        if (4 * r + t < n_blocks) block_compute(t, 4 * r + t);
    }
    lds_barrier();  // every wave is done with the tiles
    if (r == 0) PASTA_CLK(3);
    if (r == 1) PASTA_CLK(4);
  }
  PASTA_CLK(6);

  // ---- this wave's rows leave through its own tile: [32 rows][32 pieces of 4 floats], piece c of
  // row r at c ^ r, then 512-byte rows go out whole
  if (R > 0) {
    f32x4* otile = reinterpret_cast<f32x4*>(&lds.tile[w]);
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int b4 = 0; b4 < 4; ++b4) {
        const int cc = 8 * mt + 2 * b4 + hh;
        otile[l32 * 32 + (cc ^ l32)] = f32x4{O[mt][4 * b4], O[mt][4 * b4 + 1], O[mt][4 * b4 + 2], O[mt][4 * b4 + 3]};
      }
    const float l_all = l_run + __shfl_xor(l_run, 32, kWave);
    if (hh == 0 && l32 < R) p.part_ml[part_row0 + l32] = make_float2(m_run, l_all);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int pass = 0; pass < 16; ++pass) {
      const int rr = 2 * pass + hh, cc = l32;
      const f32x4 val = otile[rr * 32 + (cc ^ rr)];
      if (rr < R) *reinterpret_cast<f32x4*>(p.part_acc + (part_row0 + rr) * D + 4 * cc) = val;
    }
  }
  PASTA_CLK(7);
}

}  // namespace pasta
