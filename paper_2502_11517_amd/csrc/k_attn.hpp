// K2 + K3 on the matrix cores, one launch.
//
// K2, shared prefix.  Every stream forked from the same thread sees the same prefix rows
// of the pool (arxiv 2502.11517, Section 3, "Efficiency": a forked thread attends to the
// spawning thread's tokens that existed before the fork; the appendix on the naive
// interpreter names the cost of duplicating that prefix per thread).  Here the prefix K/V
// rows of one kv head are read from HBM ONCE per step and used for all R = n_streams * G
// query rows stacked together, so  S = Q_stack K^T  and  O = P V  are small dense
// contractions.  Work item = (request, kv head, split-K chunk of the common prefix).
//
// K3, private segments.  A stream's own rows are interleaved with the other streams' rows
// in the pool (Section 3, "Efficiency"; Figure 2c).  Work item = (stream, kv head, chunk of
// the stream's private list).  A chunk that lies inside one (start, count, stride) range
// is addressed arithmetically; otherwise its ranges are expanded to physical rows in LDS.
// Rows are gathered with the same 128-bit loads (16 lanes = one 256-byte row of one kv
// head).  Only the G query rows of that stream are live.
//
// Both kinds run the same tile loop in a work-group of four wavefronts, 64 tokens per
// tile.  The loop is built around bytes in flight, because that is what bounds a decode
// step: every thread keeps TWO tiles of loads (16 x 16 B) outstanding in registers while
// the work-group computes on a third that sits in LDS.
//   * registers -> LDS with a 16-byte XOR swizzle;
//   * wave w computes S^T for tokens 16w..16w+15 against all rows with
//     v_mfma_f32_16x16x32_bf16 (A = K rows, B = Q rows, both from LDS), fp32 accumulate;
//   * row maxima: across the four 16-lane groups of a wave by lane shuffles, across the
//     waves through LDS, so the work-group shares one running max per row;
//   * P = 2^(S - m) is rounded to bf16 and written to LDS in B-operand order; wave w then
//     accumulates O^T for head-dim slice 32w..32w+31 over the tile's 64 tokens with
//     v_mfma_f32_32x32x16_bf16, A = V^T fetched with the transposing LDS read.
// A work item ends with one partial (m, l, acc[D]) per live row for the merge kernel.
// Logits are kept in log2 units.
#pragma once
#include "pasta_dev.hpp"

namespace pasta {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;  // a plain 16-byte register quad
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kTile = 64;            // tokens per LDS tile
constexpr int kAttnThreads = 256;    // four wavefronts
constexpr int kAttnMaxRows = 128;    // stacked query rows one work-group can carry (RT <= 4)
constexpr int kGatherMax = 256;      // most tokens (and ranges) of one private work item

inline bool attn_kernel_supports(int D, int G) { return D == 128 && G >= 1; }

template <int RT>
struct AttnLds {
  u32x4 kt[kTile * 16];     // K tile [row][16 pieces], piece p of row r at p ^ (r & 15); once
                            // S is done it holds P^T [rt][4 steps][2 halves][32 rows]: 8 tokens
                            // (16 B) each, RT * 4 KB
  u32x4 vt[kTile * 16];     // V tile, same swizzle
  u32x4 q[RT * 32 * 16];    // stacked Q rows, same swizzle (rows >= R are zero)
  float tmax[4][RT * 32];   // per-wave row maxima of the current tile
  float lsum[4][RT * 32];   // per-wave row sums at the end of the item
  int rows[kGatherMax];          // listed gather items: physical row of every token
  DevRange ranges[kGatherMax];   // listed gather items: the ranges the item overlaps
};

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  f32x2 f = {a, b};
  bf16x2 h = __builtin_convertvector(f, bf16x2);  // v_cvt_pk_bf16_f32, round to nearest even
  return *reinterpret_cast<uint32_t*>(&h);
}

// Transposing LDS read: within each 16-lane block, lane i receives element (i % 4) of the
// 8-byte datum addressed by block lane 4 e + i / 4, for e = 0..3.  With block lane j
// pointing at row (j / 4), columns 4 (j % 4).., lane i ends up with column i of 4 rows.
__device__ __forceinline__ s16x4 lds_read_tr16(const uint16_t* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)p);
}

// 16 bytes per lane from global memory straight into LDS (global_load_lds_dwordx4): lane l's
// datum lands at lds_base + 16 l, lds_base wave-uniform; counted by vmcnt like any load.
__device__ __forceinline__ void load_to_lds16(const void* src, void* lds_base) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                   (__attribute__((address_space(3))) void*)lds_base, 16, 0, 0);
}

// s_waitcnt vmcnt(N) alone (N < 64): vector-memory loads return in issue order, so this waits
// for every load except the N issued last.
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// Work-group barrier that orders LDS traffic only: unlike __syncthreads() it does not drain the
// vector-memory counter, so global loads issued before it stay in flight across it.  LDS filled
// by load_to_lds16 needs the matching wait_vmcnt before this barrier.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

struct TileRegs { u32x4 k[4], v[4]; };  // one thread's share of a 64-token tile

// Phase clocks for kernel tuning (compiled in only with -DPASTA_PHASE_CLOCKS): thread 0 of every
// work-group stores the 100 MHz wall clock at a few points into the tail of the partials buffer.
#ifdef PASTA_PHASE_CLOCKS
#define PASTA_CLK(n) do { if (threadIdx.x == 0 && blockIdx.x < 512) p.part_ml[p.clock_row0 + (long long)blockIdx.x * 8 + (n)] = \
    __builtin_bit_cast(float2, (unsigned long long)__builtin_amdgcn_s_memrealtime()); } while (0)
#else
#define PASTA_CLK(n) do {} while (0)
#endif

template <int RT, bool PAGED, bool GATHER>
__device__ __forceinline__ void attn_item(const DecodeParams& p, AttnLds<RT>& lds, const int32_t* meta, int wi) {
  constexpr int D = 128;
  constexpr int NT = 2 * RT;  // 16-row tiles of S^T
  const int tid = threadIdx.x;
  const int lane = tid & 63, w = tid >> 6;
  const int c16 = lane & 15, q4 = lane >> 4;   // S^T layout: row nt*16 + c16, tokens 16 w + 4 q4 + i
  const int l32 = lane & 31, hh = lane >> 5;   // O^T layout: row rt*32 + l32, half hh
  const int G = p.Hq / p.Hkv;
  PASTA_CLK(0);

  // ---- decode the work item.  Token j of the item is logical slot slot0 + j * stride of
  // request `req`, except for "listed" gather items, whose rows come from LDS.
  int req, g, R, n_tok, slot0, stride, gather_pos, pend0, pend_src0;
  long long part_row0;
  const int32_t* req_streams = nullptr;  // prefix, several requests: stacked row r is stream req_streams[r / G]
  int q_stream = 0;                      // gather: the one stream
  int n_req_streams = 0;
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
        if (wi >= b && wi < b + reqs[qi].n_chunks * p.Hkv) break;
      }
      rq = reqs[qi];
      req_streams = meta + p.off_req_streams + rq.stream0;
    }
    // kv head = work-group index mod Hkv: with 8 kv heads every work-group of head g (private
    // items included, their index is item * Hkv + g) lands on XCD g, whose L2 then holds all of
    // that head's partials for the merge
    const int wl = wi - rq.wg_begin;
    const int c = wl / p.Hkv;
    g = wl % p.Hkv;
    req = rq.req;
    R = rq.n_streams * G;
    n_req_streams = rq.n_streams;
    slot0 = c * rq.chunk_tokens;
    stride = 1;
    n_tok = min(rq.chunk_tokens, rq.pc - slot0);
    part_row0 = rq.part_base + (long long)(g * rq.n_chunks + c) * R;
    gather_pos = slot0;
    pend0 = rq.pend0;
    pend_src0 = rq.pend_src0;
  } else {
    const int item = wi / p.Hkv;
    g = wi % p.Hkv;
    const DevItem it = reinterpret_cast<const DevItem*>(meta + p.off_items)[item];
    req = it.req;
    R = G;
    q_stream = it.stream;
    n_tok = it.tok_count;
    slot0 = it.slot0;
    stride = it.stride;
    part_row0 = p.priv_part_base + (long long)(item * p.Hkv + g) * G;
    gather_pos = it.gather_pos;
    pend0 = it.pend0;
    pend_src0 = it.pend_src0;
    listed = it.n_ranges > 1;
    if (listed) {  // ranges the item overlaps -> LDS, then every token of the item -> physical row
      const DevRange* ranges = reinterpret_cast<const DevRange*>(meta + p.off_ranges);
      const int nr = it.n_ranges;
      for (int r = tid; r < nr; r += kAttnThreads) lds.ranges[r] = ranges[it.range_first + r];
      __syncthreads();
      for (int j = tid; j < n_tok; j += kAttnThreads) {
        const int tok = it.tok_begin + j;
        int lo = 0, hi = nr - 1;  // last range with cum <= tok
        while (lo < hi) {
          const int mid = (lo + hi + 1) >> 1;
          if (lds.ranges[mid].cum <= tok) lo = mid; else hi = mid - 1;
        }
        const DevRange rg = lds.ranges[lo];
        const int slot = rg.start + (tok - rg.cum) * rg.stride;
        const int phys = phys_row(p.lay, p.page_table, req, slot);
        // rows of a deferred append are kept as -(1 + row in k_pend)
        lds.rows[j] = slot >= pend0 ? -1 - (pend_src0 + (slot - pend0)) : phys;
        if (p.dbg_rows && g == 0) p.dbg_rows[gather_pos + j] = phys;
      }
      __syncthreads();
    }
  }
  const int n_tiles = (n_tok + kTile - 1) / kTile;

  // ---- tile loads: thread -> piece (tid & 15) of rows (tid >> 4) + 16 i, i < 4
  const char* kb = reinterpret_cast<const char*>(p.k);
  const char* vb = reinterpret_cast<const char*>(p.v);
  const int piece = tid & 15, rbase = tid >> 4;  // rbase 0..15
  const char* kpend = reinterpret_cast<const char*>(p.k_pend);
  const char* vpend = reinterpret_cast<const char*>(p.v_pend);
  auto phys_of = [&](int j) -> int {  // physical pool row of token j (not for listed items)
    const int t = slot0 + j * stride;
    if constexpr (PAGED) {
      const int pp = p.page_table[req * p.lay.pages_per_request + (t >> p.lay.page_shift)];
      return (pp << p.lay.page_shift) | (t & p.lay.page_mask);
    } else {
      return req * p.lay.pool_tokens + t;
    }
  };
  // Source of token j's row: the pool, or the rows of a deferred append.  Branch-free so that
  // a tile's loads issue together.  Returns the byte offset; is_pend picks the base.
  auto src_of = [&](int j, bool& is_pend) -> long long {
    const int t = slot0 + j * stride;
    int phys = phys_of(j);
    int pidx = pend_src0 + (t - pend0);
    is_pend = t >= pend0;
    if constexpr (GATHER) {
      const int code = lds.rows[j];  // j < kGatherMax; meaningful only for listed items
      if (listed) { is_pend = code < 0; pidx = -1 - code; phys = code; }
    }
    const long long off_pool = (elem_off(p.lay, is_pend ? 0 : phys, g) + piece * 8) * 2;
    const long long off_pend = (((long long)pidx * p.Hkv + g) * D + piece * 8) * 2;
    return is_pend ? off_pend : off_pool;
  };
  auto load_tile = [&](TileRegs& tr, int tile) {
    long long off[4];
    bool pnd[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int j = min(tile * kTile + rbase + 16 * i, n_tok - 1);  // rows past the end repeat the last one
      off[i] = src_of(j, pnd[i]);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      tr.k[i] = *reinterpret_cast<const u32x4*>((pnd[i] ? kpend : kb) + off[i]);
      tr.v[i] = *reinterpret_cast<const u32x4*>((pnd[i] ? vpend : vb) + off[i]);
    }
  };
  TileRegs ta, tb;
  load_tile(ta, 0);  // first: nothing else on the way to these loads
  if (n_tiles > 1) load_tile(tb, 1);
  PASTA_CLK(1);

  // ---- stacked Q rows -> LDS (loads issued behind the tiles', stored before them)
  {
    const u32x4* qg = reinterpret_cast<const u32x4*>(p.q);
    u32x4 qr[RT * 2];
#pragma unroll
    for (int i = 0; i < RT * 2; ++i) {
      const int idx = tid + i * kAttnThreads;
      const int r = idx >> 4, pc16 = idx & 15;
      qr[i] = u32x4{0u, 0u, 0u, 0u};
      if (r < R) {
        const int s = GATHER ? q_stream : (req_streams ? req_streams[r / G] : r / G);
        qr[i] = qg[((long long)s * p.Hq + (g * G + r % G)) * 16 + pc16];
      }
    }
#pragma unroll
    for (int i = 0; i < RT * 2; ++i) {
      const int idx = tid + i * kAttnThreads;
      const int r = idx >> 4, pc16 = idx & 15;
      lds.q[r * 16 + (pc16 ^ (r & 15))] = qr[i];
    }
  }

  if (p.dbg_rows && g == 0 && !listed) {  // listed items reported their rows while expanding
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

  f32x16 O[RT];                 // O^T: d = 32 w + 8 (i / 4) + 4 hh + i % 4, row rt*32 + l32
  float m_run[NT], l_run[NT];   // per 16-row tile: row nt*16 + c16 (l_run: this lane's tokens only)
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int i = 0; i < 16; ++i) O[rt][i] = 0.f;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) { m_run[nt] = -INFINITY; l_run[nt] = 0.f; }

  const uint16_t* vt16 = reinterpret_cast<const uint16_t*>(lds.vt);
  u32x4* pt = lds.kt;  // the K tile is dead once every wave has its S^T (barrier below)
  uint16_t* pt16 = reinterpret_cast<uint16_t*>(pt);

  auto compute_tile = [&](int t0) {
    // ---- S^T = K Q^T for this wave's 16 tokens: A = K[16 tok x 32 d], B = Q^T[32 d x 16 rows]
    f32x4 S[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) S[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int krow = 16 * w + c16;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const int pc = (4 * kk + q4) ^ c16;  // (krow & 15) == c16, and Q row (nt*16 + c16) & 15 == c16
      const u32x4 ar = lds.kt[krow * 16 + pc];
      const bf16x8 A = *reinterpret_cast<const bf16x8*>(&ar);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const u32x4 br = lds.q[(nt * 16 + c16) * 16 + pc];
        S[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, *reinterpret_cast<const bf16x8*>(&br), S[nt], 0, 0, 0);
      }
    }
    // scale to log2 units, mask the ragged end, wave-level row max
    const int tok_lane0 = t0 + 16 * w + 4 * q4;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      float mx = -INFINITY;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float s = (tok_lane0 + i) < n_tok ? S[nt][i] * p.scale_log2e : -INFINITY;
        S[nt][i] = s;
        mx = fmaxf(mx, s);
      }
      mx = fmaxf(mx, __shfl_xor(mx, 16, kWave));
      mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
      if (q4 == 0) lds.tmax[w][nt * 16 + c16] = mx;
    }
    __syncthreads();  // tmax visible; every wave is done with the K tile

    // ---- P = 2^(S - m) -> LDS in B-operand order; running sums; rescale O
    // contraction slot (ks, hh', e) of P V is token 16 ks + 8 hh' + e; this lane's 4 tokens
    // are ks = w, hh' = q4 / 2, e = 4 (q4 % 2) + i
    float corr[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int r = nt * 16 + c16;
      const float mt = fmaxf(fmaxf(lds.tmax[0][r], lds.tmax[1][r]), fmaxf(lds.tmax[2][r], lds.tmax[3][r]));
      const float mn = fmaxf(m_run[nt], mt);  // finite: every tile holds a valid token
      corr[nt] = fast_exp2(m_run[nt] - mn);
      m_run[nt] = mn;
      float e[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) e[i] = fast_exp2(S[nt][i] - mn);
      l_run[nt] = l_run[nt] * corr[nt] + (e[0] + e[1]) + (e[2] + e[3]);
      u32x2 pk;
      pk[0] = pack_bf16x2(e[0], e[1]);
      pk[1] = pack_bf16x2(e[2], e[3]);
      const int rt = nt >> 1, row32 = (nt & 1) * 16 + c16;
      *reinterpret_cast<u32x2*>(pt16 + ((((rt * 4 + w) * 2 + (q4 >> 1)) * 32 + row32) * 8 + 4 * (q4 & 1))) = pk;
    }
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      // this lane's O^T row is in 16-row tile 2 rt + ((lane >> 4) & 1); picked with a bit mask so
      // that the compiler keeps corr[] in registers instead of indexing it in scratch memory
      const uint32_t msk = 0u - (uint32_t)((lane >> 4) & 1);
      const float cr = __uint_as_float((__float_as_uint(corr[2 * rt + 1]) & msk) | (__float_as_uint(corr[2 * rt]) & ~msk));
#pragma unroll
      for (int i = 0; i < 16; ++i) O[rt][i] *= cr;
    }
    __syncthreads();  // P visible

    // ---- O^T[d = 32 w + dd][r] += V^T P^T over the tile's 64 tokens.
    // Lane (dd, hh) needs V[16 ks + 8 hh + e][32 w + dd], e < 8: two transposing reads, each
    // over 4 consecutive token rows x 16 columns per 16-lane block.
    const int bl = lane & 15;             // lane inside its 16-lane block
    const int cblk = (lane >> 4) & 1;     // which 16 columns of the 32-wide M-tile
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      s16x4 part[2];
#pragma unroll
      for (int e4 = 0; e4 < 2; ++e4) {
        const int trow = 16 * ks + 8 * hh + 4 * e4 + (bl >> 2);
        const int col = 32 * w + 16 * cblk + 4 * (bl & 3);
        part[e4] = lds_read_tr16(vt16 + (trow * 16 + ((col >> 3) ^ (trow & 15))) * 8 + (col & 7));
      }
      u32x4 a4;
      a4[0] = reinterpret_cast<const uint32_t*>(&part[0])[0];
      a4[1] = reinterpret_cast<const uint32_t*>(&part[0])[1];
      a4[2] = reinterpret_cast<const uint32_t*>(&part[1])[0];
      a4[3] = reinterpret_cast<const uint32_t*>(&part[1])[1];
      const bf16x8 A = *reinterpret_cast<const bf16x8*>(&a4);
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        const u32x4 br = pt[((rt * 4 + ks) * 2 + hh) * 32 + l32];
        O[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, *reinterpret_cast<const bf16x8*>(&br), O[rt], 0, 0, 0);
      }
    }
  };

  auto store_tile = [&](const TileRegs& tr) {  // rows rbase + 16 i all have (row & 15) == rbase
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      lds.kt[(rbase + 16 * i) * 16 + (piece ^ rbase)] = tr.k[i];
      lds.vt[(rbase + 16 * i) * 16 + (piece ^ rbase)] = tr.v[i];
    }
  };

  // two tiles of loads stay in flight while a third is computed on
  for (int t = 0; t < n_tiles; t += 2) {
    store_tile(ta);
    __syncthreads();
    if (t == 0) PASTA_CLK(2);
    if (t + 2 < n_tiles) load_tile(ta, t + 2);
    compute_tile(t * kTile);
    __syncthreads();  // tile buffers free
    if (t == 0) PASTA_CLK(3);
    if (t + 1 < n_tiles) {
      store_tile(tb);
      __syncthreads();
      if (t == 0) PASTA_CLK(4);
      if (t + 3 < n_tiles) load_tile(tb, t + 3);
      compute_tile((t + 1) * kTile);
      __syncthreads();
      if (t == 0) PASTA_CLK(5);
    }
  }
  PASTA_CLK(6);

  // ---- partial out: l summed over the wave's 16-lane groups and over the waves
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    float lw = l_run[nt];
    lw += __shfl_xor(lw, 16, kWave);
    lw += __shfl_xor(lw, 32, kWave);
    if (q4 == 0) lds.lsum[w][nt * 16 + c16] = lw;
  }
  // O^T goes through LDS (over the dead K/V tiles: 32 rows x 128 floats = 16 KB per row tile)
  // so that every partial row leaves as one coalesced 512-byte line.  The stores are
  // non-temporal: partials are read once, by the merge kernel, from another XCD, so there is
  // no point in leaving them dirty in this XCD's L2 for the end-of-kernel write-back.
  float* ot = reinterpret_cast<float*>(lds.kt);  // [32 rows][128 + 4 pad]
  constexpr int OTS = 132;
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    __syncthreads();  // rt == 0: lsum visible and tiles dead; rt > 0: previous row tile stored
#pragma unroll
    for (int b = 0; b < 4; ++b)
      *reinterpret_cast<f32x4*>(ot + l32 * OTS + 32 * w + 8 * b + 4 * hh) =
          f32x4{O[rt][4 * b], O[rt][4 * b + 1], O[rt][4 * b + 2], O[rt][4 * b + 3]};
    __syncthreads();
    // 256 threads = 8 rows x 32 lanes x 16 B per pass, 4 passes for the 32 rows
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) {
      const int rr = pass * 8 + (tid >> 5), r = rt * 32 + rr;
      if (r < R) {
        const f32x4 val = *reinterpret_cast<const f32x4*>(ot + rr * OTS + 4 * (tid & 31));
        __builtin_nontemporal_store(val, reinterpret_cast<f32x4*>(p.part_acc + (part_row0 + r) * D + 4 * (tid & 31)));
      }
    }
  }
  if (w == 0 && q4 == 0) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int r = nt * 16 + c16;
      if (r < R)
        p.part_ml[part_row0 + r] =
            make_float2(m_run[nt], lds.lsum[0][r] + lds.lsum[1][r] + lds.lsum[2][r] + lds.lsum[3][r]);
    }
  }
  PASTA_CLK(7);
}

// One launch for all partials of a decode step: work-groups [0, n_priv_wgs) are private
// (gather) items -- they have the longer dependency chain, so they start first -- and the
// rest are shared-prefix items.
template <int RT, bool PAGED>
__global__ __launch_bounds__(kAttnThreads, (RT == 1 ? 3 : (RT == 2 ? 2 : 1))) void k_attn(DecodeParams p) {
  __shared__ AttnLds<RT> lds;
  const int32_t* meta = meta_of(p);
  if (p.pend_n > 0) {
    // The deferred append's copy into the pool (K1's job).  No work-group of this launch reads
    // those pool rows -- lists that name them are served from k_pend / v_pend -- so the copy
    // needs no ordering against the rest of the launch.
    const int pieces = p.Hkv * 16;  // 16-byte pieces per row
    const int total = 2 * p.pend_n * pieces;
    const int32_t* dst = pend_dst_of(p);
    for (int t = blockIdx.x * kAttnThreads + threadIdx.x; t < total; t += gridDim.x * kAttnThreads) {
      const bool is_v = t >= total / 2;
      const int u = is_v ? t - total / 2 : t;
      const int row = u / pieces, gh = (u % pieces) >> 4, pc16 = u & 15;
      const u32x4 val = reinterpret_cast<const u32x4*>(is_v ? p.v_pend : p.k_pend)[u];
      char* base = reinterpret_cast<char*>(const_cast<void*>(is_v ? p.v : p.k));
      *reinterpret_cast<u32x4*>(base + (elem_off(p.lay, dst[row], gh) + pc16 * 8) * 2) = val;
    }
  }
  const int n_priv_wgs = p.n_mfma_items * p.Hkv;
  if ((int)blockIdx.x < n_priv_wgs)
    attn_item<1, PAGED, true>(p, reinterpret_cast<AttnLds<1>&>(lds), meta, blockIdx.x);
  else
    attn_item<RT, PAGED, false>(p, lds, meta, blockIdx.x - n_priv_wgs);
}

inline int launch_attn(int max_rows, dim3 grid, hipStream_t st, const DecodeParams& p) {
  if (max_rows > kAttnMaxRows) return PASTA_E_INVAL;
  const bool paged = p.lay.paged != 0;
  if (max_rows <= 32) {
    return PASTA_E_INVAL;  // served by k_attn_w
  } else if (max_rows <= 64) {
    if (paged) k_attn<2, true><<<grid, kAttnThreads, 0, st>>>(p); else k_attn<2, false><<<grid, kAttnThreads, 0, st>>>(p);
  } else {
    if (paged) k_attn<4, true><<<grid, kAttnThreads, 0, st>>>(p); else k_attn<4, false><<<grid, kAttnThreads, 0, st>>>(p);
  }
  return PASTA_OK;
}

}  // namespace pasta
