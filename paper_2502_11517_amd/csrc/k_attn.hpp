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
// the stream's private list); the list's (start, count, stride) ranges are expanded to
// physical rows in LDS and the rows are gathered with the same 128-bit loads (16 lanes =
// one 256-byte row of one kv head).  Only the G query rows of that stream are live.
//
// Both kinds run the same tile loop in a work-group of two wavefronts, 64 tokens per tile:
//   * tile loads are issued one tile ahead into registers (16 x 16 B per lane), then stored
//     to LDS with a 16-byte XOR swizzle;
//   * wave w computes S^T for tokens 32w..32w+31 against all rows with
//     v_mfma_f32_32x32x16_bf16 (A = K rows, B = Q rows, both from LDS), fp32 accumulate;
//   * the tile's row maxima are exchanged through LDS so both waves share one running max
//     (lane shuffle across the two 32-lane halves, then LDS across waves);
//   * P = 2^(S - m) is rounded to bf16 and parked in LDS (over the dead K tile) in B-operand
//     order; wave w accumulates O^T for head-dim slice 64w..64w+63 over the tile's 64 tokens,
//     A = V^T read with the transposing LDS load.  The token order inside a contraction
//     step is a free bijection, chosen so that P needs no permutation.
// A work item ends with one partial (m, l, acc[D]) per live row for the merge kernel.
// Logits are kept in log2 units.
#pragma once
#include "pasta_dev.hpp"

namespace pasta {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;  // a plain 16-byte register quad

constexpr int kTile = 64;            // tokens per LDS tile
constexpr int kAttnThreads = 128;    // two wavefronts
constexpr int kAttnMaxRows = 128;    // stacked query rows one work-group can carry (RT <= 4)
constexpr int kGatherMax = 256;      // most tokens (and ranges) of one private work item

inline bool attn_kernel_supports(int D, int G) { return D == 128 && G >= 1; }

template <int RT>
struct AttnLds {
  u32x4 kt[kTile * 16];   // K tile [row][16 pieces], piece p of row r at p ^ (r & 15);
                          // reused for P: [rt][4 steps][2 halves][32 rows] pieces
  u32x4 vt[kTile * 16];   // V tile, same swizzle
  u32x4 q[RT * 32 * 16];  // stacked Q rows, same swizzle (rows >= R are zero)
  float tmax[2][RT * 32]; // per-wave row maxima of the current tile
  float lsum[2][RT * 32]; // per-wave row sums at the end of the item
  int rows[kGatherMax];          // gather items: physical row of every token of the item
  DevRange ranges[kGatherMax];   // gather items: the ranges the item overlaps
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
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (s16x4 __attribute__((address_space(3)))*)(uintptr_t)(const __attribute__((address_space(3))) uint16_t*)p);
}

template <int RT, bool PAGED, bool GATHER>
__device__ __forceinline__ void attn_item(const DecodeParams& p, AttnLds<RT>& lds, const int32_t* meta, int wi) {
  constexpr int D = 128;
  const int tid = threadIdx.x;
  const int lane = tid & 63, w = tid >> 6;
  const int l32 = lane & 31, hh = lane >> 5;
  const int G = p.Hq / p.Hkv;
  const DevStream* streams = reinterpret_cast<const DevStream*>(meta + p.off_streams);

  // ---- decode the work item
  int req, g, R, tok0, tok1, gather_base;
  long long part_row0;
  const int32_t* req_streams = nullptr;  // prefix: stream of stacked row r is req_streams[r / G]
  int q_stream = 0;                      // gather: the one stream
  int n_req_streams = 0;
  if constexpr (!GATHER) {
    const DevReq* reqs = reinterpret_cast<const DevReq*>(meta + p.off_reqs);
    int qi = 0;
    for (; qi < p.n_reqs - 1; ++qi) {
      const int b = reqs[qi].wg_begin;
      if (wi >= b && wi < b + reqs[qi].n_chunks * p.Hkv) break;
    }
    const DevReq rq = reqs[qi];
    const int wl = wi - rq.wg_begin;
    const int c = wl % rq.n_chunks;
    g = wl / rq.n_chunks;
    req = rq.req;
    R = rq.n_streams * G;
    n_req_streams = rq.n_streams;
    tok0 = c * rq.chunk_tokens;
    tok1 = min(tok0 + rq.chunk_tokens, rq.pc);
    req_streams = meta + p.off_req_streams + rq.stream0;
    part_row0 = rq.part_base + (long long)(g * rq.n_chunks + c) * R;
    gather_base = 0;
  } else {
    const int item = wi / p.Hkv;
    g = wi % p.Hkv;
    const DevItem it = reinterpret_cast<const DevItem*>(meta + p.off_items)[item];
    const DevStream st = streams[it.stream];
    req = st.req;
    R = G;
    q_stream = it.stream;
    tok0 = 0;
    tok1 = it.tok_count;
    part_row0 = p.priv_part_base + (long long)(item * p.Hkv + g) * G;
    gather_base = st.gather_base + st.pc + it.tok_begin;
    // ranges the item overlaps -> LDS, then every token of the item -> physical row
    const DevRange* ranges = reinterpret_cast<const DevRange*>(meta + p.off_ranges);
    int nr = st.range_end - it.range_first;
    if (nr > it.tok_count) nr = it.tok_count;
    for (int r = tid; r < nr; r += kAttnThreads) lds.ranges[r] = ranges[it.range_first + r];
    __syncthreads();
    for (int j = tid; j < it.tok_count; j += kAttnThreads) {
      const int tok = it.tok_begin + j;
      int lo = 0, hi = nr - 1;  // last range with cum <= tok
      while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (lds.ranges[mid].cum <= tok) lo = mid; else hi = mid - 1;
      }
      const DevRange rg = lds.ranges[lo];
      const int phys = phys_row(p.lay, p.page_table, req, rg.start + (tok - rg.cum) * rg.stride);
      lds.rows[j] = phys;
      if (p.dbg_rows && g == 0) p.dbg_rows[gather_base + j] = phys;
    }
    // the barrier that publishes lds.rows is the one after the Q store below
  }

  // ---- stacked Q rows -> LDS
  {
    const u32x4* qg = reinterpret_cast<const u32x4*>(p.q);
#pragma unroll
    for (int i = 0; i < RT * 4; ++i) {
      const int idx = tid + i * kAttnThreads;
      const int r = idx >> 4, piece = idx & 15;
      u32x4 val = {0u, 0u, 0u, 0u};
      if (r < R) {
        const int s = GATHER ? q_stream : req_streams[r / G];
        val = qg[((long long)s * p.Hq + (g * G + r % G)) * 16 + piece];
      }
      lds.q[r * 16 + (piece ^ (r & 15))] = val;
    }
  }
  if constexpr (GATHER) __syncthreads();

  // ---- tile loads: thread -> piece (tid & 15) of rows (tid >> 4) + 8 i
  const char* kb = reinterpret_cast<const char*>(p.k);
  const char* vb = reinterpret_cast<const char*>(p.v);
  const int piece = tid & 15, rbase = tid >> 4;  // rbase 0..7
  auto row_of = [&](int t) -> int {  // branch-free so that a tile's 16 loads issue together
    if constexpr (GATHER) {
      return lds.rows[t];
    } else if constexpr (PAGED) {
      const int pp = p.page_table[req * p.lay.pages_per_request + (t >> p.lay.page_shift)];
      return (pp << p.lay.page_shift) | (t & p.lay.page_mask);
    } else {
      return req * p.lay.pool_tokens + t;
    }
  };
  u32x4 kr[8], vr[8];
  auto load_tile = [&](int t0) {
    long long off[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int tok = min(t0 + rbase + 8 * i, tok1 - 1);  // rows past the end repeat the last one
      off[i] = (elem_off(p.lay, row_of(tok), g) + piece * 8) * 2;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      kr[i] = *reinterpret_cast<const u32x4*>(kb + off[i]);
      vr[i] = *reinterpret_cast<const u32x4*>(vb + off[i]);
    }
  };
  load_tile(tok0);

  if constexpr (!GATHER) {
    if (p.dbg_rows && g == 0) {
      for (int t = tok0 + tid; t < tok1; t += kAttnThreads) {
        const int phys = row_of(t);
        for (int j = 0; j < n_req_streams; ++j) p.dbg_rows[streams[req_streams[j]].gather_base + t] = phys;
      }
    }
  }

  f32x16 O[RT][2];  // O^T for d = 64 w + 32 mt + ..., rows r
  float m_run[RT], l_run[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    m_run[rt] = -INFINITY;
    l_run[rt] = 0.f;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i) O[rt][mt][i] = 0.f;
  }

  const uint16_t* vt16 = reinterpret_cast<const uint16_t*>(lds.vt);
  for (int t0 = tok0; t0 < tok1; t0 += kTile) {
    // registers -> LDS: row rbase + 8 i, piece ^ (row & 15)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = rbase + 8 * i;
      lds.kt[r * 16 + (piece ^ (r & 15))] = kr[i];
      lds.vt[r * 16 + (piece ^ (r & 15))] = vr[i];
    }
    __syncthreads();
    if (t0 + kTile < tok1) load_tile(t0 + kTile);  // next tile in flight

    // ---- S^T = K Q^T for this wave's 32 tokens
    f32x16 S[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
      for (int i = 0; i < 16; ++i) S[rt][i] = 0.f;
    const int krow = 32 * w + l32;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const int pc = (2 * kk + hh) ^ (l32 & 15);
      const u32x4 ar = lds.kt[krow * 16 + pc];
      const bf16x8 A = *reinterpret_cast<const bf16x8*>(&ar);
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        const u32x4 br = lds.q[(rt * 32 + l32) * 16 + pc];
        S[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, *reinterpret_cast<const bf16x8*>(&br), S[rt], 0, 0, 0);
      }
    }
    // scale to log2 units, mask the ragged end, wave-level row max
    // S^T register i of lane (r, hh) is token 32 w + 8 (i / 4) + 4 hh + i % 4
    const int tok_lane0 = t0 + 32 * w + 4 * hh;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      float mx = -INFINITY;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int tok = tok_lane0 + 8 * (i >> 2) + (i & 3);
        const float s = tok < tok1 ? S[rt][i] * p.scale_log2e : -INFINITY;
        S[rt][i] = s;
        mx = fmaxf(mx, s);
      }
      mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
      if (hh == 0) lds.tmax[w][rt * 32 + l32] = mx;
    }
    __syncthreads();  // K tile is dead from here on; tmax visible

    // ---- P = 2^(S - m), parked in LDS in B-operand order; rescale O
    u32x4* pl = lds.kt;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const int r = rt * 32 + l32;
      const float mn = fmaxf(m_run[rt], fmaxf(lds.tmax[0][r], lds.tmax[1][r]));  // finite: a tile holds a valid token
      const float corr = fast_exp2(m_run[rt] - mn);
      m_run[rt] = mn;
      float ps = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float e = fast_exp2(S[rt][i] - mn);
        S[rt][i] = e;
        ps += e;
      }
      l_run[rt] = l_run[rt] * corr + ps;
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) O[rt][mt][i] *= corr;
      // contraction step ks = 2 w + s holds this wave's registers 8 s .. 8 s + 7
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        u32x4 pk;
        pk[0] = pack_bf16x2(S[rt][8 * s + 0], S[rt][8 * s + 1]);
        pk[1] = pack_bf16x2(S[rt][8 * s + 2], S[rt][8 * s + 3]);
        pk[2] = pack_bf16x2(S[rt][8 * s + 4], S[rt][8 * s + 5]);
        pk[3] = pack_bf16x2(S[rt][8 * s + 6], S[rt][8 * s + 7]);
        pl[((rt * 4 + 2 * w + s) * 2 + hh) * 32 + l32] = pk;
      }
    }
    __syncthreads();  // P visible

    // ---- O^T[d slice of this wave][r] += V^T P^T over the tile's 64 tokens.
    // Contraction slot (ks, hh, e) is token 32 (ks / 2) + 16 (ks % 2) + 8 (e / 4) + 4 hh + e % 4.
    // Lane (dd, hh) of M-tile mt needs V[those 8 tokens][64 w + 32 mt + dd]: two transposing
    // reads, each over 4 consecutive token rows x 16 columns per 16-lane block.
    const int bl = lane & 15;                 // lane inside its 16-lane block
    const int cblk = (lane >> 4) & 1;         // which 16 columns of the 32-wide M-tile
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bf16x8 A[2];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        s16x4 part[2];
#pragma unroll
        for (int e4 = 0; e4 < 2; ++e4) {
          const int trow = 32 * (ks >> 1) + 16 * (ks & 1) + 8 * e4 + 4 * hh + (bl >> 2);
          const int col = 64 * w + 32 * mt + 16 * cblk + 4 * (bl & 3);
          part[e4] = lds_read_tr16(vt16 + (trow * 16 + ((col >> 3) ^ (trow & 15))) * 8 + (col & 7));
        }
        u32x4 a4;
        a4[0] = reinterpret_cast<const uint32_t*>(&part[0])[0];
        a4[1] = reinterpret_cast<const uint32_t*>(&part[0])[1];
        a4[2] = reinterpret_cast<const uint32_t*>(&part[1])[0];
        a4[3] = reinterpret_cast<const uint32_t*>(&part[1])[1];
        A[mt] = *reinterpret_cast<const bf16x8*>(&a4);
      }
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        const u32x4 br = pl[((rt * 4 + ks) * 2 + hh) * 32 + l32];
        const bf16x8 B = *reinterpret_cast<const bf16x8*>(&br);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
          O[rt][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[mt], B, O[rt][mt], 0, 0, 0);
      }
    }
    __syncthreads();  // tile buffers free for the next round
  }

  // ---- partial out: l summed over halves and waves; O^T lane (r, hh), register i of M-tile
  // mt is d = 64 w + 32 mt + 8 (i / 4) + 4 hh + i % 4
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const float lw = l_run[rt] + __shfl_xor(l_run[rt], 32, kWave);
    if (hh == 0) lds.lsum[w][rt * 32 + l32] = lw;
  }
  __syncthreads();
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int r = rt * 32 + l32;
    if (r < R) {
      float* dst = p.part_acc + (part_row0 + r) * D + 64 * w + 4 * hh;
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int b = 0; b < 4; ++b)
          *reinterpret_cast<float4*>(dst + 32 * mt + 8 * b) =
              make_float4(O[rt][mt][4 * b], O[rt][mt][4 * b + 1], O[rt][mt][4 * b + 2], O[rt][mt][4 * b + 3]);
      if (w == 0 && hh == 0) p.part_ml[part_row0 + r] = make_float2(m_run[rt], lds.lsum[0][r] + lds.lsum[1][r]);
    }
  }
}

// One launch for all partials of a decode step: work-groups [0, n_priv_wgs) are private
// (gather) items -- they have the longer dependency chain, so they start first -- and the
// rest are shared-prefix items.
template <int RT, bool PAGED>
__global__ __launch_bounds__(kAttnThreads) void k_attn(DecodeParams p) {
  __shared__ AttnLds<RT> lds;
  const int32_t* meta = p.meta ? p.meta : p.inline_meta;
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
    if (paged) k_attn<1, true><<<grid, kAttnThreads, 0, st>>>(p); else k_attn<1, false><<<grid, kAttnThreads, 0, st>>>(p);
  } else if (max_rows <= 64) {
    if (paged) k_attn<2, true><<<grid, kAttnThreads, 0, st>>>(p); else k_attn<2, false><<<grid, kAttnThreads, 0, st>>>(p);
  } else {
    if (paged) k_attn<4, true><<<grid, kAttnThreads, 0, st>>>(p); else k_attn<4, false><<<grid, kAttnThreads, 0, st>>>(p);
  }
  return PASTA_OK;
}

}  // namespace pasta
