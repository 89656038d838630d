// K2 -- shared-prefix split-K partial attention on the matrix cores.
//
// Every stream forked from the same thread sees the same prefix rows of the pool
// (arxiv 2502.11517, Section 3, "Efficiency": a forked thread attends to the spawning
// thread's tokens that existed before the fork; the appendix on the naive interpreter
// names the cost of duplicating that prefix per thread).  Here the prefix K/V rows of one
// kv head are read from HBM ONCE per step and used for all R = n_streams * G query rows
// stacked together, which makes  S = Q_stack K^T  and  O = P V  small dense contractions.
//
// One work-group (4 wavefronts) = (request, kv head, split-K chunk).  Per 128-token tile:
//   * 128-bit coalesced global loads (16 lanes = one 256-byte row) into registers, issued
//     one tile ahead, then stored to LDS with a 16-byte XOR swizzle;
//   * wave w computes S^T for tokens 32w..32w+31 against all R rows with
//     v_mfma_f32_32x32x16_bf16 (A = K rows from LDS, B = Q rows from LDS), fp32 accumulate;
//   * the tile's row maxima are exchanged through LDS, so all waves share one running max;
//   * P = 2^(S - m) is rounded to bf16 and parked in LDS (over the dead K tile) in exactly
//     the B-operand order, and wave w accumulates O^T for head-dim slice 32w..32w+31 over
//     all 128 tokens (A = V^T gathered from LDS).  The token order inside a contraction step
//     is a free bijection; it is chosen so that P never has to be permuted.
// The chunk ends with one partial (m, l, acc[D]) per stacked row for the merge kernel.
// Logits are kept in log2 units.
#pragma once
#include "pasta_dev.hpp"

namespace pasta {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;  // a plain 16-byte register quad

constexpr int kPrefixMaxRows = 128;  // stacked query rows one work-group can carry (RT <= 4)

inline bool prefix_kernel_supports(int D, int G) { return D == 128 && G >= 1; }

template <int RT>
struct PrefixLds {
  u32x4 kt[kPrefixTile * 16];   // K tile [row][16 pieces], piece p of row r at p ^ (r & 15);
                                // reused for P: [rt][8 steps][2 halves][32 rows] pieces
  u32x4 vt[kPrefixTile * 16];   // V tile, same swizzle
  u32x4 q[RT * 32 * 16];        // stacked Q rows, same swizzle (rows >= R are zero)
  float tmax[4][RT * 32];       // per-wave row maxima of the current tile
  float lsum[4][RT * 32];       // per-wave row sums at the end of the chunk
};

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  f32x2 f = {a, b};
  bf16x2 h = __builtin_convertvector(f, bf16x2);  // v_cvt_pk_bf16_f32, round to nearest even
  return *reinterpret_cast<uint32_t*>(&h);
}

template <int RT, bool PAGED>
__global__ __launch_bounds__(256) void k_prefix(DecodeParams p) {
  constexpr int D = 128;
  __shared__ PrefixLds<RT> lds;
  const int tid = threadIdx.x;
  const int lane = tid & 63, w = tid >> 6;
  const int l32 = lane & 31, hh = lane >> 5;

  // ---- which (request, kv head, chunk)
  const DevReq* reqs = reinterpret_cast<const DevReq*>(p.meta + p.off_reqs);
  int qi = 0;
  for (; qi < p.n_reqs - 1; ++qi) {
    const int b = reqs[qi].wg_begin;
    if ((int)blockIdx.x >= b && (int)blockIdx.x < b + reqs[qi].n_chunks * p.Hkv) break;
  }
  const DevReq rq = reqs[qi];
  const int wl = blockIdx.x - rq.wg_begin;
  const int g = wl / rq.n_chunks, c = wl % rq.n_chunks;
  const int G = p.Hq / p.Hkv;
  const int R = rq.n_streams * G;
  const int tok0 = c * rq.chunk_tokens;
  const int tok1 = min(tok0 + rq.chunk_tokens, rq.pc);
  const int32_t* req_streams = p.meta + p.off_req_streams + rq.stream0;

  // ---- stacked Q rows -> LDS (row r = stream (r / G) of the request, query head g*G + r % G)
  {
    const u32x4* qg = reinterpret_cast<const u32x4*>(p.q);
#pragma unroll
    for (int i = 0; i < RT * 2; ++i) {
      const int idx = tid + i * 256;
      const int r = idx >> 4, piece = idx & 15;
      u32x4 val = {0u, 0u, 0u, 0u};
      if (r < R) {
        const int s = req_streams[r / G];
        val = qg[((long long)s * p.Hq + (g * G + r % G)) * 16 + piece];
      }
      lds.q[r * 16 + (piece ^ (r & 15))] = val;
    }
  }

  // ---- tile loads: thread -> piece (tid & 15) of rows (tid >> 4) + 16 i
  const char* kb = reinterpret_cast<const char*>(p.k);
  const char* vb = reinterpret_cast<const char*>(p.v);
  const int piece = tid & 15, rbase = tid >> 4;
  // row of logical slot t of this request (branch-free so that the tile's 16 loads issue together)
  auto row_of = [&](int t) -> int {
    if constexpr (PAGED) {
      const int pp = p.page_table[rq.req * p.lay.pages_per_request + (t >> p.lay.page_shift)];
      return (pp << p.lay.page_shift) | (t & p.lay.page_mask);
    } else {
      return rq.req * p.lay.pool_tokens + t;
    }
  };
  u32x4 kr[8], vr[8];
  auto load_tile = [&](int t0) {
    long long off[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int tok = min(t0 + rbase + 16 * i, tok1 - 1);  // rows past the end repeat the last one
      off[i] = (elem_off(p.lay, row_of(tok), g) + piece * 8) * 2;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      kr[i] = *reinterpret_cast<const u32x4*>(kb + off[i]);
      vr[i] = *reinterpret_cast<const u32x4*>(vb + off[i]);
    }
  };
  load_tile(tok0);

  if (p.dbg_rows && g == 0) {
    const DevStream* streams = reinterpret_cast<const DevStream*>(p.meta + p.off_streams);
    for (int t = tok0 + tid; t < tok1; t += 256) {
      const int phys = row_of(t);
      for (int j = 0; j < rq.n_streams; ++j) p.dbg_rows[streams[req_streams[j]].gather_base + t] = phys;
    }
  }

  f32x16 O[RT];
  float m_run[RT], l_run[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    m_run[rt] = -INFINITY;
    l_run[rt] = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) O[rt][i] = 0.f;
  }

  const uint16_t* vt16 = reinterpret_cast<const uint16_t*>(lds.vt);
  for (int t0 = tok0; t0 < tok1; t0 += kPrefixTile) {
    // registers -> LDS (rows rbase + 16 i all have (row & 15) == rbase)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      lds.kt[(rbase + 16 * i) * 16 + (piece ^ rbase)] = kr[i];
      lds.vt[(rbase + 16 * i) * 16 + (piece ^ rbase)] = vr[i];
    }
    __syncthreads();
    if (t0 + kPrefixTile < tok1) load_tile(t0 + kPrefixTile);  // next tile in flight

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
      const float mt = fmaxf(fmaxf(lds.tmax[0][r], lds.tmax[1][r]), fmaxf(lds.tmax[2][r], lds.tmax[3][r]));
      const float mn = fmaxf(m_run[rt], mt);  // finite: every tile holds a valid token
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
      for (int i = 0; i < 16; ++i) O[rt][i] *= corr;
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        u32x4 pk;
        pk[0] = pack_bf16x2(S[rt][8 * s + 0], S[rt][8 * s + 1]);
        pk[1] = pack_bf16x2(S[rt][8 * s + 2], S[rt][8 * s + 3]);
        pk[2] = pack_bf16x2(S[rt][8 * s + 4], S[rt][8 * s + 5]);
        pk[3] = pack_bf16x2(S[rt][8 * s + 6], S[rt][8 * s + 7]);
        pl[((rt * 8 + 2 * w + s) * 2 + hh) * 32 + l32] = pk;
      }
    }
    __syncthreads();  // P visible

    // ---- O^T[d slice of this wave][r] += V^T P^T over the tile's 128 tokens
    const int dcol = 32 * w + l32;            // head-dim index this lane supplies to A
    const int vpiece = dcol >> 3, vin = dcol & 7;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      // contraction slot (ks, hh, e) <-> token 32 (ks/2) + 8 (2 (ks%2) + e/4) + 4 hh + e%4
      uint32_t av[4];
#pragma unroll
      for (int e2 = 0; e2 < 4; ++e2) {
        uint32_t pr[2];
#pragma unroll
        for (int x = 0; x < 2; ++x) {
          const int e = 2 * e2 + x;
          const int tr = 32 * (ks >> 1) + 8 * (2 * (ks & 1) + (e >> 2)) + 4 * hh + (e & 3);
          pr[x] = vt16[(tr * 16 + (vpiece ^ (tr & 15))) * 8 + vin];
        }
        av[e2] = pr[0] | (pr[1] << 16);
      }
      const u32x4 a4 = {av[0], av[1], av[2], av[3]};
      const bf16x8 A = *reinterpret_cast<const bf16x8*>(&a4);
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        const u32x4 br = pl[((rt * 8 + ks) * 2 + hh) * 32 + l32];
        O[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, *reinterpret_cast<const bf16x8*>(&br), O[rt], 0, 0, 0);
      }
    }
    __syncthreads();  // tile buffers free for the next round
  }

  // ---- partial out: l summed over halves and waves; O^T lane (r, hh) holds d = 32w + 8b + 4hh + j
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const float lw = l_run[rt] + __shfl_xor(l_run[rt], 32, kWave);
    if (hh == 0) lds.lsum[w][rt * 32 + l32] = lw;
  }
  __syncthreads();
  const long long row0 = rq.part_base + (long long)(g * rq.n_chunks + c) * R;
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int r = rt * 32 + l32;
    if (r < R) {
      float* dst = p.part_acc + (row0 + r) * D + 32 * w + 4 * hh;
#pragma unroll
      for (int b = 0; b < 4; ++b)
        *reinterpret_cast<float4*>(dst + 8 * b) =
            make_float4(O[rt][4 * b], O[rt][4 * b + 1], O[rt][4 * b + 2], O[rt][4 * b + 3]);
      if (w == 0 && hh == 0)
        p.part_ml[row0 + r] = make_float2(m_run[rt], lds.lsum[0][r] + lds.lsum[1][r] + lds.lsum[2][r] + lds.lsum[3][r]);
    }
  }
}

inline int launch_prefix(int D, int G, int max_rows, dim3 grid, hipStream_t st, const DecodeParams& p) {
  (void)G;
  if (D != 128 || max_rows > kPrefixMaxRows) return PASTA_E_INVAL;
  const bool paged = p.lay.paged != 0;
  if (max_rows <= 32) {
    if (paged) k_prefix<1, true><<<grid, 256, 0, st>>>(p); else k_prefix<1, false><<<grid, 256, 0, st>>>(p);
  } else if (max_rows <= 64) {
    if (paged) k_prefix<2, true><<<grid, 256, 0, st>>>(p); else k_prefix<2, false><<<grid, 256, 0, st>>>(p);
  } else {
    if (paged) k_prefix<4, true><<<grid, 256, 0, st>>>(p); else k_prefix<4, false><<<grid, 256, 0, st>>>(p);
  }
  return PASTA_OK;
}

}  // namespace pasta
