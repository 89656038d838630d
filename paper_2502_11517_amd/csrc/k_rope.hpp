// Rotary position embedding by GIVEN position ids.  In PASTA a token decoded after a promise
// gets an estimated position id, because the asynchronous block before it has only a predicted
// length (arxiv 2502.11517, Section 4, "Training a PASTA-SFT model"; appendix "Positional
// Embedding"); the ids are the caller's, the rotation is the base model's.  It is applied to K
// on its way into the pool (K1) and, ahead of a decode step's attention launch, to Q and to the
// K rows of a deferred append (k_rope_prep).  Half-split planes over the whole head dim: plane
// f = (x[f], x[f + D/2]) turns by position * theta^(-2f/D).
//
// Precision: position * frequency reaches tens of thousands of radians, so the product is
// taken in fp64 from a table of theta^(-2f/D) / (2 pi) (fp64, D/2 entries, in the workspace)
// and reduced to a fraction of a revolution before it becomes fp32; the rotation itself is
// fp32, rounded once to the pool dtype.
#pragma once
#include "pasta_dev.hpp"

namespace pasta {

// FAST: the hardware's v_cos_f32 / v_sin_f32 (argument in revolutions), good to about 1e-6
// absolute -- ample under a bf16 rounding.  Otherwise the library's sincospi (about 1 ulp).
template <bool FAST>
__device__ __forceinline__ void rope_cos_sin(const double* tab, int f, int pos, float& c, float& s) {
  const double rev = (double)pos * tab[f];
  const float fr = (float)(rev - __builtin_floor(rev));
  if constexpr (FAST) {
    c = __builtin_amdgcn_cosf(fr);
    s = __builtin_amdgcn_sinf(fr);
  } else {
    sincospif(2.f * fr, &s, &c);
  }
}

// One 16-byte piece of a bf16 head row (8 elements, first plane index f0), `par` the piece D/2
// elements away; `upper` says that `own` holds the second components of its planes.
template <bool FAST>
__device__ __forceinline__ void rope_piece_bf16(const uint32_t (&own)[4], const uint32_t (&par)[4],
                                                uint32_t (&out)[4], bool upper, int f0, int pos,
                                                const double* tab) {
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    float r[2];
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
      const float x = hf ? bf16_hi(own[w]) : bf16_lo(own[w]);
      const float y = hf ? bf16_hi(par[w]) : bf16_lo(par[w]);
      float c, s;
      rope_cos_sin<FAST>(tab, f0 + 2 * w + hf, pos, c, s);
      r[hf] = upper ? x * c + y * s : x * c - y * s;
    }
    out[w] = (uint32_t)f32_to_bf16_rne(r[0]) | ((uint32_t)f32_to_bf16_rne(r[1]) << 16);
  }
}

// The same for an fp32 row: 4 elements per piece.
__device__ __forceinline__ void rope_piece_f32(const uint32_t (&own)[4], const uint32_t (&par)[4],
                                               uint32_t (&out)[4], bool upper, int f0, int pos,
                                               const double* tab) {
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const float x = __uint_as_float(own[w]), y = __uint_as_float(par[w]);
    float c, s;
    rope_cos_sin<false>(tab, f0 + w, pos, c, s);
    out[w] = __float_as_uint(upper ? x * c + y * s : x * c - y * s);
  }
}

// A piece of either dtype, addressed inside a [..][D] array of 16-byte pieces: `src` points at
// piece 0 of the head row, `piece` < pieces_per_head.
__device__ __forceinline__ uint4 rope_row_piece(const uint4* src, int piece, int pieces_per_head, bool is_f32,
                                                int pos, const double* tab) {
  const int half = pieces_per_head >> 1;
  const bool upper = piece >= half;
  const uint4 o = src[piece], q = src[upper ? piece - half : piece + half];
  const uint32_t own[4] = {o.x, o.y, o.z, o.w}, par[4] = {q.x, q.y, q.z, q.w};
  uint32_t out[4];
  const int f0 = (upper ? piece - half : piece) * (is_f32 ? 4 : 8);
  if (is_f32) rope_piece_f32(own, par, out, upper, f0, pos, tab);
  else rope_piece_bf16<true>(own, par, out, upper, f0, pos, tab);  // the same arithmetic wherever bf16 keys are turned
  return make_uint4(out[0], out[1], out[2], out[3]);
}

// What a decode step has to turn before its attention launch, in one small launch: the Q rows
// (into q_rot, [n][Hq][D]) and the K rows of a deferred rotating append (into k_rot,
// [pend_n][Hkv][D]; the attention launch then reads and copies those instead of the caller's
// unrotated rows).  One thread per 16-byte piece; pieces [0, n_q_pieces) are Q's.  Rotating
// inside the attention kernel was tried first and costs more than this launch: with loads that
// go straight into LDS in flight the compiler makes every other wait a wait for all of them.
// DecodeParams comes first (the metadata may ride inside it).
__global__ __launch_bounds__(256) void k_rope_prep(DecodeParams p, uint4* q_rot, uint4* k_rot, int pieces_per_head,
                                                  int is_f32, long long n_q_pieces) {
  const long long n_k_pieces = p.pend_rope ? (long long)p.pend_n * p.Hkv * pieces_per_head : 0;
  const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n_q_pieces + n_k_pieces) return;
  if (t < n_q_pieces) {
    const int piece = (int)(t % pieces_per_head);
    const long long row = t / pieces_per_head;  // (stream, query head)
    const int s = (int)(row / p.Hq);
    const DevStream* streams = reinterpret_cast<const DevStream*>(meta_of(p) + p.off_streams);
    const uint4* src = reinterpret_cast<const uint4*>(p.q) + row * pieces_per_head;
    q_rot[t] = rope_row_piece(src, piece, pieces_per_head, is_f32 != 0, streams[s].pos, p.rope_tab);
  } else {
    const long long u = t - n_q_pieces;
    const int piece = (int)(u % pieces_per_head);
    const long long rh = u / pieces_per_head;  // (deferred row, kv head)
    const int row = (int)(rh / p.Hkv);
    const uint4* src = reinterpret_cast<const uint4*>(p.k_pend) + rh * pieces_per_head;
    k_rot[u] = rope_row_piece(src, piece, pieces_per_head, is_f32 != 0, pend_pos_of(p)[row], p.rope_tab);
  }
}

}  // namespace pasta
