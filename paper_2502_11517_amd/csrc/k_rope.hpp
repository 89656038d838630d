// Rotary position embedding by GIVEN position ids.  In PASTA a token decoded after a promise
// gets an estimated position id, because the asynchronous block before it has only a predicted
// length (arxiv 2502.11517, Section 4, "Training a PASTA-SFT model"; appendix "Positional
// Embedding"); the ids are the caller's, the rotation is the base model's.  It is applied
// where the data is touched anyway: to K on its way into the pool (K1), to Q on its way into
// the attention kernel.  Half-split planes over the whole head dim: plane f = (x[f], x[f + D/2])
// turns by position * theta^(-2f/D).
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

// The table in the workspace: D/2 entries theta^(-2f/D) / (2 pi), then, for D = 128, the same
// numbers factored as f = 8 a + b: 8 entries theta^(-16a/D) / (2 pi) and 8 entries theta^(-2b/D).
// The attention kernel uses the factors: the second set is the same for every lane (it sits in
// scalar registers), the first is one number per lane, so nothing of the table has to be
// fetched after the K/V loads have been issued.
constexpr int kRopeTabFactorA = 64;  // first index of the a-factors (D = 128)
constexpr int kRopeTabFactorB = 72;  // first index of the b-factors
constexpr int kRopeTabEntries = 80;

// One 16-byte piece of a bf16 head row with D = 128, for the attention kernel: plane indices
// 8 a .. 8 a + 7; fa = the a-factor of this piece, tab_b = the eight b-factors (uniform).
__device__ __forceinline__ void rope_piece_bf16_factored(const uint32_t (&own)[4], const uint32_t (&par)[4],
                                                         uint32_t (&out)[4], bool upper, int pos, double fa,
                                                         const double (&tab_b)[8]) {
  const double pa = (double)pos * fa;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    float r[2];
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
      const float x = hf ? bf16_hi(own[w]) : bf16_lo(own[w]);
      const float y = hf ? bf16_hi(par[w]) : bf16_lo(par[w]);
      const double rev = pa * tab_b[2 * w + hf];
      const float fr = (float)(rev - __builtin_floor(rev));
      const float c = __builtin_amdgcn_cosf(fr), s = __builtin_amdgcn_sinf(fr);
      r[hf] = upper ? x * c + y * s : x * c - y * s;
    }
    out[w] = (uint32_t)f32_to_bf16_rne(r[0]) | ((uint32_t)f32_to_bf16_rne(r[1]) << 16);
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

// Q of a decode step, rotated into a buffer of its own ([n][Hq][D], pool dtype): for the paths
// that do not rotate Q inside the attention kernel (fp32, D = 64, the vector-ALU walker).
// One thread per 16-byte piece.  DecodeParams comes first (the metadata may ride inside it).
__global__ __launch_bounds__(256) void k_rope_q(DecodeParams p, uint4* q_rot, int pieces_per_head, int is_f32) {
  const long long total = (long long)p.n_streams * p.Hq * pieces_per_head;
  const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= total) return;
  const int piece = (int)(t % pieces_per_head);
  const long long row = t / pieces_per_head;  // (stream, query head)
  const int s = (int)(row / p.Hq);
  const DevStream* streams = reinterpret_cast<const DevStream*>(meta_of(p) + p.off_streams);
  const uint4* src = reinterpret_cast<const uint4*>(p.q) + row * pieces_per_head;
  q_rot[t] = rope_row_piece(src, piece, pieces_per_head, is_f32 != 0, streams[s].pos, p.rope_tab);
}

}  // namespace pasta
