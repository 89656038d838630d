// K4 -- log-sum-exp merge of the split partials.  Splitting a stream's visible set between
// the shared-prefix kernel's chunks and the private-segment items is this build's device;
// the identity used is  sum_t e^{z_t} v_t = sum_i e^{m_i} acc_i  over the parts i, so
//   m = max_i m_i,  l = sum_i l_i 2^{m_i - m},  out = sum_i acc_i 2^{m_i - m} / l
// (m in log2 units).  Parts with l_i = 0 (nothing visible in them) contribute nothing.
// One wavefront per (stream, query head); lanes own D/64 output elements.
#pragma once
#include "pasta_dev.hpp"

namespace pasta {

template <typename T, int D, int G>
__global__ __launch_bounds__(256) void k_merge(DecodeParams p) {
  constexpr int EPL = D / kWave;  // elements per lane (1 or 2)
  const int lane = threadIdx.x & (kWave - 1);
  const int wid = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (wid >= p.n_streams * p.Hq) return;
  const int s = wid / p.Hq, h = wid % p.Hq;
  const int g = h / G, gi = h % G;
  const DevStream st = reinterpret_cast<const DevStream*>(p.meta + p.off_streams)[s];
  const DevReq rq = reinterpret_cast<const DevReq*>(p.meta + p.off_reqs)[st.req_idx];
  const int R = rq.n_streams * G;
  const int n_pre = rq.n_chunks;
  const int n_parts = n_pre + (st.item_end - st.item_begin);
  auto part_row = [&](int i) -> int {
    if (i < n_pre) return rq.part_base + (g * rq.n_chunks + i) * R + st.local * G + gi;
    return p.priv_part_base + ((st.item_begin + (i - n_pre)) * p.Hkv + g) * G + gi;
  };

  float mx = -INFINITY;
  for (int i = lane; i < n_parts; i += kWave) {
    const float2 ml = p.part_ml[part_row(i)];
    if (ml.y > 0.f) mx = fmaxf(mx, ml.x);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, kWave));

  float L = 0.f, o[EPL];
#pragma unroll
  for (int x = 0; x < EPL; ++x) o[x] = 0.f;
  for (int i = 0; i < n_parts; ++i) {
    const int row = part_row(i);
    const float2 ml = p.part_ml[row];
    const float w = (ml.y > 0.f) ? fast_exp2(ml.x - mx) : 0.f;
    L += ml.y * w;
    const float* a = p.part_acc + (long long)row * D + lane * EPL;
    if (EPL == 2) {
      const float2 av = *reinterpret_cast<const float2*>(a);
      o[0] = fmaf(av.x, w, o[0]);
      o[EPL - 1] = fmaf(av.y, w, o[EPL - 1]);
    } else {
      o[0] = fmaf(a[0], w, o[0]);
    }
  }
  const float inv = 1.f / L;
  const long long ob = ((long long)s * p.Hq + h) * D + lane * EPL;
  if constexpr (sizeof(T) == 4) {
    float* out = reinterpret_cast<float*>(p.out) + ob;
#pragma unroll
    for (int x = 0; x < EPL; ++x) out[x] = o[x] * inv;
  } else {
    uint16_t* out = reinterpret_cast<uint16_t*>(p.out) + ob;
#pragma unroll
    for (int x = 0; x < EPL; ++x) out[x] = f32_to_bf16_rne(o[x] * inv);
  }
  if (p.lse && lane == 0) p.lse[(long long)s * p.Hq + h] = (mx + __log2f(L)) * kLn2;
}

}  // namespace pasta
