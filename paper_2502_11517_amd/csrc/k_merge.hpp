// K4 -- log-sum-exp merge of the split partials.  Splitting a stream's visible set between
// the shared-prefix chunks and the private-segment items is this build's device; the
// identity used is  sum_t e^{z_t} v_t = sum_i e^{m_i} acc_i  over the parts i, so
//   m = max_i m_i,  l = sum_i l_i 2^{m_i - m},  out = sum_i acc_i 2^{m_i - m} / l
// (m in log2 units).  Parts with l_i = 0 (nothing visible in them) contribute nothing.
// One work-group of 512 threads per (stream, query head): the threads form 512/D groups,
// group k sums parts k, k + 512/D, ... with one head-dim element per thread (a part's row is
// read as one coalesced 4D-byte line) and several loads in flight; the groups are then
// added through LDS.
#pragma once
#include "pasta_dev.hpp"

namespace pasta {

constexpr int kMergeThreads = 512;

template <typename T, int D, int G>
__global__ __launch_bounds__(kMergeThreads) void k_merge(DecodeParams p) {
  constexpr int NGRP = kMergeThreads / D;
  constexpr int UNR = 16;
  __shared__ float red[kMergeThreads / kWave];
  __shared__ float osum[NGRP][D];
  __shared__ float lsum[NGRP];
  const int tid = threadIdx.x;
  const int s = blockIdx.x / p.Hq, h = blockIdx.x % p.Hq;
  const int g = h / G, gi = h % G;
  const int32_t* meta = meta_of(p);
  const DevStream st = reinterpret_cast<const DevStream*>(meta + p.off_streams)[s];
  int R, n_pre, part_base;
  if (p.single_req) {  // scalars from the kernel arguments: one table look-up less
    R = p.req0.n_streams * G; n_pre = p.req0.n_chunks; part_base = p.req0.part_base;
  } else {
    const DevReq rq = reinterpret_cast<const DevReq*>(meta + p.off_reqs)[st.req_idx];
    R = rq.n_streams * G; n_pre = rq.n_chunks; part_base = rq.part_base;
  }
  const int n_parts = n_pre + (st.item_end - st.item_begin);
  const int pre0 = part_base + g * n_pre * R + st.local * G + gi;                // + i * R
  const int priv0 = p.priv_part_base + (st.item_begin * p.Hkv + g) * G + gi;     // + j * Hkv * G
  auto part_row = [&](int i) -> int {
    return i < n_pre ? pre0 + i * R : priv0 + (i - n_pre) * p.Hkv * G;
  };

  // ---- this thread's first batch of (m, l, acc) loads goes out before anything waits
  const int grp = tid / D, d = tid % D;
  float2 ml[UNR];
  float a[UNR];
  auto load_batch = [&](int i0) {
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int i = i0 + u * NGRP;
      const int row = part_row(i < n_parts ? i : i0);
      ml[u] = p.part_ml[row];
      a[u] = p.part_acc[(long long)row * D + d];
      if (i >= n_parts) ml[u].y = 0.f;
    }
  };
  if (grp < n_parts) load_batch(grp);

  // ---- global max over the parts that hold something
  float mx = -INFINITY;
  for (int i = tid; i < n_parts; i += kMergeThreads) {
    const float2 v = p.part_ml[part_row(i)];
    if (v.y > 0.f) mx = fmaxf(mx, v.x);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, kWave));
  if ((tid & 63) == 0) red[tid >> 6] = mx;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < kMergeThreads / kWave; ++i) mx = fmaxf(mx, red[i]);

  // ---- weighted sums, one head-dim element per thread, parts strided over the groups
  float o = 0.f, L = 0.f;
  for (int i0 = grp; i0 < n_parts; i0 += NGRP * UNR) {
    if (i0 != grp) load_batch(i0);
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const float wgt = (ml[u].y > 0.f) ? fast_exp2(ml[u].x - mx) : 0.f;
      L = fmaf(ml[u].y, wgt, L);
      o = fmaf(a[u], wgt, o);
    }
  }
  osum[grp][d] = o;
  if (d == 0) lsum[grp] = L;
  __syncthreads();
  if (grp == 0) {
#pragma unroll
    for (int k = 1; k < NGRP; ++k) { o += osum[k][d]; L += lsum[k]; }
    const long long ob = ((long long)s * p.Hq + h) * D + d;
    const float val = o / L;
    if constexpr (sizeof(T) == 4) reinterpret_cast<float*>(p.out)[ob] = val;
    else reinterpret_cast<uint16_t*>(p.out)[ob] = f32_to_bf16_rne(val);
    if (p.lse && d == 0) p.lse[(long long)s * p.Hq + h] = (mx + __log2f(L)) * kLn2;
  }
}

}  // namespace pasta
