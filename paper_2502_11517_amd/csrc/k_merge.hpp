// K4 -- log-sum-exp merge of the split partials.  Splitting a stream's visible set between
// the shared-prefix chunks and the private-segment items is this build's device; the
// identity used is  sum_t e^{z_t} v_t = sum_i e^{m_i} acc_i  over the parts i, so
//   m = max_i m_i,  l = sum_i l_i 2^{m_i - m},  out = sum_i acc_i 2^{m_i - m} / l
// (m in log2 units).  Parts with l_i = 0 (nothing visible in them) contribute nothing.
// One work-group of NT threads per (stream, query head): the threads form NT/D groups,
// group k takes parts k, k + NT/D, ... with one head-dim element per thread (a part's
// row is read as one coalesced 4D-byte line).  The kernel is a chain of memory round
// trips, kept to one (a step of one request with few streams: all the merge needs rides in the
// kernel arguments) or two (the stream's record, then all its parts in one list).  The maximum
// and the sum over the groups are taken by group 0 after one LDS exchange.
// NT = 1024 for steps with few output rows (they are a chain of latencies, and wide work-groups
// shorten it); with many rows the launch is bound by the rate at which wavefronts can be
// started, and NT = 256 starts a quarter as many.
#pragma once
#include "pasta_dev.hpp"

namespace pasta {

constexpr int kMergeThreads = 1024;      // few rows
constexpr int kMergeThreadsSmall = 256;  // many rows
constexpr int kMergeManyRows = 512;      // from this many (stream, query head) rows on: the small form

template <typename T, int D, int G, int NT>
__global__ __launch_bounds__(NT) void k_merge(DecodeParams p) {
  constexpr int kMergeThreads = NT;
  constexpr int NGRP = kMergeThreads / D;
  constexpr int UNR = 8;  // parts per thread and batch
  __shared__ float msum[NGRP];
  __shared__ float osum[NGRP][D];
  __shared__ float lsum[NGRP];
  const int tid = threadIdx.x;
  const int grp = tid / D, d = tid % D;
  // grid (Hkv, G, streams): the linear work-group index is (s * G + gi) * Hkv + g, whose remainder
  // mod Hkv is the kv head, as in the attention launch, so that with 8 kv heads the partials are
  // read on the XCD whose L2 holds them (three grid dimensions spare the kernel the divisions)
  const int g = blockIdx.x, gi = blockIdx.y, s = blockIdx.z;
  const int h = g * G + gi;
  const int32_t* meta = meta_of(p);
  const DevStream* stp = reinterpret_cast<const DevStream*>(meta + p.off_streams) + s;
  // The running state of this thread: max-free accumulation is not possible, so each batch
  // is folded with the running max of what the thread has seen (one more online softmax).
  // No early exit and no branch on the loaded values: with one, the compiler requests a part's
  // accumulator only after its (m, l) has arrived and been looked at -- two memory round trips
  // per batch instead of one.
  float m_t = -INFINITY, l_t = 0.f, o_t = 0.f;
  auto fold = [&](const float2* ml, const float* a, int n_valid) {
    float mb = m_t;
#pragma unroll
    for (int u = 0; u < UNR; ++u) mb = fmaxf(mb, (u < n_valid && ml[u].y > 0.f) ? ml[u].x : -INFINITY);
    const float mref = mb == -INFINITY ? 0.f : mb;  // nothing seen yet: every weight below is 0
    const float c = fast_exp2(m_t - mref);           // 0 when m_t was -inf
    l_t *= c;
    o_t *= c;
    m_t = mb;
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const float wgt = (u < n_valid && ml[u].y > 0.f) ? fast_exp2(ml[u].x - mref) : 0.f;
      l_t = fmaf(ml[u].y, wgt, l_t);
      o_t = fmaf(a[u], wgt, o_t);
    }
  };
  // parts [0, n_a) of kind A (row a0 + i * a_step), then parts [0, n_b) of kind B, as ONE list:
  // group grp takes list entries grp, grp + NGRP, ..., UNR of them per batch
  auto run = [&](int a0, int a_step, int n_a, int b0, int b_step, int n_b) {
    const int n = n_a + n_b;
    for (int i0 = grp; i0 < n; i0 += NGRP * UNR) {
      float2 ml[UNR];
      float a[UNR];
      const int n_valid = min(UNR, (n - i0 + NGRP - 1) / NGRP);
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        ml[u] = make_float2(-INFINITY, 0.f);
        a[u] = 0.f;
        if (u < n_valid) {  // the same in all lanes of a wave: a scalar branch, no load for what is not there
          const int i = i0 + u * NGRP;
          const int row = i < n_a ? a0 + i * a_step : b0 + (i - n_a) * b_step;
          ml[u] = p.part_ml[row];
          a[u] = p.part_acc[(long long)row * D + d];
        }
      }
      fold(ml, a, n_valid);
    }
  };
  // shared-prefix part i of this (stream, head): row pre0 + i * R; private part j: row priv0 + j * Hkv * G
  int pre0, n_pre, R, item_begin, n_priv;
  if (p.single_req == 2) {  // one request, few streams: everything rides in the kernel arguments -- one round trip
    const int32_t* si = s_items_of(p);
    item_begin = si[2 * s];
    n_priv = si[2 * s + 1];
    R = p.req0.n_streams * G;  // stream i is stacked-row block i
    n_pre = p.req0.n_chunks;
    pre0 = p.req0.part_base + s * G;
  } else {  // the stream's record first (it carries what the merge needs of its request), then all parts
    pre0 = stp->m_pre0;
    n_pre = stp->m_n_pre;
    R = stp->m_R;
    item_begin = stp->item_begin;
    n_priv = stp->item_end - item_begin;
  }
  run(pre0 + g * n_pre * R + gi, R, n_pre, p.priv_part_base + (item_begin * p.Hkv + g) * G + gi, p.Hkv * G, n_priv);

  // ---- the groups meet once: each leaves its (m, l, o) in LDS as it is, group 0 takes the common
  // max, rescales and adds (a group's m and l are the same for all its head-dim elements)
  osum[grp][d] = o_t;
  if (d == 0) { msum[grp] = m_t; lsum[grp] = l_t; }
  __syncthreads();
  if (grp == 0) {
    float mg[NGRP], mx = -INFINITY;
#pragma unroll
    for (int k = 0; k < NGRP; ++k) { mg[k] = msum[k]; mx = fmaxf(mx, mg[k]); }
    float o = 0.f, L = 0.f;
#pragma unroll
    for (int k = 0; k < NGRP; ++k) {
      const float c = (mg[k] == -INFINITY) ? 0.f : fast_exp2(mg[k] - mx);
      o = fmaf(osum[k][d], c, o);
      L = fmaf(lsum[k], c, L);
    }
    const long long ob = ((long long)s * p.Hq + h) * D + d;
    const float val = o / L;
    if constexpr (sizeof(T) == 4) reinterpret_cast<float*>(p.out)[ob] = val;
    else reinterpret_cast<uint16_t*>(p.out)[ob] = f32_to_bf16_rne(val);
    if (p.lse && d == 0) p.lse[(long long)s * p.Hq + h] = (mx + __log2f(L)) * kLn2;
  }
}

}  // namespace pasta
