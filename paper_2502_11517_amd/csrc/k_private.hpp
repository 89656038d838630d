// K3, vector-ALU form -- per-stream private-segment partial attention (arxiv 2502.11517,
// Section 3, "Efficiency": a thread attends only to its own rows of the interleaved pool
// plus the spawning thread's rows that existed before the fork; Figure 2b/2c).  This form
// serves fp32 pools, D = 64, and the whole visible list when the matrix-core kernel is
// switched off; bf16 D = 128 private segments normally go through k_attn's gather items.
//
// One wavefront walks one work item = (stream, kv head, chunk of <= 128 tokens of the
// stream's private list).  The list is a sequence of (start, count, stride) ranges of
// logical slots; the wave first expands its chunk into physical rows in LDS, then streams
// the rows: a row of one kv head is D*e bytes = LPR lanes x 16 B, so one 128-bit load
// instruction per wave fetches 64/LPR whole rows.  Each LPR-lane group keeps its own online
// softmax state (m, l, acc) for the rows it sees, for all G query heads of the kv head; the
// dot products are reduced inside the group with lane shuffles, the groups are combined at
// the end, and the wave writes one partial (m, l, acc[D]) per query head for the merge.
// Logits are kept in log2 units (scale * log2 e folded into q).
#pragma once
#include "pasta_dev.hpp"

namespace pasta {

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int kVec = 4;
  static __device__ __forceinline__ void unpack(const uint4& r, float* f) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
    f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  }
};
template <> struct Elem<uint16_t> {  // bf16 bit patterns
  static constexpr int kVec = 8;
  static __device__ __forceinline__ void unpack(const uint4& r, float* f) {
    f[0] = bf16_lo(r.x); f[1] = bf16_hi(r.x); f[2] = bf16_lo(r.y); f[3] = bf16_hi(r.y);
    f[4] = bf16_lo(r.z); f[5] = bf16_hi(r.z); f[6] = bf16_lo(r.w); f[7] = bf16_hi(r.w);
  }
};

// sum over the LPR lanes of a row group (LPR a power of two, groups aligned)
template <int LPR>
__device__ __forceinline__ float group_sum(float x) {
#pragma unroll
  for (int off = 1; off < LPR; off <<= 1) x += __shfl_xor(x, off, kWave);
  return x;
}

struct PrivLds {
  int rows[4][kPrivChunk];          // physical rows of the chunk, per wave
  DevRange ranges[4][kPrivChunk];   // the ranges the chunk overlaps, per wave
};

template <typename T, int D, int G>
__device__ __forceinline__ void private_item(const DecodeParams& p, PrivLds& lds, int item_idx, int g) {
  constexpr int VEC = Elem<T>::kVec;
  constexpr int LPR = D / VEC;        // lanes per row
  constexpr int TPI = kWave / LPR;    // rows per wave load
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x >> 6;
  const int sub = lane / LPR, dl = lane % LPR;

  const int32_t* meta = meta_of(p);
  // the work item and the ranges it overlaps: from the blob, or -- device-resident lists -- derived from
  // the stream's record, the ranges picked among the candidates that the arena holds
  DevItem it;
  DevStream st;
  int r_first = 0, nr = 1;         // blob: ranges [r_first, r_first + nr) of the blob; device: candidates
  int tok_base = 0;                // index of the item's first token in the space that `cum` counts
  bool synth = false;              // the piece is plain slots [slot0, slot0 + cnt): no range to look up
  if (!p.dev_tables) {
    it = reinterpret_cast<const DevItem*>(meta + p.off_items)[item_idx];
    st = reinterpret_cast<const DevStream*>(meta + p.off_streams)[it.stream];
    r_first = it.range_first;
    nr = it.n_ranges;
    tok_base = it.tok_begin;
  } else {
    const int si = dev_stream_of_item(p, meta, item_idx);
    st = reinterpret_cast<const DevStream*>(meta + p.off_streams)[si];
    bool in_ranges;
    it = dev_item(p, st, si, item_idx, in_ranges);
    tok_base = it.tok_begin;
    synth = !in_ranges;
    if (in_ranges) r_first = dev_item_candidates(p, st, it.tok_begin, it.tok_count, kPrivChunk, nr);
  }
  const int cnt = it.tok_count;
  // where the item's rows go in the debug gather map
  const int gather0 = p.dev_tables ? it.gather_pos : st.gather_base + st.pc + it.tok_begin;

  if (synth) {
    if (lane == 0) lds.ranges[wave][0] = DevRange{it.slot0, cnt, 1, tok_base};
    nr = 1;
  } else if (!p.dev_tables) {
    const DevRange* ranges = reinterpret_cast<const DevRange*>(meta + p.off_ranges);
    for (int r = lane; r < nr; r += kWave) lds.ranges[wave][r] = ranges[r_first + r];
  } else {
    for (int r = lane; r < nr; r += kWave) lds.ranges[wave][r] = dev_range_at(p, st, r_first + r);
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

  // -- expand token index -> physical row
  for (int j = lane; j < cnt; j += kWave) {
    const int tok = tok_base + j;
    int lo = 0, hi = nr - 1;  // last range with cum <= tok
    while (lo < hi) {
      int mid = (lo + hi + 1) >> 1;
      if (lds.ranges[wave][mid].cum <= tok) lo = mid; else hi = mid - 1;
    }
    const DevRange rg = lds.ranges[wave][lo];
    const int slot = rg.start + (tok - rg.cum) * rg.stride;
    const int phys = phys_row(p.lay, p.page_table, st.req, slot);
    lds.rows[wave][j] = phys;
    if (p.dbg_rows && g == 0) p.dbg_rows[gather0 + j] = phys;
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

  // -- this lane's slice of the G query rows, pre-scaled
  float qv[G][VEC];
  {
    const char* qb = reinterpret_cast<const char*>(p.q);
#pragma unroll
    for (int i = 0; i < G; ++i) {
      const long long e = ((long long)it.stream * p.Hq + (g * G + i)) * D + dl * VEC;
      const uint4 raw = *reinterpret_cast<const uint4*>(qb + e * sizeof(T));
      Elem<T>::unpack(raw, qv[i]);
#pragma unroll
      for (int x = 0; x < VEC; ++x) qv[i][x] *= p.scale_log2e;
    }
  }

  float m[G], l[G], acc[G][VEC];
#pragma unroll
  for (int i = 0; i < G; ++i) {
    m[i] = -INFINITY; l[i] = 0.f;
#pragma unroll
    for (int x = 0; x < VEC; ++x) acc[i][x] = 0.f;
  }

  const char* kb = reinterpret_cast<const char*>(p.k);
  const char* vb = reinterpret_cast<const char*>(p.v);
  constexpr int UNR = 2;
  for (int base = 0; base < cnt; base += TPI * UNR) {
    uint4 kr[UNR], vr[UNR];
    bool valid[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int j = base + u * TPI + sub;
      valid[u] = j < cnt;
      const int row = lds.rows[wave][valid[u] ? j : cnt - 1];
      const long long off = (elem_off(p.lay, row, g) + dl * VEC) * (long long)sizeof(T);
      kr[u] = *reinterpret_cast<const uint4*>(kb + off);
      vr[u] = *reinterpret_cast<const uint4*>(vb + off);
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      float kf[VEC], vf[VEC];
      Elem<T>::unpack(kr[u], kf);
      Elem<T>::unpack(vr[u], vf);
#pragma unroll
      for (int i = 0; i < G; ++i) {
        float s = 0.f;
#pragma unroll
        for (int x = 0; x < VEC; ++x) s = fmaf(qv[i][x], kf[x], s);
        s = group_sum<LPR>(s);
        if (!valid[u]) s = -INFINITY;
        const float mn = fmaxf(m[i], s);
        // mn == -inf only while nothing valid has been seen: keep the state untouched
        const float corr = (mn == -INFINITY) ? 1.f : fast_exp2(m[i] - mn);
        const float pw = (mn == -INFINITY) ? 0.f : fast_exp2(s - mn);
        m[i] = mn;
        l[i] = l[i] * corr + pw;
#pragma unroll
        for (int x = 0; x < VEC; ++x) acc[i][x] = fmaf(pw, vf[x], acc[i][x] * corr);
      }
    }
  }

  // -- combine the TPI row groups of the wave
#pragma unroll
  for (int off = LPR; off < kWave; off <<= 1) {
#pragma unroll
    for (int i = 0; i < G; ++i) {
      const float om = __shfl_xor(m[i], off, kWave);
      const float ol = __shfl_xor(l[i], off, kWave);
      const float mn = fmaxf(m[i], om);
      const float a = (mn == -INFINITY) ? 0.f : fast_exp2(m[i] - mn);
      const float b = (mn == -INFINITY) ? 0.f : fast_exp2(om - mn);
      m[i] = mn;
      l[i] = l[i] * a + ol * b;
#pragma unroll
      for (int x = 0; x < VEC; ++x) {
        const float oa = __shfl_xor(acc[i][x], off, kWave);
        acc[i][x] = acc[i][x] * a + oa * b;
      }
    }
  }

  if (sub == 0) {
    const int row0 = p.priv_part_base + (item_idx * p.Hkv + g) * G;
#pragma unroll
    for (int i = 0; i < G; ++i) {
      float* dst = p.part_acc + (long long)(row0 + i) * D + dl * VEC;
#pragma unroll
      for (int x = 0; x < VEC; x += 4)
        *reinterpret_cast<float4*>(dst + x) = make_float4(acc[i][x], acc[i][x + 1], acc[i][x + 2], acc[i][x + 3]);
      if (dl == 0) p.part_ml[row0 + i] = make_float2(m[i], l[i]);
    }
  }
}

// stand-alone launch: 4 waves per work-group, one (item, kv head) per wave
template <typename T, int D, int G>
__global__ __launch_bounds__(256) void k_private(DecodeParams p) {
  __shared__ PrivLds lds;
  const int wid = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (wid >= p.n_items * p.Hkv) return;  // whole wave leaves; no block-wide barrier is used
  private_item<T, D, G>(p, lds, wid / p.Hkv, wid % p.Hkv);
}

}  // namespace pasta
