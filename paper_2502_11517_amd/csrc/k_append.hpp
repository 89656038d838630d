// K1 -- KV-append scatter (arxiv 2502.11517, Section 3, "Efficiency"; Figure 2c):
// every active thread's new K/V row goes to the next free slot of the shared pool, so rows
// of concurrently decoding threads end up in neighbouring slots.  A pure copy: each lane
// moves one 16-byte piece of one (row, kv head) from k_new/v_new to its pool position.
// With the rotary option the K pieces are turned by the row's position id on the way (V never).
#pragma once
#include "k_rope.hpp"

namespace pasta {

constexpr int kAppendInline = 32;  // destination rows that travel in the kernel arguments
constexpr int kPatchMax = 64;      // most entries of the device-resident lists one launch brings up to date

struct AppendParams {
  const uint4* k_new;   // [n_rows][Hkv][D] as 16-byte pieces
  const uint4* v_new;
  void* k;              // layer base
  void* v;
  const int32_t* dst_rows;           // physical row per appended row (device), or null:
  int32_t inline_rows[kAppendInline];  // then the rows are here
  Layout lay;
  int n_rows, Hkv;
  int pieces_per_head;  // D * elem_bytes / 16
  int elem_shift;       // log2(elem_bytes)
  // rotary embedding of K (rope_tab == nullptr: plain copy)
  const double* rope_tab;             // theta^(-2f/D) / (2 pi), f < D/2 (device)
  const int32_t* pos_rows;            // position id per appended row (device), or null:
  int32_t inline_pos[kAppendInline];  // then the ids are here
  // The append also extends the device-resident visibility lists (the lists that decode steps in
  // maintained mode read): entries of the range arena and of the range index that this call's rows
  // changed or created, computed by the host from its mirror.
  DevRange* arena;
  int32_t* cidx;
  int n_rpatch, n_cpatch;
  int32_t rp_idx[kPatchMax];
  DevRange rp_val[kPatchMax];
  int32_t cp_idx[kPatchMax];
  int32_t cp_val[kPatchMax];
};

static_assert(sizeof(AppendParams) <= 4096, "kernel arguments are limited to 4 KB");

__global__ __launch_bounds__(256) void k_append(AppendParams p) {
  const long long total = (long long)p.n_rows * p.Hkv * p.pieces_per_head;
  long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (t < p.n_rpatch) p.arena[p.rp_idx[t]] = p.rp_val[t];
  else if (t < p.n_rpatch + p.n_cpatch) p.cidx[p.cp_idx[t - p.n_rpatch]] = p.cp_val[t - p.n_rpatch];
  if (t >= 2 * total) return;
  const bool is_v = t >= total;
  if (is_v) t -= total;
  const int piece = (int)(t % p.pieces_per_head);
  const long long rh = t / p.pieces_per_head;
  const int g = (int)(rh % p.Hkv);
  const int row = (int)(rh / p.Hkv);
  const int phys = p.dst_rows ? p.dst_rows[row] : p.inline_rows[row];
  const long long off_bytes = (elem_off(p.lay, phys, g) << p.elem_shift) + (long long)piece * 16;
  uint4 val;
  if (p.rope_tab && !is_v) {
    const int pos = p.pos_rows ? p.pos_rows[row] : p.inline_pos[row];
    val = rope_row_piece(p.k_new + rh * p.pieces_per_head, piece, p.pieces_per_head, p.elem_shift == 2, pos,
                         p.rope_tab);
  } else {
    val = (is_v ? p.v_new : p.k_new)[t];
  }
  *reinterpret_cast<uint4*>(reinterpret_cast<char*>(is_v ? p.v : p.k) + off_bytes) = val;
}

// Carries a piece of a decode step's plan to the device inside its own kernel arguments: a plan too large
// for the attention launch's arguments, but small (a few KB: one fixed-size record per stream), gets to
// device memory this way in one or two tiny launches -- no copy engine, and no kernel reading host memory.
constexpr int kRelayWords = 960;
struct RelayParams {
  int32_t* dst;
  int n_words;
  int32_t words[kRelayWords];
};
static_assert(sizeof(RelayParams) <= 4096, "kernel arguments are limited to 4 KB");

__global__ __launch_bounds__(256) void k_meta_relay(RelayParams p) {
  typedef const char __attribute__((address_space(4))) * kernarg_ptr;
  kernarg_ptr ka = (kernarg_ptr)__builtin_amdgcn_kernarg_segment_ptr();
  const int32_t __attribute__((address_space(4)))* src =
      (const int32_t __attribute__((address_space(4)))*)(ka + __builtin_offsetof(RelayParams, words));
  for (int i = threadIdx.x; i < p.n_words; i += 256) p.dst[i] = src[i];
}

}  // namespace pasta
