// Small device-side tools of the matrix-core attention kernel: register vector types, bf16
// packing, the transposing LDS read, loads straight into LDS, explicit wait counts.
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

constexpr int kTile = 64;            // split-K chunk lengths are multiples of this many tokens
constexpr int kAttnThreads = 256;    // four wavefronts
constexpr int kGatherMax = 256;      // most tokens (and ranges) of one private work item

inline bool attn_kernel_supports(int D, int G) { return D == 128 && G >= 1; }

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

// A 32-bit word of read-only device memory at a wave-uniform address, through the scalar
// data path (s_load_dword): it neither occupies the vector-memory queue nor counts in vmcnt.
// Only for memory that no launch in flight writes (the page table).
__device__ __forceinline__ int32_t scalar_load_i32(const int32_t* ptr, int idx) {
  typedef const int32_t __attribute__((address_space(4))) * const_ptr;
  return ((const_ptr)(uintptr_t)ptr)[idx];
}

// Phase clocks for kernel tuning (compiled in only with -DPASTA_TUNING=2, which the library build never sets): thread 0 of every
// work-group stores the 100 MHz wall clock at a few points into the tail of the partials buffer.
#if defined(PASTA_TUNING) && PASTA_TUNING >= 2
#ifndef PASTA_CLK_WGS
#define PASTA_CLK_WGS 512  // work-groups that have a row of eight clocks
#endif
#define PASTA_CLK(n) do { if (threadIdx.x == 0 && blockIdx.x < PASTA_CLK_WGS) p.part_ml[p.clock_row0 + (long long)blockIdx.x * 8 + (n)] = \
    __builtin_bit_cast(float2, (unsigned long long)__builtin_amdgcn_s_memrealtime()); } while (0)
#else
#define PASTA_CLK(n) do {} while (0)
#endif

}  // namespace pasta
