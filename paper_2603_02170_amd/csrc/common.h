// Shared device-side types and helpers for the SageBwd kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sage {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef unsigned short v8us __attribute__((ext_vector_type(8)));
typedef unsigned short v4us __attribute__((ext_vector_type(4)));

constexpr int kBlock = 64;  // B_q = B_kv: rows that share one quantisation scale

// ---------------------------------------------------------------------------
// Operand layouts written by the pre-pass.  Both cover a tensor X^ [N, d] of one
// head as consecutive 1 KiB fragments of 64 lanes x 16 bytes, so that a wave loads
// an MFMA operand with one 16-byte access per lane at `lane * 16`.
//
// F  ("row fragments", contraction over d):
//    fragment (rb, s), rb = 32-row block, s = 32-channel step; lane (r, h), r = lane % 32,
//    h = lane / 32, byte t:   X^[32 rb + r][32 s + 16 h + t]
// TF ("transposed fragments", contraction over rows):
//    fragment (rb, cb), cb = 32-channel block; lane (c, h), byte t = 4a + b:
//    X^[32 rb + 8a + 4h + b][32 cb + c]
//    The row order 8a + 4h + b is the order in which a 32x32 MFMA accumulator holds
//    its rows (register 4a + b of lane half h), so a quantised accumulator tile is
//    directly the matching operand of the next MFMA.
// Fragment index within a head: rb * (d / 32) + (s or cb).
// ---------------------------------------------------------------------------

__device__ __forceinline__ float bf16_bits_to_float(unsigned short u) {
  return __uint_as_float(((unsigned)u) << 16);
}

// round-to-nearest-even float -> bf16 bits (finite inputs; NaN kept quiet)
__device__ __forceinline__ unsigned short float_to_bf16_bits(float f) {
  unsigned u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (unsigned short)(u >> 16);
}

// max over the two 32-lane halves of a wave, result in every lane
__device__ __forceinline__ int half_swap_max_i32(int v) {
  auto r = __builtin_amdgcn_permlane32_swap((unsigned)v, (unsigned)v, false, false);
  int a = (int)r[0], b = (int)r[1];
  return a > b ? a : b;
}
__device__ __forceinline__ float half_swap_max_f32(float v) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_swap_sum_f32(float v) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// max over all 64 lanes of a NON-NEGATIVE float (result in every lane).  Non-negative floats
// order like their bit patterns, so the reduction runs on unsigned integers: four DPP steps
// inside each row of 16 lanes (the `old` value 0 is the identity of an unsigned max, which lets the
// compiler fold each lane permutation into the max instruction), then the row and half-wave swaps
// of gfx950.  No LDS traffic.
__device__ __forceinline__ float wave_max_nonneg_f32(float v) {
  unsigned u = __float_as_uint(v);
  unsigned t;
  t = (unsigned)__builtin_amdgcn_update_dpp(0, (int)u, 0xB1, 0xf, 0xf, false);   // quad_perm [1,0,3,2]
  u = u > t ? u : t;
  t = (unsigned)__builtin_amdgcn_update_dpp(0, (int)u, 0x4E, 0xf, 0xf, false);   // quad_perm [2,3,0,1]
  u = u > t ? u : t;
  t = (unsigned)__builtin_amdgcn_update_dpp(0, (int)u, 0x141, 0xf, 0xf, false);  // row_half_mirror
  u = u > t ? u : t;
  t = (unsigned)__builtin_amdgcn_update_dpp(0, (int)u, 0x140, 0xf, 0xf, false);  // row_mirror
  u = u > t ? u : t;
  auto r16 = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  u = r16[0] > r16[1] ? r16[0] : r16[1];
  auto r32 = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  u = r32[0] > r32[1] ? r32[0] : r32[1];
  return __uint_as_float(u);
}

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// One 16-byte piece per lane, global -> LDS, no registers in between.  The LDS address is
// `lds_base + lane * 16` (the hardware adds the lane offset to the wave-uniform base).
__device__ __forceinline__ void async_copy_16(const void* gsrc_lane, void* lds_base) {
  __builtin_amdgcn_global_load_lds((gptr_t)gsrc_lane, (lptr_t)lds_base, 16, 0, 0);
}
__device__ __forceinline__ void async_copy_4(const void* gsrc_lane, void* lds_base) {
  __builtin_amdgcn_global_load_lds((gptr_t)gsrc_lane, (lptr_t)lds_base, 4, 0, 0);
}

// Immediate of `s_waitcnt vmcnt(n)` alone (the LDS / scalar and export counters are left at their
// maxima = no wait): the six bits of n sit in bits 3:0 and 15:14.
constexpr int vmcnt_only(int n) { return 0x0F70 | (n & 15) | ((n >> 4) << 14); }
// Keeps memory operations in program order across this point (for the compiler; no instruction).
__device__ __forceinline__ void compiler_fence() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
}

// Workgroup barrier that waits for this wave's LDS traffic only.  (__syncthreads() would
// also drain the asynchronous global->LDS copies that are meant to stay in flight.)
__device__ __forceinline__ void barrier_lds_only() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}
// Same, after all of this wave's global-memory operations (the async copies included).
__device__ __forceinline__ void barrier_all_memory() {
  __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0), as a builtin so the compiler's own wait tracking sees it
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Where row n of head bh = b * H + h of one of the caller's [.., N, d] tensors starts, in elements:
// dense [B, H, N, d] has strides (H N d, N d, d), token-major [B, N, H, d] has (N H d, d, H d).
struct RowView {
  size_t batch_stride, head_stride, row_stride;
  int H;
  __host__ __device__ size_t row(int bh, size_t n) const {
    return (size_t)(bh / H) * batch_stride + (size_t)(bh % H) * head_stride + n * row_stride;
  }
};

// Workgroup id -> (head, work item of the head).  Consecutive ids go round-robin over the 8 XCDs, so
// with a multiple of 8 heads every head's workgroups are given one XCD and share its L2.  The heads of
// an XCD are taken `head_set` at a time, and inside such a set the items go heaviest first over ALL its
// heads (item 0 of every head, then item 1, ...): with the causal mask the last workgroups to start
// are then the lightest of several heads, not of one.  That shortens the tail of short-sequence
// launches (13 % of the step at N = 2048); at N = 8192 the compute kernels lose 2 % to it (several
// heads' operands compete for the L2), so they take one head at a time there.
// Other head counts are laid out densely, head after head: no workgroup is without
// work (it would still queue for a whole workgroup's LDS and wave slots before it could exit) and a
// single head spreads over all XCDs instead of one.
struct WorkItem {
  int head, item;
};
// head_set > 0: that many heads of an XCD per set; head_set < 0: the dense layout (written as a set of
// one head on a machine of one XCD, so that the mapping below stays one formula)
__host__ __device__ inline int head_set_for(int items, int heads, bool always = false) {
  if (heads % 8 != 0) return -1;
  const int per_xcd = heads / 8;
  int hs = (always || items <= 32) ? 4 : 1;
  while (hs > 1 && per_xcd % hs != 0) hs >>= 1;
  return hs;
}
__host__ __device__ inline int grid_for(int heads, int items) { return heads * items; }
__device__ inline WorkItem work_item(int block, int items, int head_set) {
  const int xcds = head_set < 0 ? 1 : 8, hs = head_set < 0 ? 1 : head_set;
  const int xcd = block % xcds, slot = block / xcds;
  const int hset = slot / (items * hs), rem = slot % (items * hs);
  return WorkItem{xcd + xcds * (hset * hs + rem % hs), rem / hs};
}

}  // namespace sage
