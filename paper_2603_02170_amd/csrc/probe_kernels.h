// Machine probes for the roofline context (gfx950): what this GPU sustains on the two resources the
// attention kernels are priced against, measured with the same clocks, power limit and memory system
// they run under.  Not part of the method.
#pragma once

#include "common.h"

namespace sage {

// Dense MFMA issue: every wave runs `iters` rounds of four independent accumulator chains of the
// matrix instruction the attention kernels use (INT8 32x32x32, or bf16 32x32x16), operands held in
// registers, nothing else in the loop.  Two waves per SIMD.  The operands are lane-dependent random
// codes ANDed with `mask`: all ones for the figure that compares with real work; zero gives the same
// instruction stream on all-zero operands, which draws less power and shows what the clock then allows.
// Operations per wave: iters * 4 * 2 * 32 * 32 * K.
template <bool BF16>
__global__ void __launch_bounds__(256, 2) probe_mfma_kernel(int iters, int seed, int mask, int* sink) {
  const int lane = threadIdx.x & 63;
  unsigned x = (unsigned)(seed + lane * 0x9E3779B9u + blockIdx.x * 0x85EBCA6Bu) | 1u;
  auto next = [&]() {
    x ^= x << 13;
    x ^= x >> 17;
    x ^= x << 5;
    return x;
  };
  int total = 0;
  if constexpr (!BF16) {
    v4i a[2], b[2];
#pragma unroll
    for (int k = 0; k < 2; k++)
#pragma unroll
      for (int r = 0; r < 4; r++) {
        a[k][r] = (int)next() & mask;
        b[k][r] = (int)next() & mask;
      }
    v16i acc[4];
#pragma unroll
    for (int c = 0; c < 4; c++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[c][r] = 0;
    for (int it = 0; it < iters; it++) {
#pragma unroll
      for (int c = 0; c < 4; c++) acc[c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[c & 1], b[c >> 1], acc[c], 0, 0, 0);
    }
#pragma unroll
    for (int c = 0; c < 4; c++)
#pragma unroll
      for (int r = 0; r < 16; r++) total ^= acc[c][r];
  } else {
    // bf16 values +-1, +-0.5 (sign and low exponent bit from the generator): the sums stay finite
    v8bf a[2], b[2];
#pragma unroll
    for (int k = 0; k < 2; k++) {
      v8us ua, ub;
#pragma unroll
      for (int r = 0; r < 8; r++) {
        const unsigned u = next();
        ua[r] = (unsigned short)((0x3F00u | ((u & 1u) << 7) | ((u & 2u) << 14)) & (unsigned)mask);
        ub[r] = (unsigned short)((0x3F00u | ((u & 4u) << 5) | ((u & 8u) << 12)) & (unsigned)mask);
      }
      a[k] = __builtin_bit_cast(v8bf, ua);
      b[k] = __builtin_bit_cast(v8bf, ub);
    }
    v16f acc[4];
#pragma unroll
    for (int c = 0; c < 4; c++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[c][r] = 0.f;
    for (int it = 0; it < iters; it++) {
#pragma unroll
      for (int c = 0; c < 4; c++) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c & 1], b[c >> 1], acc[c], 0, 0, 0);
    }
#pragma unroll
    for (int c = 0; c < 4; c++)
#pragma unroll
      for (int r = 0; r < 16; r++) total ^= (int)__float_as_uint(acc[c][r]);
  }
  // keeps the accumulators alive; the stored value means nothing (one word, whichever lane comes last)
  if (total == seed) *sink = total;
}

// Streaming memory traffic: every lane moves 16-byte pieces, consecutive lanes consecutive pieces, the
// workgroups striding over the buffer.  COPY: read src, write dst.  Otherwise read only (the pieces
// are folded into one word per lane, stored only if it matches `seed`).
template <bool COPY>
__global__ void __launch_bounds__(256) probe_stream_kernel(const v4i* __restrict__ src, v4i* __restrict__ dst, size_t pieces,
                                                           int seed, int* sink) {
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  int fold = 0;
  for (; i + 3 * stride < pieces; i += 4 * stride) {
    const v4i v0 = __builtin_nontemporal_load(src + i);
    const v4i v1 = __builtin_nontemporal_load(src + i + stride);
    const v4i v2 = __builtin_nontemporal_load(src + i + 2 * stride);
    const v4i v3 = __builtin_nontemporal_load(src + i + 3 * stride);
    if constexpr (COPY) {
      __builtin_nontemporal_store(v0, dst + i);
      __builtin_nontemporal_store(v1, dst + i + stride);
      __builtin_nontemporal_store(v2, dst + i + 2 * stride);
      __builtin_nontemporal_store(v3, dst + i + 3 * stride);
    } else {
      const v4i x = (v0 ^ v1) ^ (v2 ^ v3);
      fold ^= (x[0] ^ x[1]) ^ (x[2] ^ x[3]);
    }
  }
  for (; i < pieces; i += stride) {
    const v4i v = __builtin_nontemporal_load(src + i);
    if constexpr (COPY) __builtin_nontemporal_store(v, dst + i);
    else fold ^= (v[0] ^ v[1]) ^ (v[2] ^ v[3]);
  }
  if (!COPY && fold == seed) *sink = fold;
}

}  // namespace sage
