// Pre-pass kernels: K-smoothing mean, optional Q-smoothing block mean, the per-block
// INT8 quantiser psi, delta = rowsum(dO o O), and the export (inspection) kernels.
//
// Paper: Sec. 3 "Quantization" (X^ = round(X / delta_X), delta_X = max|X| / 127),
// Sec. 3 "Q and K Smoothing" (mu_K over the whole key tensor, mu_Qi per block),
// Algorithm 1 "Quantization" line, Algorithm 2 line 2 (D) and line 6 (psi(dO_i)).
//
// The stored INT8 codes and FP32 scales are a bit-exact contract, so the arithmetic
// here is fixed: mean = (float64 sum) / N rounded once to FP32; x - mu in FP32;
// a = max|x|; s = a / 127 and r = 127 / a as IEEE FP32 divisions; q = rne(x * r).
#pragma once

#include "common.h"

namespace sage {

#pragma clang fp contract(off)

// Rows of K per workgroup of the mean reduction: the host picks the largest of these that still gives
// the launch a few workgroups per CU (the consumer sums one partial per chunk and channel).
inline int mean_chunk_rows(int heads, int N) {
  int rows = 1024;
  while (rows > 128 && (long long)heads * ((N + rows - 1) / rows) < 1024) rows >>= 1;
  return rows;
}

// ---- QK-norm fused into the pre-pass (paper Sec. 4, "Stabilizing Outliers with QK-Norm") ----------
// y = x / sqrt(mean_c x^2 + eps) * gamma per token, rounded to bf16: the tensor a bf16 model hands to the
// attention, so the fused pre-pass gives the bits of "normalise, then quantise".  Arithmetic (part of the
// bit-exact contract): sum of squares in float64 (exact for bf16 inputs), r = 1 / sqrt(sum / D + eps) in
// float64 rounded once to FP32, y = bf16((x *_f32 r) *_f32 gamma).
struct QkNorm {
  const float* gamma;   // [D] per-channel gain, or nullptr: no normalisation
  float eps;
};
__device__ __forceinline__ float qknorm_rscale(double sumsq, int D, float eps) {
  return (float)(1.0 / sqrt(sumsq / (double)D + (double)eps));
}
__device__ __forceinline__ float qknorm_apply(float x, float r, float g) {
  return bf16_bits_to_float(float_to_bf16_bits((x * r) * g));
}

// ---- K mean, stage 1: float64 column sums of a chunk of rows -----------------------
// (bf16 data of ordinary range sum exactly in float64, so the result does not depend on the order
// or on the chunk size.)  Stage 2, the sum over the chunks, the division by N and the one rounding to
// FP32, runs at the start of every workgroup that quantises a block of K (prepass_quant_kernel).
template <int D>
__global__ void __launch_bounds__(256) kmean_partial_kernel(const unsigned short* __restrict__ K, RowView view,
                                                            double* __restrict__ kpart, int N,
                                                            int nchunk, int chunk_rows, QkNorm norm) {
  constexpr int TPR = D / 8;          // threads per row, 8 channels (16 bytes) each
  constexpr int RPP = 256 / TPR;      // rows per pass
  __shared__ double red[256][8];
  const int t = threadIdx.x;
  const int chunk = blockIdx.x, bh = blockIdx.y;
  const int row0 = chunk * chunk_rows;
  const int rows = min(chunk_rows, N - row0);
  const unsigned short* base = K + view.row(bh, row0);
  double acc[8];
#pragma unroll
  for (int e = 0; e < 8; e++) acc[e] = 0.0;
  const int tr = t / TPR, tc = t % TPR;
  int r = tr;
  if (norm.gamma != nullptr) {
    // the mean is taken over the normalised keys: the TPR threads of a row share its sum of squares
    float g[8];
#pragma unroll
    for (int e = 0; e < 8; e++) g[e] = norm.gamma[tc * 8 + e];
    for (int r0 = 0; r0 < rows; r0 += RPP) {      // whole passes: the shuffles need every lane
      r = r0 + tr;
      v8us v = {0, 0, 0, 0, 0, 0, 0, 0};
      if (r < rows) v = *(const v8us*)(base + (size_t)r * view.row_stride + tc * 8);
      double ss = 0.0;
#pragma unroll
      for (int e = 0; e < 8; e++) {
        const float x = bf16_bits_to_float(v[e]);
        ss += (double)(x * x);
      }
#pragma unroll
      for (int off = 1; off < TPR; off <<= 1) ss += __shfl_xor(ss, off, 64);
      if (r < rows) {
        const float rs = qknorm_rscale(ss, D, norm.eps);
#pragma unroll
        for (int e = 0; e < 8; e++) acc[e] += (double)qknorm_apply(bf16_bits_to_float(v[e]), rs, g[e]);
      }
    }
    r = rows;   // nothing left for the plain loops below
  }
  // four independent 16-byte loads in flight per thread
  for (; r + 3 * RPP < rows; r += 4 * RPP) {
    v8us v[4];
#pragma unroll
    for (int u = 0; u < 4; u++) v[u] = *(const v8us*)(base + (size_t)(r + u * RPP) * view.row_stride + tc * 8);
#pragma unroll
    for (int u = 0; u < 4; u++)
#pragma unroll
      for (int e = 0; e < 8; e++) acc[e] += (double)bf16_bits_to_float(v[u][e]);
  }
  for (; r < rows; r += RPP) {
    v8us v = *(const v8us*)(base + (size_t)r * view.row_stride + tc * 8);
#pragma unroll
    for (int e = 0; e < 8; e++) acc[e] += (double)bf16_bits_to_float(v[e]);
  }
#pragma unroll
  for (int e = 0; e < 8; e++) red[t][e] = acc[e];
  __syncthreads();
  if (t < D) {
    double s = 0.0;
    for (int g = 0; g < RPP; g++) s += red[g * TPR + t / 8][t % 8];
    kpart[((size_t)bh * nchunk + chunk) * D + t] = s;
  }
}

__global__ void fill_zero_f32_kernel(float* __restrict__ p, size_t n) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = 0.f;
}

// ---- psi on one 64-row block (of a numerics block of 64 or 128 rows) -------------
struct QuantJob {
  const unsigned short* src;   // bf16, rows addressed through `view`
  RowView view;                // where the rows of src (and of O) lie in the caller's tensor
  int N, Np;                   // rows of src that exist; rows of the workspace tensors (N rounded up to 64)
  int q_like;                  // host side only: a Q-like tensor (numerics blocks of B_q rows) or a K-like one (B_kv)
  int8_t* outF;                // F layout or nullptr
  int8_t* outTF;               // TF layout or nullptr
  float* scale;                // [BH, N/64]
  const double* mean_part;     // K-smoothing: float64 column sums [BH, nchunk, D] of the whole head; the
                               // mean (sum / N, rounded once to FP32) is subtracted from every row.  Else nullptr
  int nchunk;
  float* mu_head_out;          // [BH, D]: where block 0 of each head stores that mean
  float* mu_block_out;         // [BH, N/64, D]: if set, the block mean is computed, stored and subtracted
  const unsigned short* O;     // bf16 [BH, N, D] or nullptr: delta = rowsum(src o O)
  float* delta;                // [BH, N]: -rowsum(src o O)
  const float* lse;            // [BH, N] or nullptr: nl2 = -lse * log2(e) for the backward
  float* nl2;                  // [BH, N]
  QkNorm norm;                 // QK-norm applied to src before anything else (Q and K jobs), or gamma == nullptr
  unsigned short* norm_out;    // if set: the normalised rows as dense bf16 [BH, Np, D] (for the Q-smoothing bias)
};
struct QuantJobs {
  QuantJob job[4];
};

// Per job: N = rows of the caller's tensor, Np = N rounded up to a multiple of 64 = rows of its workspace
// tensors (Q-like and K-like tensors may have different lengths).  Rows N .. Np-1 do not exist: they are
// read as zeros AFTER the smoothing (so they change no absmax), enter no mean, get delta = 0 and
// -L*log2(e) = -inf (P = 0 in the backward).  The grid's x extent covers the longest job.
//
// SUB = 64-row blocks per numerics block (Algorithm 1 leaves B_q, B_kv free): 1, or 2 for blocks of 128 rows.
// A workgroup always writes ONE 64-row block; with SUB = 2 it also reads the other half of its numerics
// block (its "partner") and takes the block mean and the absmax over both, so that the two workgroups of a
// numerics block arrive at the same scale (and mean) without exchanging anything, and store it once per
// 64-row block: the attention kernels index scales, means and bias rows by 64-row block whatever the
// numerics block is.
template <int D, int SUB>
__global__ void __launch_bounds__(256) prepass_quant_kernel(QuantJobs jobs) {
  constexpr int CPR = D / 16;            // 16-channel chunks per row
  constexpr int NCH = 64 * CPR / 256;    // chunks per thread (1 for D=64, 2 for D=128)
  constexpr int NTF = 4 * D / 256;       // TF chunks per thread
  static_assert(SUB == 1 || SUB == 2, "numerics blocks of 64 or 128 rows");
  __shared__ __attribute__((aligned(16))) int8_t tile[64 * D];
  __shared__ float colbuf[64 * D / 4];   // used by the block mean only (16 rows at a time)
  __shared__ float mu_s[D];
  __shared__ float wmax[4];

  const QuantJob jb = jobs.job[blockIdx.z];
  const int t = threadIdx.x;
  const int blk = blockIdx.x, bh = blockIdx.y;
  const int N = jb.N, Np = jb.Np;
  const RowView view = jb.view;
  const int nblk = Np / kBlock;
  if (blk >= nblk) return;
  const size_t tile_off = view.row(bh, (size_t)blk * kBlock);               // in the caller's tensors
  const int rows_here = min(kBlock, N - blk * kBlock);                      // rows of this block that exist
  // the partner block (SUB = 2): the other 64 rows of this numerics block, possibly past the end
  const int pblk = blk ^ 1;
  const int rows_partner = SUB == 2 ? max(0, min(kBlock, N - pblk * kBlock)) : 0;

  // rows of 64-row block `b` (the first `rows` of them exist) as FP32, 16 channels per chunk
  auto load_rows = [&](float (&v)[NCH][16], const int b, const int rows) {
    const size_t off = view.row(bh, (size_t)b * kBlock);
#pragma unroll
    for (int it = 0; it < NCH; it++) {
      const int c = t + 256 * it;
      const int row = c / CPR, ch = c % CPR;
      v8us lo = {0, 0, 0, 0, 0, 0, 0, 0}, hi = {0, 0, 0, 0, 0, 0, 0, 0};
      if (row < rows) {
        const unsigned short* p = jb.src + off + (size_t)row * view.row_stride + ch * 16;
        lo = *(const v8us*)p;
        hi = *(const v8us*)(p + 8);
      }
#pragma unroll
      for (int e = 0; e < 8; e++) {
        v[it][e] = bf16_bits_to_float(lo[e]);
        v[it][8 + e] = bf16_bits_to_float(hi[e]);
      }
    }
  };
  // QK-norm of the rows held in `v`: the CPR threads of a row (consecutive lanes) share its sum of squares
  auto qk_normalise = [&](float (&v)[NCH][16], const int rows, unsigned short* out_rows) {
#pragma unroll
    for (int it = 0; it < NCH; it++) {
      const int c = t + 256 * it;
      const int row = c / CPR, ch = c % CPR;
      double ss = 0.0;
#pragma unroll
      for (int e = 0; e < 16; e++) ss += (double)(v[it][e] * v[it][e]);
#pragma unroll
      for (int off = 1; off < CPR; off <<= 1) ss += __shfl_xor(ss, off, 64);
      if (row < rows) {
        const float rs = qknorm_rscale(ss, D, jb.norm.eps);
        const float* g = jb.norm.gamma + ch * 16;
#pragma unroll
        for (int e = 0; e < 16; e++) v[it][e] = qknorm_apply(v[it][e], rs, g[e]);
      }
      if (out_rows != nullptr) {
        v8us lo, hi;
#pragma unroll
        for (int e = 0; e < 8; e++) {
          lo[e] = float_to_bf16_bits(v[it][e]);        // exact: the values are bf16 already (zero in missing rows)
          hi[e] = float_to_bf16_bits(v[it][8 + e]);
        }
        unsigned short* o = out_rows + (size_t)row * D + ch * 16;
        *(v8us*)o = lo;
        *(v8us*)(o + 8) = hi;
      }
    }
  };
  // v -= mu_s on the rows that exist
  auto subtract_mu = [&](float (&v)[NCH][16], const int rows) {
#pragma unroll
    for (int it = 0; it < NCH; it++) {
      const int row = (t + 256 * it) / CPR, ch = (t + 256 * it) % CPR;
      if (row < rows) {
#pragma unroll
        for (int e = 0; e < 16; e++) v[it][e] = v[it][e] - mu_s[ch * 16 + e];
      }
    }
  };
  // float64 column sums of the rows held in `v` (zeros where a row does not exist), thread t < D taking
  // channel t; in 4 passes of 16 rows through `colbuf` to bound LDS
  auto add_column_sums = [&](const float (&v)[NCH][16], double& part) {
    for (int pass = 0; pass < 4; pass++) {
      __syncthreads();
#pragma unroll
      for (int it = 0; it < NCH; it++) {
        const int c = t + 256 * it;
        const int row = c / CPR, ch = c % CPR;
        if (row / 16 == pass) {
#pragma unroll
          for (int e = 0; e < 16; e++) colbuf[(row % 16) * D + ch * 16 + e] = v[it][e];
        }
      }
      __syncthreads();
      if (t < D) {
        for (int r = 0; r < 16; r++) part += (double)colbuf[r * D + t];
      }
    }
  };

  float x[NCH][16];
  float xp[SUB == 2 ? NCH : 1][16];      // the partner's rows (SUB = 2)
  load_rows(x, blk, rows_here);
  if constexpr (SUB == 2) load_rows(xp, pblk, rows_partner);

  if (jb.norm.gamma != nullptr) {
    qk_normalise(x, rows_here,
                 jb.norm_out != nullptr ? jb.norm_out + ((size_t)bh * Np + (size_t)blk * kBlock) * D : nullptr);
    if constexpr (SUB == 2) qk_normalise(xp, rows_partner, nullptr);
  }

  // delta = rowsum(dO o O), FP32 (not part of the bit-exact contract)
  if (jb.O != nullptr) {
#pragma unroll
    for (int it = 0; it < NCH; it++) {
      const int c = t + 256 * it;
      const int row = c / CPR, ch = c % CPR;
      v8us lo = {0, 0, 0, 0, 0, 0, 0, 0}, hi = {0, 0, 0, 0, 0, 0, 0, 0};
      if (row < rows_here) {
        const unsigned short* p = jb.O + tile_off + (size_t)row * view.row_stride + ch * 16;
        lo = *(const v8us*)p;
        hi = *(const v8us*)(p + 8);
      }
      float acc = 0.f;
#pragma unroll
      for (int e = 0; e < 8; e++) {
        acc += x[it][e] * bf16_bits_to_float(lo[e]);
        acc += x[it][8 + e] * bf16_bits_to_float(hi[e]);
      }
#pragma unroll
      for (int off = 1; off < CPR; off <<= 1) acc += __shfl_xor(acc, off, 64);
      // stored negated: the backward starts the dP accumulators from -delta (dP - delta in one chain)
      if (ch == 0) jb.delta[(size_t)bh * Np + (size_t)blk * kBlock + row] = -acc;
    }
  }

  if (jb.lse != nullptr && t < 64) {
    const size_t row = (size_t)blk * kBlock + t;
    jb.nl2[(size_t)bh * Np + row] = t < rows_here ? -jb.lse[(size_t)bh * N + row] * 1.4426950408889634f : -INFINITY;
  }

  if (jb.mean_part != nullptr) {
    // mu_K: the chunk sums of the head, added in float64, divided by N, rounded once to FP32
    if (t < D) {
      double s = 0.0;
      for (int k = 0; k < jb.nchunk; k++) s += jb.mean_part[((size_t)bh * jb.nchunk + k) * D + t];
      const float m = (float)(s / (double)N);
      mu_s[t] = m;
      if (blk == 0) jb.mu_head_out[(size_t)bh * D + t] = m;
    }
    __syncthreads();
    subtract_mu(x, rows_here);
    if constexpr (SUB == 2) subtract_mu(xp, rows_partner);
  }

  if (jb.mu_block_out != nullptr) {
    // block mean over the rows of the numerics block that exist: float64 sum (exact for bf16 data), one rounding
    double part = 0.0;   // thread t < D accumulates channel t
    add_column_sums(x, part);
    if constexpr (SUB == 2) add_column_sums(xp, part);
    if (t < D) {
      const float m = (float)(part / (double)(rows_here + rows_partner));
      mu_s[t] = m;
      jb.mu_block_out[((size_t)bh * nblk + blk) * D + t] = m;
    }
    __syncthreads();
    subtract_mu(x, rows_here);
    if constexpr (SUB == 2) subtract_mu(xp, rows_partner);
  }

  // block absmax
  float a = 0.f;
#pragma unroll
  for (int it = 0; it < NCH; it++)
#pragma unroll
    for (int e = 0; e < 16; e++) a = fmaxf(a, fabsf(x[it][e]));
  if constexpr (SUB == 2) {
#pragma unroll
    for (int it = 0; it < NCH; it++)
#pragma unroll
      for (int e = 0; e < 16; e++) a = fmaxf(a, fabsf(xp[it][e]));
  }
  a = wave_max_nonneg_f32(a);
  if ((t & 63) == 0) wmax[t >> 6] = a;
  __syncthreads();
  a = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
  const bool nz = a > 0.f;
  const float s = nz ? a / 127.0f : 0.f;
  const float r = nz ? 127.0f / a : 0.f;
  if (t == 0) jb.scale[(size_t)bh * nblk + blk] = s;

  const size_t frag_base = ((size_t)bh * (Np / 32) + (size_t)blk * 2) * (D / 32) * 1024;
#pragma unroll
  for (int it = 0; it < NCH; it++) {
    const int c = t + 256 * it;
    const int row = c / CPR, ch = c % CPR;
    v4i packed;
#pragma unroll
    for (int w = 0; w < 4; w++) {
      unsigned u = 0;
#pragma unroll
      for (int e = 0; e < 4; e++) {
        float y = __builtin_rintf(x[it][4 * w + e] * r);
        y = fminf(fmaxf(y, -127.f), 127.f);
        u |= ((unsigned)((int)y) & 0xffu) << (8 * e);
      }
      packed[w] = (int)u;
    }
    if (jb.outTF != nullptr) *(v4i*)(tile + row * D + ch * 16) = packed;
    if (jb.outF != nullptr) {
      const int rb = row / 32, sstep = ch / 2, h = ch % 2;
      const int lane = (row % 32) + 32 * h;
      *(v4i*)(jb.outF + frag_base + ((size_t)(rb * (D / 32) + sstep) * 64 + lane) * 16) = packed;
    }
  }
  if (jb.outTF != nullptr) {
    __syncthreads();
#pragma unroll
    for (int it = 0; it < NTF; it++) {
      const int c = t + 256 * it;            // (rb, cb, lane)
      const int lane = c % 64, cb = (c / 64) % (D / 32), rb = c / (64 * (D / 32));
      const int col = 32 * cb + (lane % 32), h = lane / 32;
      v4i packed;
#pragma unroll
      for (int aa = 0; aa < 4; aa++) {
        unsigned u = 0;
#pragma unroll
        for (int b = 0; b < 4; b++) {
          const int row = 32 * rb + 8 * aa + 4 * h + b;
          u |= ((unsigned)(unsigned char)tile[row * D + col]) << (8 * b);
        }
        packed[aa] = (int)u;
      }
      *(v4i*)(jb.outTF + frag_base + ((size_t)(rb * (D / 32) + cb) * 64 + lane) * 16) = packed;
    }
  }
}

// ---- inspection: fragment layouts back to row-major -----------------------------
// One thread per 16-byte fragment chunk.  transposed = 0: F layout, 1: TF layout.
__global__ void export_fragments_kernel(const int8_t* __restrict__ frag, int8_t* __restrict__ out,
                                        size_t n_chunks, int N, int D, int transposed) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i >= n_chunks) return;
  const int fpr = D / 32;                     // fragments per 32-row block
  const int lane = (int)(i % 64);
  const size_t f = i / 64;                    // global fragment index
  const int sc = (int)(f % fpr);
  const size_t rbg = f / fpr;                 // 32-row block over all heads (N % 32 == 0)
  const size_t head = rbg / (N / 32);
  const int rb = (int)(rbg % (N / 32));
  v4i v = *(const v4i*)(frag + i * 16);
  const int r = lane % 32, h = lane / 32;
  int8_t* obase = out + head * (size_t)N * D;
  if (!transposed) {
    *(v4i*)(obase + (size_t)(32 * rb + r) * D + 32 * sc + 16 * h) = v;
  } else {
#pragma unroll
    for (int aa = 0; aa < 4; aa++)
#pragma unroll
      for (int b = 0; b < 4; b++)
        obase[(size_t)(32 * rb + 8 * aa + 4 * h + b) * D + 32 * sc + r] = (int8_t)((v[aa] >> (8 * b)) & 0xff);
  }
}

// out = sign * in (sign = +-1: exact)
__global__ void copy_f32_kernel(const float* __restrict__ in, float* __restrict__ out, size_t n, float sign) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) out[i] = sign * in[i];
}

// ---- Q-smoothing: logit bias table -------------------------------------------------
// bias[bh][I][k] = sm_scale*log2(e) * mu_Q[I] . K_sm[k]  (the mu_Qi K_sm^T term of the
// Sec. 3 decomposition; the two mu_K terms are constant along a softmax row and dropped).
// FP32 from the unquantised K - mu_K.  Causal: blocks I < block(k) are never read (nor written).
template <int D>
__global__ void __launch_bounds__(256) qsmooth_bias_kernel(const unsigned short* __restrict__ K, RowView view,
                                                           const float* __restrict__ muK,
                                                           const float* __restrict__ muQ,
                                                           float* __restrict__ bias, int N, int Np, int nqblk,
                                                           int causal_shift, float scale_log2e) {
  // (N = rows of K as the caller holds it, Np = N rounded up to the block: keys that do not exist count as
  // zero rows; nqblk = Q blocks; causal_shift < 0: no mask, else Q block I sees key blocks <= I + causal_shift.)
  // One workgroup per (key block, head): a [Q blocks] x [64 keys] x [D channels] FP32 product on
  // the FP32 matrix instruction (32x32x2).  The smoothed keys go through LDS once (coalesced
  // reads); every wave keeps half of them as B operands in registers and takes 32 Q blocks at a
  // time as the A operand.  The contraction order is free, so lane (row, half) pairs channel
  // 8 v + 4 half + e with step (v, e): both operands then come from 16-byte reads.
  constexpr int LD = D + 4;                      // floats per LDS row (keeps rows 16-byte aligned)
  __shared__ __attribute__((aligned(16))) float ks[64 * LD];
  const int t = threadIdx.x;
  const int kblk = blockIdx.x, bh = blockIdx.y;
  const int nblk = Np / kBlock;
  const unsigned short* src = K + view.row(bh, (size_t)kblk * kBlock);
  const int rows_here = min(kBlock, N - kblk * kBlock);
  const float* mk = muK + (size_t)bh * D;
  {
    constexpr int NCH = 64 * D / 8 / 256;        // 16-byte chunks (8 channels) per thread
    v8us raw[NCH];
#pragma unroll
    for (int u = 0; u < NCH; u++) {
      raw[u] = v8us{0, 0, 0, 0, 0, 0, 0, 0};
      const int ch = t + 256 * u;
      if (ch / (D / 8) < rows_here) raw[u] = *(const v8us*)(src + (size_t)(ch / (D / 8)) * view.row_stride + 8 * (ch % (D / 8)));
    }
#pragma unroll
    for (int u = 0; u < NCH; u++) {
      const int ch = t + 256 * u, row = ch / (D / 8), c0 = 8 * (ch % (D / 8));
      const bool there = row < rows_here;
      const v4f m0 = *(const v4f*)(mk + c0), m1 = *(const v4f*)(mk + c0 + 4);
      v4f f0, f1;
#pragma unroll
      for (int e = 0; e < 4; e++) {
        f0[e] = there ? bf16_bits_to_float(raw[u][e]) - m0[e] : 0.f;
        f1[e] = there ? bf16_bits_to_float(raw[u][4 + e]) - m1[e] : 0.f;
      }
      *(v4f*)(ks + row * LD + c0) = f0;
      *(v4f*)(ks + row * LD + c0 + 4) = f1;
    }
  }
  __syncthreads();
  const int lane = t & 63, r = lane & 31, half = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  // wave = (Q-block tile parity, key half): each wave keeps one half of the keys as B operands
  const int kt = wave & 1;
  v4f kb[D / 8];                                 // B operands: key 32 kt + r
#pragma unroll
  for (int v = 0; v < D / 8; v++) kb[v] = *(const v4f*)(ks + (32 * kt + r) * LD + 8 * v + 4 * half);
  const int first = causal_shift >= 0 ? max(kblk - causal_shift, 0) : 0;   // Q blocks that cannot see the key block are never read
  for (int it = first / 32 + (wave >> 1); 32 * it < nqblk; it += 2) {
    const int I = min(32 * it + r, nqblk - 1);   // rows past the end repeat the last one (not stored)
    const float* mq = muQ + ((size_t)bh * nqblk + I) * D + 4 * half;
    v16f acc[2];                                 // two chains over alternate steps, summed at the end
#pragma unroll
    for (int c = 0; c < 2; c++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[c][e] = 0.f;
#pragma unroll
    for (int v = 0; v < D / 8; v++) {
      const v4f a4 = *(const v4f*)(mq + 8 * v);
#pragma unroll
      for (int e = 0; e < 4; e++)
        acc[e & 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a4[e], kb[v][e], acc[e & 1], 0, 0, 0);
    }
    // accumulator register e of lane (r, half): Q block 32 it + 8 (e / 4) + 4 half + e % 4, key 32 kt + r
#pragma unroll
    for (int e = 0; e < 16; e++) {
      const int Io = 32 * it + 8 * (e >> 2) + 4 * half + (e & 3);
      if (Io >= first && Io < nqblk)
        bias[((size_t)bh * nqblk + Io) * Np + (size_t)kblk * kBlock + 32 * kt + r] = (acc[0][e] + acc[1][e]) * scale_log2e;
    }
  }
}

// ---- inspection: the psi(dS) tiles the backward left in its scratch, as a row-major [Np, Np] matrix ----
// Tile (i, j) holds four 1 KiB fragments (32-query block qb, 32-key block kb): lane (key, half), byte
// 4 a + b = psi(dS)[64 i + 32 qb + 8 a + 4 half + b][64 j + 32 kb + key] (a quantised accumulator quadrant
// as the backward kernel holds it).  Tiles above the causal diagonal
// were never written: they are returned as zeros.  One thread per 16 bytes.
__global__ void export_ds_kernel(const int8_t* __restrict__ tiles, const float* __restrict__ scales,
                                 int8_t* __restrict__ ds_out, float* __restrict__ scale_out, int nqblk, int Np,
                                 int pitch, int causal_shift) {
  // [nqblk * 64, Np] out; causal_shift < 0: no mask, else tile (i, j) exists iff j <= i + causal_shift
  const int nblk = Np / kBlock;
  const size_t c = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (c >= (size_t)nqblk * nblk * 256) return;
  const int tile = (int)(c / 256), i = tile / nblk, j = tile % nblk;
  const int frag = (int)(c % 256) / 64, lane = (int)(c % 64);
  const bool there = causal_shift < 0 || j <= i + causal_shift;
  v4i v = {0, 0, 0, 0};
  if (there) v = *(const v4i*)(tiles + ((size_t)i * pitch + j) * 4096 + (c % 256) * 16);   // `pitch` tiles per Q-block row
  // fragment (qb, kb), lane (key, h), byte 4 a + b = psi(dS)[32 qb + 8 a + 4 h + b][32 kb + key]
  const int qrow0 = 64 * i + 32 * (frag >> 1) + 4 * (lane >> 5), key = 64 * j + 32 * (frag & 1) + (lane & 31);
  if (ds_out != nullptr) {
#pragma unroll
    for (int a = 0; a < 4; a++)
#pragma unroll
      for (int b = 0; b < 4; b++) ds_out[(size_t)(qrow0 + 8 * a + b) * Np + key] = (int8_t)((v[a] >> (8 * b)) & 0xff);
  }
  if (scale_out != nullptr && c % 256 == 0) scale_out[tile] = there ? scales[(size_t)i * pitch + j] : 0.f;
}

}  // namespace sage
