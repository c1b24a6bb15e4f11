// Fused INT8 attention forward (paper Algorithm 1) for gfx950.
//
// One wave owns 32 queries; a workgroup of NW waves owns 32*NW consecutive queries of
// one head and walks the KV blocks (64 keys each), staging K^ and V^ fragments in LDS.
//
// The logits are formed TRANSPOSED, S^T = K^ Q^^T (keys x queries), with the 32x32x32
// INT8 MFMA: an accumulator lane then holds one query (column) and 16 keys (rows) per
// 32-key block, so that
//   - the row max / row sum of the softmax are in-lane reductions plus one exchange
//     between the two half-waves,
//   - the per-token quantised P^ (Algorithm 1 line 9), packed four codes to a register,
//     is already the B operand of O^T = V^^T P^^T (the TF layout of V^ orders its keys
//     the way the accumulator holds them), with no trip through LDS.
//
// Per-token quantisation: P~/s_P with s_P = exp(rowmax(S_ij) - m_ij)/127 equals
// 127 * exp(S_ij - rowmax(S_ij)), which does not depend on the running max.  The kernel
// evaluates that form (never 0/0) and keeps the running reference m only for the FP32
// accumulators: O += beta * s_V * (P^ V^), l += beta * sum(127 p), beta = exp(rowmax - m).
// m is raised only when a tile's row max exceeds it by more than kTau (in log2 units); the
// result is unchanged because O/l and m + log l do not depend on the reference chosen.
#pragma once

#include "common.h"

namespace sage {

struct FwdArgs {
  const int8_t* QF;     // F layout
  const int8_t* KF;     // F layout
  const int8_t* VT;     // TF layout
  const float* sQ;      // [BH, N/64]
  const float* sK;
  const float* sV;
  const float* bias;    // Q-smoothing: [BH, N/64, N] = sm_scale*log2e * mu_Qi . K_sm[k], else nullptr
  unsigned short* O;    // bf16 [BH, N, D]
  float* LSE;           // [BH, N]
  int BH, N;
  int n_qtiles;         // workgroups per head
  float scale_log2e;    // sm_scale * log2(e)
};

constexpr float kTau = 8.0f;
constexpr float kLog2_127 = 6.98868468677216585f;
constexpr float kLn2 = 0.69314718055994531f;

// One KV tile for one wave.  MASK = the tile straddles the causal diagonal for this wave
// (a separate instantiation so the full tiles carry no masking code).
template <int D, bool QSMOOTH, bool MASK>
__device__ __forceinline__ void fwd_tile(const int8_t* __restrict__ Kt, const int8_t* __restrict__ Vt,
                                         const v4i (&qf)[D / 32], v16f (&oacc)[D / 32], float& m_ref,
                                         float& l_part, const float c, const float sv,
                                         const float* __restrict__ bias_row, const int k0, const int q,
                                         const int lane, const int h) {
  constexpr int KS = D / 32;
  // ---- S^T = K^ Q^^T : two 32-key blocks, interleaved so consecutive MFMAs are independent ----
  v16i sacc[2];
#pragma unroll
  for (int kb = 0; kb < 2; kb++)
#pragma unroll
    for (int r = 0; r < 16; r++) sacc[kb][r] = 0;
#pragma unroll
  for (int s = 0; s < KS; s++) {
#pragma unroll
    for (int kb = 0; kb < 2; kb++) {
      const v4i a = *(const v4i*)(Kt + (kb * KS + s) * 1024 + lane * 16);
      sacc[kb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, qf[s], sacc[kb], 0, 0, 0);
    }
  }
  float x[2][16];
  float mloc;   // row max of the tile in the log2 domain
  if constexpr (!QSMOOTH) {
    // the scale is one positive scalar per tile, so the row max can be taken on the integers
    int mi = INT_MIN;
#pragma unroll
    for (int kb = 0; kb < 2; kb++)
#pragma unroll
      for (int r = 0; r < 16; r++) {
        int v = sacc[kb][r];
        if constexpr (MASK) {
          const int key = k0 + 32 * kb + 8 * (r >> 2) + 4 * h + (r & 3);
          v = key > q ? INT_MIN : v;
          sacc[kb][r] = v;
        }
        mi = max(mi, v);
      }
    mi = half_swap_max_i32(mi);
    mloc = (float)mi * c;
    const float off = kLog2_127 - mloc;
#pragma unroll
    for (int kb = 0; kb < 2; kb++)
#pragma unroll
      for (int r = 0; r < 16; r++) {
        float v = __builtin_fmaf((float)sacc[kb][r], c, off);
        if constexpr (MASK) v = sacc[kb][r] == INT_MIN ? -INFINITY : v;
        x[kb][r] = v;
      }
  } else {
    float mf = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; kb++)
#pragma unroll
      for (int aa = 0; aa < 4; aa++) {
        const int key = k0 + 32 * kb + 8 * aa + 4 * h;
        const v4f b4 = *(const v4f*)(bias_row + key);
#pragma unroll
        for (int b = 0; b < 4; b++) {
          float v = __builtin_fmaf((float)sacc[kb][4 * aa + b], c, b4[b]);
          if constexpr (MASK) v = (key + b) > q ? -INFINITY : v;
          x[kb][4 * aa + b] = v;
          mf = fmaxf(mf, v);
        }
      }
    mloc = half_swap_max_f32(mf);
    const float off = kLog2_127 - mloc;
#pragma unroll
    for (int kb = 0; kb < 2; kb++)
#pragma unroll
      for (int r = 0; r < 16; r++) x[kb][r] = x[kb][r] + off;
  }
  // ---- online softmax reference ----
  if (__builtin_amdgcn_ballot_w64(mloc > m_ref + kTau) != 0) {
    const float m_new = fmaxf(m_ref, mloc);
    const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);   // 0 on the first tile
    l_part *= alpha;
#pragma unroll
    for (int cb = 0; cb < KS; cb++)
#pragma unroll
      for (int r = 0; r < 16; r++) oacc[cb][r] *= alpha;
    m_ref = m_new;
  }
  const float beta = __builtin_amdgcn_exp2f(mloc - m_ref);
  // ---- P^ = rne(127 exp(S - rowmax)), packed as the B operand; row sum of 127 p ----
  v4i pf[2];
  float psum = 0.f;
#pragma unroll
  for (int kb = 0; kb < 2; kb++)
#pragma unroll
    for (int aa = 0; aa < 4; aa++) {
      unsigned u = 0;
#pragma unroll
      for (int b = 0; b < 4; b++) {
        const float e = __builtin_amdgcn_exp2f(x[kb][4 * aa + b]);
        psum += e;
        u = __builtin_amdgcn_cvt_pk_u8_f32(e, b, u);
      }
      pf[kb][aa] = (int)u;
    }
  l_part = __builtin_fmaf(beta, psum, l_part);
  const float w = beta * sv;
  // ---- O^T += (V^^T P^^T) * w : all MFMAs first, then the conversions ----
  v16i t[KS];
#pragma unroll
  for (int cb = 0; cb < KS; cb++) {
#pragma unroll
    for (int r = 0; r < 16; r++) t[cb][r] = 0;
#pragma unroll
    for (int kb = 0; kb < 2; kb++) {
      const v4i a = *(const v4i*)(Vt + (kb * KS + cb) * 1024 + lane * 16);
      t[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, pf[kb], t[cb], 0, 0, 0);
    }
  }
#pragma unroll
  for (int cb = 0; cb < KS; cb++)
#pragma unroll
    for (int r = 0; r < 16; r++) oacc[cb][r] = __builtin_fmaf((float)t[cb][r], w, oacc[cb][r]);
}

template <int D, bool CAUSAL, bool QSMOOTH, int NW>
__global__ void __launch_bounds__(64 * NW, (NW == 8 ? 1 : 2)) sage_fwd_kernel(FwdArgs args) {
  constexpr int KS = D / 32;                 // k-steps of Q K^T; also channel blocks of O
  constexpr int TILE_BYTES = 64 * D;         // one K^ or V^ tile of 64 keys
  constexpr int QT = 32 * NW;                // queries per workgroup
  constexpr int CHUNKS = 2 * TILE_BYTES / 16 / (64 * NW);  // 16-byte chunks per thread per tile pair
  static_assert(CHUNKS >= 1, "tile too small for this workgroup");

  __shared__ __attribute__((aligned(16))) int8_t lds[2][2 * TILE_BYTES];   // [buf][K tile | V tile]

  // XCD-aware mapping: consecutive workgroup ids go round-robin over the 8 XCDs, so all
  // query tiles of one head are given ids with the same residue and share one L2.
  const int g = blockIdx.x;
  const int xcd = g & 7, slot = g >> 3;
  const int bh = xcd + 8 * (slot / args.n_qtiles);
  if (bh >= args.BH) return;
  // heaviest (last) query tiles first under the causal mask
  const int qt = args.n_qtiles - 1 - (slot % args.n_qtiles);

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int ql = lane & 31, h = lane >> 5;
  const int N = args.N;
  const int q0 = qt * QT + 32 * wave;        // first query of this wave
  const int q = q0 + ql;
  const int nblk = N / kBlock;

  const int8_t* KFh = args.KF + (size_t)bh * N * D;
  const int8_t* VTh = args.VT + (size_t)bh * N * D;
  const float* sKh = args.sK + (size_t)bh * nblk;
  const float* sVh = args.sV + (size_t)bh * nblk;

  // Q^ fragments stay in registers for the whole loop
  v4i qf[KS];
  {
    const int8_t* p = args.QF + (size_t)bh * N * D + (size_t)(q0 / 32) * KS * 1024 + lane * 16;
#pragma unroll
    for (int s = 0; s < KS; s++) qf[s] = *(const v4i*)(p + s * 1024);
  }
  const float cq = args.sQ[(size_t)bh * nblk + q0 / kBlock] * args.scale_log2e;
  const float* bias_row = QSMOOTH ? args.bias + ((size_t)bh * nblk + q0 / kBlock) * N : nullptr;

  const int n_tiles = CAUSAL ? (qt * QT + QT) / kBlock : nblk;

  v16f oacc[KS];
#pragma unroll
  for (int cb = 0; cb < KS; cb++)
#pragma unroll
    for (int r = 0; r < 16; r++) oacc[cb][r] = 0.f;
  float m_ref = -INFINITY;   // log2 domain
  float l_part = 0.f;        // this lane's share of sum(127 p) relative to m_ref

  // stage tile 0
  v4i pre[CHUNKS];
  {
#pragma unroll
    for (int c = 0; c < CHUNKS; c++) {
      const int idx = (tid + c * 64 * NW) * 16;
      const int8_t* src = idx < TILE_BYTES ? KFh + idx : VTh + (idx - TILE_BYTES);
      pre[c] = *(const v4i*)src;
    }
#pragma unroll
    for (int c = 0; c < CHUNKS; c++) *(v4i*)(&lds[0][(tid + c * 64 * NW) * 16]) = pre[c];
  }
  __syncthreads();

  for (int j = 0; j < n_tiles; j++) {
    const int buf = j & 1;
    if (j + 1 < n_tiles) {
#pragma unroll
      for (int c = 0; c < CHUNKS; c++) {
        const int idx = (tid + c * 64 * NW) * 16;
        const int8_t* src = idx < TILE_BYTES ? KFh + (size_t)(j + 1) * TILE_BYTES + idx
                                             : VTh + (size_t)(j + 1) * TILE_BYTES + (idx - TILE_BYTES);
        pre[c] = *(const v4i*)src;
      }
    }

    const int k0 = j * kBlock;
    const bool active = !CAUSAL || (k0 <= q0 + 31);
    if (active) {
      const int8_t* Kt = &lds[buf][0];
      const int8_t* Vt = &lds[buf][TILE_BYTES];
      const float c = cq * sKh[j];
      const float sv = sVh[j];
      const bool diag = CAUSAL && (k0 + 63 > q0);   // some key of the tile may exceed some query
      if (diag) fwd_tile<D, QSMOOTH, true>(Kt, Vt, qf, oacc, m_ref, l_part, c, sv, bias_row, k0, q, lane, h);
      else fwd_tile<D, QSMOOTH, false>(Kt, Vt, qf, oacc, m_ref, l_part, c, sv, bias_row, k0, q, lane, h);
    }

    if (j + 1 < n_tiles) {
#pragma unroll
      for (int c = 0; c < CHUNKS; c++) *(v4i*)(&lds[buf ^ 1][(tid + c * 64 * NW) * 16]) = pre[c];
    }
    __syncthreads();
  }

  // ---- epilogue: O = O / l, L = m + log(l) (l carries a factor 127) ----
  const float l_tot = half_swap_sum_f32(l_part);
  const float inv_l = 1.0f / l_tot;
  unsigned short* Oh = args.O + ((size_t)bh * N + q) * D;
#pragma unroll
  for (int cb = 0; cb < KS; cb++)
#pragma unroll
    for (int aa = 0; aa < 4; aa++) {
      v4us o;
#pragma unroll
      for (int b = 0; b < 4; b++) o[b] = float_to_bf16_bits(oacc[cb][4 * aa + b] * inv_l);
      *(v4us*)(Oh + 32 * cb + 8 * aa + 4 * h) = o;
    }
  if (h == 0) args.LSE[(size_t)bh * N + q] = (m_ref + __builtin_amdgcn_logf(l_tot) - kLog2_127) * kLn2;
}

}  // namespace sage
