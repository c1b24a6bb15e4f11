// Fused INT8 attention backward (paper Algorithm 2) for gfx950.
//
// A workgroup of 4 waves owns one KV block j (64 keys) and walks the Q blocks i.  Per
// (i, j) tile:
//   phase A  each wave takes one 32x32 quadrant (qb, kb) of the tile:
//            S = Q^ K^^T on INT8 MFMA, dP = dO V^T on bf16 MFMA (the one unquantised matmul),
//            P = exp(S - L), dS = P o (dP - delta); tile-wide max P and max |dS| are exchanged
//            through LDS; psi(P), psi(dS) are written to LDS as MFMA operand fragments.
//   phase B  each wave takes one 32-channel slice of the outputs and contracts over the whole
//            tile: dV^T += dO^^T P^, dK^T += Q^^T dS^ (accumulated in FP32 registers with the
//            per-tile scales).  psi(dS_ij) and its scale are also stored to a scratch buffer.
// A second kernel (sage_bwd_dq_kernel) owns one Q block per workgroup and forms
//   dQ_i = sum_j s_dS(i,j) s_K(j) sm_scale * (dS^_ij K^_j)
// from the stored INT8 tiles: a plain scaled INT8 GEMM with no atomics, so dQ is
// deterministic.  (A first version added dQ with FP32 atomics from the first kernel; at
// N=8192 the 4.3e9 atomic adds alone took 13 ms.)
//
// S is formed untransposed (queries x keys): an accumulator lane then holds one key and 16
// queries, which is the B-operand form of the two contractions over queries (dV, dK).  The
// contraction over keys (dQ) needs dS^ with one query per lane; that copy is scattered to
// LDS bytewise (no VALU work) in the key order of the TF layout of K^, and copied out from
// there in 16-byte pieces.
#pragma once

#include "common.h"

namespace sage {

struct BwdArgs {
  const int8_t* QF;    // F layout   (S recompute, A operand)
  const int8_t* QT;    // TF layout  (dK, A operand)
  const int8_t* KF;    // F layout   (S recompute, B operand)
  const int8_t* dOT;   // TF layout  (dV, A operand)
  const unsigned short* V;    // bf16 [BH, N, D]
  const unsigned short* dO;   // bf16 [BH, N, D]
  const float* sQ;
  const float* sK;
  const float* sdO;
  const float* LSE;    // [BH, N]
  const float* delta;  // [BH, N]
  const float* bias;   // Q-smoothing logit bias [BH, N/64, N] (log2 domain) or nullptr
  const float* muQ;    // Q-smoothing block means [BH, N/64, D] or nullptr
  int8_t* dSq;         // psi(dS) tiles [heads, N/64, N/64, 4096], A fragments (q block, key step)
  float* sdS;          // their scales [heads, N/64, N/64]
  int bh0;             // first head of this launch (the scratch above is indexed from it)
  unsigned short* dK;  // bf16 [BH, N, D]
  unsigned short* dV;
  int BH, N;
  float sm_scale;
  float scale_log2e;
};

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kRoundMagic = 12582912.0f;   // 1.5 * 2^23: x + magic has rne(x) in its low mantissa bits

template <int D, bool CAUSAL, bool QSMOOTH>
__global__ void __launch_bounds__(256, 2) sage_bwd_kernel(BwdArgs args) {
  constexpr int KS = D / 32;     // INT8 k-steps over d; channel blocks
  constexpr int KB = D / 16;     // bf16 k-steps over d
  constexpr int NPB = KS / 2;    // 32-row blocks per wave in phase B (2 for D=128, 1 for D=64)
  constexpr int TILE = 64 * D;   // bytes of one INT8 tile

  __shared__ __attribute__((aligned(16))) int8_t s_qf[TILE];
  __shared__ __attribute__((aligned(16))) int8_t s_qt[TILE];
  __shared__ __attribute__((aligned(16))) int8_t s_dot[TILE];
  __shared__ __attribute__((aligned(16))) int8_t s_dof[2 * TILE];   // bf16 dO as A fragments
  __shared__ __attribute__((aligned(16))) float s_l[64];            // L * log2(e)
  __shared__ __attribute__((aligned(16))) float s_dl[64];           // delta
  __shared__ __attribute__((aligned(16))) int8_t s_pb[4096];        // psi(P)  B fragments (q step, key block)
  __shared__ __attribute__((aligned(16))) int8_t s_dsb[4096];       // psi(dS) B fragments
  __shared__ __attribute__((aligned(16))) int8_t s_dst[4096];       // psi(dS) A fragments (q block, key step)
  __shared__ float s_red[4][2];
  __shared__ float s_cs[2][64];                                     // Q-smoothing: column sums of dS
  __shared__ __attribute__((aligned(16))) float s_muq[D];

  const int g = blockIdx.x;
  const int xcd = g & 7, slot = g >> 3;
  const int N = args.N;
  const int nblk = N / kBlock;
  const int hl = xcd + 8 * (slot / nblk);   // head within this launch
  if (hl >= args.BH) return;
  const int bh = args.bh0 + hl;
  const int j = slot % nblk;          // small j = most Q blocks under the causal mask: scheduled first

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int ll = lane & 31, h = lane >> 5;
  const int qb = wave >> 1, kb = wave & 1;                 // phase A quadrant
  const int cb = (D == 128) ? wave : (wave & 1);           // phase B channel block
  const int blk0 = (D == 128) ? 0 : (wave >> 1);           // phase B first 32-row block

  const size_t head = (size_t)bh * N * D;
  const float sKj = args.sK[(size_t)bh * nblk + j];

  // ---- operands that stay in registers for the whole loop ----
  v4i kfr[KS];
  {
    const int8_t* p = args.KF + head + ((size_t)(2 * j + kb) * KS) * 1024 + lane * 16;
#pragma unroll
    for (int s = 0; s < KS; s++) kfr[s] = *(const v4i*)(p + s * 1024);
  }
  v8bf vfr[KB];
  {
    const unsigned short* p = args.V + head + (size_t)(64 * j + 32 * kb + ll) * D + 8 * h;
#pragma unroll
    for (int s = 0; s < KB; s++) vfr[s] = *(const v8bf*)(p + 16 * s);
  }
  v16f dvacc[NPB], dkacc[NPB], dkbias[QSMOOTH ? NPB : 1];
#pragma unroll
  for (int t = 0; t < NPB; t++)
#pragma unroll
    for (int r = 0; r < 16; r++) {
      dvacc[t][r] = 0.f;
      dkacc[t][r] = 0.f;
      if constexpr (QSMOOTH) dkbias[t][r] = 0.f;
    }

  const int i_first = CAUSAL ? j : 0;
  // slot of key kappa = lane%32 inside a TF-ordered 32-key step: kappa = 8a + 4h' + b -> (h', 4a + b)
  const int tk_h = (ll >> 2) & 1, tk_t = 4 * (ll >> 3) + (ll & 3);

  // Staging of one Q block through registers.  Set A feeds phase A (Q^ row fragments, bf16 dO
  // fragments, L, delta), set B feeds phase B (Q^ and dO^ transposed fragments, mu_Q).
  constexpr int NI8 = TILE / 16 / 256;        // 16-byte pieces per thread of one INT8 tile
  constexpr int NBF = 2 * TILE / 16 / 256;    // same for the bf16 dO tile
  v4i ra_qf[NI8], ra_do[NBF], rb_qt[NI8], rb_dot[NI8];
  float ra_l = 0.f;
  v4f rb_muq = {0.f, 0.f, 0.f, 0.f};
  auto load_a = [&](int i) {
    const size_t toff = head + (size_t)i * TILE;
#pragma unroll
    for (int c = 0; c < NI8; c++) ra_qf[c] = *(const v4i*)(args.QF + toff + (tid + 256 * c) * 16);
    const unsigned short* src = args.dO + head + (size_t)i * 64 * D;
#pragma unroll
    for (int c = 0; c < NBF; c++) {
      const int cidx = tid + 256 * c;
      ra_do[c] = *(const v4i*)(src + (size_t)(cidx / (D / 8)) * D + (cidx % (D / 8)) * 8);
    }
    if (tid < 64) ra_l = args.LSE[(size_t)bh * N + 64 * i + tid] * kLog2e;
    else if (tid < 128) ra_l = args.delta[(size_t)bh * N + 64 * i + tid - 64];
  };
  auto store_a = [&]() {
#pragma unroll
    for (int c = 0; c < NI8; c++) *(v4i*)(s_qf + (tid + 256 * c) * 16) = ra_qf[c];
    // bf16 dO rows -> A fragments (32-row block, 16-channel step), lane = row + 32*(channel half);
    // the slot inside a fragment is XOR-swizzled with the step so these stores spread over banks
#pragma unroll
    for (int c = 0; c < NBF; c++) {
      const int cidx = tid + 256 * c;
      const int row = cidx / (D / 8), ch = cidx % (D / 8);
      const int s = ch >> 1, hh = ch & 1;
      const int slot_ = ((row & 31) + 32 * hh) ^ (s & 7);
      *(v4i*)(s_dof + (((row >> 5) * KB + s) * 64 + slot_) * 16) = ra_do[c];
    }
    if (tid < 64) s_l[tid] = ra_l;
    else if (tid < 128) s_dl[tid - 64] = ra_l;
  };
  auto load_b = [&](int i) {
    const size_t toff = head + (size_t)i * TILE;
#pragma unroll
    for (int c = 0; c < NI8; c++) {
      rb_qt[c] = *(const v4i*)(args.QT + toff + (tid + 256 * c) * 16);
      rb_dot[c] = *(const v4i*)(args.dOT + toff + (tid + 256 * c) * 16);
    }
    if constexpr (QSMOOTH) {
      if (tid < D / 4) rb_muq = *(const v4f*)(args.muQ + ((size_t)bh * nblk + i) * D + 4 * tid);
    }
  };
  auto store_b = [&]() {
#pragma unroll
    for (int c = 0; c < NI8; c++) {
      *(v4i*)(s_qt + (tid + 256 * c) * 16) = rb_qt[c];
      *(v4i*)(s_dot + (tid + 256 * c) * 16) = rb_dot[c];
    }
    if constexpr (QSMOOTH) {
      if (tid < D / 4) *(v4f*)(s_muq + 4 * tid) = rb_muq;
    }
  };

  load_a(nblk - 1);
  load_b(nblk - 1);
  store_a();
  store_b();
  __syncthreads();

  for (int i = nblk - 1; i >= i_first; i--) {
    const bool has_next = i > i_first;
    if (has_next) load_a(i - 1);

    // ---------------- phase A: quadrant (qb, kb) ----------------
    v16i sacc;
#pragma unroll
    for (int r = 0; r < 16; r++) sacc[r] = 0;
#pragma unroll
    for (int s = 0; s < KS; s++) {
      v4i a = *(const v4i*)(s_qf + ((qb * KS + s) * 64 + lane) * 16);
      sacc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, kfr[s], sacc, 0, 0, 0);
    }
    v16f dp;
#pragma unroll
    for (int r = 0; r < 16; r++) dp[r] = 0.f;
#pragma unroll
    for (int s = 0; s < KB; s++) {
      v8bf a = *(const v8bf*)(s_dof + ((qb * KB + s) * 64 + (lane ^ (s & 7))) * 16);
      dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, vfr[s], dp, 0, 0, 0);
    }
    const float sQi = args.sQ[(size_t)bh * nblk + i];
    const float sdOi = args.sdO[(size_t)bh * nblk + i];
    const float c = sQi * sKj * args.scale_log2e;
    float bias_l = 0.f;
    if constexpr (QSMOOTH) bias_l = args.bias[((size_t)bh * nblk + i) * N + 64 * j + 32 * kb + ll];
    const bool diag = CAUSAL && (i == j);
    float p[16], ds[16];
    float pm = 0.f, dm = 0.f, cs = 0.f;
#pragma unroll
    for (int aa = 0; aa < 4; aa++) {
      const v4f l4 = *(const v4f*)(s_l + 32 * qb + 8 * aa + 4 * h);
      const v4f d4 = *(const v4f*)(s_dl + 32 * qb + 8 * aa + 4 * h);
#pragma unroll
      for (int b = 0; b < 4; b++) {
        const int r = 4 * aa + b;
        const float x = __builtin_fmaf((float)sacc[r], c, bias_l - l4[b]);
        p[r] = __builtin_amdgcn_exp2f(x);
      }
      if (diag) {
#pragma unroll
        for (int b = 0; b < 4; b++)
          if ((32 * qb + 8 * aa + 4 * h + b) < (32 * kb + ll)) p[4 * aa + b] = 0.f;
      }
#pragma unroll
      for (int b = 0; b < 4; b++) {
        const int r = 4 * aa + b;
        ds[r] = p[r] * (dp[r] - d4[b]);
        pm = fmaxf(pm, p[r]);
        dm = fmaxf(dm, fabsf(ds[r]));
        if constexpr (QSMOOTH) cs += ds[r];
      }
    }
    pm = wave_max_f32(pm);
    dm = wave_max_f32(dm);
    if (lane == 0) {
      s_red[wave][0] = pm;
      s_red[wave][1] = dm;
    }
    if constexpr (QSMOOTH) {
      cs = half_swap_sum_f32(cs);
      if (h == 0) s_cs[qb][32 * kb + ll] = cs;
    }
    __syncthreads();   // (1) tile maxima visible; phase A reads of the staging buffers are done

    if (has_next) store_a();
    pm = fmaxf(fmaxf(s_red[0][0], s_red[1][0]), fmaxf(s_red[2][0], s_red[3][0]));
    dm = fmaxf(fmaxf(s_red[0][1], s_red[1][1]), fmaxf(s_red[2][1], s_red[3][1]));
    const float rP = pm > 0.f ? 127.0f / pm : 0.f;
    const float sP = pm / 127.0f;
    const float rS = dm > 0.f ? 127.0f / dm : 0.f;
    const float sS = dm / 127.0f;
    {
      v4i pf, df;
      int8_t* tbase = s_dst + ((qb * 2 + kb) * 64 + 32 * tk_h) * 16 + tk_t;
#pragma unroll
      for (int aa = 0; aa < 4; aa++) {
        unsigned up = 0;
        unsigned ub[4];
#pragma unroll
        for (int b = 0; b < 4; b++) {
          const int r = 4 * aa + b;
          up = __builtin_amdgcn_cvt_pk_u8_f32(p[r] * rP, b, up);
          ub[b] = __float_as_uint(__builtin_fmaf(ds[r], rS, kRoundMagic));
          tbase[(8 * aa + 4 * h + b) * 16] = (int8_t)ub[b];
        }
        pf[aa] = (int)up;
        const unsigned lo = __builtin_amdgcn_perm(ub[1], ub[0], 0x0c0c0400u);
        const unsigned hi = __builtin_amdgcn_perm(ub[3], ub[2], 0x04000c0cu);
        df[aa] = (int)(lo | hi);
      }
      *(v4i*)(s_pb + ((qb * 2 + kb) * 64 + lane) * 16) = pf;
      *(v4i*)(s_dsb + ((qb * 2 + kb) * 64 + lane) * 16) = df;
    }
    __syncthreads();   // (2) quantised tiles visible
    if (has_next) load_b(i - 1);

    // psi(dS_ij) and its scale go to the scratch buffer for the dQ kernel
    {
      const size_t tile = ((size_t)hl * nblk + i) * nblk + j;
      *(v4i*)(args.dSq + tile * 4096 + tid * 16) = *(const v4i*)(s_dst + tid * 16);
      if (tid == 0) args.sdS[tile] = sS;
    }

    // ---------------- phase B: channel block cb ----------------
    const float w_dv = sP * sdOi;
    const float w_dk = sS * sQi * args.sm_scale;
#pragma unroll
    for (int t = 0; t < NPB; t++) {
      const int kbo = blk0 + t;
      v16i av, ak;
#pragma unroll
      for (int r = 0; r < 16; r++) {
        av[r] = 0;
        ak[r] = 0;
      }
#pragma unroll
      for (int qs = 0; qs < 2; qs++) {
        const v4i a1 = *(const v4i*)(s_dot + ((qs * KS + cb) * 64 + lane) * 16);
        const v4i b1 = *(const v4i*)(s_pb + ((qs * 2 + kbo) * 64 + lane) * 16);
        av = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, b1, av, 0, 0, 0);
        const v4i a2 = *(const v4i*)(s_qt + ((qs * KS + cb) * 64 + lane) * 16);
        const v4i b2 = *(const v4i*)(s_dsb + ((qs * 2 + kbo) * 64 + lane) * 16);
        ak = __builtin_amdgcn_mfma_i32_32x32x32_i8(a2, b2, ak, 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < 16; r++) {
        dvacc[t][r] = __builtin_fmaf((float)av[r], w_dv, dvacc[t][r]);
        dkacc[t][r] = __builtin_fmaf((float)ak[r], w_dk, dkacc[t][r]);
      }
      if constexpr (QSMOOTH) {
        // dK_bias = (dS^T 1) mu_Q^T with the unquantised column sums of this tile
        const float csv = s_cs[0][32 * kbo + ll] + s_cs[1][32 * kbo + ll];
#pragma unroll
        for (int aa = 0; aa < 4; aa++) {
          const v4f m4 = *(const v4f*)(s_muq + 32 * cb + 8 * aa + 4 * h);
#pragma unroll
          for (int b = 0; b < 4; b++) dkbias[t][4 * aa + b] = __builtin_fmaf(csv, m4[b], dkbias[t][4 * aa + b]);
        }
      }
    }
    __syncthreads();   // (3) phase B reads done: the phase-B staging and exchange buffers are free
    if (has_next) store_b();
  }

  // ---- write dV, dK (bf16) ----
#pragma unroll
  for (int t = 0; t < NPB; t++) {
    const int key = 64 * j + 32 * (blk0 + t) + ll;
    unsigned short* pv = args.dV + head + (size_t)key * D + 32 * cb + 4 * h;
    unsigned short* pk = args.dK + head + (size_t)key * D + 32 * cb + 4 * h;
#pragma unroll
    for (int aa = 0; aa < 4; aa++) {
      v4us ov, ok;
#pragma unroll
      for (int b = 0; b < 4; b++) {
        float kv = dkacc[t][4 * aa + b];
        if constexpr (QSMOOTH) kv = __builtin_fmaf(dkbias[t][4 * aa + b], args.sm_scale, kv);
        ov[b] = float_to_bf16_bits(dvacc[t][4 * aa + b]);
        ok[b] = float_to_bf16_bits(kv);
      }
      *(v4us*)(pv + 8 * aa) = ov;
      *(v4us*)(pk + 8 * aa) = ok;
    }
  }
}

// ---------------------------------------------------------------------------------
// dQ_i = sum_j (dS^_ij K^_j) * s_dS(i,j) * s_K(j) * sm_scale        (Algorithm 2, the dQ line)
// One workgroup per Q block; each wave owns a 32-channel slice and streams its operands
// straight from global memory / L2 (no LDS, no barriers): A = stored psi(dS) fragments,
// B = K^ in TF layout.
struct DqArgs {
  const int8_t* dSq;
  const float* sdS;
  const int8_t* KT;
  const float* sK;
  unsigned short* dQ;   // bf16 [BH, N, D]
  int BH, N, bh0;
  float sm_scale;
};

template <int D, bool CAUSAL>
__global__ void __launch_bounds__(256, 2) sage_bwd_dq_kernel(DqArgs args) {
  constexpr int KS = D / 32;
  constexpr int NPB = KS / 2;
  const int g = blockIdx.x;
  const int xcd = g & 7, slot = g >> 3;
  const int N = args.N;
  const int nblk = N / kBlock;
  const int hl = xcd + 8 * (slot / nblk);
  if (hl >= args.BH) return;
  const int bh = args.bh0 + hl;
  const int i = nblk - 1 - (slot % nblk);      // longest rows first under the causal mask
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int ll = lane & 31, h = lane >> 5;
  const int cb = (D == 128) ? wave : (wave & 1);
  const int blk0 = (D == 128) ? 0 : (wave >> 1);
  const size_t head = (size_t)bh * N * D;
  const int n_j = CAUSAL ? i + 1 : nblk;

  const int8_t* ds_row = args.dSq + ((size_t)hl * nblk + i) * nblk * 4096 + lane * 16;
  const float* sc_row = args.sdS + ((size_t)hl * nblk + i) * nblk;
  const float* sKh = args.sK + (size_t)bh * nblk;
  const int8_t* kt = args.KT + head + (size_t)cb * 1024 + lane * 16;

  v16f acc[NPB];
#pragma unroll
  for (int t = 0; t < NPB; t++)
#pragma unroll
    for (int r = 0; r < 16; r++) acc[t][r] = 0.f;

  v4i a_cur[NPB][2], b_cur[2];
  auto load_tile = [&](int j, v4i (&a)[NPB][2], v4i (&b)[2]) {
#pragma unroll
    for (int ks = 0; ks < 2; ks++) {
      b[ks] = *(const v4i*)(kt + (size_t)(2 * j + ks) * KS * 1024);
#pragma unroll
      for (int t = 0; t < NPB; t++) a[t][ks] = *(const v4i*)(ds_row + (size_t)j * 4096 + ((blk0 + t) * 2 + ks) * 1024);
    }
  };
  load_tile(0, a_cur, b_cur);
  for (int j = 0; j < n_j; j++) {
    v4i a_nxt[NPB][2], b_nxt[2];
    if (j + 1 < n_j) load_tile(j + 1, a_nxt, b_nxt);
    const float w = sc_row[j] * sKh[j] * args.sm_scale;
#pragma unroll
    for (int t = 0; t < NPB; t++) {
      v16i q;
#pragma unroll
      for (int r = 0; r < 16; r++) q[r] = 0;
#pragma unroll
      for (int ks = 0; ks < 2; ks++) q = __builtin_amdgcn_mfma_i32_32x32x32_i8(a_cur[t][ks], b_cur[ks], q, 0, 0, 0);
#pragma unroll
      for (int r = 0; r < 16; r++) acc[t][r] = __builtin_fmaf((float)q[r], w, acc[t][r]);
    }
    if (j + 1 < n_j) {
#pragma unroll
      for (int ks = 0; ks < 2; ks++) {
        b_cur[ks] = b_nxt[ks];
#pragma unroll
        for (int t = 0; t < NPB; t++) a_cur[t][ks] = a_nxt[t][ks];
      }
    }
  }
  // accumulator lane = channel, registers = query rows 8a + 4h + b of the 32-row block
#pragma unroll
  for (int t = 0; t < NPB; t++) {
    unsigned short* dst = args.dQ + head + (size_t)(64 * i + 32 * (blk0 + t) + 4 * h) * D + 32 * cb + ll;
#pragma unroll
    for (int aa = 0; aa < 4; aa++)
#pragma unroll
      for (int b = 0; b < 4; b++) dst[(size_t)(8 * aa + b) * D] = float_to_bf16_bits(acc[t][4 * aa + b]);
  }
}

}  // namespace sage
