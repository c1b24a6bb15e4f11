// Fused INT8 attention forward (paper Algorithm 1) for gfx950.
//
// One wave owns 32 queries; a workgroup of NW waves owns 32*NW consecutive queries of
// one head and walks the KV blocks (64 keys each).  K^ and V^ fragments are copied
// global -> LDS asynchronously into a ring of four tile buffers, one barrier per tile.
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
// Software pipeline inside a wave: the MFMAs of S_{j+1} are issued before the softmax of
// tile j, and the MFMAs of one 32-channel block of P^V^ before the FP32 update of the
// previous block, so that the matrix pipe works underneath the vector work of the same wave.
//
// Per-token quantisation: P~/s_P with s_P = exp(rowmax(S_ij) - m_ij)/127 equals
// 127 * exp(S_ij - rowmax(S_ij)), which does not depend on the running max.  The kernel
// evaluates that form (never 0/0) and keeps the running reference m only for the FP32
// accumulators: O += beta * s_V * (P^ V^), l += beta * sum(127 p), beta = exp(rowmax - m).
// m is raised only when a tile's row max exceeds it by more than kTau (in log2 units); the
// result is unchanged because O/l and m + log l do not depend on the reference chosen.
//
// INT32 -> FP32 without a conversion instruction: the P^V^ accumulators start from the bit
// pattern B0 of the float C0 = 1/(2 pi) (an inline constant of the ISA; the compiler keeps the
// splat in 16 registers because several MFMAs start from it).  B0's mantissa leaves more than 2^20 codes to either end of its binade, so for
// every possible sum |a| <= 64 * 127 * 127 the bits B0 + a read as the float C0 + a * 2^-26
// exactly.  The FP32 accumulators take w * 2^26 * (C0 + a * 2^-26) with ONE fused multiply-add
// per value and so carry the bias C0 * 2^26 * sum(w), the same for every channel of a query;
// it is subtracted every kBiasPeriod tiles and at the end.  Between corrections the bias stays
// below about 2^26 times the weight of a tile, so each addition still resolves a * w to about
// one part in 10^4 of a typical tile's contribution.  Measured at N = 8192 against the CPU oracle:
// relative L1 of O 2.5e-4 (6e-5 when the bias is subtracted after every tile, 4e-4 with a period
// of 16), an order of magnitude below the rounding of the bf16 output and the 1e-2 tolerance.
// The logits' accumulators use the same start where the tile scales allow it (SBIAS in fwd_tile;
// |s| <= 128 * 127 * 127 still fits the binade): O then sits 5e-4 from the oracle, L 4e-5.
#pragma once

#include <type_traits>

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
  unsigned short* O;    // bf16, rows addressed through `oview` (dense [BH, N, D] or the caller's token-major tensor)
  RowView oview;
  float* LSE;           // [BH, nq_valid]
  int BH, N;            // N = rows of the K-like workspace tensors (N_kv rounded up to a multiple of 64)
  int nvalid;           // keys >= nvalid do not exist (nvalid = N unless N_kv is not a multiple of 64)
  int Nq;               // rows of the Q-like workspace tensors (N_q rounded up to a multiple of 64)
  int nq_valid;         // query rows >= nq_valid do not exist
  int shift;            // causal: query i sees keys k <= i + shift (N_kv - N_q, a multiple of 64)
  int n_qtiles;         // workgroups per head
  int head_set;         // heads per XCD whose work items are interleaved (see work_item)
  float scale_log2e;    // sm_scale * log2(e)
};

constexpr float kTau = 8.0f;
constexpr float kLog2_127 = 6.98868468677216585f;
constexpr float kLn2 = 0.69314718055994531f;
constexpr int kBiasBits = 0x3E22F983;         // bit pattern of 1/(2 pi): an inline constant of the ISA
constexpr float kBiasC0 = 0.15915494309189532f;
constexpr float kTwo26 = 67108864.0f;
constexpr int kBiasPeriod = 8;                // tiles between two subtractions of the accumulated bias

// Keeps the computation of `v` where it is written: without a use at this point the compiler
// sinks the vector work of a chunk past the scheduling barriers into the next basic block.
__device__ __forceinline__ void pin(float& v) { asm volatile("" : "+v"(v)); }

// S^T accumulators of one 64-key tile (two 32-key blocks), interleaved so that consecutive
// MFMAs are independent.
template <int D, bool SBIAS>
__device__ __forceinline__ void fwd_s_mfma(const int8_t* __restrict__ Kt, const v4i (&qf)[D / 32], v16i (&sacc)[2],
                                           const int lane) {
  constexpr int KS = D / 32;
#pragma unroll
  for (int kb = 0; kb < 2; kb++)
#pragma unroll
    for (int r = 0; r < 16; r++) sacc[kb][r] = SBIAS ? kBiasBits : 0;
#pragma unroll
  for (int s = 0; s < KS; s++) {
#pragma unroll
    for (int kb = 0; kb < 2; kb++) {
      const v4i a = *(const v4i*)(Kt + (kb * KS + s) * 1024 + lane * 16);
      sacc[kb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, qf[s], sacc[kb], 0, 0, 0);
    }
  }
}

// One KV tile for one wave: (optionally) the logits of the NEXT tile on the matrix pipe, the
// softmax and per-token quantisation of THIS tile (`sacc`), then O^T += V^^T P^^T.
// MASK = the tile straddles the causal diagonal for this wave.
//
// The instruction stream is laid out by hand in chunks separated by scheduling barriers: each
// chunk pairs one MFMA (and the LDS read of an operand two MFMAs ahead) with the vector work of
// four logits or of sixteen output values, so that the matrix pipe and the LDS latency hide
// under the vector instructions of the same wave.
//
// KV128 = numerics blocks of 128 keys: the per-token quantiser of P~ (Algorithm 1 line 9) then takes its row
// max over both 64-key tiles of the block.  `pair` carries the other tile's row max in (INT_MIN / -inf if
// the other tile has no visible key) and this tile's own row max out.
struct PairMax {
  int i;      // integer domain (no Q-smoothing: both tiles of a block share the scale c)
  float f;    // log2 domain (Q-smoothing)
};
template <int D, bool QSMOOTH, bool MASK, bool NEXT, bool SBIAS, bool KV128 = false>
__device__ __forceinline__ void fwd_tile(const int8_t* __restrict__ Knext, const int8_t* __restrict__ Vt,
                                         const v4i (&qf)[D / 32], v16i (&sacc)[2], v16i (&snext)[2],
                                         float (&oacc)[D / 32][16], float& w_bias, float& m_ref, float& l_part,
                                         const float c, const float sv, const float* __restrict__ bias_row,
                                         const int k0, const int q, const int lane, const int h,
                                         PairMax* pair = nullptr) {
  constexpr int KS = D / 32;
  constexpr int NSM = 2 * KS;    // MFMAs of the next tile's logits; MFMA m = (k-step m / 2, key block m % 2)
  const int8_t* kl = Knext + lane * 16;
  const int8_t* vl = Vt + lane * 16;
  auto k_frag = [&](int m) { return *(const v4i*)(kl + ((m & 1) * KS + (m >> 1)) * 1024); };
  auto v_frag = [&](int m) { return *(const v4i*)(vl + m * 1024); };   // m = kb * KS + cb

  v4i ka[3];
  if constexpr (NEXT) {
    ka[0] = k_frag(0);
    ka[1] = k_frag(1);
  }

  float x[2][16];
  float mloc;   // row max of the tile in the log2 domain
  float bmax_f = 0.f;   // SBIAS: the row max as the float its bits spell
  if constexpr (!QSMOOTH) {
    // the scale is one positive scalar per tile, so the row max can be taken on the integers
    int mi[2] = {INT_MIN, INT_MIN};
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
        mi[kb] = max(mi[kb], v);
      }
    // (with SBIAS the accumulators hold B0 + s: the same order, and B0 + s never is INT_MIN)
    int mrow = half_swap_max_i32(max(mi[0], mi[1]));
    if constexpr (KV128) {
      const int own = mrow;
      mrow = max(mrow, pair->i);
      pair->i = own;
    }
    mloc = (float)(mrow - (SBIAS ? kBiasBits : 0)) * c;
    if constexpr (SBIAS) bmax_f = __int_as_float(mrow);
  } else {
    float mf = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; kb++)
#pragma unroll
      for (int aa = 0; aa < 4; aa++) {
        const int key = k0 + 32 * kb + 8 * aa + 4 * h;
        const v4f b4 = *(const v4f*)(bias_row + (key - k0));   // the tile's 64 biases, staged in LDS
#pragma unroll
        for (int b = 0; b < 4; b++) {
          float v = __builtin_fmaf((float)sacc[kb][4 * aa + b], c, b4[b]);
          if constexpr (MASK) v = (key + b) > q ? -INFINITY : v;
          x[kb][4 * aa + b] = v;
          mf = fmaxf(mf, v);
        }
      }
    mloc = half_swap_max_f32(mf);
    if constexpr (KV128) {
      const float own = mloc;
      mloc = fmaxf(mloc, pair->f);
      pair->f = own;
    }
  }
  // ---- online softmax reference (rarely raised) ----
  if (__builtin_amdgcn_ballot_w64(mloc > m_ref + kTau) != 0) {
    const float m_new = fmaxf(m_ref, mloc);
    const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);   // 0 on the first tile
    l_part *= alpha;
    w_bias *= alpha;
#pragma unroll
    for (int cb = 0; cb < KS; cb++)
#pragma unroll
      for (int r = 0; r < 16; r++) oacc[cb][r] *= alpha;
    m_ref = m_new;
  }
  const float beta = __builtin_amdgcn_exp2f(mloc - m_ref);
  // SBIAS: the logits' accumulators started from the bits of C0, so they read as the floats
  // C0 + s * 2^-26 and x = s * c + off becomes one FMA on those floats, without a conversion; the
  // offset is formed from the row max taken the same way, so the largest logit of the row still
  // lands on log2(127) up to the rounding of the product C0 * 2^26 * c (the caller admits only
  // scales c for which that is far below the half code that would carry 127 to 128).
  const float c_eff = SBIAS ? c * kTwo26 : c;
  const float off = SBIAS ? __builtin_fmaf(-bmax_f, c_eff, kLog2_127) : kLog2_127 - mloc;
  __builtin_amdgcn_sched_barrier(0);

  // ---- slots 0..7: P^ = rne(127 exp(S - rowmax)) for four logits each, packed as the B operand;
  //      row sum of 127 p.  Matrix work issued underneath: MFMA m of the next tile's logits in
  //      slot m; the first half of O^T += V^^T P^^T (key block 0, channel block cb) in slot 4 + cb.
  // ---- slots 8..: the second half (key block 1) in slot 8 + cb, and the FP32 update of channel
  //      block cb in slots 10 + 2 cb and 11 + 2 cb.  V^ fragments are read two slots ahead. ----
  v4i pf[2];
  v4i va[4];
  v16i t[KS];
  float psum[4] = {0.f, 0.f, 0.f, 0.f};
  float w = 0.f;
  constexpr int NSLOT = 10 + 2 * KS;
  auto pv_slot = [&](int m) { return m < KS ? 4 + m : 8 + (m - KS); };   // slot of P^V^ MFMA m = (kb, cb)
#pragma unroll
  for (int sl = 0; sl < NSLOT; sl++) {
    // The softmax slots carry the long dependency chains (max, exp2, pack); a wave in them gets issue
    // priority over its SIMD neighbour, which is mostly in the matrix-heavy second half (measured: 5-7 %).
    if (sl == 0) __builtin_amdgcn_s_setprio(1);
    if (sl == 8) __builtin_amdgcn_s_setprio(0);
    // LDS reads: V^ fragment of the MFMA two slots ahead
#pragma unroll
    for (int m = 0; m < 2 * KS; m++)
      if (pv_slot(m) == sl + 2) va[m & 3] = v_frag(m);
    // matrix work of this slot
    if constexpr (NEXT) {
      if (sl < NSM) {
        if (sl + 2 < NSM) ka[(sl + 2) % 3] = k_frag(sl + 2);
        if (sl < 2) {
          v16i z;
#pragma unroll
          for (int r = 0; r < 16; r++) z[r] = SBIAS ? kBiasBits : 0;
          snext[sl & 1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ka[sl % 3], qf[sl >> 1], z, 0, 0, 0);
        } else {
          snext[sl & 1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ka[sl % 3], qf[sl >> 1], snext[sl & 1], 0, 0, 0);
        }
      }
    }
#pragma unroll
    for (int m = 0; m < 2 * KS; m++)
      if (pv_slot(m) == sl) {
        if (m < KS) {
          v16i b0;
#pragma unroll
          for (int r = 0; r < 16; r++) b0[r] = kBiasBits;
          t[m] = __builtin_amdgcn_mfma_i32_32x32x32_i8(va[m & 3], pf[0], b0, 0, 0, 0);
        }
        else t[m - KS] = __builtin_amdgcn_mfma_i32_32x32x32_i8(va[m & 3], pf[1], t[m - KS], 0, 0, 0);
      }
    // vector work of this slot
    if (sl < 8) {
      const int kb = sl >> 2, aa = sl & 3;
      unsigned u = 0;
#pragma unroll
      for (int b = 0; b < 4; b++) {
        float xv;
        if constexpr (!QSMOOTH) {
          if constexpr (SBIAS) xv = __builtin_fmaf(__int_as_float(sacc[kb][4 * aa + b]), c_eff, off);
          else xv = __builtin_fmaf((float)sacc[kb][4 * aa + b], c, off);
          if constexpr (MASK) xv = sacc[kb][4 * aa + b] == INT_MIN ? -INFINITY : xv;
        } else {
          xv = x[kb][4 * aa + b] + off;
        }
        const float e = __builtin_amdgcn_exp2f(xv);
        psum[b] += e;
        pin(psum[b]);
        u = __builtin_amdgcn_cvt_pk_u8_f32(e, b, u);
      }
      pf[kb][aa] = (int)u;
    } else if (sl == 8) {
      l_part = __builtin_fmaf(beta, (psum[0] + psum[1]) + (psum[2] + psum[3]), l_part);
      w = beta * sv * kTwo26;
      w_bias += w;
      pin(l_part);
      pin(w);
      pin(w_bias);
    } else if (sl >= 10) {
      const int cb = (sl - 10) >> 1, half = (sl - 10) & 1;
#pragma unroll
      for (int r = 8 * half; r < 8 * half + 8; r++) {
        oacc[cb][r] = __builtin_fmaf(__int_as_float(t[cb][r]), w, oacc[cb][r]);
        pin(oacc[cb][r]);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }
}

// Row max of one tile's logits `s` over the keys a lane's query sees (key <= qlim), as fwd_tile forms it:
// the integer max (no Q-smoothing) or the max of s * c + bias in the log2 domain.
template <bool QSMOOTH, bool MASK>
__device__ __forceinline__ PairMax tile_row_max(const v16i (&s)[2], const float c, const float* __restrict__ bias_row,
                                                const int k0, const int qlim, const int h) {
  PairMax m{INT_MIN, -INFINITY};
#pragma unroll
  for (int kb = 0; kb < 2; kb++)
#pragma unroll
    for (int aa = 0; aa < 4; aa++) {
      const int key = k0 + 32 * kb + 8 * aa + 4 * h;
      v4f b4 = {0.f, 0.f, 0.f, 0.f};
      if constexpr (QSMOOTH) b4 = *(const v4f*)(bias_row + (key - k0));
#pragma unroll
      for (int b = 0; b < 4; b++) {
        const bool hidden = MASK && (key + b) > qlim;
        if constexpr (QSMOOTH) {
          const float v = __builtin_fmaf((float)s[kb][4 * aa + b], c, b4[b]);
          m.f = fmaxf(m.f, hidden ? -INFINITY : v);
        } else {
          m.i = max(m.i, hidden ? INT_MIN : s[kb][4 * aa + b]);
        }
      }
    }
  if constexpr (QSMOOTH) m.f = half_swap_max_f32(m.f);
  else m.i = half_swap_max_i32(m.i);
  return m;
}

template <int D, bool CAUSAL, bool QSMOOTH, int NW, bool KV128 = false>
__global__ void __launch_bounds__(64 * NW, (NW == 4 ? (D == 64 ? 3 : 2) : 1)) sage_fwd_kernel(FwdArgs args) {
  constexpr int KS = D / 32;                 // k-steps of Q K^T; also channel blocks of O
  constexpr int TILE_BYTES = 64 * D;         // one K^ or V^ tile of 64 keys
  constexpr int PAIR = 2 * TILE_BYTES;       // K^ tile | V^ tile
  constexpr int NFRAG = PAIR / 1024;         // 1 KiB fragments per pair
  constexpr int QT = 32 * NW;                // queries per workgroup

  // Q-smoothing: the 64 logit biases of each wave's Q block and the tile's keys travel with the tile too
  constexpr int BIAS_OFF = PAIR + 64;
  constexpr int SLOT = BIAS_OFF + (QSMOOTH ? NW * 256 : 0);
  __shared__ __attribute__((aligned(16))) int8_t lds[4][SLOT];   // K^ | V^ | per-wave (s_K, s_V) | per-wave bias row

  // workgroup -> (head, query tile): a head's tiles share one XCD's L2; heaviest (last) query
  // tiles first under the causal mask, over sets of heads (see work_item)
  const WorkItem wi = work_item(blockIdx.x, args.n_qtiles, args.head_set);
  const int bh = wi.head;
  if (bh >= args.BH) return;
  const int qt = args.n_qtiles - 1 - wi.item;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ql = lane & 31, h = lane >> 5;
  const int N = args.N;
  const int q0 = qt * QT + 32 * wave;        // first query of this wave
  const int q = q0 + ql;
  // last visible key of this lane's query: under the causal mask the query's own position among the
  // keys (a query row that does not exist may see keys that do not exist: it is dropped anyway), else
  // the last key
  const int qlim = CAUSAL ? q + args.shift : args.nvalid - 1;
  const int nblk = N / kBlock;               // KV blocks
  const int nqblk = args.Nq / kBlock;        // Q blocks

  const int8_t* KFh = args.KF + (size_t)bh * N * D;
  const int8_t* VTh = args.VT + (size_t)bh * N * D;
  const float* sKh = args.sK + (size_t)bh * nblk;
  const float* sVh = args.sV + (size_t)bh * nblk;

  // Q^ fragments stay in registers for the whole loop
  v4i qf[KS];
  {
    const int8_t* p = args.QF + (size_t)bh * args.Nq * D + (size_t)(q0 / 32) * KS * 1024 + lane * 16;
#pragma unroll
    for (int s = 0; s < KS; s++) qf[s] = *(const v4i*)(p + s * 1024);
  }
  const float cq = args.sQ[(size_t)bh * nqblk + q0 / kBlock] * args.scale_log2e;
  const float* bias_row = QSMOOTH ? args.bias + ((size_t)bh * nqblk + q0 / kBlock) * N : nullptr;

  const int n_tiles = CAUSAL ? (qt * QT + QT + args.shift) / kBlock : nblk;   // barrier count, uniform in the workgroup
  const int last = CAUSAL ? (q0 + 31 + args.shift) / kBlock : nblk - 1;       // this wave's last tile (masked if causal)

  float oacc[KS][16];
#pragma unroll
  for (int cb = 0; cb < KS; cb++)
#pragma unroll
    for (int r = 0; r < 16; r++) oacc[cb][r] = 0.f;
  float w_bias = 0.f;        // sum of the tile weights since the last bias subtraction (see the header)
  float m_ref = -INFINITY;   // log2 domain
  float l_part = 0.f;        // this lane's share of sum(127 p) relative to m_ref

  // Asynchronous copy of tile j (K^ fragments, then V^ fragments) into a ring slot; the
  // 1 KiB fragments are dealt round-robin to the waves.
  auto stage_load = [&](int j, int8_t* dst) {
#pragma unroll
    for (int k = 0; k < (NFRAG + NW - 1) / NW; k++) {
      const int o = wave + NW * k;           // wave-uniform
      if (o < NFRAG) {
        const int8_t* src = o < NFRAG / 2 ? KFh + (size_t)j * TILE_BYTES + o * 1024
                                          : VTh + (size_t)j * TILE_BYTES + (o - NFRAG / 2) * 1024;
        async_copy_16(src + lane * 16, dst + o * 1024);
      }
    }
    // the two block scales of the tile, one private copy per wave (lanes 0 and 1 carry them)
    if (lane < 2) async_copy_4((lane == 0 ? sKh : sVh) + j, dst + PAIR + wave * 8);
    if constexpr (QSMOOTH) async_copy_4(bias_row + j * kBlock + lane, dst + BIAS_OFF + wave * 256);
  };

  int8_t* cur = &lds[0][0];
  int8_t* nxt = &lds[1][0];
  int8_t* nx2 = &lds[2][0];
  int8_t* nx3 = &lds[3][0];
  stage_load(0, cur);
  if (n_tiles > 1) stage_load(1, nxt);
  if (n_tiles > 2) stage_load(2, nx2);
  barrier_all_memory();


  // Iteration j: tile j + 3 starts to load into the slot that tile j - 1 occupied (every wave is
  // past the barrier that ended iteration j - 1, so nobody reads it any more); this wave forms
  // S_{j+1} from slot `nxt` and finishes tile j with V^ from slot `cur`; before the barrier at
  // the end it waits for the copies of tile j + 2 (issued one iteration earlier), while its copies
  // of tile j + 3 stay in flight.  The block scales travel with the tiles, so the loop has no
  // register-returning global loads whose waits would also drain the copies.  Every wave of
  // the workgroup runs n_tiles iterations (the barriers must match): its unmasked tiles, its last
  // tile, then iterations that only keep the ring moving.
  constexpr int CPW = (NFRAG + NW - 1) / NW + (QSMOOTH ? 1 : 0);   // copies per wave and tile (every wave issues all of them)
  static_assert(NFRAG % NW == 0, "every wave must issue the same number of copies");
  auto end_iter = [&](const bool issued) {
    if (issued) {
      __builtin_amdgcn_s_waitcnt(0x0F70 | (CPW + 1));   // vmcnt: all but this iteration's copies
      barrier_lds_only();
    } else {
      barrier_all_memory();
    }
    int8_t* t = cur;
    cur = nxt;
    nxt = nx2;
    nx2 = nx3;
    nx3 = t;
  };
  // subtracts the bias that the output accumulators carry (see the header)
  auto unbias = [&]() {
    const float corr = kBiasC0 * w_bias;
#pragma unroll
    for (int cb = 0; cb < KS; cb++)
#pragma unroll
      for (int r = 0; r < 16; r++) oacc[cb][r] -= corr;
    w_bias = 0.f;
  };
  // The logits' accumulators can start from the bits of C0 as well (SBIAS, see fwd_tile), which
  // saves the INT32 -> FP32 conversion of every logit; that needs C0 * 2^26 * c, about 1e7 c, to
  // stay small against the half code between 127 and 128 in the log2 domain, so the wave takes
  // that path only if its largest tile scale c is below 1e-3 (QK-normed inputs sit near 1e-4).
  bool use_sbias = false;
  if constexpr (!QSMOOTH) {
    float smax = 0.f;
    for (int jj = lane; jj < n_tiles; jj += 64) smax = fmaxf(smax, sKh[jj]);
    use_sbias = cq * wave_max_nonneg_f32(smax) < 1e-3f;
  }
  auto run = [&](auto sbias_tag) __attribute__((always_inline)) {
    constexpr bool SBIAS = decltype(sbias_tag)::value;
    v16i sA[2], sB[2];
    fwd_s_mfma<D, SBIAS>(cur, qf, sA, lane);
    // KV128: numerics blocks of 128 keys = pairs of tiles (j even, j + 1).  The row max of the pair must be
    // known before either tile is quantised, so before the even tile the logits of the odd one are formed
    // once just for their row max (8 or 4 MFMAs that nothing overlaps) and dropped; fwd_tile then forms them
    // again under the even tile's softmax as it always does (the matrix pipe has the time, and holding them
    // instead would cost 32 registers this kernel does not have).  The odd tile takes the even tile's own
    // row max, which fwd_tile leaves in `pm`.
    PairMax pm{INT_MIN, -INFINITY};
    auto partner_max = [&](const int jn, auto mask_tag) __attribute__((always_inline)) {
      constexpr bool MASKED = decltype(mask_tag)::value;
      v16i sT[2];
      fwd_s_mfma<D, SBIAS>(nxt, qf, sT, lane);      // tile jn = j + 1 sits in the next ring slot
      const v2f scn = *(const v2f*)(nxt + PAIR + wave * 8);
      // (with SBIAS the accumulators hold B0 + s: the same order)
      pm = tile_row_max<QSMOOTH, MASKED>(sT, cq * scn[0], (const float*)(nxt + BIAS_OFF + wave * 256), jn * kBlock, qlim, h);
    };
    auto full_iter = [&](const int j, v16i (&sc)[2], v16i (&sn)[2]) __attribute__((always_inline)) {
      const bool issue = j + 3 < n_tiles;
      if (issue) stage_load(j + 3, nx3);
      const v2f sc2 = *(const v2f*)(cur + PAIR + wave * 8);
      fwd_tile<D, QSMOOTH, false, true, SBIAS, KV128>(nxt, cur + TILE_BYTES, qf, sc, sn, oacc, w_bias, m_ref, l_part,
                                        cq * sc2[0], sc2[1], (const float*)(cur + BIAS_OFF + wave * 256), j * kBlock, q, lane, h, &pm);
      if ((j & (kBiasPeriod - 1)) == kBiasPeriod - 1) unbias();
      end_iter(issue);
    };
    int j = 0;
    for (; j + 1 < last; j += 2) {
      if constexpr (KV128) partner_max(j + 1, std::false_type{});
      full_iter(j, sA, sB);
      full_iter(j + 1, sB, sA);
    }
    // (j is even here: either the last tile itself, which then has no partner, or the tile before it)
    if constexpr (KV128) pm = PairMax{INT_MIN, -INFINITY};
    if (j < last) {
      if constexpr (KV128) partner_max(j + 1, std::true_type{});
      full_iter(j, sA, sB);
#pragma unroll
      for (int kb = 0; kb < 2; kb++) sA[kb] = sB[kb];
      j++;
    }
    {
      const bool issue = j + 3 < n_tiles;
      if (issue) stage_load(j + 3, nx3);
      const v2f sc2 = *(const v2f*)(cur + PAIR + wave * 8);
      // (the last tile always takes the masked path: without the causal mask it hides the keys past nvalid)
      fwd_tile<D, QSMOOTH, true, false, SBIAS, KV128>(nxt, cur + TILE_BYTES, qf, sA, sB, oacc, w_bias, m_ref, l_part,
                                        cq * sc2[0], sc2[1], (const float*)(cur + BIAS_OFF + wave * 256), j * kBlock, qlim, lane, h, &pm);
      end_iter(issue);
      j++;
    }
    for (; j < n_tiles; j++) {
      const bool issue = j + 3 < n_tiles;
      if (issue) stage_load(j + 3, nx3);
      end_iter(issue);
    }
    unbias();
    // ---- epilogue: O = O / l, L = m + log(l) (l carries a factor 127) ----
    const float l_tot = half_swap_sum_f32(l_part);
    const float inv_l = 1.0f / l_tot;
    if (q >= args.nq_valid) return;                    // a query row that does not exist
    unsigned short* Oh = args.O + args.oview.row(bh, q);
#pragma unroll
    for (int cb = 0; cb < KS; cb++)
#pragma unroll
      for (int aa = 0; aa < 4; aa++) {
        v4us o;
#pragma unroll
        for (int b = 0; b < 4; b++) o[b] = float_to_bf16_bits(oacc[cb][4 * aa + b] * inv_l);
        *(v4us*)(Oh + 32 * cb + 8 * aa + 4 * h) = o;
      }
    // (LSE is [BH, nq_valid]: the caller's own row count)
    if (h == 0) args.LSE[(size_t)bh * args.nq_valid + q] = (m_ref + __builtin_amdgcn_logf(l_tot) - kLog2_127) * kLn2;
  };
  // (each path runs to the end of the kernel, so that no register state has to be merged)
  if (__builtin_amdgcn_readfirstlane((int)use_sbias)) run(std::true_type{});
  else run(std::false_type{});
}

}  // namespace sage
