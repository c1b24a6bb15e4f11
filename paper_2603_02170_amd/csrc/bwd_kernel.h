// Fused INT8 attention backward (paper Algorithm 2) for gfx950.
//
// sage_bwd_kernel: a workgroup of 8 waves owns two adjacent KV blocks (one per group of 4
// waves) and walks the Q blocks i from the last one down.  The operands of the coming Q blocks
// are copied global -> LDS asynchronously (LDS-DMA loads) into double buffers.  Per (i, j) tile
// and group there are three phases:
//   phase A  each wave takes one 32x32 quadrant (qb, kb) of the tile:
//            S = Q^ K^^T on INT8 MFMA, dP = dO V^T on bf16 MFMA (the one unquantised matmul),
//            P = exp(S - L), dS = P o (dP - delta), kept in registers; the wave maxima of P and
//            |dS| go to LDS.
//   phase Q  with the tile-wide maxima: psi(P), psi(dS) to LDS as MFMA operand fragments, and
//            the psi(dS) fragments also to the scratch buffer (the dQ kernel transposes them).
//   phase B  each wave takes one 32-channel slice of the outputs and contracts over the whole
//            tile: dV^T += dO^^T P^, dK^T += Q^^T dS^ (accumulated in FP32 registers with the
//            per-tile scales).
// The phases are software-pipelined over ONE workgroup barrier per tile (see the kernel).
// A second kernel (sage_bwd_dq_kernel) owns two Q blocks per workgroup and forms
//   dQ_i = sum_j s_dS(i,j) s_K(j) sm_scale * (dS^_ij K^_j)
// from the stored INT8 tiles: a plain scaled INT8 GEMM with no atomics, so dQ is
// deterministic.  It is bound by the memory pipeline (the tiles are read once, from HBM), so
// its work goes into how the copies are issued and how dQ leaves, not into its arithmetic.
// (A first version added dQ with FP32 atomics from the first kernel; at N=8192 the 4.3e9
// atomic adds alone took 13 ms.)
//
// S is formed untransposed (queries x keys): an accumulator lane then holds one key and 16
// queries, which is the B-operand form of the two contractions over queries (dV, dK).  The
// contraction over keys (dQ) needs dS^ with one query per lane; scattering it bytewise through
// LDS cost more LDS time than all operand reads together, hence a transposing MFMA (one matrix
// instruction against a permutation matrix), which runs in the dQ kernel: that kernel waits for
// memory and has the issue slots to spare, this one does not.
#pragma once

#include <type_traits>

#include "common.h"

namespace sage {

struct BwdArgs {
  const int8_t* QF;    // F layout   (S recompute, A operand)
  const int8_t* QT;    // TF layout  (dK, A operand)
  const int8_t* KF;    // F layout   (S recompute, B operand)
  const int8_t* dOT;   // TF layout  (dV, A operand)
  const unsigned short* V;    // bf16, rows addressed through `cv` (dense [BH, N, D] or the caller's token-major tensors)
  const unsigned short* dO;   // bf16, likewise
  RowView cv;                 // rows of the K-like tensors V, dK, dV
  RowView cvq;                // rows of the Q-like tensor dO
  const float* sQ;
  const float* sK;
  const float* sdO;
  const float* nL2;    // [BH, N]  -LSE * log2(e)
  const float* delta;  // [BH, N]  -rowsum(dO o O)
  const float* bias;   // Q-smoothing logit bias [BH, N/64, N] (log2 domain) or nullptr
  const float* muQ;    // Q-smoothing block means [BH, N/64, D] or nullptr
  int8_t* dSq;         // psi(dS) tiles [heads, N/64, ds_pitch, 4096]: the four quadrant fragments as phase Q forms them
  int ds_pitch;        // tiles per Q-block row of that array (>= N/64)
  float* sdS;          // their scales [heads, N/64, ds_pitch]
  float* tmax;         // B_q = 128: (max P, max |dS|) of the tiles of the even Q blocks [heads, N/64, ds_pitch][2], see MODE
  int bh0;             // first head of this launch (the scratch above is indexed from it)
  unsigned short* dK;  // bf16 [BH, N, D]
  unsigned short* dV;
  int BH, N;           // N = rows of the K-like workspace tensors (N_kv rounded up to a multiple of 64)
  int nvalid;          // keys >= nvalid do not exist (nvalid = N unless N_kv is not a multiple of 64)
  int Nq;              // rows of the Q-like workspace tensors (N_q rounded up to a multiple of 64)
  int nq_valid;        // query rows >= nq_valid do not exist
  int shift_blocks;    // causal: Q block i sees KV blocks j <= i + shift_blocks ((N_kv - N_q) / 64), diagonal at equality
  int head_set;        // heads per XCD whose work items are interleaved (see work_item)
  float sm_scale;
  float scale_log2e;
};

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kRoundMagic = 12582912.0f;   // 1.5 * 2^23: x + magic has rne(x) in its low mantissa bits
constexpr int kMagicBits = 0x4B400000;       // its bit pattern

template <int D>
struct BwdStageA {            // operands of phase A for one Q block
  int8_t qf[64 * D];          // Q^  F fragments
  int8_t dof[128 * D];        // bf16 dO as A fragments (32-row block, 16-channel step), XOR-swizzled slots
  float nl2[64];              // -L * log2(e)
  float dl[64];               // -delta
  float bias[128];            // Q-smoothing logit bias of this Q block for the workgroup's 128 keys
  float sc[64];               // s_Q[i] in every entry
};
template <int D>
struct BwdStageB {            // operands of phase B for one Q block
  int8_t qt[64 * D];          // Q^  TF fragments
  int8_t dot[64 * D];         // dO^ TF fragments
  float muq[D];               // Q-smoothing block mean
  float sc[64];               // s_Q[i] in the even entries, s_dO[i] in the odd ones
};
struct BwdExchange {          // per group of 4 waves and tile parity
  int8_t pb[4096];            // psi(P)  B fragments (q step, key block)
  int8_t dsb[4096];           // psi(dS) B fragments
};

// phase A element-wise work of one quadrant (`dp` holds dP - delta, or dP with -delta passed in `dl`); MASK = some entries of the tile are masked: query row
// qrow0 + 8 aa + b of the tile sees key column kcol only up to column klim_row (the row itself on
// the causal diagonal, 63 elsewhere) and only if the key exists (kcol < kvalid)
template <bool MASK, bool QSMOOTH>
__device__ __forceinline__ void bwd_quadrant(const v16i& sacc, const v16f& dp, const float* __restrict__ nl2,
                                             const float* __restrict__ dl, const float c, const float bias_l,
                                             const int qrow0, const int kcol, const bool diag, const int kvalid,
                                             float (&p)[16], float (&ds)[16], float& pm, float& dm, float& cs) {
  float pm2[2] = {0.f, 0.f}, dm2[2] = {0.f, 0.f};
  cs = 0.f;
#pragma unroll
  for (int aa = 0; aa < 4; aa++) {
    const v4f l4 = *(const v4f*)(nl2 + 8 * aa);
    v4f d4 = {0.f, 0.f, 0.f, 0.f};
    if constexpr (QSMOOTH) d4 = *(const v4f*)(dl + 8 * aa);     // -delta
#pragma unroll
    for (int b = 0; b < 4; b++) {
      const int r = 4 * aa + b;
      const float off = QSMOOTH ? bias_l + l4[b] : l4[b];
      float pv = __builtin_amdgcn_exp2f(__builtin_fmaf((float)sacc[r], c, off));
      if constexpr (MASK) pv = ((diag && (qrow0 + 8 * aa + b) < kcol) || kcol >= kvalid) ? 0.f : pv;
      // (without Q-smoothing the dP accumulators started from -delta)
      const float dsv = QSMOOTH ? pv * (dp[r] + d4[b]) : pv * dp[r];
      p[r] = pv;
      ds[r] = dsv;
      pm2[aa & 1] = fmaxf(pm2[aa & 1], pv);
      dm2[aa & 1] = fmaxf(dm2[aa & 1], fabsf(dsv));
      if constexpr (QSMOOTH) cs += dsv;
    }
  }
  pm = fmaxf(pm2[0], pm2[1]);
  dm = fmaxf(dm2[0], dm2[1]);
}

// Schedule.  The tiles of a group (Q blocks i = nblk-1 .. i_first against its KV block) go
// through three phases,
//   A  S = Q^K^^T (INT8), dP = dO V^T (bf16), P, dS in registers, wave maxima to LDS,
//   Q  psi(P), psi(dS) with the tile maxima -> LDS operand fragments,
//   B  dV^T += dO^^T P^, dK^T += Q^^T dS^ (INT8) with FP32 accumulation,
// software-pipelined over the workgroup's ONE barrier per tile: interval t runs Q of tile t-1,
// A of tile t and B of tile t-2, so every phase finds its cross-wave inputs complete and the
// matrix work of one tile runs under the vector work of its neighbours.
//
// MODE.  psi(P) and psi(dS) share one scale per numerics block of B_q queries x B_kv keys (Algorithm 2 lines
// 6 and 9).  With B_q = 64 (kBwdFused) the block lies inside one interval of this kernel and the maxima come
// from the interval's own phase A.  With B_q = 128 a block spans two consecutive Q blocks (2m + 1, which the
// walk meets first, and 2m), one interval apart, with no registers or LDS left to hold a tile back.  The tile
// of Q block 2m finds its partner's maxima in the previous interval's; the tile of 2m + 1 needs maxima the
// walk has not reached.  So the kernel runs twice: kBwdMaxOnly visits the EVEN Q blocks only, does phase A
// alone and stores each tile's two maxima to args.tmax; kBwdPairedRows is the full kernel, whose phase Q
// combines its own maxima with the stored ones of the tile below (odd Q blocks; staged into LDS one interval
// ahead) or with the previous interval's (even Q blocks).  P and dS are recomputed bit for bit, so the maxima
// are exactly those of the values quantised.
constexpr int kBwdFused = 0, kBwdMaxOnly = 1, kBwdPairedRows = 2;

// KV128: numerics blocks of 128 keys.  In that direction the block is the two tiles the workgroup's
// two groups hold in the same interval, so phase Q takes the maxima over both groups' phase A (a group whose
// tile does not exist in an interval, above the diagonal or past the last KV block, contributes zeros); 64 x 128
// blocks therefore need one sweep only.
template <int D, bool CAUSAL, bool QSMOOTH, int MODE = kBwdFused, bool KV128 = false>
__global__ void __launch_bounds__(512, 1) sage_bwd_kernel(BwdArgs args) {
  constexpr int ISTEP = MODE == kBwdMaxOnly ? 2 : 1;     // Q blocks between two tiles of the walk
  constexpr int KS = D / 32;     // INT8 k-steps over d; channel blocks
  constexpr int KB = D / 16;     // bf16 k-steps over d
  constexpr int NPB = KS / 2;    // 32-row blocks per wave in phase B (2 for D=128, 1 for D=64)
  constexpr int TILE = 64 * D;   // bytes of one INT8 tile
  constexpr int NF = TILE / 1024;  // 1 KiB fragments per INT8 tile

  // One LDS object: with several, the compiler tags every LDS access with the variable it touches and
  // then makes reads of buffers that no asynchronous copy ever writes wait for all copies in flight.
  struct Lds {
    BwdStageA<D> stA[2];
    BwdStageB<D> stB[2];
    BwdExchange xch[2][2];                          // [group][tile parity]
    int8_t vst[2][2 * D * 64];                      // [group]: bf16 V_j as B fragments (key block, 16-channel step)
    unsigned red[2][2][4][2];                       // [group][tile parity][wave][max P, max |dS|] as bit patterns
    float csum[QSMOOTH ? 2 * 3 * 2 * 64 : 1];       // [group][tile % 3][q half][key]: column sums of dS
    float tmx[MODE == kBwdPairedRows ? 2 * 2 * 64 : 1];   // [tile parity][group][even lanes: max P, odd lanes: max |dS|]
  };
  __shared__ __attribute__((aligned(16))) Lds L;
  auto& stA = L.stA;
  auto& stB = L.stB;
  auto& xch = L.xch;
  auto& vst = L.vst;
  auto& red = L.red;
  auto& csum = L.csum;
  auto& tmx = L.tmx;

  const int gidx = blockIdx.x;
  const int N = args.N;
  const int nblk = N / kBlock;        // KV blocks
  const int nqblk = args.Nq / kBlock; // Q blocks
  const int sb = CAUSAL ? args.shift_blocks : 0;
  const int npair = (nblk + 1) / 2;
  const WorkItem wi = work_item(gidx, npair, args.head_set);
  const int hl = wi.head;             // head within this launch
  if (hl >= args.BH) return;
  const int bh = args.bh0 + hl;
  const int jp = wi.item;             // small jp = most Q blocks under the causal mask: scheduled first

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave >> 2, w4 = wave & 3, gtid = tid & 255;
  const int ll = lane & 31, h = lane >> 5;
  const int qb = w4 >> 1, kb = w4 & 1;                     // phase A quadrant
  const int cb = (D == 128) ? w4 : (w4 & 1);               // phase B channel block
  const int blk0 = (D == 128) ? 0 : (w4 >> 1);             // phase B first 32-row block
  const int j = 2 * jp + grp;
  const bool gvalid = j < nblk;
  const int jc = gvalid ? j : nblk - 1;                    // clamped: an idle group still loads in bounds
  const int kvalid = min(64, args.nvalid - 64 * jc);       // key columns of this group's KV block that exist

  const size_t head = (size_t)bh * N * D;                  // in the dense K-like workspace tensors
  const size_t qhead = (size_t)bh * args.Nq * D;           // in the Q-like ones
  const size_t chead = args.cv.row(bh, 0);                 // in V, dK, dV
  const size_t rs = args.cv.row_stride;
  const size_t cqhead = args.cvq.row(bh, 0);               // in dO
  const size_t rsq = args.cvq.row_stride;
  const float sKj = args.sK[(size_t)bh * nblk + jc];

  // ---- operands that stay in registers for the whole loop ----
  v4i kfr[KS];
  {
    const int8_t* p = args.KF + head + ((size_t)(2 * jc + kb) * KS) * 1024 + lane * 16;
#pragma unroll
    for (int s = 0; s < KS; s++) kfr[s] = *(const v4i*)(p + s * 1024);
  }
  // bf16 V_j (B operand of dP): staged once in LDS as 1 KiB fragments (key block kb, 16-channel
  // step s), lane (key, half) holding V[key][16 s + 8 half .. + 8]; 16 fragments (d = 128) dealt
  // to the group's 4 waves.  Keeping it in registers instead would cost 32 of them, which the
  // prefetch of the streamed operands needs more.
#pragma unroll
  for (int k = 0; k < (2 * KB + 3) / 4; k++) {
    const int f = w4 + 4 * k;
    if (f < 2 * KB) {
      const int fkb = f / KB, fs = f % KB;
      // (a key row that does not exist re-reads the last one that does: its P is masked to zero)
      const int vrow = min(64 * jc + 32 * fkb + ll, args.nvalid - 1);
      async_copy_16(args.V + chead + (size_t)vrow * rs + 16 * fs + 8 * h, vst[grp] + f * 1024);
    }
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

  const int i_first = CAUSAL ? max(2 * jp - sb, 0) : 0;
  // tile t of this workgroup is Q block itop - ISTEP * t, down to i_first (kBwdMaxOnly: the even blocks only)
  const int itop = MODE == kBwdMaxOnly ? ((nqblk - 1) & ~1) : nqblk - 1;
  const int T = itop >= i_first ? (itop - i_first) / ISTEP + 1 : 0;
  // Asynchronous staging (global -> LDS, no registers) of the phase-A operands of Q block i.
  // Written without branches where the fragment counts divide evenly among the 8 waves (d = 128):
  // which array a wave copies from is a compile-time fact per copy, and the small vectors are
  // copied by every wave (duplicates of identical data), so that the steady-state interval stays
  // one basic block.  Every address is a wave-uniform base plus a 32-bit lane offset.
  // (LAST: Q block i may be the partial last block; query rows that do not exist re-read the last one
  // that does: their P is zero because the pre-pass gave them -L = -inf)
  auto load_A = [&](int i, BwdStageA<D>& st, auto last_tag) {
    constexpr bool LAST = decltype(last_tag)::value;
    const size_t toff = qhead + (size_t)i * TILE;
    const unsigned lane16 = lane * 16;
#pragma unroll
    for (int k = 0; k < (3 * NF + 7) / 8; k++) {
      const int o = wave + 8 * k;            // wave-uniform
      const bool all_q = 8 * k + 7 < NF, none_q = 8 * k >= NF;       // compile-time when NF % 8 == 0
      const bool in_range = 8 * k + 7 < 3 * NF || o < 3 * NF;
      if (all_q || (!none_q && o < NF)) {
        async_copy_16(args.QF + toff + o * 1024 + lane16, st.qf + o * 1024);
      } else if (in_range) {
        // bf16 dO fragment f = (32-row block, 16-channel step s); LDS slot l holds the piece of
        // (row, channel half) = (l ^ (s & 7)) so that the A-operand reads stay conflict-free
        const int f = o - NF;
        const int rb = f / KB, sst = f % KB;
        const unsigned orig = lane ^ (sst & 7);
        if constexpr (LAST) {
          const int row = min(64 * i + 32 * rb + (int)(orig & 31), args.nq_valid - 1);
          async_copy_16(args.dO + cqhead + (size_t)row * rsq + 16 * sst + 8 * (orig >> 5), st.dof + f * 1024);
        } else {
          const size_t loff = (orig & 31) * (2 * rsq) + (orig >> 5) * 16;          // bytes: row, channel half
          const char* base = (const char*)(args.dO + cqhead + (size_t)(64 * i + 32 * rb) * rsq + 16 * sst);
          async_copy_16(base + loff, st.dof + f * 1024);
        }
      }
    }
    // -L*log2e (even waves) or delta (odd waves), and s_Q[i] broadcast to 64 entries
    const float* vsrc = ((wave & 1) ? args.delta : args.nL2) + (size_t)bh * args.Nq + 64 * i;
    async_copy_4((const char*)vsrc + lane * 4, (wave & 1) ? st.dl : st.nl2);
    async_copy_4(args.sQ + (size_t)bh * nqblk + i, st.sc);
    if constexpr (QSMOOTH) {
      const char* brow = (const char*)(args.bias + ((size_t)bh * nqblk + i) * N + 128 * jp);
      if (wave == 5) async_copy_4(brow + lane * 4, st.bias);
      if (wave == 6 && 2 * jp + 1 < nblk) async_copy_4(brow + 256 + lane * 4, st.bias + 64);
    }
  };
  // ... and of its phase-B operands.
  auto load_B = [&](int i, BwdStageB<D>& st) {
    const size_t toff = qhead + (size_t)i * TILE;
    const unsigned lane16 = lane * 16;
#pragma unroll
    for (int k = 0; k < (2 * NF + 7) / 8; k++) {
      const int o = wave + 8 * k;
      const bool all_q = 8 * k + 7 < NF, none_q = 8 * k >= NF;
      const bool in_range = 8 * k + 7 < 2 * NF || o < 2 * NF;
      if (all_q || (!none_q && o < NF)) async_copy_16(args.QT + toff + o * 1024 + lane16, st.qt + o * 1024);
      else if (in_range) async_copy_16(args.dOT + toff + (o - NF) * 1024 + lane16, st.dot + (o - NF) * 1024);
    }
    // s_Q[i] (even lanes) and s_dO[i] (odd lanes)
    async_copy_4(((lane & 1) ? args.sdO : args.sQ) + (size_t)bh * nqblk + i, st.sc);
    if constexpr (QSMOOTH) {
      const char* mq = (const char*)(args.muQ + ((size_t)bh * nqblk + i) * D);
      if (wave == 3) async_copy_4(mq + lane * 4, st.muq);
      if (D == 128 && wave == 4) async_copy_4(mq + 256 + lane * 4, st.muq + 64);
    }
  };

  load_A(itop, stA[0], std::true_type{});
  barrier_all_memory();

  float p[16], ds[16];           // P and dS of the tile between its phases A and Q
  float sP_q = 0.f, sS_q = 0.f;  // tile scales found by the last phase Q
  unsigned prev_p = 0u, prev_d = 0u;   // kBwdPairedRows: the maxima (bit patterns) of the tile the last phase Q handled
  // One interval.  STEADY = all three phases are active and tile t is not on the diagonal: the
  // body is then free of branches, one basic block in which the compiler interleaves the three
  // independent phases (the LDS and MFMA latencies of one hide under the vector work of the others).
  auto interval = [&](const int t, auto steady_tag) __attribute__((always_inline)) {
    constexpr bool STEADY = decltype(steady_tag)::value;
    const float sP_b = sP_q, sS_b = sS_q;      // scales of tile t - 2 (its phase Q ran in the last interval)
    const int ib = itop - ISTEP * (t - 2);     // Q blocks of the three tiles in flight
    const int iq = itop - ISTEP * (t - 1);
    const int ia = itop - ISTEP * t;
    const bool act_b = MODE != kBwdMaxOnly && (STEADY || (t >= 2 && gvalid && (!CAUSAL || ib + sb >= j)));
    const bool act_q = STEADY || (t >= 1 && t - 1 < T && gvalid && (!CAUSAL || iq + sb >= j));
    const bool act_a = STEADY || (t < T && gvalid && (!CAUSAL || ia + sb >= j));

    // operands of the coming intervals; the copies are issued in two batches so that the eight
    // waves do not queue up behind each other at the memory pipeline
    if (STEADY || t + 1 < T) load_A(ia - ISTEP, stA[(t + 1) & 1], std::false_type{});

    __builtin_amdgcn_sched_barrier(0);
    // ---------------- phase Q of tile t - 1 ----------------
    if (act_q) {
      BwdExchange& X = xch[grp][(t - 1) & 1];
      // (the maxima are non-negative floats: they order like their bit patterns, and integer maxima
      // need no NaN canonicalisation of the loaded values)
      const unsigned(&R)[4][2] = red[grp][(t - 1) & 1];
      unsigned pu = max(max(R[0][0], R[1][0]), max(R[2][0], R[3][0]));
      unsigned du = max(max(R[0][1], R[1][1]), max(R[2][1], R[3][1]));
      if constexpr (KV128) {
        const unsigned(&R2)[4][2] = red[grp ^ 1][(t - 1) & 1];
        pu = max(pu, max(max(R2[0][0], R2[1][0]), max(R2[2][0], R2[3][0])));
        du = max(du, max(max(R2[0][1], R2[1][1]), max(R2[2][1], R2[3][1])));
      }
      if constexpr (MODE == kBwdPairedRows) {
        // the other Q block of the numerics block: below (iq odd: the stored maxima of tile (iq - 1, j), and of
        // its neighbour in the 128-key block, where those tiles exist) or above (iq even: the last interval's)
        const unsigned own_p = pu, own_d = du;
        if (iq & 1) {
          const unsigned* tm = (const unsigned*)(tmx + (((t - 1) & 1) * 2 + grp) * 64);
          if constexpr (KV128) {
            const int j0 = j & ~1;
            if (!CAUSAL || j0 <= iq - 1 + sb) {
              pu = max(pu, tm[0]);
              du = max(du, tm[1]);
            }
            if (j0 + 1 < nblk && (!CAUSAL || j0 + 1 <= iq - 1 + sb)) {
              pu = max(pu, tm[2]);
              du = max(du, tm[3]);
            }
          } else if (!CAUSAL || j <= iq - 1 + sb) {
            pu = max(pu, tm[0]);
            du = max(du, tm[1]);
          }
        } else if (iq + 1 < nqblk) {
          pu = max(pu, prev_p);
          du = max(du, prev_d);
        }
        prev_p = own_p;
        prev_d = own_d;
      }
      const float pm = __uint_as_float(pu), dm = __uint_as_float(du);
      if constexpr (MODE == kBwdMaxOnly) {
        // this tile's two maxima, for the pass over the numerics blocks; nothing is quantised in this mode
        if (w4 == 0 && lane == 0) {
          const size_t tile = ((size_t)hl * nqblk + iq) * args.ds_pitch + j;
          *(v2f*)(args.tmax + 2 * tile) = v2f{pm, dm};
        }
      } else {
      // the per-tile scales of P and dS are internal (never stored bit-exactly): 127/a via rcp
      const float rP = pm > 0.f ? 127.0f * __builtin_amdgcn_rcpf(pm) : 0.f;
      const float rS = dm > 0.f ? 127.0f * __builtin_amdgcn_rcpf(dm) : 0.f;
      sP_q = pm * (1.0f / 127.0f);
      sS_q = dm * (1.0f / 127.0f);
      v4i pf, df;
#pragma unroll
      for (int aa = 0; aa < 4; aa++) {
        unsigned ub[4];
#pragma unroll
        for (int b = 0; b < 4; b++) ub[b] = __float_as_uint(__builtin_fmaf(ds[4 * aa + b], rS, kRoundMagic));
        const unsigned lo = __builtin_amdgcn_perm(ub[1], ub[0], 0x0c0c0400u);
        const unsigned hi = __builtin_amdgcn_perm(ub[3], ub[2], 0x04000c0cu);
        df[aa] = (int)(lo | hi);
      }
#pragma unroll
      for (int aa = 0; aa < 4; aa++) {
        unsigned up = 0;
#pragma unroll
        for (int b = 0; b < 4; b++) up = __builtin_amdgcn_cvt_pk_u8_f32(p[4 * aa + b] * rP, b, up);
        pf[aa] = (int)up;
      }
      *(v4i*)(X.pb + ((qb * 2 + kb) * 64 + lane) * 16) = pf;
      *(v4i*)(X.dsb + ((qb * 2 + kb) * 64 + lane) * 16) = df;
      {
        // the same fragment goes to the scratch buffer for the dQ kernel: fragment (qb, kb), lane (key, h),
        // byte 4 a + b = psi(dS)[32 qb + 8 a + 4 h + b][32 kb + key]
        // (tiles and scales share one index: a second index product costs the Q-smoothing instantiation a spill)
        const size_t tile = ((size_t)hl * nqblk + iq) * args.ds_pitch + j;
        *(v4i*)(args.dSq + tile * 4096 + ((qb * 2 + kb) * 64 + lane) * 16) = df;
        args.sdS[tile] = sS_q;   // the same value from every lane: no branch
      }
      }
    }
    if constexpr (MODE != kBwdMaxOnly) {
      if (STEADY || (t >= 1 && t - 1 < T)) load_B(iq, stB[(t - 1) & 1]);
    }
    if constexpr (MODE == kBwdPairedRows) {
      // tile t has its phase Q in the next interval: if its Q block is odd, the stored maxima of the tile below
      // it (and, with 128-key blocks, of that tile's neighbour: entries j0 and j0 + 1 are adjacent; the rows of
      // the table are three entries longer than a row of tiles).  Each wave copies its group's two or four
      // floats: lanes 0, 1 (, 2, 3) = max P, max |dS| (, of the neighbour); the other lanes repeat them.
      if ((STEADY || t < T) && (ia & 1)) {
        const size_t tile = ((size_t)hl * nqblk + ia - 1) * args.ds_pitch + (KV128 ? (jc & ~1) : jc);
        async_copy_4(args.tmax + 2 * tile + (lane & (KV128 ? 3 : 1)), tmx + ((t & 1) * 2 + grp) * 64);
      }
    }

    __builtin_amdgcn_sched_barrier(0);
    // The two waves of a SIMD are wave w (first group) and w + 4 (second group); the arbiter favours the
    // older one, which then idles at the interval's barrier.  Raising the younger wave's priority for
    // its MFMA-dense phase evens the two out (measured: 2-3 % of the kernel).
    if (STEADY && grp == 1) __builtin_amdgcn_s_setprio(1);
    // ---------------- phase A of tile t: quadrant (qb, kb) ----------------
    if (act_a) {
      const BwdStageA<D>& st = stA[t & 1];
      // The two MFMA chains (S over INT8 steps, dP over bf16 steps) are interleaved, and the LDS
      // reads of their operands run two bf16 steps ahead of the MFMAs that consume them.
      v4i qa[KS];
      v8bf da[KB], vb[KB];
      const int8_t* qfp = st.qf + (qb * KS * 64 + lane) * 16;
      const int8_t* vbp = vst[grp] + (kb * KB * 64 + lane) * 16;
      auto ld = [&](int s) {
        if (s % 2 == 0) qa[s / 2] = *(const v4i*)(qfp + (s / 2) * 1024);
        da[s] = *(const v8bf*)(st.dof + ((qb * KB + s) * 64 + (lane ^ (s & 7))) * 16);
        vb[s] = *(const v8bf*)(vbp + s * 1024);
      };
      ld(0);
      ld(1);
      v16i sacc;
      v16f dp;
      // dS = P o (dP - delta): the dP chain starts from -delta of the rows this lane's registers hold
      // (register 4a + b = query 8a + 4h + b of the quadrant), which saves the subtraction per entry.
      // (Not with Q-smoothing: that instantiation has no register to spare, and anything that lengthens
      // a live range there ends in a scratch access inside the loop, whose wait drains the staging copies.)
      if constexpr (QSMOOTH) {
#pragma unroll
        for (int r = 0; r < 16; r++) dp[r] = 0.f;
      } else {
        const float* dl = st.dl + 32 * qb + 4 * h;
#pragma unroll
        for (int aa = 0; aa < 4; aa++) {
          const v4f d4 = *(const v4f*)(dl + 8 * aa);
#pragma unroll
          for (int b = 0; b < 4; b++) dp[4 * aa + b] = d4[b];
        }
      }
#pragma unroll
      for (int r = 0; r < 16; r++) sacc[r] = 0;
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int s = 0; s < KB; s++) {
        if (s + 2 < KB) ld(s + 2);
        if (s % 2 == 0) sacc = __builtin_amdgcn_mfma_i32_32x32x32_i8(qa[s / 2], kfr[s / 2], sacc, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(da[s], vb[s], dp, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
      const float c = st.sc[0] * sKj * args.scale_log2e;
      float bias_l = 0.f;
      if constexpr (QSMOOTH) bias_l = st.bias[64 * grp + 32 * kb + ll];
      const float* nl2 = st.nl2 + 32 * qb + 4 * h;
      float pm, dm, cs;
      if (!STEADY && ((CAUSAL && ia + sb == j) || kvalid < 64))
        bwd_quadrant<true, QSMOOTH>(sacc, dp, nl2, st.dl + 32 * qb + 4 * h, c, bias_l, 32 * qb + 4 * h, 32 * kb + ll, CAUSAL && ia + sb == j, kvalid,
                                    p, ds, pm, dm, cs);
      else
        bwd_quadrant<false, QSMOOTH>(sacc, dp, nl2, st.dl + 32 * qb + 4 * h, c, bias_l, 0, 0, false, 64, p, ds, pm, dm, cs);
      pm = wave_max_nonneg_f32(pm);
      dm = wave_max_nonneg_f32(dm);
      // every lane stores the same pair (one LDS write, no branch)
      red[grp][t & 1][w4][0] = __float_as_uint(pm);
      red[grp][t & 1][w4][1] = __float_as_uint(dm);
      if constexpr (QSMOOTH) {
        cs = half_swap_sum_f32(cs);
        if (h == 0) csum[((grp * 3 + t % 3) * 2 + qb) * 64 + 32 * kb + ll] = cs;
      }
    } else if constexpr (KV128) {
      // no tile for this group in this interval: nothing for the other group's block maxima
      red[grp][t & 1][w4][0] = 0u;
      red[grp][t & 1][w4][1] = 0u;
    }

    __builtin_amdgcn_sched_barrier(0);
    if (STEADY) __builtin_amdgcn_s_setprio(0);
    // ---------------- phase B of tile t - 2: channel block cb ----------------
    if (act_b) {
      const BwdStageB<D>& st = stB[t & 1];
      const BwdExchange& X = xch[grp][t & 1];
      const float w_dv = sP_b * st.sc[1];
      const float w_dk = sS_b * st.sc[0] * args.sm_scale;
#pragma unroll
      for (int tt = 0; tt < NPB; tt++) {
        const int kbo = blk0 + tt;
        v16i av, ak;
#pragma unroll
        for (int r = 0; r < 16; r++) {
          av[r] = 0;
          ak[r] = 0;
        }
#pragma unroll
        for (int qs = 0; qs < 2; qs++) {
          const v4i a1 = *(const v4i*)(st.dot + ((qs * KS + cb) * 64 + lane) * 16);
          const v4i b1 = *(const v4i*)(X.pb + ((qs * 2 + kbo) * 64 + lane) * 16);
          av = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, b1, av, 0, 0, 0);
          const v4i a2 = *(const v4i*)(st.qt + ((qs * KS + cb) * 64 + lane) * 16);
          const v4i b2 = *(const v4i*)(X.dsb + ((qs * 2 + kbo) * 64 + lane) * 16);
          ak = __builtin_amdgcn_mfma_i32_32x32x32_i8(a2, b2, ak, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 16; r++) {
          dvacc[tt][r] = __builtin_fmaf((float)av[r], w_dv, dvacc[tt][r]);
          dkacc[tt][r] = __builtin_fmaf((float)ak[r], w_dk, dkacc[tt][r]);
        }
        if constexpr (QSMOOTH) {
          // dK_bias = (dS^T 1) mu_Q^T with the unquantised column sums of this tile
          const float* cs2 = csum + ((grp * 3 + (t - 2) % 3) * 2) * 64;
          const float csv = cs2[32 * kbo + ll] + cs2[64 + 32 * kbo + ll];
#pragma unroll
          for (int aa = 0; aa < 4; aa++) {
            const v4f m4 = *(const v4f*)(st.muq + 32 * cb + 8 * aa + 4 * h);
#pragma unroll
            for (int b = 0; b < 4; b++) dkbias[tt][4 * aa + b] = __builtin_fmaf(csv, m4[b], dkbias[tt][4 * aa + b]);
          }
        }
      }
    }
    barrier_all_memory();   // the interval's LDS traffic, copies and stores are complete
  };
  // steady intervals: t >= 2 (all three tiles exist), tile t above the diagonal and not the last row
  // (a KV block with keys that do not exist masks them in every tile: no branch-free intervals for its group)
  // (under the mask: while Q block itop - ISTEP * t lies above the group's diagonal block j - sb)
  const int t_steady_end = (!gvalid || kvalid < 64) ? 0 : (CAUSAL ? min((itop + sb - j + ISTEP - 1) / ISTEP, T - 1) : T - 1);
  int t = 0;
  for (; t < 2 && t < T + 2; t++) interval(t, std::false_type{});
  for (; t < t_steady_end; t++) interval(t, std::true_type{});
  for (; t < T + 2; t++) interval(t, std::false_type{});

  if (!gvalid) return;

  // ---- write dV, dK (bf16) ----
#pragma unroll
  for (int t = 0; t < NPB; t++) {
    const int key = 64 * j + 32 * (blk0 + t) + ll;
    unsigned short* pv = args.dV + chead + (size_t)key * rs + 32 * cb + 4 * h;
    unsigned short* pk = args.dK + chead + (size_t)key * rs + 32 * cb + 4 * h;
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
      if (key < args.nvalid) {
        *(v4us*)(pv + 8 * aa) = ov;
        *(v4us*)(pk + 8 * aa) = ok;
      }
    }
  }
}

// ---------------------------------------------------------------------------------
// dQ_i = sum_j (dS^_ij K^_j) * s_dS(i,j) * s_K(j) * sm_scale        (Algorithm 2, the dQ line)
// A = the stored psi(dS) fragments, transposed here, B = K^ in TF layout.
struct DqArgs {
  const int8_t* dSq;
  int ds_pitch;         // tiles per Q-block row of dSq
  const float* sdS;
  const int8_t* KT;
  const float* sK;
  unsigned short* dQ;   // bf16, rows addressed through `cv` (dense [BH, N_q, D] or the caller's token-major tensor)
  RowView cv;
  int BH, N, bh0;       // N = rows of the K-like workspace tensors (a multiple of 64)
  int Nq;               // rows of the Q-like ones
  int nvalid;           // query rows >= nvalid do not exist
  int shift_blocks;     // causal: Q block i sees KV blocks j <= i + shift_blocks
  int head_set;         // heads per XCD whose work items are interleaved (see work_item)
  float sm_scale;
};

// A workgroup of 4 waves owns TWO Q blocks (128 queries) and walks the KV blocks j; wave (Q block, row half)
// owns 32 query rows and ALL d channels.  A stored psi(dS) fragment holds one KEY per lane and 16 queries in
// its bytes (the form the backward kernel's own products need); the product over keys needs one QUERY per
// lane, so each fragment is transposed on arrival by one MFMA against a permutation matrix: read as an A
// operand it is the matrix (key, permuted query), and the accumulator comes back with lane = query and
// registers = keys in the order of the TF layout of K^; the low bytes of the INT32 results are the codes.
// Each wave streams its own 2 KiB per tile from HBM straight into registers (one 16-byte load per lane
// and fragment, nothing shared, no LDS): kStages tiles ahead.  The K^ tile (TF layout, from L2) is
// shared by the four waves and travels global -> LDS asynchronously through a ring that runs the same
// number of stages ahead, together with the three scales of the stage; one barrier per stage.  Both
// streams are issued by every wave in the same order and complete in order, so one count of outstanding
// memory operations (`s_waitcnt vmcnt`) covers the K^ copies and the compiler's own waits cover the
// registers.  Three workgroups share a CU: about 96 KiB of psi(dS) in flight per CU.
// (Every lane takes part in the scale copy: a memory operation under a lane mask sits behind a branch,
// and with a path that skips it the compiler stops counting the loads in flight and waits for all of
// them before each use.)  Measured: the kernel runs at the speed of its psi(dS) stream alone (no
// arithmetic, no K^ copies: 0.51 ms of 0.54 at the headline shape, about 4.4 TB/s, where a plain read
// stream over the same bytes reaches 5.6 TB/s on this GPU); ring depths 3 to 7, two or three workgroups
// per CU and non-temporal loads change nothing.
template <int D, bool CAUSAL>
__global__ void __launch_bounds__(256, 3) sage_bwd_dq_kernel(DqArgs args) {
  constexpr int KS = D / 32;               // channel blocks
  constexpr int TILE = 64 * D;             // bytes of one K^ tile
  constexpr int DSB = 4096;                // bytes of one psi(dS) tile
  constexpr int kStages = 4;               // stages in flight (3 to 7 measured the same)
  constexpr int NS = kStages + 1;          // ring slots
  constexpr int KSLOT = TILE + 256;        // K^ tile | s_dS of Q block 0, of Q block 1, s_K (lanes 3.. repeat s_K)
  constexpr int KC = TILE / 4096;          // K^ copies per wave and stage (the tile's 1 KiB fragments dealt to 4 waves)
  constexpr int OPS = 2 + KC + 1;          // memory operations per wave and stage: 2 psi(dS) loads, K^ copies, scales

  __shared__ __attribute__((aligned(16))) int8_t lds[NS * KSLOT];

  const int g = blockIdx.x;
  const int N = args.N;
  const int nblk = N / kBlock;                         // KV blocks
  const int nqblk = args.Nq / kBlock;                  // Q blocks
  const int sb = CAUSAL ? args.shift_blocks : 0;
  const int npair = (nqblk + 1) / 2;
  const WorkItem wi = work_item(g, npair, args.head_set);
  const int hl = wi.head;
  if (hl >= args.BH) return;
  const int bh = args.bh0 + hl;
  const int i0 = 2 * (npair - 1 - wi.item);            // longest rows first under the causal mask
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ll = lane & 31, h = lane >> 5;
  const int iq = wave >> 1, qb = wave & 1;             // Q block of the pair, 32-row half of it
  const bool valid = i0 + iq < nqblk;
  const int i = valid ? i0 + iq : i0;                  // clamped: the loads stay in bounds
  const int i1 = i0 + 1 < nqblk ? i0 + 1 : i0;
  const size_t head = (size_t)bh * N * D;
  const int n_j = CAUSAL ? min(i0 + 2 + sb, nblk) : nblk;            // stages of the workgroup
  const int j_last = CAUSAL ? i + sb : nblk - 1;       // last tile of this wave's Q block that was written

  // this wave's fragments of tile (i, j): (row half qb, key step 0 / 1) at j * DSB, + 1024
  const int8_t* dsw = args.dSq + ((size_t)hl * nqblk + i) * args.ds_pitch * DSB + qb * 2048 + lane * 16;
  const int8_t* kth = args.KT + head + wave * 1024 + lane * 16;
  // per stage lanes 0, 1, 2 fetch s_dS of Q block 0, s_dS of Q block 1, s_K
  const size_t sc_off = lane == 0 ? ((size_t)hl * nqblk + i0) * args.ds_pitch : ((size_t)hl * nqblk + i1) * args.ds_pitch;
  const float* sc_src = lane < 2 ? args.sdS + sc_off : args.sK + (size_t)bh * nblk;

  // Stage indices past the end are clamped: the loads then re-read the last stage (into registers or a
  // slot that nobody reads any more), and every wave issues the same operations in every iteration.
  auto load_ds = [&](int j, v4i (&a)[2]) __attribute__((always_inline)) {
    const int jc = j < j_last ? j : j_last;
    const int8_t* p = dsw + (size_t)jc * DSB;
    a[0] = *(const v4i*)p;
    a[1] = *(const v4i*)(p + 1024);
  };
  auto load_k = [&](int j, int sl) __attribute__((always_inline)) {
    const int jc = j < n_j ? j : n_j - 1;
    const int8_t* src = kth + (size_t)jc * TILE;
    int8_t* dst = lds + sl * KSLOT + wave * 1024;
    async_copy_16(src, dst);
    if constexpr (KC == 2) async_copy_16(src + 4096, dst + 4096);
    async_copy_4(sc_src + jc, lds + sl * KSLOT + TILE);   // (the same values from every wave; lanes 2.. all carry s_K)
  };

  v16f acc[KS];
#pragma unroll
  for (int cb = 0; cb < KS; cb++)
#pragma unroll
    for (int r = 0; r < 16; r++) acc[cb][r] = 0.f;

  // B operand of the transposing MFMA: a stored fragment, read as an A operand, has contraction index
  // k = 16 h + 4 a + b for the query 8 a + 4 h + b; column n of the permutation matrix picks the k that
  // stands for query n.  Lane (n, hh) holds k = 16 hh + t in byte t.
  v4i tperm;
#pragma unroll
  for (int aa = 0; aa < 4; aa++) {
    unsigned u = 0;
#pragma unroll
    for (int b = 0; b < 4; b++) u |= (unsigned)((8 * aa + 4 * h + b) == ll) << (8 * b);
    tperm[aa] = (int)u;
  }
  auto transposed = [&](const v4i& f) __attribute__((always_inline)) {
    v16i z;
#pragma unroll
    for (int r = 0; r < 16; r++) z[r] = 0;
    const v16i tr = __builtin_amdgcn_mfma_i32_32x32x32_i8(f, tperm, z, 0, 0, 0);
    v4i o;
#pragma unroll
    for (int aa = 0; aa < 4; aa++) {
      const unsigned lo = __builtin_amdgcn_perm((unsigned)tr[4 * aa + 1], (unsigned)tr[4 * aa], 0x0c0c0400u);
      const unsigned hi = __builtin_amdgcn_perm((unsigned)tr[4 * aa + 3], (unsigned)tr[4 * aa + 2], 0x04000c0cu);
      o[aa] = (int)(lo | hi);
    }
    return o;
  };

  v4i a[kStages][2];
#pragma unroll
  for (int s = 0; s < kStages; s++) {
    load_ds(s, a[s]);
    load_k(s, s);
    compiler_fence();                      // the waits below count operations in issue order
  }
  static_assert((kStages - 1) * OPS < 64, "vmcnt has six bits");
  __builtin_amdgcn_s_waitcnt(vmcnt_only((kStages - 1) * OPS));   // stage 0 has landed
  barrier_lds_only();

  // Iteration j: contract stage j (registers a[j % kStages], ring slot j % NS), then start stage
  // j + kStages into the same registers and into the slot that stage j - 1 occupied (every wave is past
  // the barrier that ended iteration j - 1); before the barrier at the end, wait until this wave's
  // copies of stage j + 1 have landed (everything but the kStages - 1 youngest stages).
  // The loop is unrolled over the kStages register sets and runs whole rounds (the stages past n_j only
  // keep the counts even: clamped loads, no arithmetic), so that every path through the body issues the
  // same memory operations and the compiler's count of the loads in flight stays exact.
  int sk = 0;                              // slot of stage j
  for (int j0 = 0; j0 < n_j; j0 += kStages) {
#pragma unroll
    for (int s = 0; s < kStages; s++) {
      const int j = j0 + s;
      if (j < n_j && valid && (!CAUSAL || j <= i + sb)) {
        const int8_t* kp = lds + sk * KSLOT;
        const float* sc = (const float*)(kp + TILE);
        const float w = sc[iq] * sc[2] * args.sm_scale;
        const v4i a0 = transposed(a[s][0]), a1 = transposed(a[s][1]);
#pragma unroll
        for (int cb = 0; cb < KS; cb++) {
          const v4i b0 = *(const v4i*)(kp + cb * 1024 + lane * 16);
          const v4i b1 = *(const v4i*)(kp + (KS + cb) * 1024 + lane * 16);
          v16i q;
#pragma unroll
          for (int r = 0; r < 16; r++) q[r] = 0;
          q = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, b0, q, 0, 0, 0);
          q = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, b1, q, 0, 0, 0);
#pragma unroll
          for (int r = 0; r < 16; r++) acc[cb][r] = __builtin_fmaf((float)q[r], w, acc[cb][r]);
        }
      }
      load_ds(j + kStages, a[s]);
      load_k(j + kStages, sk == 0 ? NS - 1 : sk - 1);
      __builtin_amdgcn_s_waitcnt(vmcnt_only((kStages - 1) * OPS));
      barrier_lds_only();
      sk = sk == NS - 1 ? 0 : sk + 1;
    }
  }
  barrier_all_memory();    // the clamped copies past the last stage have landed before the ring is reused
  // ---- write dQ (bf16): the accumulators hold one channel per lane and 16 query rows in registers, so
  // the two 64 x D blocks go through LDS (the ring is drained) and leave as 16-byte row pieces ----
  constexpr int LDQ = D + 8;                                   // padded row, in bf16 elements
  static_assert(2 * 64 * LDQ * 2 <= NS * KSLOT, "the dQ staging must fit the ring");
  unsigned short* stg = (unsigned short*)lds;                  // [Q block][row][LDQ]
  if (valid) {
#pragma unroll
    for (int cb = 0; cb < KS; cb++)
#pragma unroll
      for (int aa = 0; aa < 4; aa++)
#pragma unroll
        for (int b = 0; b < 4; b++)
          stg[(iq * 64 + 32 * qb + 8 * aa + 4 * h + b) * LDQ + 32 * cb + ll] = float_to_bf16_bits(acc[cb][4 * aa + b]);
  }
  barrier_lds_only();
  constexpr int CPR = D / 8;                                   // 16-byte pieces per row
  for (int c = tid; c < 2 * 64 * CPR; c += 256) {
    const int qblk = c / (64 * CPR), row = (c / CPR) % 64, pc = c % CPR;
    if (i0 + qblk < nqblk && 64 * (i0 + qblk) + row < args.nvalid)
      *(v8us*)(args.dQ + args.cv.row(bh, 64 * (i0 + qblk) + row) + 8 * pc) = *(const v8us*)(stg + (qblk * 64 + row) * LDQ + 8 * pc);
  }
}

}  // namespace sage
