// C-ABI host side of the SageBwd library: argument validation, workspace layout,
// kernel launches.  See include/sagebwd.h for the contract of every entry point.
#include "sagebwd.h"

#include <hip/hip_runtime.h>
#include <math.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "common.h"
#include "prepass_kernels.h"
#include "fwd_kernel.h"
#include "bwd_kernel.h"
#include "probe_kernels.h"

// Workspace of sagebwd_fwd_static: one array per GPU, held until the process ends.  In host code the
// name `scratch` is only a handle for hipGetSymbolAddress; the device address it returns (per device)
// is what the kernels are given.
static __device__ __align__(256) unsigned char scratch[SAGEBWD_STATIC_SCRATCH_BYTES];

namespace {

using namespace sage;

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each GPU, looked up once

// Device address of this GPU's copy of `scratch` (the current device's), or nullptr on failure.
void* static_scratch_for_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

constexpr size_t kDefaultDsBudget = (size_t)8 << 30;   // bytes of INT8 dS scratch the backward holds at once unless told otherwise

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// Rows of every workspace tensor: the caller's N rounded up to the 64-row block.  When the two differ
// the kernels run on the rounded shape: the rows that do not exist are zero rows behind a key mask in
// the workspace, are never read from the caller's tensors (loaders clamp) and never stored.
inline int padded_rows(int N) { return (N + 63) / 64 * 64; }

// Numerics block sizes (rows that share one quantisation scale): 64 unless the caller says 128.
inline int block_q(const sagebwd_params& p) { return p.bq > 0 ? p.bq : 64; }
inline int block_kv(const sagebwd_params& p) { return p.bkv > 0 ? p.bkv : 64; }
inline bool big_blocks(const sagebwd_params& p) { return block_q(p) != 64 || block_kv(p) != 64; }

// Keys per head: N_kv, or N when the caller leaves it 0 (square attention).
inline int kv_len(const sagebwd_params& p) { return p.Nkv > 0 ? p.Nkv : p.N; }

// Where the rows of one of the caller's bf16 tensors start, in elements (times `scale`); `rows` = its
// sequence length (N for Q, O, dO, dQ; N_kv for K, V, dK, dV).
inline RowView caller_view(const sagebwd_params& p, size_t scale, int rows) {
  const size_t N = rows, H = p.H, d = p.d;
  RowView v;
  v.H = p.H;
  if (p.layout == SAGEBWD_LAYOUT_BNHD) {
    v.batch_stride = N * H * d * scale; v.head_stride = d * scale; v.row_stride = H * d * scale;
  } else {
    v.batch_stride = H * N * d * scale; v.head_stride = N * d * scale; v.row_stride = d * scale;
  }
  return v;
}


// Byte offsets of every buffer inside the caller's workspace.  What the forward needs comes first
// (`fwd_total` bytes), so that a forward-only caller can pass a much smaller buffer.
struct Workspace {
  size_t kpart, muK, muQ, sQ, sK, sV;
  size_t QF, KF, VT;        // forward operands (QF, KF also feed the backward's S recompute)
  size_t bias;              // Q-smoothing: logit bias table [BH, N/64, N]
  size_t Knorm;             // QK-norm with Q-smoothing: the normalised K as dense bf16 [BH, Nk, d] (the bias kernel reads it)
  size_t QT, KT;            // backward operands (TF layouts) that depend on Q and K only
  size_t fwd_total;         // the forward's need (with SAGEBWD_FLAG_SHARE_QUANTIZED it includes QT, KT)
  size_t sdO, delta, nl2, dOT;
  size_t dSq;               // psi(dS) tiles of one head group [heads_per_group, N/64, N/64, 4096]
  size_t sdS;               // their scales [heads_per_group, N/64, ds_pitch]
  int heads_per_group;      // the backward runs in groups of heads that share the dS scratch
  int ds_pitch;             // tiles per Q-block row of the dS scratch
  size_t tmax;              // B_q = 128: (max P, max |dS|) per tile of the even Q blocks, from the backward's first sweep
  size_t total;
  int nchunk, chunk_rows;   // K-mean reduction: chunks per head, rows per chunk
};

Workspace make_layout(const sagebwd_params& p) {
  Workspace w;
  // Nq, Nk: rows of the Q-like and K-like workspace tensors
  const size_t BH = (size_t)p.B * p.H, Nq = padded_rows(p.N), Nk = padded_rows(kv_len(p)), d = p.d;
  const size_t nqblk = Nq / 64, nkblk = Nk / 64;
  const bool qs = (p.smooth & SAGEBWD_SMOOTH_Q) != 0;
  const bool share = (p.flags & SAGEBWD_FLAG_SHARE_QUANTIZED) != 0;
  w.chunk_rows = mean_chunk_rows((int)BH, kv_len(p));
  w.nchunk = (kv_len(p) + w.chunk_rows - 1) / w.chunk_rows;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
  w.kpart = take(BH * w.nchunk * d * sizeof(double));
  w.muK = take(BH * d * 4);
  w.muQ = take(qs ? BH * nqblk * d * 4 : 0);
  w.sQ = take(BH * nqblk * 4);
  w.sK = take(BH * nkblk * 4);
  w.sV = take(BH * nkblk * 4);
  w.QF = take(BH * Nq * d);
  w.KF = take(BH * Nk * d);
  w.VT = take(BH * Nk * d);
  w.bias = take(qs ? BH * nqblk * Nk * 4 : 0);
  w.Knorm = take(qs && (p.flags & SAGEBWD_FLAG_QK_NORM) ? BH * Nk * d * 2 : 0);
  if (!share) w.fwd_total = off;
  w.QT = take(BH * Nq * d);
  w.KT = take(BH * Nk * d);
  if (share) w.fwd_total = off;
  w.sdO = take(BH * nqblk * 4);
  w.delta = take(BH * Nq * 4);
  w.nl2 = take(BH * Nq * 4);
  w.dOT = take(BH * Nq * d);
  // dS scratch: one 4 KiB tile per (Q block, KV block) and head, capped at the budget by processing the
  // heads in groups.
  // Rows of the dS scratch are three tiles longer than they need to be: with a power-of-two row length
  // the workgroups of the dQ kernel, which walk their rows at the same pace, read addresses that differ
  // in the high bits only (measured: 4 % of that kernel).
  w.ds_pitch = (int)nkblk + 3;
  const size_t ds_head = nqblk * (size_t)w.ds_pitch * 4096;   // bytes of dS scratch per head
  const size_t budget = p.scratch_budget != 0 ? (size_t)p.scratch_budget : kDefaultDsBudget;
  size_t hpg = budget / ds_head;
  if (hpg < 1) hpg = 1;
  if (hpg > BH) hpg = BH;
  w.heads_per_group = (int)hpg;
  w.dSq = take(hpg * ds_head);
  w.sdS = take(hpg * nqblk * (size_t)w.ds_pitch * 4);
  w.tmax = take(block_q(p) == 128 ? hpg * nqblk * (size_t)w.ds_pitch * 8 : 0);
  w.total = off;
  return w;
}

int check_params(const sagebwd_params* p) {
  if (p == nullptr) return SAGEBWD_INVALID_ARG;
  if (p->B <= 0 || p->H <= 0 || p->N <= 0 || p->d <= 0) return SAGEBWD_INVALID_ARG;
  if (p->layout != SAGEBWD_LAYOUT_BHND && p->layout != SAGEBWD_LAYOUT_BNHD) return SAGEBWD_INVALID_ARG;
  if ((p->flags & ~(SAGEBWD_FLAG_SHARE_QUANTIZED | SAGEBWD_FLAG_QK_NORM)) != 0 || p->Nkv < 0 || p->reserved != 0)
    return SAGEBWD_INVALID_ARG;
  if (p->flags & SAGEBWD_FLAG_QK_NORM) {
    if (p->qk_gamma_q == nullptr || p->qk_gamma_k == nullptr || !(p->qk_norm_eps >= 0.f) || isinf(p->qk_norm_eps))
      return SAGEBWD_INVALID_ARG;
  } else if (p->qk_gamma_q != nullptr || p->qk_gamma_k != nullptr) {
    return SAGEBWD_INVALID_ARG;
  }
  if (p->bq < 0 || p->bkv < 0) return SAGEBWD_INVALID_ARG;
  if ((p->smooth & ~(SAGEBWD_SMOOTH_K | SAGEBWD_SMOOTH_Q)) != 0) return SAGEBWD_INVALID_ARG;
  if (p->causal != 0 && p->causal != 1) return SAGEBWD_INVALID_ARG;
  if (!(p->sm_scale >= 0.f) || isinf(p->sm_scale)) return SAGEBWD_INVALID_ARG;
  if (p->d != 64 && p->d != 128) return SAGEBWD_UNSUPPORTED_SHAPE;
  if ((p->bq != 0 && p->bq != 64 && p->bq != 128) || (p->bkv != 0 && p->bkv != 64 && p->bkv != 128))
    return SAGEBWD_UNSUPPORTED_SHAPE;
  const int Nk = kv_len(*p);
  if (p->N > (1 << 30) || Nk > (1 << 30)) return SAGEBWD_UNSUPPORTED_SHAPE;
  // under the mask the last query sits on the last key; the kernels keep one diagonal tile per Q block,
  // which needs the two lengths to differ by whole blocks
  if (p->causal && (Nk < p->N || (Nk - p->N) % 64 != 0)) return SAGEBWD_UNSUPPORTED_SHAPE;
  const double elems = (double)p->B * p->H * (double)padded_rows(p->N > Nk ? p->N : Nk) * p->d;
  if (elems >= 1099511627776.0) return SAGEBWD_UNSUPPORTED_SHAPE;
  if ((double)p->B * p->H > 65535.0) return SAGEBWD_UNSUPPORTED_SHAPE;   // grid.y limit
  return SAGEBWD_OK;
}

float logit_scale(const sagebwd_params& p) {
  return p.sm_scale > 0.f ? p.sm_scale : (float)(1.0 / sqrt((double)p.d));
}

// ---- timing -----------------------------------------------------------------
struct TimedSpan {
  hipEvent_t a, b;
};
// Benchmark hook: the only process-wide state of the library, guarded by one mutex.
std::mutex g_timing_mutex;
int g_timing = 0;   // bit k set: bracket kernel k (sagebwd_kernel) with events
std::vector<TimedSpan> g_spans[SAGEBWD_KERNEL_COUNT];
std::vector<TimedSpan> g_pool;

struct ScopedTimer {
  int k;
  hipStream_t st;
  TimedSpan span;
  bool on;
  ScopedTimer(int kernel, hipStream_t s) : k(kernel), st(s), on(false) {
    std::lock_guard<std::mutex> lock(g_timing_mutex);
    on = ((g_timing >> kernel) & 1) != 0;
    if (!on) return;
    if (!g_pool.empty()) {
      span = g_pool.back();
      g_pool.pop_back();
    } else if (hipEventCreate(&span.a) != hipSuccess || hipEventCreate(&span.b) != hipSuccess) {
      on = false;
      return;
    }
    (void)hipEventRecord(span.a, st);
  }
  ~ScopedTimer() {
    if (!on) return;
    (void)hipEventRecord(span.b, st);
    std::lock_guard<std::mutex> lock(g_timing_mutex);
    g_spans[k].push_back(span);
  }
};

#define SAGE_LAUNCH_CHECK()                                   \
  do {                                                        \
    if (hipGetLastError() != hipSuccess) return SAGEBWD_HIP_ERROR; \
  } while (0)

// ---- pre-pass ---------------------------------------------------------------
// want_qk: smooth and quantise Q and K (F layouts; with want_tf also the backward's TF layouts);
// want_v: quantise V; dO != nullptr: quantise dO and form delta and -L*log2(e).
template <int D>
int run_prepass(const void* Q, const void* K, const void* V, const void* dO, const void* O, const float* LSE,
                const sagebwd_params& p, char* ws, const Workspace& w, bool want_qk, bool want_tf, bool want_v,
                hipStream_t st) {
  const int BH = p.B * p.H, Nq = p.N, Nk = kv_len(p), Nqp = padded_rows(Nq), Nkp = padded_rows(Nk);
  const bool ks = (p.smooth & SAGEBWD_SMOOTH_K) != 0;
  const bool qs = (p.smooth & SAGEBWD_SMOOTH_Q) != 0;
  const RowView qview = caller_view(p, 1, Nq), kview = caller_view(p, 1, Nk);     // in bf16 elements
  float* muK = (float*)(ws + w.muK);
  const bool qkn = (p.flags & SAGEBWD_FLAG_QK_NORM) != 0;
  const QkNorm norm_q{qkn ? p.qk_gamma_q : nullptr, p.qk_norm_eps}, norm_k{qkn ? p.qk_gamma_k : nullptr, p.qk_norm_eps};
  if (want_qk) {
    if (ks) {
      kmean_partial_kernel<D><<<dim3(w.nchunk, BH), 256, 0, st>>>((const unsigned short*)K, kview,
                                                                   (double*)(ws + w.kpart), Nk, w.nchunk, w.chunk_rows,
                                                                   norm_k);
      SAGE_LAUNCH_CHECK();
    } else {
      fill_zero_f32_kernel<<<(BH * D + 255) / 256, 256, 0, st>>>(muK, (size_t)BH * D);
      SAGE_LAUNCH_CHECK();
    }
  }
  QuantJobs jobs;
  memset(&jobs, 0, sizeof(jobs));
  int nj = 0;
  auto q_like = [&](QuantJob& j) { j.view = qview; j.N = Nq; j.Np = Nqp; j.q_like = 1; };
  auto k_like = [&](QuantJob& j) { j.view = kview; j.N = Nk; j.Np = Nkp; j.q_like = 0; };
  if (want_qk) {
    // K first: the mean reduction has just read it, so these blocks find it in the memory-side cache.
    // F layout, and TF layout for the backward (dQ = dS^ K^)
    k_like(jobs.job[nj]);
    jobs.job[nj].src = (const unsigned short*)K;
    jobs.job[nj].outF = (int8_t*)(ws + w.KF);
    jobs.job[nj].outTF = want_tf ? (int8_t*)(ws + w.KT) : nullptr;
    jobs.job[nj].scale = (float*)(ws + w.sK);
    jobs.job[nj].mean_part = ks ? (const double*)(ws + w.kpart) : nullptr;
    jobs.job[nj].nchunk = w.nchunk;
    jobs.job[nj].mu_head_out = muK;
    jobs.job[nj].norm = norm_k;
    jobs.job[nj].norm_out = (qkn && qs) ? (unsigned short*)(ws + w.Knorm) : nullptr;
    nj++;
    // Q: F layout (S = Q^ K^^T in both passes) and, for the backward, TF layout (dK = dS^^T Q^)
    q_like(jobs.job[nj]);
    jobs.job[nj].src = (const unsigned short*)Q;
    jobs.job[nj].outF = (int8_t*)(ws + w.QF);
    jobs.job[nj].outTF = want_tf ? (int8_t*)(ws + w.QT) : nullptr;
    jobs.job[nj].scale = (float*)(ws + w.sQ);
    jobs.job[nj].mu_block_out = qs ? (float*)(ws + w.muQ) : nullptr;
    jobs.job[nj].norm = norm_q;
    nj++;
  }
  if (want_v) {
    // V: TF layout (O = P^ V^ contracts over keys); the backward uses the bf16 V only
    k_like(jobs.job[nj]);
    jobs.job[nj].src = (const unsigned short*)V;
    jobs.job[nj].outTF = (int8_t*)(ws + w.VT);
    jobs.job[nj].scale = (float*)(ws + w.sV);
    nj++;
  }
  if (dO != nullptr) {
    // dO: TF layout (dV = P^^T dO^ contracts over queries), plus delta when O is given
    q_like(jobs.job[nj]);
    jobs.job[nj].src = (const unsigned short*)dO;
    jobs.job[nj].outTF = (int8_t*)(ws + w.dOT);
    jobs.job[nj].scale = (float*)(ws + w.sdO);
    jobs.job[nj].O = (const unsigned short*)O;
    jobs.job[nj].delta = (float*)(ws + w.delta);
    jobs.job[nj].lse = LSE;
    jobs.job[nj].nl2 = (float*)(ws + w.nl2);
    nj++;
  }
  if (nj > 0) {
    // one launch per numerics block size in use (64-row blocks per numerics block: 1 or 2); Q-like jobs
    // quantise per B_q rows, K-like jobs per B_kv rows
    const int nblk_max = (Nqp > Nkp ? Nqp : Nkp) / 64;
    for (int sub = 1; sub <= 2; sub++) {
      QuantJobs part;
      memset(&part, 0, sizeof(part));
      int np = 0;
      for (int k = 0; k < nj; k++) {
        if ((jobs.job[k].q_like ? block_q(p) : block_kv(p)) / 64 == sub) part.job[np++] = jobs.job[k];
      }
      if (np == 0) continue;
      if (sub == 1) prepass_quant_kernel<D, 1><<<dim3(nblk_max, BH, np), 256, 0, st>>>(part);
      else prepass_quant_kernel<D, 2><<<dim3(nblk_max, BH, np), 256, 0, st>>>(part);
      SAGE_LAUNCH_CHECK();
    }
  }
  if (qs && want_qk) {
    const float sl2 = logit_scale(p) * 1.4426950408889634f;
    // with QK-norm the bias is formed from the normalised keys, which the quantiser's K blocks left in the workspace
    RowView dense;
    dense.H = p.H;
    dense.batch_stride = (size_t)p.H * Nkp * D; dense.head_stride = (size_t)Nkp * D; dense.row_stride = D;
    qsmooth_bias_kernel<D><<<dim3(Nkp / 64, BH), 256, 0, st>>>(
        qkn ? (const unsigned short*)(ws + w.Knorm) : (const unsigned short*)K, qkn ? dense : kview, muK,
        (const float*)(ws + w.muQ), (float*)(ws + w.bias), Nk, Nkp, Nqp / 64, p.causal ? (Nk - Nq) / 64 : -1, sl2);
    SAGE_LAUNCH_CHECK();
  }
  return SAGEBWD_OK;
}

template <int D>
int prepass_for_forward(const void* Q, const void* K, const void* V, const sagebwd_params& p, char* ws,
                        const Workspace& w, hipStream_t st) {
  const bool share = (p.flags & SAGEBWD_FLAG_SHARE_QUANTIZED) != 0;
  return run_prepass<D>(Q, K, V, nullptr, nullptr, nullptr, p, ws, w, true, share, true, st);
}
template <int D>
int prepass_for_backward(const void* Q, const void* K, const void* V, const void* dO, const void* O, const float* LSE,
                         const sagebwd_params& p, char* ws, const Workspace& w, bool reuse, hipStream_t st) {
  return run_prepass<D>(Q, K, V, dO, O, LSE, p, ws, w, !reuse, true, false, st);
}

// Waves per forward workgroup (32 queries each).  Four, with two (d = 128) or three (d = 64)
// workgroups per CU: the waves that share a SIMD then belong to different workgroups and do not
// wait at each other's barriers (measured 7 % faster than one 8-wave workgroup per CU, although
// that stages every K^/V^ tile once for twice as many queries).
int pick_fwd_waves(int N) { return N % 128 == 0 ? 4 : 2; }

// kv128: numerics blocks of 128 keys (the per-token quantiser of P~ takes its row max over two tiles)
template <int D, bool CAUSAL, bool QS>
int launch_fwd_nw(const FwdArgs& a, int nw, bool kv128, hipStream_t st) {
  FwdArgs args = a;
  args.n_qtiles = a.Nq / (32 * nw);
  args.head_set = head_set_for(args.n_qtiles, a.BH);
  const int grid = grid_for(a.BH, args.n_qtiles);
  if (kv128) {
    if (nw == 4) sage_fwd_kernel<D, CAUSAL, QS, 4, true><<<grid, 256, 0, st>>>(args);
    else sage_fwd_kernel<D, CAUSAL, QS, 2, true><<<grid, 128, 0, st>>>(args);
  } else {
    if (nw == 4) sage_fwd_kernel<D, CAUSAL, QS, 4><<<grid, 256, 0, st>>>(args);
    else sage_fwd_kernel<D, CAUSAL, QS, 2><<<grid, 128, 0, st>>>(args);
  }
  SAGE_LAUNCH_CHECK();
  return SAGEBWD_OK;
}

template <int D>
int launch_fwd(const FwdArgs& a, bool causal, bool qs, bool kv128, hipStream_t st) {
  const int nw = pick_fwd_waves(a.Nq);
  if (causal) return qs ? launch_fwd_nw<D, true, true>(a, nw, kv128, st) : launch_fwd_nw<D, true, false>(a, nw, kv128, st);
  return qs ? launch_fwd_nw<D, false, true>(a, nw, kv128, st) : launch_fwd_nw<D, false, false>(a, nw, kv128, st);
}

template <int D, int MODE, bool KV128 = false>
int launch_bwd(const BwdArgs& a, bool causal, bool qs, hipStream_t st) {
  const int npair = (a.N / 64 + 1) / 2;     // one workgroup per pair of KV blocks
  BwdArgs args = a;
  args.head_set = head_set_for(npair, a.BH);
  const int grid = grid_for(a.BH, npair);
  if (causal) {
    if (qs) sage_bwd_kernel<D, true, true, MODE, KV128><<<grid, 512, 0, st>>>(args);
    else sage_bwd_kernel<D, true, false, MODE, KV128><<<grid, 512, 0, st>>>(args);
  } else {
    if (qs) sage_bwd_kernel<D, false, true, MODE, KV128><<<grid, 512, 0, st>>>(args);
    else sage_bwd_kernel<D, false, false, MODE, KV128><<<grid, 512, 0, st>>>(args);
  }
  SAGE_LAUNCH_CHECK();
  return SAGEBWD_OK;
}

template <int D>
int launch_bwd_dq(const DqArgs& a, bool causal, hipStream_t st) {
  const int npair = (a.Nq / 64 + 1) / 2;    // one workgroup per pair of Q blocks
  DqArgs args = a;
  args.head_set = head_set_for(npair, a.BH, true);   // memory-bound: gains from head sets at every length
  const int grid = grid_for(a.BH, npair);
  if (causal) sage_bwd_dq_kernel<D, true><<<grid, 256, 0, st>>>(args);
  else sage_bwd_dq_kernel<D, false><<<grid, 256, 0, st>>>(args);
  SAGE_LAUNCH_CHECK();
  return SAGEBWD_OK;
}

// The forward on a workspace that holds at least w.fwd_total bytes (arguments already validated).
int forward_impl(const void* Q, const void* K, const void* V, void* O, float* LSE, const sagebwd_params& p,
                 char* ws, const Workspace& w, hipStream_t st) {
  int rc;
  {
    ScopedTimer tm(SAGEBWD_KERNEL_PREPASS_FWD, st);
    rc = p.d == 64 ? prepass_for_forward<64>(Q, K, V, p, ws, w, st) : prepass_for_forward<128>(Q, K, V, p, ws, w, st);
  }
  if (rc != SAGEBWD_OK) return rc;
  FwdArgs a;
  a.QF = (const int8_t*)(ws + w.QF);
  a.KF = (const int8_t*)(ws + w.KF);
  a.VT = (const int8_t*)(ws + w.VT);
  a.sQ = (const float*)(ws + w.sQ);
  a.sK = (const float*)(ws + w.sK);
  a.sV = (const float*)(ws + w.sV);
  const bool qs = (p.smooth & SAGEBWD_SMOOTH_Q) != 0;
  a.bias = qs ? (const float*)(ws + w.bias) : nullptr;
  a.O = (unsigned short*)O;
  a.oview = caller_view(p, 1, p.N);
  a.LSE = LSE;
  a.BH = p.B * p.H;
  a.N = padded_rows(kv_len(p));
  a.nvalid = kv_len(p);
  a.Nq = padded_rows(p.N);
  a.nq_valid = p.N;
  a.shift = p.causal ? kv_len(p) - p.N : 0;
  a.n_qtiles = 0;
  a.scale_log2e = logit_scale(p) * 1.4426950408889634f;
  {
    ScopedTimer tm(SAGEBWD_KERNEL_FWD, st);
    const bool kv128 = block_kv(p) == 128;
    rc = p.d == 64 ? launch_fwd<64>(a, p.causal != 0, qs, kv128, st) : launch_fwd<128>(a, p.causal != 0, qs, kv128, st);
  }
  return rc;
}

// Times `reps` launches of `launch` on `st` with one pair of events around them, after one untimed launch;
// waits for them.  Returns the mean milliseconds per launch through *ms.
template <class F>
int time_probe(F launch, int reps, hipStream_t st, double* ms) {
  hipEvent_t a = nullptr, b = nullptr;
  if (hipEventCreate(&a) != hipSuccess) return SAGEBWD_HIP_ERROR;
  if (hipEventCreate(&b) != hipSuccess) {
    (void)hipEventDestroy(a);
    return SAGEBWD_HIP_ERROR;
  }
  int rc = SAGEBWD_OK;
  launch();
  if (hipEventRecord(a, st) != hipSuccess) rc = SAGEBWD_HIP_ERROR;
  for (int r = 0; r < reps && rc == SAGEBWD_OK; r++) launch();
  if (rc == SAGEBWD_OK && hipEventRecord(b, st) != hipSuccess) rc = SAGEBWD_HIP_ERROR;
  if (rc == SAGEBWD_OK && hipEventSynchronize(b) != hipSuccess) rc = SAGEBWD_HIP_ERROR;
  float t = 0.f;
  if (rc == SAGEBWD_OK && hipEventElapsedTime(&t, a, b) != hipSuccess) rc = SAGEBWD_HIP_ERROR;
  if (rc == SAGEBWD_OK && hipGetLastError() != hipSuccess) rc = SAGEBWD_HIP_ERROR;
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  *ms = (double)t / reps;
  return rc;
}


}  // namespace

extern "C" {

int sagebwd_workspace_bytes(const sagebwd_params* params, size_t* fwd_bytes, size_t* bwd_bytes) {
  int rc = check_params(params);
  if (rc != SAGEBWD_OK) return rc;
  const Workspace w = make_layout(*params);
  if (fwd_bytes != nullptr) *fwd_bytes = w.fwd_total;
  if (bwd_bytes != nullptr) *bwd_bytes = w.total;
  return SAGEBWD_OK;
}

int sagebwd_quantize(const void* Q, const void* K, const void* V, const void* dO, const void* O,
                     const sagebwd_params* params, void* workspace, size_t workspace_bytes,
                     void* stream) {
  int rc = check_params(params);
  if (rc != SAGEBWD_OK) return rc;
  if (Q == nullptr || K == nullptr || V == nullptr || workspace == nullptr) return SAGEBWD_INVALID_ARG;
  if (O != nullptr && dO == nullptr) return SAGEBWD_INVALID_ARG;
  const Workspace w = make_layout(*params);
  if (workspace_bytes < w.total) return SAGEBWD_WORKSPACE_TOO_SMALL;
  hipStream_t st = (hipStream_t)stream;
  char* ws = (char*)workspace;
  // the inspection pre-pass fills every layout: forward operands first, then the backward's
  {
    ScopedTimer tm(SAGEBWD_KERNEL_PREPASS_FWD, st);
    rc = params->d == 64 ? prepass_for_forward<64>(Q, K, V, *params, ws, w, st)
                         : prepass_for_forward<128>(Q, K, V, *params, ws, w, st);
  }
  if (rc != SAGEBWD_OK || dO == nullptr) return rc;
  {
    ScopedTimer tm(SAGEBWD_KERNEL_PREPASS_BWD, st);
    rc = params->d == 64 ? prepass_for_backward<64>(Q, K, V, dO, O, nullptr, *params, ws, w, false, st)
                         : prepass_for_backward<128>(Q, K, V, dO, O, nullptr, *params, ws, w, false, st);
  }
  return rc;
}

int sagebwd_export_quantized(const sagebwd_params* params, const void* workspace,
                             size_t workspace_bytes, int which, int8_t* q_out, float* scale_out,
                             void* stream) {
  int rc = check_params(params);
  if (rc != SAGEBWD_OK) return rc;
  if (workspace == nullptr) return SAGEBWD_INVALID_ARG;
  const Workspace w = make_layout(*params);
  if (workspace_bytes < w.total) return SAGEBWD_WORKSPACE_TOO_SMALL;
  size_t qoff, soff;
  int transposed;
  switch (which) {
    case SAGEBWD_TENSOR_Q: qoff = w.QF; soff = w.sQ; transposed = 0; break;
    case SAGEBWD_TENSOR_K: qoff = w.KF; soff = w.sK; transposed = 0; break;
    case SAGEBWD_TENSOR_V: qoff = w.VT; soff = w.sV; transposed = 1; break;
    case SAGEBWD_TENSOR_DO: qoff = w.dOT; soff = w.sdO; transposed = 1; break;
    default: return SAGEBWD_INVALID_ARG;
  }
  hipStream_t st = (hipStream_t)stream;
  const char* ws = (const char*)workspace;
  const size_t BH = (size_t)params->B * params->H;
  const bool k_like = which == SAGEBWD_TENSOR_K || which == SAGEBWD_TENSOR_V;
  const int Np = padded_rows(k_like ? kv_len(*params) : params->N);
  if (q_out != nullptr) {
    const size_t n_chunks = BH * Np * params->d / 16;
    export_fragments_kernel<<<(unsigned)((n_chunks + 255) / 256), 256, 0, st>>>(
        (const int8_t*)(ws + qoff), q_out, n_chunks, Np, params->d, transposed);
    SAGE_LAUNCH_CHECK();
  }
  if (scale_out != nullptr) {
    const size_t n = BH * (Np / 64);
    copy_f32_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>((const float*)(ws + soff), scale_out, n, 1.0f);
    SAGE_LAUNCH_CHECK();
  }
  return SAGEBWD_OK;
}

int sagebwd_export_stats(const sagebwd_params* params, const void* workspace, size_t workspace_bytes,
                         float* mu_K, float* mu_Q, float* delta, void* stream) {
  int rc = check_params(params);
  if (rc != SAGEBWD_OK) return rc;
  if (workspace == nullptr) return SAGEBWD_INVALID_ARG;
  const Workspace w = make_layout(*params);
  if (workspace_bytes < w.total) return SAGEBWD_WORKSPACE_TOO_SMALL;
  if (mu_Q != nullptr && !(params->smooth & SAGEBWD_SMOOTH_Q)) return SAGEBWD_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  const char* ws = (const char*)workspace;
  const size_t BH = (size_t)params->B * params->H;
  auto copy = [&](size_t off, float* out, size_t n, float sign = 1.0f) {
    unsigned grid = (unsigned)((n + 255) / 256);
    if (grid > 65535u * 16u) grid = 65535u * 16u;
    copy_f32_kernel<<<grid, 256, 0, st>>>((const float*)(ws + off), out, n, sign);
  };
  if (mu_K != nullptr) { copy(w.muK, mu_K, BH * params->d); SAGE_LAUNCH_CHECK(); }
  const size_t Np = padded_rows(params->N);
  if (mu_Q != nullptr) { copy(w.muQ, mu_Q, BH * (Np / 64) * params->d); SAGE_LAUNCH_CHECK(); }
  if (delta != nullptr) { copy(w.delta, delta, BH * Np, -1.0f); SAGE_LAUNCH_CHECK(); }   // the workspace holds -delta
  return SAGEBWD_OK;
}

int sagebwd_export_ds(const sagebwd_params* params, const void* workspace, size_t workspace_bytes, int head,
                      int8_t* ds_out, float* scale_out, void* stream) {
  int rc = check_params(params);
  if (rc != SAGEBWD_OK) return rc;
  if (workspace == nullptr || head < 0 || head >= params->B * params->H) return SAGEBWD_INVALID_ARG;
  const Workspace w = make_layout(*params);
  if (workspace_bytes < w.total) return SAGEBWD_WORKSPACE_TOO_SMALL;
  // the scratch holds the heads of the LAST group the backward processed: only a backward that ran
  // in one group leaves every head behind
  if (w.heads_per_group < params->B * params->H) return SAGEBWD_UNSUPPORTED_SHAPE;
  const int Nkp = padded_rows(kv_len(*params)), nkblk = Nkp / 64, nqblk = padded_rows(params->N) / 64;
  const char* ws = (const char*)workspace;
  const size_t n = (size_t)nqblk * nkblk * 256;
  export_ds_kernel<<<(unsigned)((n + 255) / 256), 256, 0, (hipStream_t)stream>>>(
      (const int8_t*)(ws + w.dSq) + (size_t)head * nqblk * w.ds_pitch * 4096,
      (const float*)(ws + w.sdS) + (size_t)head * nqblk * w.ds_pitch, ds_out, scale_out, nqblk, Nkp, w.ds_pitch,
      params->causal ? (kv_len(*params) - params->N) / 64 : -1);
  SAGE_LAUNCH_CHECK();
  return SAGEBWD_OK;
}

int sagebwd_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                const sagebwd_params* params, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_params(params);
  if (rc != SAGEBWD_OK) return rc;
  if (Q == nullptr || K == nullptr || V == nullptr || O == nullptr || LSE == nullptr || workspace == nullptr)
    return SAGEBWD_INVALID_ARG;
  const Workspace w = make_layout(*params);
  if (workspace_bytes < w.fwd_total) return SAGEBWD_WORKSPACE_TOO_SMALL;
  return forward_impl(Q, K, V, O, LSE, *params, (char*)workspace, w, (hipStream_t)stream);
}

int sagebwd_fwd_static(const void* Q, const void* K, const void* V, void* O, float* LSE,
                       const sagebwd_params* params, void* stream) {
  int rc = check_params(params);
  if (rc != SAGEBWD_OK) return rc;
  if (Q == nullptr || K == nullptr || V == nullptr || O == nullptr || LSE == nullptr) return SAGEBWD_INVALID_ARG;
  // the backward of such a call would need the caller's workspace anyway: nothing is shared through `scratch`
  if ((params->flags & SAGEBWD_FLAG_SHARE_QUANTIZED) != 0) return SAGEBWD_INVALID_ARG;
  const Workspace w = make_layout(*params);
  if (w.fwd_total > (size_t)SAGEBWD_STATIC_SCRATCH_BYTES) return SAGEBWD_STATIC_SCRATCH_TOO_SMALL;
  char* ws = (char*)static_scratch_for_current_device();
  if (ws == nullptr) return SAGEBWD_HIP_ERROR;
  // every byte of the forward's workspace that a kernel reads is written earlier in the same call
  // (the pre-pass fills all operand rows, the missing ones of a partial block as zero codes), so nothing
  // the previous call left in the array has to be cleared
  return forward_impl(Q, K, V, O, LSE, *params, ws, w, (hipStream_t)stream);
}

int sagebwd_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                const float* LSE, void* dQ, void* dK, void* dV, const sagebwd_params* params,
                void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_params(params);
  if (rc != SAGEBWD_OK) return rc;
  if (Q == nullptr || K == nullptr || V == nullptr || O == nullptr || dO == nullptr || LSE == nullptr ||
      dQ == nullptr || dK == nullptr || dV == nullptr || workspace == nullptr)
    return SAGEBWD_INVALID_ARG;
  const Workspace w = make_layout(*params);
  if (workspace_bytes < w.total) return SAGEBWD_WORKSPACE_TOO_SMALL;
  hipStream_t st = (hipStream_t)stream;
  char* ws = (char*)workspace;
  const int BH = params->B * params->H, d = params->d;
  const int Nk = kv_len(*params), Nkp = padded_rows(Nk), Nqp = padded_rows(params->N);
  const int shift_blocks = params->causal ? (Nk - params->N) / 64 : 0;
  const bool qs = (params->smooth & SAGEBWD_SMOOTH_Q) != 0;
  {
    ScopedTimer tm(SAGEBWD_KERNEL_PREPASS_BWD, st);
    const bool reuse = (params->flags & SAGEBWD_FLAG_SHARE_QUANTIZED) != 0;   // Q^, K^ as the forward left them
    rc = d == 64 ? prepass_for_backward<64>(Q, K, V, dO, O, LSE, *params, ws, w, reuse, st)
                 : prepass_for_backward<128>(Q, K, V, dO, O, LSE, *params, ws, w, reuse, st);
    if (rc != SAGEBWD_OK) return rc;
  }
  BwdArgs a;
  a.QF = (const int8_t*)(ws + w.QF);
  a.QT = (const int8_t*)(ws + w.QT);
  a.KF = (const int8_t*)(ws + w.KF);
  a.dOT = (const int8_t*)(ws + w.dOT);
  a.cv = caller_view(*params, 1, Nk);           // in bf16 elements
  a.cvq = caller_view(*params, 1, params->N);
  a.V = (const unsigned short*)V;
  a.dO = (const unsigned short*)dO;
  a.sQ = (const float*)(ws + w.sQ);
  a.sK = (const float*)(ws + w.sK);
  a.sdO = (const float*)(ws + w.sdO);
  a.nL2 = (const float*)(ws + w.nl2);
  a.delta = (const float*)(ws + w.delta);
  a.bias = qs ? (const float*)(ws + w.bias) : nullptr;
  a.muQ = qs ? (const float*)(ws + w.muQ) : nullptr;
  a.dSq = (int8_t*)(ws + w.dSq);
  a.ds_pitch = w.ds_pitch;
  a.sdS = (float*)(ws + w.sdS);
  a.tmax = nullptr;
  const bool big = big_blocks(*params);
  a.dK = (unsigned short*)dK;
  a.dV = (unsigned short*)dV;
  a.N = Nkp;
  a.nvalid = Nk;
  a.Nq = Nqp;
  a.nq_valid = params->N;
  a.shift_blocks = shift_blocks;
  a.sm_scale = logit_scale(*params);
  a.scale_log2e = a.sm_scale * 1.4426950408889634f;
  DqArgs q;
  q.cv = a.cvq;
  q.dSq = a.dSq;
  q.ds_pitch = w.ds_pitch;
  q.sdS = a.sdS;
  q.KT = (const int8_t*)(ws + w.KT);
  q.sK = a.sK;
  q.dQ = (unsigned short*)dQ;
  q.nvalid = params->N;
  q.N = Nkp;
  q.Nq = Nqp;
  q.shift_blocks = shift_blocks;
  q.sm_scale = a.sm_scale;
  for (int h0 = 0; h0 < BH; h0 += w.heads_per_group) {
    const int nh = BH - h0 < w.heads_per_group ? BH - h0 : w.heads_per_group;
    a.bh0 = q.bh0 = h0;
    a.BH = q.BH = nh;
    {
      ScopedTimer tm(SAGEBWD_KERNEL_BWD, st);
      const bool causal = params->causal != 0;
      if (!big) {
        rc = d == 64 ? launch_bwd<64, kBwdFused>(a, causal, qs, st) : launch_bwd<128, kBwdFused>(a, causal, qs, st);
        if (rc != SAGEBWD_OK) return rc;
      } else if (block_q(*params) == 64) {
        // 64 x 128: the numerics block is the pair of tiles a workgroup holds at once
        rc = d == 64 ? launch_bwd<64, kBwdFused, true>(a, causal, qs, st) : launch_bwd<128, kBwdFused, true>(a, causal, qs, st);
        if (rc != SAGEBWD_OK) return rc;
      } else {
        // 128-row Q blocks: phase A alone on the even Q blocks for their tiles' maxima, then the full kernel,
        // which pairs every Q block with its neighbour (see the modes in bwd_kernel.h)
        a.tmax = (float*)(ws + w.tmax);
        rc = d == 64 ? launch_bwd<64, kBwdMaxOnly>(a, causal, qs, st) : launch_bwd<128, kBwdMaxOnly>(a, causal, qs, st);
        if (rc != SAGEBWD_OK) return rc;
        if (block_kv(*params) == 128)
          rc = d == 64 ? launch_bwd<64, kBwdPairedRows, true>(a, causal, qs, st) : launch_bwd<128, kBwdPairedRows, true>(a, causal, qs, st);
        else
          rc = d == 64 ? launch_bwd<64, kBwdPairedRows>(a, causal, qs, st) : launch_bwd<128, kBwdPairedRows>(a, causal, qs, st);
        if (rc != SAGEBWD_OK) return rc;
      }
    }
    {
      ScopedTimer tm(SAGEBWD_KERNEL_BWD_DQ, st);
      rc = d == 64 ? launch_bwd_dq<64>(q, params->causal != 0, st) : launch_bwd_dq<128>(q, params->causal != 0, st);
      if (rc != SAGEBWD_OK) return rc;
    }
  }
  return rc;
}

int sagebwd_set_timing(int kernels) {
  if (kernels < 0 || kernels > SAGEBWD_TIMING_ALL) return SAGEBWD_INVALID_ARG;
  std::lock_guard<std::mutex> lock(g_timing_mutex);
  g_timing = kernels;
  return SAGEBWD_OK;
}

int sagebwd_read_timing(int kernel, double* total_ms, int* launches) {
  if (kernel < 0 || kernel >= SAGEBWD_KERNEL_COUNT || total_ms == nullptr || launches == nullptr)
    return SAGEBWD_INVALID_ARG;
  double tot = 0.0;
  int n = 0;
  std::lock_guard<std::mutex> lock(g_timing_mutex);
  for (TimedSpan& s : g_spans[kernel]) {
    if (hipEventSynchronize(s.b) != hipSuccess) return SAGEBWD_HIP_ERROR;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, s.a, s.b) != hipSuccess) return SAGEBWD_HIP_ERROR;
    tot += ms;
    n++;
    g_pool.push_back(s);
  }
  g_spans[kernel].clear();
  *total_ms = tot;
  *launches = n;
  return SAGEBWD_OK;
}

int sagebwd_probe_mfma(int kind, int iters, int reps, void* sink, void* stream, double* ms, double* ops) {
  if (kind < 0 || kind > (SAGEBWD_PROBE_MFMA_BF16 | SAGEBWD_PROBE_MFMA_ZERO_OPERANDS) || iters < 1 || iters > (1 << 20) || reps < 1 ||
      reps > 1000 || sink == nullptr || ms == nullptr || ops == nullptr)
    return SAGEBWD_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  int cus = 0, dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
    return SAGEBWD_HIP_ERROR;
  // two workgroups of four waves per CU = two waves per SIMD, eight rounds of them
  const int grid = cus * 2 * 8;
  const bool bf16 = (kind & SAGEBWD_PROBE_MFMA_BF16) != 0;
  const int mask = (kind & SAGEBWD_PROBE_MFMA_ZERO_OPERANDS) ? 0 : -1;
  auto launch = [&]() {
    if (bf16) probe_mfma_kernel<true><<<grid, 256, 0, st>>>(iters, 0x5A6E, mask, (int*)sink);
    else probe_mfma_kernel<false><<<grid, 256, 0, st>>>(iters, 0x5A6E, mask, (int*)sink);
  };
  *ops = (double)grid * 4.0 * iters * 4.0 * 2.0 * 32 * 32 * (bf16 ? 16 : 32);
  return time_probe(launch, reps, st, ms);
}

int sagebwd_probe_stream(int kind, const void* src, void* dst, size_t bytes, int reps, void* sink, void* stream, double* ms) {
  if ((kind != SAGEBWD_PROBE_STREAM_COPY && kind != SAGEBWD_PROBE_STREAM_READ) || src == nullptr || bytes < 16 || bytes % 16 != 0 ||
      reps < 1 || reps > 1000 || sink == nullptr || ms == nullptr || (kind == SAGEBWD_PROBE_STREAM_COPY && dst == nullptr))
    return SAGEBWD_INVALID_ARG;
  if (((uintptr_t)src | (uintptr_t)dst) % 16 != 0) return SAGEBWD_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  int cus = 0, dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
    return SAGEBWD_HIP_ERROR;
  const size_t pieces = bytes / 16;
  size_t want = (pieces + 255) / 256;
  const int grid = (int)(want < (size_t)cus * 8 ? want : (size_t)cus * 8);
  const bool copy = kind == SAGEBWD_PROBE_STREAM_COPY;
  auto launch = [&]() {
    if (copy) probe_stream_kernel<true><<<grid, 256, 0, st>>>((const v4i*)src, (v4i*)dst, pieces, 0x5A6E, (int*)sink);
    else probe_stream_kernel<false><<<grid, 256, 0, st>>>((const v4i*)src, nullptr, pieces, 0x5A6E, (int*)sink);
  };
  return time_probe(launch, reps, st, ms);
}

const char* sagebwd_strerror(int status) {
  switch (status) {
    case SAGEBWD_OK: return "ok";
    case SAGEBWD_INVALID_ARG: return "invalid argument (null pointer, bad flag or size)";
    case SAGEBWD_UNSUPPORTED_SHAPE: return "unsupported shape (need d in {64,128}, numerics blocks of 64 or 128, sizes within the stated limits)";
    case SAGEBWD_WORKSPACE_TOO_SMALL: return "workspace too small (see sagebwd_workspace_bytes)";
    case SAGEBWD_HIP_ERROR: return "HIP runtime error";
    case SAGEBWD_STATIC_SCRATCH_TOO_SMALL:
      return "problem too large for the built-in scratch of sagebwd_fwd_static (use sagebwd_fwd with a workspace)";
    default: return "unknown status";
  }
}

}  // extern "C"
