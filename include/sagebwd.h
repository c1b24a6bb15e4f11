/*
 * sagebwd.h -- C ABI of the SageBwd hot path on one MI355X (gfx950).
 *
 * SageBwd is a trainable INT8 attention: the forward computes
 * O = softmax(sm_scale * Q K^T) V with Q K^T and P V on INT8 with per-block
 * scales (paper Sec. 3 "SageBwd", Algorithm 1); the backward recomputes P and
 * forms dV, dP, dS, dQ, dK with every matmul on INT8 except dP = dO V^T
 * (paper Sec. 3 gradient equations, Algorithm 2).
 *
 * Conventions shared by every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The library
 *     allocates and frees no device memory; scratch lives in a caller-owned
 *     workspace of sagebwd_workspace_bytes() bytes (256-byte aligned).  Apart from the
 *     benchmark hooks at the end of this file the library keeps no state between calls:
 *     everything that shapes a call, the scratch budget included, is in sagebwd_params.
 *   - Tensors are dense and contiguous: Q, O, dO, dQ are bf16 [B, H, N, d], K, V, dK, dV are bf16
 *     [B, H, Nkv, d] (or [B, N, H, d] / [B, Nkv, H, d], see sagebwd_params.layout); LSE is float32
 *     [B, H, N].  Nkv = N unless sagebwd_params.Nkv says otherwise (cross attention, chunked prefill,
 *     decoding against a cache: the paper states the method for one length, nothing in it couples the two).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work
 *     is enqueued on it and the call returns without synchronising.  The entry points
 *     only launch kernels (no allocation, no memset, no host synchronisation), so
 *     sagebwd_fwd / sagebwd_bwd may be recorded under stream capture and replayed.
 *   - Return value: SAGEBWD_OK (0) or a negative sagebwd_status.  Arguments are
 *     validated on the host before anything is launched; on error nothing runs.
 *   - Numerics blocks are B_q = B_kv = 64 (one FP32 scale per 64 rows x d channels); Algorithm 1
 *     takes both as inputs, sagebwd_params carries them, other values are SAGEBWD_UNSUPPORTED_SHAPE.
 *   - Bit-exact contract: the stored INT8 tensors Q^, K^, V^, dO^, their scales and the smoothing
 *     means equal the paper's definitions evaluated in FP32 bit for bit.  The quantisers inside
 *     the attention loops (P^ of the forward, psi(P) and psi(dS) of the backward) depend on the
 *     hardware exp2 and are held to a tolerance (codes within one step), as are O, LSE, dQ, dK, dV.
 *   - Supported shapes: d in {64, 128}; N >= 1; B*H*Np*d < 2^40, where Np is N rounded
 *     up to a multiple of 64.  The paper assumes N/B_q and N/B_kv integral (Algorithm 1
 *     line 2); for other N the last block is a partial block whose missing rows do not
 *     exist: they enter no mean, no block maximum, no softmax and receive no gradient.
 *     (The kernels run on Np rows of workspace operands with the missing keys masked; the
 *     caller's tensors are read and written on their N rows only.)
 */
#ifndef SAGEBWD_H
#define SAGEBWD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum sagebwd_status {
  SAGEBWD_OK = 0,
  SAGEBWD_INVALID_ARG = -1,        /* null pointer, non-positive size, unknown selector */
  SAGEBWD_UNSUPPORTED_SHAPE = -2,  /* d not in {64,128}, numerics blocks other than 64 or 128, sizes beyond the stated limits */
  SAGEBWD_WORKSPACE_TOO_SMALL = -3,
  SAGEBWD_HIP_ERROR = -4,          /* a HIP runtime call or launch failed */
  SAGEBWD_STATIC_SCRATCH_TOO_SMALL = -5 /* sagebwd_fwd_static: the forward's workspace exceeds the built-in scratch */
} sagebwd_status;

/* Smoothing flags (paper Sec. 3 "Q and K Smoothing"). */
#define SAGEBWD_SMOOTH_K 1 /* subtract the token mean of K of each head before quantising */
#define SAGEBWD_SMOOTH_Q 2 /* subtract the mean of each 64-row Q block; logits get the bias back */

/* Layouts of the bf16 tensors (LSE is float32 [B, H, N] in both). */
#define SAGEBWD_LAYOUT_BHND 0 /* [B, H, N, d]: what the kernels read and write directly */
#define SAGEBWD_LAYOUT_BNHD 1 /* [B, N, H, d], token-major as most frameworks hold activations: read and
                                 written in place through row strides (rows lie H*d elements apart) */

/* Flags.
 * SAGEBWD_FLAG_SHARE_QUANTIZED: the backward takes psi(Q), psi(K), their scales and the smoothing
 * means from the forward instead of forming them again (Algorithm 2 lists them among its inputs
 * "from the forward").  With the flag set, sagebwd_fwd also leaves Q^ and K^ in the operand layouts
 * of the backward (its workspace need grows by 2*B*H*Np*d bytes, see sagebwd_workspace_bytes), and
 * sagebwd_bwd re-runs only the dO part of the pre-pass.  The caller guarantees that the same
 * workspace, params, Q and K are passed to both calls and that nothing wrote the workspace in
 * between (another sagebwd_fwd on it included).  Results are bit-identical to the calls without
 * the flag.  Without the flag sagebwd_bwd relies on nothing an earlier call left behind. */
#define SAGEBWD_FLAG_SHARE_QUANTIZED 1
/* SAGEBWD_FLAG_QK_NORM: Q and K are the projections BEFORE the model's QK-norm (paper Sec. 4,
 * "Stabilizing Outliers with QK-Norm": RMS normalisation of every token of Q and K); the pre-pass applies
 *     y = x / sqrt(mean_c(x^2) + qk_norm_eps) * gamma      per token and head, gamma = qk_gamma_q / qk_gamma_k,
 * rounds y to bf16 (the tensor a bf16 model would hand to the attention) and goes on with the smoothing
 * and the quantiser, so one pass over Q and K replaces the model's normalisation kernel plus this
 * library's pre-pass, with the bits of running the two one after the other.  Arithmetic (part of the
 * bit-exact contract): sum of squares in float64, r = 1 / sqrt(sum / d + eps) in float64 rounded once to
 * FP32, y = bf16((x *_f32 r) *_f32 gamma).  O, LSE, dV are unchanged in meaning; dQ and dK are the
 * gradients with respect to the NORMALISED Q and K (the chain rule through the normalisation is the
 * caller's).  qk_gamma_q and qk_gamma_k are device pointers to d floats each, shared by all heads. */
#define SAGEBWD_FLAG_QK_NORM 2

typedef struct sagebwd_params {
  int32_t B, H, N, d; /* N = rows of Q, O, dO, dQ (and of K, V, dK, dV unless Nkv is set) */
  int32_t causal;  /* 0 / 1: key index <= query index (+ Nkv - N when the lengths differ) */
  int32_t smooth;  /* OR of SAGEBWD_SMOOTH_* ; the paper's default is SAGEBWD_SMOOTH_K */
  float sm_scale;  /* logit scale; 0 selects 1/sqrt(d) (paper Sec. 4: S = Q K^T / sqrt(d)) */
  int32_t layout;  /* SAGEBWD_LAYOUT_*: how the caller holds Q, K, V, O, dO, dQ, dK, dV */
  int32_t bq, bkv; /* numerics block sizes B_q, B_kv (Algorithm 1, input line): 0 (= 64), 64 or 128 each.
                      Q and dO share one psi scale (and Q its smoothing mean) per B_q rows, K and V per B_kv
                      rows, psi(P~) of the forward its row max per B_kv keys, psi(P) and psi(dS) of the backward
                      one scale per B_q x B_kv block; blocks start at row / key 0.  The kernels' tiles stay
                      64 x 64: every stored or exported scale, mean and bias row is kept once per 64-row block
                      (the value of the numerics block it lies in).  64 x 64 is the fast path: B_kv = 128
                      costs the forward about a tenth, B_q = 128 a second sweep of the backward (see
                      sagebwd_bwd).  Forward and backward must be given the same sizes. */
  int32_t flags;   /* OR of SAGEBWD_FLAG_* */
  int32_t Nkv;     /* rows of K, V, dK, dV; 0 selects N (square attention).  With causal = 1 the last
                      query is aligned with the last key (query i sees keys k <= i + Nkv - N), which needs
                      Nkv >= N and Nkv - N a multiple of 64 (else SAGEBWD_UNSUPPORTED_SHAPE); a decoding
                      step whose queries see the whole cache is the call with causal = 0 */
  uint64_t scratch_budget;   /* upper bound, in bytes, on the INT8 dS scratch that sagebwd_bwd holds at
                                once; 0 selects 8 GiB.  The backward needs Np*(Nkp+192) bytes per head and
                                processes the heads in groups that fit the bound (at least one head per
                                group); the workspace size follows from it. */
  const float* qk_gamma_q;   /* SAGEBWD_FLAG_QK_NORM: DEVICE pointers to the d gains of Q and of K; */
  const float* qk_gamma_k;   /*   must be NULL without the flag                                      */
  float qk_norm_eps;         /* SAGEBWD_FLAG_QK_NORM: >= 0, added to the mean square */
  int32_t reserved;          /* must be 0 */
} sagebwd_params;

/* Which quantised tensor sagebwd_export_quantized() copies out. */
typedef enum sagebwd_tensor {
  SAGEBWD_TENSOR_Q = 0,
  SAGEBWD_TENSOR_K = 1,
  SAGEBWD_TENSOR_V = 2,
  SAGEBWD_TENSOR_DO = 3
} sagebwd_tensor;

/* Kernels whose device time sagebwd_read_timing() reports. */
typedef enum sagebwd_kernel {
  SAGEBWD_KERNEL_PREPASS_FWD = 0, /* smoothing + psi(Q), psi(K), psi(V)            */
  SAGEBWD_KERNEL_FWD = 1,         /* fused forward (Algorithm 1 loop)              */
  SAGEBWD_KERNEL_PREPASS_BWD = 2, /* psi(dO), delta, and the backward's operand layouts */
  SAGEBWD_KERNEL_BWD = 3,         /* fused backward (Algorithm 2 loop): dK, dV, psi(dS) */
  SAGEBWD_KERNEL_BWD_DQ = 4,      /* dQ = sum_j psi(dS_ij) K^_j from the stored tiles */
  SAGEBWD_KERNEL_COUNT = 5
} sagebwd_kernel;

/* Bytes of workspace the calls need for these params (host computation only): *fwd_bytes for
 * sagebwd_fwd, *bwd_bytes (never smaller) for sagebwd_bwd, sagebwd_quantize and the export hooks.
 * The forward's part is a prefix of the backward's, so a buffer of *bwd_bytes serves every call.
 * Either pointer may be NULL. */
int sagebwd_workspace_bytes(const sagebwd_params* params, size_t* fwd_bytes, size_t* bwd_bytes);

/*
 * Pre-pass (paper Sec. 3 smoothing equations; Algorithm 1 "Quantization" line;
 * Algorithm 2 line 2 and the psi(dO_i) of its line 6).
 *   mu_K = mean over the N tokens of K[b,h] (only with SAGEBWD_SMOOTH_K), K_sm = K - mu_K;
 *   psi per 64-row block of Q (or Q - mu_Qi), K_sm, V:  a = max|x|, s = a/127,
 *   q = rne(x * (127/a)) in FP32, clamped to [-127,127]; a == 0 gives s = 0, q = 0.
 *   If dO is non-NULL: psi(dO) per 64-row block; if O is also non-NULL,
 *   delta = rowsum(dO o O) in FP32.
 * Results are left in `workspace` in the library's internal operand layouts (1 KiB fragments in
 * the order the matrix instructions consume them, Q^ and K^ twice), which is why there is no call
 * that returns raw pointers into the workspace: use sagebwd_export_quantized() /
 * sagebwd_export_stats() to read them in row-major form.  dO and O may be NULL.
 */
int sagebwd_quantize(const void* Q, const void* K, const void* V, const void* dO, const void* O,
                     const sagebwd_params* params, void* workspace, size_t workspace_bytes,
                     void* stream);

/*
 * Copy one quantised tensor out of a workspace filled by sagebwd_quantize (or by
 * sagebwd_fwd / sagebwd_bwd, which run the same pre-pass) into row-major form:
 *   q_out      int8    [B, H, Np, d]     (Np = the tensor's row count, N or Nkv, rounded up to a multiple
 *                                         of 64; the rows past it are zero)
 *   scale_out  float32 [B, H, Np/64]
 * Either output may be NULL.  SAGEBWD_TENSOR_DO requires that dO was given.
 * This is a test / inspection hook for the bit-exact part of the contract.
 */
int sagebwd_export_quantized(const sagebwd_params* params, const void* workspace,
                             size_t workspace_bytes, int which /* sagebwd_tensor */,
                             int8_t* q_out, float* scale_out, void* stream);

/* Copy the smoothing means out of the workspace: mu_K float32 [B, H, d] (zeros when
 * K-smoothing is off), mu_Q float32 [B, H, Np/64, d] (only written with
 * SAGEBWD_SMOOTH_Q), delta float32 [B, H, Np] (only after a pre-pass that had dO and O);
 * Np = N rounded up to a multiple of 64.
 * Any pointer may be NULL. */
int sagebwd_export_stats(const sagebwd_params* params, const void* workspace,
                         size_t workspace_bytes, float* mu_K, float* mu_Q, float* delta,
                         void* stream);

/*
 * Copy the quantised score gradient psi(dS) (Algorithm 2, the dS line and its quantisation) that the
 * last sagebwd_bwd on this workspace left in its scratch, for one head = b * H + h:
 *   ds_out     int8    [Np, Nkp] row-major (query, key); tiles above the causal diagonal are zero
 *   scale_out  float32 [Np/64, Nkp/64], one scale per 64x64 tile (dS ~ scale * code; with larger numerics
 *              blocks the tiles of a block carry the same scale)
 * Np, Nkp = N, Nkv rounded up to a multiple of 64.  Either output may be NULL.  Only defined when the backward
 * ran all heads in one group (B*H*Np*(Np+192) bytes within params->scratch_budget), otherwise
 * SAGEBWD_UNSUPPORTED_SHAPE.  A test / inspection hook: the in-loop quantisers depend on the
 * hardware's exp2, so their codes are compared with a tolerance of one step, not bit for bit.
 */
int sagebwd_export_ds(const sagebwd_params* params, const void* workspace, size_t workspace_bytes,
                      int head, int8_t* ds_out, float* scale_out, void* stream);

/*
 * Forward (paper Algorithm 1 with K-smoothing applied before psi(K), Sec. 3):
 *   S_ij = (Q^_i K^_j^T) * s_Q * s_K * sm_scale  [+ mu_Qi K_sm_j^T * sm_scale with Q-smoothing],
 *   online softmax over the KV blocks, per-token quantisation of P~ relative to the
 *   row max of the tile, O_i += (P^_ij V^_j) * s_P * s_V, O = O / l, L = m + log l.
 * Writes O bf16 [B,H,N,d] and LSE float32 [B,H,N].  LSE is the log-sum-exp of the
 * SMOOTHED logits (it differs from the unsmoothed one by a per-row constant) and is
 * meant to be handed back to sagebwd_bwd unchanged.
 */
int sagebwd_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                const sagebwd_params* params, void* workspace, size_t workspace_bytes,
                void* stream);

/*
 * sagebwd_fwd for callers that cannot allocate device memory or pass a workspace: code under
 * stream capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels
 * and results (bit for bit) as sagebwd_fwd, but the forward's workspace is a built-in device array of
 * SAGEBWD_STATIC_SCRATCH_BYTES that every GPU the library runs on holds until the process ends.
 * The call allocates and frees nothing (its first call on a device looks the array's address up).
 *   - Problems whose forward workspace (*fwd_bytes of sagebwd_workspace_bytes) exceeds the array
 *     are rejected with SAGEBWD_STATIC_SCRATCH_TOO_SMALL before anything is launched; roughly
 *     3*B*H*Np*d bytes plus the small vectors, e.g. up to B*H = 8 heads of N = 8192, d = 128.
 *   - SAGEBWD_FLAG_SHARE_QUANTIZED is rejected (SAGEBWD_INVALID_ARG): the backward reads a caller's
 *     workspace, not this array.
 *   - All calls on one GPU share the one array: two calls that overlap in time on the same GPU
 *     (different streams or threads) race.  Calls in stream order on one stream are safe; nothing
 *     has to be cleared between calls (every byte read is written earlier in the same call).
 */
#define SAGEBWD_STATIC_SCRATCH_BYTES (32u << 20)
int sagebwd_fwd_static(const void* Q, const void* K, const void* V, void* O, float* LSE,
                       const sagebwd_params* params, void* stream);

/*
 * Backward (paper Algorithm 2; gradient equations of Sec. 3):
 *   delta = rowsum(dO o O);  P_ij = exp(S_ij - L_i);
 *   dV_j += psi(P_ij)^T psi(dO_i) * s_P * s_dO                      (INT8)
 *   dP_ij = dO_i V_j^T                                              (bf16, unquantised)
 *   dS_ij = P_ij o (dP_ij - delta_i)
 *   dQ_i += psi(dS_ij) K^_j * s_dS * s_K * sm_scale                 (INT8)
 *   dK_j += psi(dS_ij)^T Q^_i * s_dS * s_Q * sm_scale [+ bias branch with Q-smoothing] (INT8)
 * Inputs are the caller's bf16 Q, K, V, O, dO and the LSE of sagebwd_fwd run with the
 * same params; the pre-pass is re-run inside, so the workspace need not survive
 * between the two calls (unless SAGEBWD_FLAG_SHARE_QUANTIZED is set).  dQ, dK, dV
 * (bf16 [B,H,N,d]) are overwritten.
 * The quantised dS tiles are staged in the workspace (Np*(Np+192) bytes per head, at most
 * params->scratch_budget at a time: larger problems are processed in groups of heads) and dQ is
 * formed from them by a second kernel, so all three gradients are deterministic (no atomics).
 * Numerics blocks (params->bq, bkv): psi(P) and psi(dS) take one scale per B_q x B_kv block, over the entries
 * on or below the causal diagonal.  64 x 64 and 64 x 128 run in one sweep; with B_q = 128 the maxima of a block
 * span tiles the kernel reaches in different iterations, so it first sweeps S, dP, P, dS of every second Q block
 * for the maxima alone and then runs in full against them (about 1.3 x the time of the 64 x 64 backward).
 */
int sagebwd_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                const float* LSE, void* dQ, void* dK, void* dV, const sagebwd_params* params,
                void* workspace, size_t workspace_bytes, void* stream);

/* ---- benchmark hooks (not calls of the method; the only process-wide state of the library) ----
 * Per-kernel device timing.  `kernels` is a mask (bit k = sagebwd_kernel k, SAGEBWD_TIMING_ALL = all,
 * 0 = off): every entry point brackets the selected kernels it launches with HIP events on the caller's
 * stream.  An event between two kernels keeps the second from starting until the first has drained
 * (about 10 us on an MI355X), so a benchmark that wants the step undisturbed selects the one kernel it
 * prices.  sagebwd_read_timing waits for the recorded events of `kernel`, returns their summed
 * milliseconds and the launch count since the last read, and resets both.  The mask and the recorded
 * events are shared by all threads of the process (guarded by a mutex); do not enable it under stream
 * capture. */
#define SAGEBWD_TIMING_ALL 31
int sagebwd_set_timing(int kernels);
int sagebwd_read_timing(int kernel /* sagebwd_kernel */, double* total_ms, int* launches);

/* Machine probes (not calls of the method): what this GPU sustains, under the clocks and the power
 * limit the attention kernels run under, on the two resources they are priced against.  Each call
 * launches its kernel once untimed and `reps` (1..1000) times between two events on `stream`, waits
 * for them and returns the mean milliseconds per launch through *ms.  `sink` is a device address of
 * at least 4 bytes that the kernels may or may not write one word to.  Nothing is allocated.
 *
 * sagebwd_probe_mfma: every wave of a grid that fills the GPU (two waves per SIMD) issues
 * `iters` (1..2^20) rounds of four independent accumulator chains of the matrix instruction the
 * attention kernels use, operands in registers; *ops = operations of one launch (2 per multiply-add). */
#define SAGEBWD_PROBE_MFMA_INT8 0 /* 32x32x32 INT8 -> INT32 */
#define SAGEBWD_PROBE_MFMA_BF16 1 /* 32x32x16 bf16 -> FP32  */
#define SAGEBWD_PROBE_MFMA_ZERO_OPERANDS 2 /* OR into kind: all-zero operands instead of random codes (the same
                                             instructions at lower power: what the clock then allows) */
int sagebwd_probe_mfma(int kind, int iters, int reps, void* sink /* device */, void* stream, double* ms /* host */,
                       double* ops /* host */);
/* sagebwd_probe_stream: 16-byte pieces per lane over `bytes` (a multiple of 16) of device memory at
 * `src` (16-byte aligned): copied to `dst` (COPY: `bytes` read and `bytes` written per launch), or
 * read and folded into a word (READ: `dst` is ignored).  Buffers well beyond the 256 MB memory-side
 * cache measure HBM. */
#define SAGEBWD_PROBE_STREAM_COPY 0
#define SAGEBWD_PROBE_STREAM_READ 1
int sagebwd_probe_stream(int kind, const void* src /* device */, void* dst /* device */, size_t bytes, int reps,
                         void* sink /* device */, void* stream, double* ms /* host */);

/* Static description of a status code. */
const char* sagebwd_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* SAGEBWD_H */
