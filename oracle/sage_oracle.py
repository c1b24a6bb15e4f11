"""Plain NumPy oracle of SageBwd: the INT8 attention forward (Algorithm 1) and
backward (Algorithm 2) of the paper, written in a non-tiled form.

TEST INFRASTRUCTURE ONLY -- never imported by the product package.

The method is an approximation of exact attention (INT8 noise), so the oracle
is the method itself, taken step by step in the paper's notation:

  psi      per-block INT8 quantiser, delta_X = max|X| / 127      (Sec. 3, "Quantization")
  smoothing  K minus its token mean; optional per-block Q mean    (Sec. 3, "Q and K Smoothing")
  forward  S = psi(Q) psi(K)^T, online softmax, per-token psi(P~),
           O = sum_j P^_ij V^_j, L = m + log l                   (Algorithm 1)
  backward D = rowsum(dO o O); P = exp(S - L); dV, dS, dQ, dK with
           per-block psi(P), psi(dO), psi(dS); dP kept unquantised (Algorithm 2, Sec. 3 "SageBwd")

"Non-tiled" means: the running max / running sum of Algorithm 1 are replaced
by the row max and row sum over all visible keys, which is what the online
recurrence evaluates to (only the floating-point order differs).  The pieces
that the paper defines per tile (the quantisers and their scales) are taken
per tile exactly as written.

Precision: the quantisers take their decisions (absmax, scale, round) in
float32, because the stored INT8 tensors and scales are part of the bit-exact
contract; every other quantity is float64.  Inputs are float32 arrays holding
bf16-representable values; outputs O, dQ, dK, dV are rounded to bf16 (returned
as float32 arrays), L is float32.

Readings taken where the paper's text is silent or garbled are listed next to
the code that uses them (R1..R17).

Block sizes: Algorithm 1 takes B_q and B_kv as inputs and fixes neither; every
function takes them as `bq`, `bkv` (default 64 x 64, the configuration the GPU
kernels implement; one must divide the other).  Q, dO and mu_Q are blocked by
bq rows, K and V by bkv rows, psi(P_ij) and psi(dS_ij) act on bq x bkv tiles, and
the forward's per-token psi(P~) on the bkv keys of a tile.

Non-square attention (the paper states the method for Q, K, V of one length N; cross
attention, chunked prefill and decoding against a cache have N_q != N_kv): Q, O, dO, dQ
have N_q rows, K, V, dK, dV have N_kv rows; nothing else changes, every step acts on its
own blocks.  Under the causal mask the last query is aligned with the last key: query i
sees keys k <= i + (N_kv - N_q) (N_kv >= N_q), which is the square mask when the
lengths agree.

Sequence lengths that are not a multiple of the block (the paper assumes N/B_q and
N/B_kv integral, Algorithm 1 line 2): the last block is a partial block whose
missing rows do not exist.  They enter no mean, no absmax, no sum, no softmax.
The code below writes that as "append zero rows AFTER the smoothing, mask the
appended keys, drop the appended query rows", which is the same thing: a zero
row changes no absmax and no integer sum, and a masked key has P = 0.
"""
from __future__ import annotations

import numpy as np

BLOCK = 64  # default B_q = B_kv: the FlashAttention tile that psi's scale is shared over.
# Algorithm 1 (its input line) leaves B_q and B_kv free; every function below takes them as
# `bq` (rows of a Q / dO block) and `bkv` (rows of a K / V block), both defaulting to 64.

_F32 = np.float32
_F64 = np.float64


# --------------------------------------------------------------------------
# small helpers
# --------------------------------------------------------------------------
def round_to_bf16(x) -> np.ndarray:
    """Round float values to the nearest bf16 (ties to even); result as float32."""
    a = np.ascontiguousarray(np.asarray(x, dtype=_F32))
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    r = (u + np.uint64(0x7FFF) + lsb) >> np.uint64(16)
    out = (r << np.uint64(16)).astype(np.uint32).view(_F32)
    nan = np.isnan(a)
    if nan.any():
        out = out.copy()
        out[nan] = np.nan
    return out.reshape(a.shape)


def qk_norm(X, gamma, eps: float = 1e-6) -> np.ndarray:
    """QK-norm of one head (Sec. 4, "Stabilizing Outliers with QK-Norm": RMS normalisation of every
    token of Q and K, with the learned per-channel gain gamma the paper mentions):
        y[n, :] = x[n, :] / sqrt(mean_c x[n, c]^2 + eps) * gamma.
    The model side of the method, here for the pre-pass that fuses it with the quantiser.  Arithmetic:
    the mean of squares in float64 (exact for bf16 inputs), r = 1 / sqrt(mean + eps) in float64 rounded
    once to float32, y = (x *_f32 r) *_f32 gamma, rounded to bf16 -- the tensor a bf16 model would hand
    to the attention.  Returns float32 holding bf16 values."""
    X = np.asarray(X, dtype=_F32)
    g = np.asarray(gamma, dtype=_F32)
    ms = (X.astype(_F64) ** 2).sum(axis=1) / _F64(X.shape[1])
    r = (_F64(1.0) / np.sqrt(ms + _F64(_F32(eps)))).astype(_F32)      # eps is a float32 parameter
    y = ((X * r[:, None]).astype(_F32) * g[None, :]).astype(_F32)
    return round_to_bf16(y)


def key_mean(K: np.ndarray) -> np.ndarray:
    """mu_K = mean_row(K) over ALL N tokens of the head (Sec. 3, smoothing eq.).

    R6/R9: summed in float64 (exact for bf16 data of ordinary dynamic range,
    hence independent of summation order), divided by N, rounded once to f32.
    """
    K = np.asarray(K, dtype=_F32)
    return (K.astype(_F64).sum(axis=0) / _F64(K.shape[0])).astype(_F32)


def block_mean(Q: np.ndarray, block: int = BLOCK) -> np.ndarray:
    """mu_{Q_i} = mean_row(Q_i) for every block of `block` rows (R17: per block, the
    Sec. 3 definition); a partial last block is averaged over the rows it has.
    Returns [ceil(N/block), d] float32 (float64 sum, one rounding)."""
    Q = np.asarray(Q, dtype=_F32)
    n, d = Q.shape
    nb = -(-n // block)
    out = np.zeros((nb, d), dtype=_F32)
    for b in range(nb):
        rows = Q[b * block:(b + 1) * block].astype(_F64)
        out[b] = (rows.sum(axis=0) / _F64(rows.shape[0])).astype(_F32)
    return out


def pad_rows(X: np.ndarray, n_pad: int) -> np.ndarray:
    """X [n, ...] with zero rows appended up to n_pad rows (see the module header)."""
    X = np.asarray(X)
    if X.shape[0] == n_pad:
        return X
    out = np.zeros((n_pad,) + X.shape[1:], dtype=X.dtype)
    out[:X.shape[0]] = X
    return out


def quantize_blocks(X: np.ndarray, block: int = BLOCK):
    """psi applied to every block of `block` rows of X [N, d] (R8: one scale per block of
    `block` rows x all d channels; 64 unless said).

    Sec. 3: X^ = round(X / delta_X), delta_X = max|X| / 127, delta in FP32.
    R5: round = nearest-even; result clamped to [-127, 127].
    R6: all in float32: a = max|x|, s = a / 127, r = 127 / a, q = rne(x * r).
    R7: an all-zero block has s = 0 and q = 0.
    Returns (q int8 [N, d], s float32 [N/block]).
    """
    X = np.ascontiguousarray(np.asarray(X, dtype=_F32))
    n, d = X.shape
    assert n % block == 0
    xb = X.reshape(n // block, block * d)
    a = np.abs(xb).max(axis=1).astype(_F32)
    nz = a > 0
    safe = np.where(nz, a, _F32(1))
    s = np.where(nz, a / _F32(127.0), _F32(0)).astype(_F32)
    r = np.where(nz, _F32(127.0) / safe, _F32(0)).astype(_F32)
    y = (xb * r[:, None]).astype(_F32)          # one f32 rounding of the product
    q = np.clip(np.rint(y), -127, 127).astype(np.int8)
    return q.reshape(n, d), s


def _quantize_tile_f32(x64: np.ndarray):
    """psi on ONE tile whose values are float64 intermediates (P_ij or dS_ij,
    Algorithm 2): the decision is taken in float32 like every other quantiser.
    Returns (q as float64 integers, scale float32); a zero tile gives (0, 0)."""
    x = x64.astype(_F32)
    a = np.abs(x).max() if x.size else _F32(0)
    a = _F32(a)
    if not a > 0:
        return np.zeros(x.shape, dtype=_F64), _F32(0)
    r = _F32(127.0) / a
    q = np.clip(np.rint((x * r).astype(_F32)), -127, 127)
    return q.astype(_F64), _F32(a / _F32(127.0))


# --------------------------------------------------------------------------
# pre-pass: smoothing + psi for Q, K, V (and dO in the backward)
# --------------------------------------------------------------------------
def _check_blocks(bq: int, bkv: int):
    assert bq >= 1 and bkv >= 1 and max(bq, bkv) % min(bq, bkv) == 0, "one block size must divide the other"


def padded_len(n: int, bq: int = BLOCK, bkv: int = BLOCK) -> int:
    """Rows after appending: n rounded up to a multiple of both block sizes."""
    big = max(bq, bkv)
    return -(-n // big) * big


def prepass_head(Q, K, V, k_smooth: bool = True, q_smooth: bool = False, bq: int = BLOCK, bkv: int = BLOCK):
    """Smoothing and per-block quantisation of one head (Algorithm 1, the
    "Quantization" step, preceded by the smoothing of Sec. 3).  Q is quantised per
    block of bq rows, K and V per block of bkv rows.

    Returns a dict with Qh, sQ, Kh, sK, Vh, sV (int8 / float32), muK [d],
    muQ [rows/bq, d] (zeros when the smoothing is off) and Ksm (float32 K - mu_K).
    When N is not a multiple of the blocks the row-indexed entries have N rounded up
    to a multiple of both, the appended rows zero (module header); "n", "nk" are the true
    N_q and N_kv (K and V may have another length than Q).
    """
    _check_blocks(bq, bkv)
    Q = np.asarray(Q, dtype=_F32)
    K = np.asarray(K, dtype=_F32)
    V = np.asarray(V, dtype=_F32)
    n, d = Q.shape
    nk = K.shape[0]
    assert V.shape[0] == nk
    n_pad, nk_pad = padded_len(n, bq, bkv), padded_len(nk, bq, bkv)
    muK = key_mean(K) if k_smooth else np.zeros(d, dtype=_F32)   # over the N_kv tokens that exist
    Ksm = (K - muK[None, :]).astype(_F32)       # f32 subtraction, R6
    if q_smooth:
        muQ = pad_rows(block_mean(Q, bq), n_pad // bq)           # blocks with no row at all: mean 0
        Qsm = (Q - np.repeat(muQ, bq, axis=0)[:n]).astype(_F32)
    else:
        muQ = np.zeros((n_pad // bq, d), dtype=_F32)
        Qsm = Q
    Qsm = pad_rows(Qsm, n_pad)
    Ksm, Vp = (pad_rows(x, nk_pad) for x in (Ksm, V))
    Qh, sQ = quantize_blocks(Qsm, bq)
    Kh, sK = quantize_blocks(Ksm, bkv)
    Vh, sV = quantize_blocks(Vp, bkv)
    return dict(Qh=Qh, sQ=sQ, Kh=Kh, sK=sK, Vh=Vh, sV=sV, muK=muK, muQ=muQ, Ksm=Ksm, n=n, nk=nk, bq=bq, bkv=bkv)


def delta_rows(dO, O) -> np.ndarray:
    """delta = rowsum(dO o O) (Sec. 3 "SageBwd"; "D" in Algorithm 2), float64
    from the bf16 values the caller holds (R16), returned as float64 [N]."""
    return (np.asarray(dO, dtype=_F64) * np.asarray(O, dtype=_F64)).sum(axis=1)


def _logits_block(pp, i0: int, n_keys: int, sm_scale: float, q_smooth: bool, key_idx=None) -> np.ndarray:
    """S for the bq queries starting at i0 against keys [0, n_keys) (or against the
    keys listed in key_idx, a sampling aid that changes no value):
    S = (Q^ K^^T) * s_Q * s_K * sm_scale (Algorithm 1, the S_ij line; R1: the
    1/sqrt(d) of Sec. 4 is applied in the dequantisation factor) plus the
    Q-smoothing bias mu_Qi K^sm^T when that smoothing is on (Sec. 3 decomposition;
    the mu_K terms are row constants and are dropped, so S lives in the smoothed
    frame, R10)."""
    bq, bkv = pp["bq"], pp["bkv"]
    I = i0 // bq
    sel = slice(0, n_keys) if key_idx is None else key_idx
    qi = pp["Qh"][i0:i0 + bq].astype(_F64)
    kj = pp["Kh"][sel].astype(_F64)
    acc = qi @ kj.T                                           # exact integers
    sk_per_key = np.repeat(pp["sK"].astype(_F64), bkv)[sel]
    S = acc * (_F64(pp["sQ"][I]) * _F64(sm_scale)) * sk_per_key[None, :]
    if q_smooth:
        bias = pp["Ksm"][sel].astype(_F64) @ pp["muQ"][I].astype(_F64)
        S = S + _F64(sm_scale) * bias[None, :]
    return S


def _visible_keys(i0: int, nk: int, causal: bool, bq: int, bkv: int, shift: int = 0) -> int:
    """Keys [0, n_keys) that the Q block starting at i0 works on: all nk without the mask; under the
    causal mask (R13; query i sees keys k <= i + shift, shift = N_kv - N_q) the KV blocks that hold a
    visible key for some row of the block (whole KV blocks, since psi's scales are per block; fully
    masked blocks are skipped)."""
    if not causal:
        return nk
    return min(nk, -(-(i0 + bq + shift) // bkv) * bkv)


# --------------------------------------------------------------------------
# forward (Algorithm 1)
# --------------------------------------------------------------------------
def forward_head(Q, K, V, causal: bool = True, k_smooth: bool = True, q_smooth: bool = False,
                 sm_scale: float | None = None, return_raw: bool = False, q_blocks=None,
                 bq: int = BLOCK, bkv: int = BLOCK):
    """INT8 attention forward of one head.  Q: [N_q, d], K, V: [N_kv, d] float32 (bf16 values).

    Returns (O [N, d] bf16-rounded float32, L [N] float32); with return_raw the
    unrounded float64 O and L come too.  `q_blocks` (iterable of bq-row block
    indices) restricts the work to those query blocks -- rows are independent --
    and leaves the other rows zero (sampling for large N).
    """
    Q = np.asarray(Q, dtype=_F32)
    n_true, d = Q.shape
    nk_true = np.asarray(K).shape[0]
    n, nk = padded_len(n_true, bq, bkv), padded_len(nk_true, bq, bkv)   # rows after appending (module header)
    shift = nk_true - n_true                          # causal: query i sees keys k <= i + shift
    assert not causal or shift >= 0, "causal attention needs N_kv >= N_q"
    if sm_scale is None:
        sm_scale = 1.0 / np.sqrt(d)
    pp = prepass_head(Q, K, V, k_smooth, q_smooth, bq, bkv)
    Vh = pp["Vh"].astype(_F64).reshape(nk // bkv, bkv, d)
    sV = pp["sV"].astype(_F64)
    O = np.zeros((n, d), dtype=_F64)
    L = np.zeros(n, dtype=_F64)
    rows = np.arange(bq)
    todo = range(n // bq) if q_blocks is None else sorted(set(int(b) for b in q_blocks))
    for i0 in (bq * b for b in todo):
        n_keys = _visible_keys(i0, nk, causal, bq, bkv, shift)    # R13: keys k <= i + shift only
        tj = n_keys // bkv
        S = _logits_block(pp, i0, n_keys, sm_scale, q_smooth)
        kk = np.arange(n_keys)
        if causal:
            S = np.where(kk[None, :] > (i0 + rows + shift)[:, None], -np.inf, S)
        S = np.where(kk[None, :] >= nk_true, -np.inf, S)          # keys that do not exist
        # softmax statistics over the whole row: what m_{i,Tn}, l_{i,Tn} evaluate to (R2, R3)
        m = S.max(axis=1)
        m = np.where(np.isfinite(m), m, 0.0)          # (appended query rows past a short K see no key: dropped below)
        l = np.exp(S - m[:, None]).sum(axis=1)        # unquantised P~ feeds l
        l = np.where(l > 0, l, 1.0)
        L[i0:i0 + bq] = m + np.log(l)
        # per KV block j: per-token quantisation of P~ (the s_P line of Algorithm 1).
        # R12: P~/s_P = exp(S - m) * 127 / exp(rowmax(S_ij) - m) = 127 exp(S - rowmax(S_ij)),
        # rounded to nearest; the value is decided in float32.  (A row whose keys in block j are
        # all masked has rowmax = -inf: its codes and its weight are zero.)
        St = S.reshape(bq, tj, bkv)
        Mloc = St.max(axis=2)                         # rowmax(S_ij), [bq, tj]
        Msafe = np.where(np.isfinite(Mloc), Mloc, 0.0)
        e = np.exp(St - Msafe[:, :, None]).astype(_F32)
        Ph = np.rint((e * _F32(127.0)).astype(_F32)).astype(_F64)      # integers 0..127
        w = np.where(np.isfinite(Mloc), np.exp(Msafe - m[:, None]), 0.0) / 127.0   # s_P relative to the final max
        PV = np.einsum("qjk,jkc->qjc", Ph, Vh[:tj])   # exact integers
        acc = np.einsum("qj,qjc->qc", w * sV[None, :tj], PV)
        O[i0:i0 + bq] = acc / l[:, None]              # R4: O_i = diag(l)^-1 O_i
    O, L = O[:n_true], L[:n_true]                     # query rows that do not exist are dropped
    Ob = round_to_bf16(O)
    Lf = L.astype(_F32)
    if return_raw:
        return Ob, Lf, O, L
    return Ob, Lf


# --------------------------------------------------------------------------
# backward (Algorithm 2)
# --------------------------------------------------------------------------
def backward_head(Q, K, V, O, dO, L, causal: bool = True, k_smooth: bool = True,
                  q_smooth: bool = False, sm_scale: float | None = None,
                  return_raw: bool = False, intermediates: dict | None = None,
                  q_blocks=None, kv_blocks=None, bq: int = BLOCK, bkv: int = BLOCK):
    """INT8 attention backward of one head.

    Inputs as the caller holds them: Q, O, dO [N_q, d], K, V [N_kv, d] (bf16 values as
    float32) and L [N_q] float32 from the forward.  Returns bf16-rounded
    (dQ [N_q, d], dK, dV [N_kv, d]); with return_raw the float64 values instead.

    If `intermediates` is a dict it receives the unquantised float64 P, dP, dS
    of the whole head, the codes psi(dS) ("dSh", integers as float64) and their
    tile scales ("sdS", [N/bq, N/bkv] float32) (tiny inputs only; used by the
    invariant tests and by the GPU check of the in-loop quantiser).

    Sampling for large N (tiles are independent given L and delta):
    `q_blocks` keeps only those Q blocks (of bq rows) -- the rows of dQ that belong to them
    are then complete, dK and dV are partial; `kv_blocks` keeps only those KV blocks (of bkv
    rows) -- the rows of dK and dV that belong to them are complete, dQ is partial.
    """
    Q = np.asarray(Q, dtype=_F32)
    n_true, d = Q.shape
    nk_true = np.asarray(K).shape[0]
    n, nk = padded_len(n_true, bq, bkv), padded_len(nk_true, bq, bkv)   # rows after appending (module header)
    shift = nk_true - n_true                                  # causal: query i sees keys k <= i + shift
    assert not causal or shift >= 0, "causal attention needs N_kv >= N_q"
    if sm_scale is None:
        sm_scale = 1.0 / np.sqrt(d)
    pp = prepass_head(Q, K, V, k_smooth, q_smooth, bq, bkv)   # same blocks and scales as forward
    dO = pad_rows(np.asarray(dO, dtype=_F32), n)
    O = pad_rows(np.asarray(O, dtype=_F32), n)
    V = pad_rows(np.asarray(V, dtype=_F32), nk)
    L = pad_rows(np.asarray(L, dtype=_F32), n)
    dOh, sdO = quantize_blocks(dO, bq)                        # psi(dO_i), per block of bq rows
    delta = delta_rows(dO, O)
    V64 = np.asarray(V, dtype=_F64)
    dO64 = np.asarray(dO, dtype=_F64)
    L64 = np.asarray(L, dtype=_F64)
    Kh = pp["Kh"].astype(_F64)
    Qh = pp["Qh"].astype(_F64)
    dQ = np.zeros((n, d), dtype=_F64)
    dK = np.zeros((nk, d), dtype=_F64)
    dV = np.zeros((nk, d), dtype=_F64)
    if intermediates is not None:
        intermediates["P"] = np.zeros((n, nk))
        intermediates["dP"] = np.zeros((n, nk))
        intermediates["dS"] = np.zeros((n, nk))
        intermediates["dSh"] = np.zeros((n, nk))
        intermediates["sdS"] = np.zeros((n // bq, nk // bkv), dtype=_F32)
    rows = np.arange(bq)
    q_todo = range(n // bq) if q_blocks is None else sorted(set(int(b) for b in q_blocks))
    kv_keep = None if kv_blocks is None else set(int(b) for b in kv_blocks)
    for i0 in (bq * b for b in q_todo):
        I = i0 // bq
        n_keys = _visible_keys(i0, nk, causal, bq, bkv, shift)
        blocks = [J for J in range(n_keys // bkv) if kv_keep is None or J in kv_keep]
        if not blocks:
            continue
        # the key columns this row block works on (all visible keys unless KV blocks are sampled)
        kk = np.concatenate([np.arange(bkv * J, bkv * J + bkv) for J in blocks])
        S = _logits_block(pp, i0, n_keys, sm_scale, q_smooth, None if kv_keep is None else kk)
        P = np.exp(S - L64[i0:i0 + bq, None])                 # P_ij = exp(S_ij - L_i)
        if causal:
            P = np.where(kk[None, :] > (i0 + rows + shift)[:, None], 0.0, P)   # R13: masked entries are 0
        # keys and query rows that do not exist
        P = np.where((kk[None, :] >= nk_true) | ((i0 + rows)[:, None] >= n_true), 0.0, P)
        dP = dO64[i0:i0 + bq] @ V64[kk].T                     # unquantised matmul (R15)
        dS = P * (dP - delta[i0:i0 + bq, None])
        if intermediates is not None:
            intermediates["P"][i0:i0 + bq, kk] = P
            intermediates["dP"][i0:i0 + bq, kk] = dP
            intermediates["dS"][i0:i0 + bq, kk] = dS
        dOh_i = dOh[i0:i0 + bq].astype(_F64)
        Qh_i = Qh[i0:i0 + bq]
        for t, J in enumerate(blocks):
            j0 = J * bkv
            c0 = t * bkv                                      # column offset of block J inside S, P, dS
            # dV_j += psi(P_ij)^T psi(dO_i) * s_P * s_dO   (R14: dynamic per-tile scale)
            Ph, sP = _quantize_tile_f32(P[:, c0:c0 + bkv])
            dV[j0:j0 + bkv] += (_F64(sP) * _F64(sdO[I])) * (Ph.T @ dOh_i)
            # psi(dS_ij); dQ_i += dS^ K^_j * s_dS * s_K ; dK_j += dS^^T Q^_i * s_dS * s_Q
            dSh, sdS = _quantize_tile_f32(dS[:, c0:c0 + bkv])
            if intermediates is not None:
                intermediates["dSh"][i0:i0 + bq, j0:j0 + bkv] = dSh
                intermediates["sdS"][I, J] = sdS
            dQ[i0:i0 + bq] += (_F64(sm_scale) * _F64(sdS) * _F64(pp["sK"][J])) * (dSh @ Kh[j0:j0 + bkv])
            dK[j0:j0 + bkv] += (_F64(sm_scale) * _F64(sdS) * _F64(pp["sQ"][I])) * (dSh.T @ Qh_i)
            if q_smooth:
                # dK_bias = (dS^T 1) mu_Q^T (ablation section); R17: from the unquantised dS
                colsum = dS[:, c0:c0 + bkv].sum(axis=0)
                dK[j0:j0 + bkv] += _F64(sm_scale) * colsum[:, None] * pp["muQ"][I].astype(_F64)[None, :]
    dQ, dK, dV = dQ[:n_true], dK[:nk_true], dV[:nk_true]
    if return_raw:
        return dQ, dK, dV
    return round_to_bf16(dQ), round_to_bf16(dK), round_to_bf16(dV)


# --------------------------------------------------------------------------
# batched wrappers: [B, H, N, d]
# --------------------------------------------------------------------------
def forward(Q, K, V, causal=True, k_smooth=True, q_smooth=False, sm_scale=None):
    Q = np.asarray(Q, dtype=_F32)
    B, H, N, d = Q.shape
    O = np.zeros((B, H, N, d), dtype=_F32)
    L = np.zeros((B, H, N), dtype=_F32)
    for b in range(B):
        for h in range(H):
            O[b, h], L[b, h] = forward_head(Q[b, h], K[b, h], V[b, h], causal, k_smooth, q_smooth, sm_scale)
    return O, L


def backward(Q, K, V, O, dO, L, causal=True, k_smooth=True, q_smooth=False, sm_scale=None):
    Q = np.asarray(Q, dtype=_F32)
    B, H, N, d = Q.shape
    dQ = np.zeros((B, H, N, d), dtype=_F32)
    dK = np.zeros_like(dQ)
    dV = np.zeros_like(dQ)
    for b in range(B):
        for h in range(H):
            dQ[b, h], dK[b, h], dV[b, h] = backward_head(
                Q[b, h], K[b, h], V[b, h], O[b, h], dO[b, h], L[b, h], causal, k_smooth, q_smooth, sm_scale)
    return dQ, dK, dV
