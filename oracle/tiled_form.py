"""Second formulation of the oracle: the method as a streaming (tiled) computation with
the online softmax of Algorithm 1 and the KV-outer loop nest of Algorithm 2, in float64.

TEST INFRASTRUCTURE ONLY.  It exists so that the non-tiled oracle can be checked against a
formulation that was written separately: nothing is imported from sage_oracle.  The
smoothing, the quantiser psi, delta and both passes are written out again here, in a
different style (scalar float32 decisions per block, math.fsum for the means, one running
state per Q block), so a mistake in either file shows up as a disagreement.

Readings shared with the non-tiled oracle (they are readings of the paper, not code):
the running max starts at -inf with one entry per query row and the running sum at 0; the
running sum and the output accumulator are both rescaled by exp(m_old - m_new) when the
max moves; the logits carry sm_scale in the dequantisation factor; the causal mask is
applied to the dequantised logits; psi rounds to nearest-even in float32 with r = 127 / a.
N_q must be a multiple of B_q and N_kv of B_kv here (small test inputs only); the two may differ
(the causal mask then aligns the last query with the last key).
"""
from __future__ import annotations

import math

import numpy as np

f32 = np.float32


def _token_mean(X):
    """Column means over all rows: exact sum (math.fsum), one division, one rounding to float32."""
    n = X.shape[0]
    return np.array([f32(math.fsum(float(v) for v in X[:, c]) / n) for c in range(X.shape[1])], dtype=f32)


def _psi(block_rows):
    """The INT8 quantiser on one block (Sec. 3 "Quantization"): codes as float64 integers and
    the float32 scale delta = max|x| / 127.  Decisions in float32."""
    x = np.asarray(block_rows, dtype=f32)
    amax = f32(max(float(x.max()), -float(x.min())))
    if not amax > 0:
        return np.zeros(x.shape), f32(0)
    inv = f32(127.0) / amax
    codes = np.rint(x * inv)                      # float32 array times float32 scalar: one rounding
    codes = np.minimum(np.maximum(codes, -127), 127)
    return codes.astype(np.float64), f32(amax / f32(127.0))


def _quantise_rows(X, block):
    parts = [_psi(X[r0:r0 + block]) for r0 in range(0, X.shape[0], block)]
    return [p[0] for p in parts], [p[1] for p in parts]


class _Prepared:
    """Smoothed and quantised operands of one head, block by block."""

    def __init__(self, Q, K, V, k_smooth, q_smooth, bq, bkv):
        Q, K, V = (np.asarray(x, dtype=f32) for x in (Q, K, V))
        n, d = Q.shape
        nk = K.shape[0]
        assert n % bq == 0 and nk % bkv == 0 and V.shape[0] == nk
        self.n, self.nk, self.d, self.bq, self.bkv = n, nk, d, bq, bkv
        self.mu_k = _token_mean(K) if k_smooth else np.zeros(d, dtype=f32)
        self.k_sm = K - self.mu_k                 # float32 - float32
        self.mu_q = []
        q_in = Q.copy()
        for r0 in range(0, n, bq):
            mu = _token_mean(Q[r0:r0 + bq]) if q_smooth else np.zeros(d, dtype=f32)
            self.mu_q.append(mu)
            q_in[r0:r0 + bq] = Q[r0:r0 + bq] - mu
        self.q_codes, self.q_scale = _quantise_rows(q_in, bq)
        self.k_codes, self.k_scale = _quantise_rows(self.k_sm, bkv)
        self.v_codes, self.v_scale = _quantise_rows(V, bkv)
        self.q_smooth = q_smooth

    def logits(self, i, j, sm_scale):
        """Dequantised S_ij (+ the mu_Qi K_sm_j^T term with Q-smoothing), float64 [bq, bkv]."""
        s = (self.q_codes[i] @ self.k_codes[j].T) * (float(self.q_scale[i]) * float(self.k_scale[j]) * sm_scale)
        if self.q_smooth:
            kj = self.k_sm[j * self.bkv:(j + 1) * self.bkv].astype(np.float64)
            s = s + sm_scale * (kj @ self.mu_q[i].astype(np.float64))[None, :]
        return s

    def masked(self, i, j):
        """Boolean [bq, bkv]: key index > query index + (N_kv - N_q) (last query on last key)."""
        qi = i * self.bq + np.arange(self.bq) + (self.nk - self.n)
        kj = j * self.bkv + np.arange(self.bkv)
        return kj[None, :] > qi[:, None]

    def all_masked(self, i, j):
        return j * self.bkv > i * self.bq + self.bq - 1 + (self.nk - self.n)


def forward_tiled(Q, K, V, causal=True, k_smooth=True, q_smooth=False, sm_scale=None, bq=64, bkv=64):
    """Forward with the online softmax: per Q block a running (max, sum, output) state that
    every visible KV block updates in turn.  Returns float64 (O, L) before output rounding."""
    pre = _Prepared(Q, K, V, k_smooth, q_smooth, bq, bkv)
    n, d = pre.n, pre.d
    sm_scale = 1.0 / math.sqrt(d) if sm_scale is None else sm_scale
    O = np.zeros((n, d))
    L = np.zeros(n)
    for i in range(n // bq):
        run_max = np.full(bq, -np.inf)
        run_sum = np.zeros(bq)
        out = np.zeros((bq, d))
        for j in range(pre.nk // bkv):
            if causal and pre.all_masked(i, j):
                break                                           # every key of this block is masked
            s = pre.logits(i, j, sm_scale)
            if causal:
                s = np.where(pre.masked(i, j), -np.inf, s)
            tile_max = s.max(axis=1)
            new_max = np.maximum(run_max, tile_max)
            live = np.isfinite(new_max)                         # rows that have seen a key so far
            ref = np.where(live, new_max, 0.0)
            p_tilde = np.exp(s - ref[:, None])
            shrink = np.where(live, np.exp(run_max - ref), 1.0)
            run_sum = shrink * run_sum + p_tilde.sum(axis=1)
            # per-token scale of P~: exp(rowmax(S_ij) - m_ij) / 127; a row with no key in this
            # block contributes nothing
            tok = np.where(np.isfinite(tile_max), np.exp(tile_max - ref), 0.0) / 127.0
            safe = np.where(tok > 0, tok, 1.0)
            p_codes = np.rint((p_tilde / safe[:, None]).astype(f32)).astype(np.float64)
            p_codes = np.where((tok > 0)[:, None], p_codes, 0.0)
            out = shrink[:, None] * out + (p_codes @ pre.v_codes[j]) * (tok * float(pre.v_scale[j]))[:, None]
            run_max = new_max
        O[i * bq:(i + 1) * bq] = out / run_sum[:, None]
        L[i * bq:(i + 1) * bq] = run_max + np.log(run_sum)
    return O, L


def backward_tiled(Q, K, V, O, dO, L, causal=True, k_smooth=True, q_smooth=False, sm_scale=None, bq=64, bkv=64):
    """Backward with the KV blocks outermost: each KV block owns its dK, dV rows and walks the
    Q blocks, adding its share to their dQ rows.  float64 outputs before rounding."""
    pre = _Prepared(Q, K, V, k_smooth, q_smooth, bq, bkv)
    n, d = pre.n, pre.d
    sm_scale = 1.0 / math.sqrt(d) if sm_scale is None else sm_scale
    dO = np.asarray(dO, dtype=f32)
    do_codes, do_scale = _quantise_rows(dO, bq)
    big_d = np.array([math.fsum(float(a) * float(b) for a, b in zip(dO[r], np.asarray(O, dtype=f32)[r])) for r in range(n)])
    lse = np.asarray(L, dtype=f32).astype(np.float64)
    v64 = np.asarray(V, dtype=f32).astype(np.float64)
    do64 = dO.astype(np.float64)
    dQ = np.zeros((n, d))
    dK = np.zeros((pre.nk, d))
    dV = np.zeros((pre.nk, d))
    for j in range(pre.nk // bkv):
        ks = slice(j * bkv, (j + 1) * bkv)
        for i in range(n // bq):
            if causal and pre.all_masked(i, j):
                continue
            qs = slice(i * bq, (i + 1) * bq)
            p = np.exp(pre.logits(i, j, sm_scale) - lse[qs, None])
            if causal:
                p = np.where(pre.masked(i, j), 0.0, p)
            p_codes, p_scale = _psi(p)
            dV[ks] += (p_codes.T @ do_codes[i]) * (float(p_scale) * float(do_scale[i]))
            dp = do64[qs] @ v64[ks].T
            ds = p * (dp - big_d[qs, None])
            ds_codes, ds_scale = _psi(ds)
            dQ[qs] += (ds_codes @ pre.k_codes[j]) * (float(ds_scale) * float(pre.k_scale[j]) * sm_scale)
            dK[ks] += (ds_codes.T @ pre.q_codes[i]) * (float(ds_scale) * float(pre.q_scale[i]) * sm_scale)
            if q_smooth:
                dK[ks] += sm_scale * np.outer(ds.sum(axis=0), pre.mu_q[i].astype(np.float64))
    return dQ, dK, dV
