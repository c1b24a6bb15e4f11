"""Second, independent formulation of the oracle: Algorithms 1 and 2 of the
paper taken in their own loop order (tile by tile, online softmax), in float64.

TEST INFRASTRUCTURE ONLY.  Used to cross-check the non-tiled oracle on small
inputs: two formulations written separately must agree.

Typos of the printed listings are repaired as follows (the non-tiled oracle is
insensitive to all three):
  R2  m starts at -inf and has one entry per query row (B_q), l starts at 0;
  R3  l_ij = exp(m_{i,j-1} - m_ij) * l_{i,j-1} + rowsum(P~_ij);
  R4  O_ij = diag(exp(m_{i,j-1} - m_ij)) O_{i,j-1} + ...  (no inverse).
The softmax scale (R1) and the causal mask (R13) enter as in the oracle.
Only K-smoothing is supported here (no Q-smoothing bias).
"""
from __future__ import annotations

import numpy as np

from .sage_oracle import BLOCK, prepass_head, quantize_blocks, delta_rows


def _psi_tile(x):
    a = np.float32(np.abs(x.astype(np.float32)).max())
    if not a > 0:
        return np.zeros_like(x, dtype=np.float64), np.float32(0)
    r = np.float32(127.0) / a
    q = np.clip(np.rint((x.astype(np.float32) * r).astype(np.float32)), -127, 127).astype(np.float64)
    return q, np.float32(a / np.float32(127.0))


def forward_tiled(Q, K, V, causal=True, k_smooth=True, sm_scale=None):
    """Algorithm 1, loop for loop.  Returns float64 (O, L) before output rounding."""
    n, d = Q.shape
    if sm_scale is None:
        sm_scale = 1.0 / np.sqrt(d)
    pp = prepass_head(Q, K, V, k_smooth, False)
    T = n // BLOCK
    O = np.zeros((n, d))
    L = np.zeros(n)
    for i in range(T):
        qi = pp["Qh"][i * BLOCK:(i + 1) * BLOCK].astype(np.float64)
        o = np.zeros((BLOCK, d))
        l = np.zeros(BLOCK)
        m = np.full(BLOCK, -np.inf)
        for j in range(T):
            if causal and j > i:
                continue
            kj = pp["Kh"][j * BLOCK:(j + 1) * BLOCK].astype(np.float64)
            vj = pp["Vh"][j * BLOCK:(j + 1) * BLOCK].astype(np.float64)
            S = (qi @ kj.T) * float(pp["sQ"][i]) * float(pp["sK"][j]) * sm_scale
            if causal and j == i:
                r = np.arange(BLOCK)
                S = np.where(r[None, :] > r[:, None], -np.inf, S)
            rowmax = S.max(axis=1)
            m_new = np.maximum(m, rowmax)
            Pt = np.exp(S - m_new[:, None])
            alpha = np.exp(m - m_new)
            l = alpha * l + Pt.sum(axis=1)
            sP = np.exp(rowmax - m_new) / 127.0
            Ph = np.rint((Pt / sP[:, None]).astype(np.float32)).astype(np.float64)
            o = alpha[:, None] * o + (Ph @ vj) * sP[:, None] * float(pp["sV"][j])
            m = m_new
        O[i * BLOCK:(i + 1) * BLOCK] = o / l[:, None]
        L[i * BLOCK:(i + 1) * BLOCK] = m + np.log(l)
    return O, L


def backward_tiled(Q, K, V, O, dO, L, causal=True, k_smooth=True, sm_scale=None):
    """Algorithm 2, loop for loop (outer loop over KV blocks).  float64 outputs."""
    n, d = Q.shape
    if sm_scale is None:
        sm_scale = 1.0 / np.sqrt(d)
    pp = prepass_head(Q, K, V, k_smooth, False)
    dOh, sdO = quantize_blocks(dO)
    D = delta_rows(dO, O)
    T = n // BLOCK
    dQ = np.zeros((n, d))
    dK = np.zeros((n, d))
    dV = np.zeros((n, d))
    V64 = V.astype(np.float64)
    dO64 = dO.astype(np.float64)
    for j in range(T):
        js = slice(j * BLOCK, (j + 1) * BLOCK)
        kj = pp["Kh"][js].astype(np.float64)
        for i in range(T):
            if causal and i < j:
                continue
            isl = slice(i * BLOCK, (i + 1) * BLOCK)
            qi = pp["Qh"][isl].astype(np.float64)
            S = (qi @ kj.T) * float(pp["sQ"][i]) * float(pp["sK"][j]) * sm_scale
            P = np.exp(S - L[isl].astype(np.float64)[:, None])
            if causal and i == j:
                r = np.arange(BLOCK)
                P = np.where(r[None, :] > r[:, None], 0.0, P)
            Ph, sP = _psi_tile(P)
            dV[js] += (Ph.T @ dOh[isl].astype(np.float64)) * float(sP) * float(sdO[i])
            dP = dO64[isl] @ V64[js].T
            dS = P * (dP - D[isl][:, None])
            dSh, sdS = _psi_tile(dS)
            dQ[isl] += (dSh @ kj) * float(sdS) * float(pp["sK"][j]) * sm_scale
            dK[js] += (dSh.T @ qi) * float(sdS) * float(pp["sQ"][i]) * sm_scale
    return dQ, dK, dV
