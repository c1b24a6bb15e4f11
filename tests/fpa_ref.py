"""Textbook full-precision attention (FPA) in float64 and error metrics.

Test-side helper: the definition O = softmax(S) V, S = sm_scale * Q K^T of the
paper's preliminaries and the gradient formulas of its "SageBwd" paragraph,
written out with no quantisation.  It is what the oracle approximates.
"""
import numpy as np


def fpa_forward(Q, K, V, causal, sm_scale):
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    S = (Q @ K.T) * sm_scale
    n, nk = S.shape
    if causal:
        # the last query is aligned with the last key (the square mask when the lengths agree)
        S = np.where(np.arange(nk)[None, :] > (np.arange(n) + (nk - n))[:, None], -np.inf, S)
    m = S.max(axis=1, keepdims=True)
    E = np.exp(S - m)
    l = E.sum(axis=1, keepdims=True)
    P = E / l
    return P @ V, (m + np.log(l))[:, 0], P


def fpa_backward(Q, K, V, dO, causal, sm_scale):
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    dO = np.asarray(dO, dtype=np.float64)
    O, lse, P = fpa_forward(Q, K, V, causal, sm_scale)
    dV = P.T @ dO
    dP = dO @ V.T
    delta = (dO * O).sum(axis=1, keepdims=True)
    dS = P * (dP - delta)
    dQ = dS @ K * sm_scale
    dK = dS.T @ Q * sm_scale
    return dict(O=O, L=lse, P=P, dP=dP, dS=dS, dQ=dQ, dK=dK, dV=dV, delta=delta[:, 0])


def cos_sim(a, b):
    a = np.asarray(a, dtype=np.float64).ravel()
    b = np.asarray(b, dtype=np.float64).ravel()
    return float(a @ b / (np.linalg.norm(a) * np.linalg.norm(b)))


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64).ravel()
    b = np.asarray(b, dtype=np.float64).ravel()
    return float(np.linalg.norm(a - b) / np.linalg.norm(b))


def rel_l1(a, b):
    a = np.asarray(a, dtype=np.float64).ravel()
    b = np.asarray(b, dtype=np.float64).ravel()
    return float(np.abs(a - b).sum() / np.abs(b).sum())
