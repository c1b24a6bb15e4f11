"""torch.autograd plumbing around the two calls of the library (no arithmetic of its own).

`sage_attention(Q, K, V, ...)` runs `sagebwd_fwd` and records what `sagebwd_bwd` needs, so that the
INT8 attention can stand where a model calls its attention (paper Sec. 5: SageBwd replaces the
attention of the training run, forward and backward).  Tensors are bf16 CUDA tensors, [B, H, N, d] or,
with `token_major`, [B, N, H, d]; K and V may have another length than Q.
"""
from __future__ import annotations

import torch

from . import binding


class _SageAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, Q, K, V, p, share):
        Q, K, V = Q.contiguous(), K.contiguous(), V.contiguous()
        # with `share` the backward takes psi(Q), psi(K) from this forward's workspace, which then has to
        # live (untouched) until the backward has run; otherwise the forward's workspace ends here
        ws = binding.alloc_workspace(p, Q.device, forward_only=not share)
        O, L = binding.sagebwd_fwd(Q, K, V, p, ws)
        ctx.save_for_backward(Q, K, V, O, L)
        ctx.p, ctx.ws = p, (ws if share else None)
        ctx.mark_non_differentiable(L)
        return O, L

    @staticmethod
    def backward(ctx, dO, _dL):
        Q, K, V, O, L = ctx.saved_tensors
        ws = ctx.ws if ctx.ws is not None else binding.alloc_workspace(ctx.p, Q.device)
        dQ, dK, dV = binding.sagebwd_bwd(Q, K, V, O, dO.contiguous(), L, ctx.p, ws)
        ctx.ws = None
        return dQ, dK, dV, None, None


def sage_attention(Q, K, V, causal: bool = True, k_smooth: bool = True, q_smooth: bool = False, sm_scale: float = 0.0,
                   token_major: bool = False, share_quantized: bool = False, return_lse: bool = False):
    """O (and the log-sum-exp, in the smoothed frame) of INT8 attention, differentiable in Q, K, V.

    share_quantized: keep the forward's workspace until the backward and let it reuse psi(Q), psi(K)
    (Algorithm 2 takes them as inputs); costs that workspace's memory between the two calls."""
    if token_major:
        B, N, H, d = Q.shape
        Nkv = K.shape[1]
    else:
        B, H, N, d = Q.shape
        Nkv = K.shape[2]
    p = binding.SageParams(B, H, N, d, causal=causal, k_smooth=k_smooth, q_smooth=q_smooth, sm_scale=sm_scale,
                           token_major=token_major, share_quantized=share_quantized, Nkv=0 if Nkv == N else Nkv)
    O, L = _SageAttention.apply(Q, K, V, p, share_quantized)
    return (O, L) if return_lse else O
