"""Seeded sweep over combinations of the options of the two calls, each compared with the CPU oracle.

The other GPU tests cover each option on shapes chosen for it; this one draws whole configurations at random
(batch, heads, N_q, N_kv, head dimension, mask, the two smoothings, layout, fused QK-norm, sharing of the
quantised operands, a small dS scratch budget, a custom scale, numerics blocks of 64 or 128), so that options meet in combinations nobody
wrote down: e.g. token-major tensors with a partial last block, Q-smoothing, a shifted diagonal and heads
processed in groups.  The forward is compared with the oracle's forward; the backward is fed the oracle's O and L
(as in the backward tests) and compared with the oracle's backward, head by head."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_02170_amd import binding, synth
from gpu_common import check_close, check_lse, to_np

pytestmark = pytest.mark.gpu

# Regression guards of this sweep (whole-tensor relative L1, about five times the worst measured on the MI355X:
# O 4.7e-4, dQ 2.7e-4, dK 2.3e-4, dV 3.6e-5).  dQ and dK sit further from the oracle here than in the other tests (their
# guards are 2e-4 and 1.5e-4): with channel offsets of twice sigma = 4 under Q-smoothing the logit bias reaches tens of units, the
# kernels hold it in FP32 where the oracle has FP64, and more psi(dS) codes land on the other side of a rounding step.
SWEEP_GUARD = {"O": 2.5e-3, "dQ": 1.4e-3, "dK": 1.1e-3, "dV": 1.8e-4}


def _check(name, got, ref):
    l1, _ = check_close(name, got, ref, guard=False)
    kind = name.split("[")[0]
    assert l1 <= SWEEP_GUARD[kind], f"{name}: rel-L1 {l1:.3e} above the regression guard {SWEEP_GUARD[kind]:.1e}"


def _draw(rng):
    d = int(rng.choice([64, 128]))
    B, H = int(rng.integers(1, 3)), int(rng.integers(1, 4))
    N = int(rng.choice([int(rng.integers(1, 64)), int(rng.integers(64, 200)), 64 * int(rng.integers(1, 5))]))
    causal = bool(rng.integers(0, 2))
    kind = int(rng.integers(0, 3))          # square, more keys than queries, any two lengths
    if kind == 0:
        Nkv = 0
    elif causal or kind == 1:
        Nkv = N + 64 * int(rng.integers(1, 4))      # under the mask the extra keys come in whole blocks
    else:
        Nkv = int(rng.integers(1, 300))
    cfg = dict(B=B, H=H, N=N, d=d, causal=causal, Nkv=Nkv,
               k_smooth=bool(rng.integers(0, 4) > 0), q_smooth=bool(rng.integers(0, 3) == 0),
               token_major=bool(rng.integers(0, 3) == 0), qk_norm=bool(rng.integers(0, 3) == 0),
               share=bool(rng.integers(0, 2)), small_budget=bool(rng.integers(0, 3) == 0),
               sm_scale=0.0 if rng.integers(0, 3) else float(rng.uniform(0.05, 0.2)),
               sigma=float(rng.choice([1.0, 2.0, 4.0])), offset=bool(rng.integers(0, 2)))
    # numerics blocks (drawn last: the earlier fields keep their values): 64 x 64 in half of the configurations
    cfg["bq"], cfg["bkv"] = ((64, 64), (64, 64), (128, 64), (64, 128), (128, 128), (128, 128))[int(rng.integers(0, 6))]
    return cfg


CONFIGS = [_draw(np.random.default_rng(7000 + i)) for i in range(48)]


def _id(c):
    bits = "".join(k[0] for k in ("causal", "k_smooth", "q_smooth", "token_major", "qk_norm", "share", "small_budget") if c[k])
    return f"B{c['B']}H{c['H']}N{c['N']}k{c['Nkv']}d{c['d']}b{c['bq']}x{c['bkv']}-{bits}"


@pytest.mark.parametrize("c", CONFIGS, ids=_id)
def test_random_configuration_against_the_oracle(c):
    B, H, N, d = c["B"], c["H"], c["N"], c["d"]
    Nk = c["Nkv"] or N
    BH = B * H
    seed = 100 * N + Nk + d
    Q, _, _, dO = synth.gaussian_inputs(N, d, sigma_qk=c["sigma"], seed=seed, heads=BH)
    _, K, V, _ = synth.gaussian_inputs(Nk, d, sigma_qk=c["sigma"], seed=seed + 1, heads=BH)
    if c["offset"]:     # channel offsets, what the smoothings are for
        Q = (Q.float() + torch.linspace(-2, 2, d) * c["sigma"]).to(torch.bfloat16)
        K = (K.float() + torch.linspace(3, -3, d) * c["sigma"]).to(torch.bfloat16)
    Q, K, V, dO = (t.reshape(B, H, t.shape[2], d) for t in (Q, K, V, dO))
    kw = {}
    gq = gk = None
    if c["qk_norm"]:
        g = torch.Generator().manual_seed(seed)
        gq = (1.0 + 0.25 * torch.randn(d, generator=g)).float()
        gk = (1.0 + 0.25 * torch.randn(d, generator=g)).float()
        kw = dict(qk_gamma_q=gq.cuda(), qk_gamma_k=gk.cuda(), qk_norm_eps=1e-6)
    if c["small_budget"]:    # dS scratch for one or two heads at a time
        pq, pk = binding.padded_rows(N), binding.padded_rows(Nk)
        kw["scratch_budget"] = int(np.random.default_rng(seed).integers(1, 3)) * pq * (pk + 192)
    p = binding.SageParams(B, H, N, d, causal=c["causal"], k_smooth=c["k_smooth"], q_smooth=c["q_smooth"],
                           sm_scale=c["sm_scale"], token_major=c["token_major"], share_quantized=c["share"], Nkv=c["Nkv"],
                           bq=c["bq"], bkv=c["bkv"], **kw)
    print(_id(c), p, flush=True)

    # what the oracle sees: the normalised tensors when the pre-pass normalises
    Qn, Kn, Vn, dOn = (to_np(t) for t in (Q, K, V, dO))
    if c["qk_norm"]:
        Qn = np.stack([[oracle.qk_norm(Qn[b, h], gq.numpy(), 1e-6) for h in range(H)] for b in range(B)])
        Kn = np.stack([[oracle.qk_norm(Kn[b, h], gk.numpy(), 1e-6) for h in range(H)] for b in range(B)])
    scale = c["sm_scale"] or None
    okw = dict(causal=c["causal"], k_smooth=c["k_smooth"], q_smooth=c["q_smooth"], sm_scale=scale, bq=c["bq"], bkv=c["bkv"])
    On = np.zeros((B, H, N, d), np.float32)
    Ln = np.zeros((B, H, N), np.float32)
    for b in range(B):
        for h in range(H):
            On[b, h], Ln[b, h] = oracle.forward_head(Qn[b, h], Kn[b, h], Vn[b, h], **okw)

    def dev(t):   # as the caller holds it
        t = t.cuda()
        return t.permute(0, 2, 1, 3).contiguous() if c["token_major"] else t

    def host(t):  # back to [B, H, N, d]
        return to_np(t.permute(0, 2, 1, 3) if c["token_major"] else t)

    Qd, Kd, Vd, dOd = (dev(t) for t in (Q, K, V, dO))
    ws = binding.alloc_workspace(p)
    O, L = binding.sagebwd_fwd(Qd, Kd, Vd, p, ws)
    torch.cuda.synchronize()
    Og, Lg = host(O), to_np(L)
    for b in range(B):
        for h in range(H):
            _check(f"O[{b},{h}]", Og[b, h], On[b, h])
            check_lse(f"L[{b},{h}]", Lg[b, h], Ln[b, h])
    # the backward on the oracle's O and L (with the sharing flag it follows the forward on the same workspace)
    Oo = dev(torch.from_numpy(On).to(torch.bfloat16))
    Lo = torch.from_numpy(Ln).cuda()
    dQ, dK, dV = binding.sagebwd_bwd(Qd, Kd, Vd, Oo, dOd, Lo, p, ws)
    torch.cuda.synchronize()
    dQ, dK, dV = host(dQ), host(dK), host(dV)
    assert dQ.shape == (B, H, N, d) and dK.shape == (B, H, Nk, d) and dV.shape == (B, H, Nk, d)
    Ob = to_np(torch.from_numpy(On).to(torch.bfloat16))
    for b in range(B):
        for h in range(H):
            rQ, rK, rV = oracle.backward_head(Qn[b, h], Kn[b, h], Vn[b, h], Ob[b, h], dOn[b, h], Ln[b, h], **okw)
            _check(f"dV[{b},{h}]", dV[b, h], rV)
            _check(f"dQ[{b},{h}]", dQ[b, h], rQ)
            _check(f"dK[{b},{h}]", dK[b, h], rK)
