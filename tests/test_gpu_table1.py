"""Accuracy of the GPU path against exact FP64 attention on the paper's sigma sweep.

Paper Table 1 (Sec. 4, "Effect of QK Standard Deviation on Quantization Error") prints the
cosine similarity and relative L2 error of O, dQ, dK, dV against full-precision attention
for Gaussian Q, K of standard deviation 1, 3, 5, 8, 10 (sigma_V = sigma_dO = 1).  The CPU
pins hold the oracle to those printed values; this test holds the HIP kernels, called through
the C ABI, to the same values with the same bands: N = 1024, d = 64, non-causal, K-smoothing on,
four seeds averaged (the table does not state its shape; see the oracle pin for that reading).
"""
import math
import os

import numpy as np
import pytest
import torch

from paper_2603_02170_amd import binding, synth
from fpa_ref import cos_sim, fpa_backward, rel_l2
from gpu_common import to_np

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_table1_sigma_sweep_on_the_gpu_path():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "table1_qk_sigma.txt")) if l.strip() and not l.startswith("#")]
    N, d, seeds = 1024, 64, 4
    names = ("O", "dQ", "dK", "dV")
    p = binding.SageParams(1, seeds, N, d, causal=False)
    for row in rows:
        sigma = float(row[0])
        paper = dict(zip(names, [(float(row[1 + 2 * i]), float(row[2 + 2 * i])) for i in range(4)]))
        # one launch per sigma: the four seeds are four heads
        Q, K, V, dO = synth.gaussian_inputs(N, d, sigma_qk=sigma, seed=1000 + int(sigma), heads=seeds)
        Qd, Kd, Vd, dOd = (t.cuda() for t in (Q, K, V, dO))
        O, L = binding.sagebwd_fwd(Qd, Kd, Vd, p)
        dQ, dK, dV = binding.sagebwd_bwd(Qd, Kd, Vd, O, dOd, L, p)
        torch.cuda.synchronize()
        got = dict(O=to_np(O), dQ=to_np(dQ), dK=to_np(dK), dV=to_np(dV))
        acc = {n: [] for n in names}
        for h in range(seeds):
            ref = fpa_backward(to_np(Q)[0, h], to_np(K)[0, h], to_np(V)[0, h], to_np(dO)[0, h], False, 1 / math.sqrt(d))
            for n in names:
                acc[n].append((cos_sim(got[n][0, h], ref[n]), rel_l2(got[n][0, h], ref[n])))
        for n in names:
            c, e = np.mean(acc[n], axis=0)
            pc, pe = paper[n]
            if sigma == 1:
                # bf16 outputs add a rounding error of about 2^-9 relative, visible at this level only
                if n == "O":
                    assert abs(e - pe) < 0.3 * pe and c > 0.9997, (sigma, n, c, e)
                else:
                    assert pe * 0.8 < e < pe * 3.2 and c > 0.998, (sigma, n, c, e)
            else:
                band = 0.15 if sigma < 8 or n in ("O", "dV") else 0.2
                assert abs(e - pe) < band * pe, (sigma, n, e, pe)
                assert abs(c - pc) < max(0.001, 0.25 * (1 - pc)), (sigma, n, c, pc)


def _errors_vs_exact(Q, K, V, dO, q_smooth, d, blocks=(64, 64)):
    """rel-l2 of O, dQ, dK, dV against exact attention: GPU path and oracle, averaged over the heads."""
    import oracle
    H, N = Q.shape[1], Q.shape[2]
    bq, bkv = blocks
    p = binding.SageParams(1, H, N, d, causal=False, q_smooth=q_smooth, bq=bq, bkv=bkv)
    Qd, Kd, Vd, dOd = (t.cuda() for t in (Q, K, V, dO))
    O, L = binding.sagebwd_fwd(Qd, Kd, Vd, p)
    g = binding.sagebwd_bwd(Qd, Kd, Vd, O, dOd, L, p)
    torch.cuda.synchronize()
    got = [to_np(x)[0] for x in (O,) + tuple(g)]
    names = ("O", "dQ", "dK", "dV")
    e_gpu, e_orc = {n: [] for n in names}, {n: [] for n in names}
    for h in range(H):
        q, k, v, do = (to_np(t)[0, h] for t in (Q, K, V, dO))
        ref = fpa_backward(q, k, v, do, False, 1 / math.sqrt(d))
        Oo, Lo = oracle.forward_head(q, k, v, causal=False, q_smooth=q_smooth, bq=bq, bkv=bkv)
        go = oracle.backward_head(q, k, v, Oo, do, Lo, causal=False, q_smooth=q_smooth, bq=bq, bkv=bkv)
        for n, a, b in zip(names, got, (Oo,) + go):
            e_gpu[n].append(rel_l2(a[h], ref[n]))
            e_orc[n].append(rel_l2(b, ref[n]))
    return {n: float(np.mean(e_gpu[n])) for n in names}, {n: float(np.mean(e_orc[n])) for n in names}


@pytest.mark.parametrize("sigma", [1.0, 5.0, 8.0])
def test_q_smoothing_ablation_on_the_sigma_sweep(sigma):
    """The paper's ablation section reports that Q-smoothing gives no consistent gain in gradient
    accuracy and can make dQ and dK marginally worse.  On the zero-mean Gaussian inputs of the sigma
    sweep the GPU path shows the same picture as the oracle: with and without Q-smoothing the errors of
    dQ and dK against exact attention stay within a few percent of each other (neither setting wins by
    more than 5 %; 12 % at sigma = 8, where the error is 0.4 to 0.5 and moves by that much from seed to
    seed), and the GPU path's errors equal the oracle's to within 2 % in both settings.  With
    channel offsets in Q (what the smoothing is for) it lowers the errors clearly."""
    N, d, H = 1024, 64, 4
    Q, K, V, dO = synth.gaussian_inputs(N, d, sigma_qk=sigma, seed=1100 + int(sigma), heads=H)
    res = {qs: _errors_vs_exact(Q, K, V, dO, qs, d) for qs in (False, True)}
    for qs in (False, True):
        gpu, orc = res[qs]
        for n in gpu:
            assert abs(gpu[n] - orc[n]) < 0.02 * orc[n] + 1e-4, (sigma, qs, n, gpu[n], orc[n])
    for n in ("dQ", "dK"):
        off, on = res[False][0][n], res[True][0][n]
        assert abs(on - off) < (0.05 if sigma < 8 else 0.12) * off, (sigma, n, off, on)
    # the same inputs with a channel offset in Q of twice their standard deviation at the ends
    Qo = (Q.float() + torch.linspace(-2, 2, d) * sigma).to(torch.bfloat16)
    off = _errors_vs_exact(Qo, K, V, dO, False, d)[0]
    on = _errors_vs_exact(Qo, K, V, dO, True, d)[0]
    for n in ("O", "dK") + (("dQ",) if sigma >= 3 else ()):     # (at sigma = 1 dQ gains only 2 %)
        assert on[n] < 0.95 * off[n], (sigma, n, off[n], on[n])


@pytest.mark.parametrize("sigma", [1.0, 5.0])
def test_accuracy_price_of_larger_numerics_blocks_on_the_sigma_sweep(sigma):
    """What blocks of 128 cost in accuracy (Algorithm 1 leaves B_q, B_kv free; a scale shared by more values is
    coarser for most of them): on the sigma sweep's inputs the GPU path's errors against exact attention equal the
    oracle's at every block size to within 2 %, and show the oracle's picture: at sigma = 1, where the errors are
    small, 128 x 128 blocks raise the gradient errors by 15 to 60 %; at sigma = 5, where psi(dS) dominates them, block
    size changes dQ and dK by about a tenth at most (+ 8 % on these seeds)."""
    N, d, H = 1024, 64, 4
    Q, K, V, dO = synth.gaussian_inputs(N, d, sigma_qk=sigma, seed=1200 + int(sigma), heads=H)
    res = {b: _errors_vs_exact(Q, K, V, dO, False, d, blocks=b) for b in ((64, 64), (128, 64), (64, 128), (128, 128))}
    for b, (gpu, orc) in res.items():
        for n in gpu:
            assert abs(gpu[n] - orc[n]) < 0.02 * orc[n] + 1e-4, (sigma, b, n, gpu[n], orc[n])
    small, big = res[(64, 64)][0], res[(128, 128)][0]
    print(sigma, {b: {n: round(v, 4) for n, v in r[0].items()} for b, r in res.items()}, flush=True)
    if sigma == 1.0:
        for n in ("dQ", "dK", "dV"):
            assert 1.15 * small[n] < big[n] < 1.6 * small[n], (n, small[n], big[n])
    else:
        for n in ("dQ", "dK"):
            assert abs(big[n] - small[n]) < 0.12 * small[n], (n, small[n], big[n])
