"""GPU parity of the fused forward against the CPU oracle (through the C ABI)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_02170_amd import binding, synth
from gpu_common import check_close, check_lse, params_for, to_np

pytestmark = pytest.mark.gpu


def _fwd_case(Q, K, V, p, heads=None):
    Qd, Kd, Vd = (t.cuda() for t in (Q, K, V))
    O, L = binding.sagebwd_fwd(Qd, Kd, Vd, p)
    torch.cuda.synchronize()
    O, L = to_np(O), to_np(L)
    Qn, Kn, Vn = (to_np(t) for t in (Q, K, V))
    B, H = Q.shape[:2]
    todo = [(b, h) for b in range(B) for h in range(H)] if heads is None else heads
    for b, h in todo:
        Or, Lr = oracle.forward_head(Qn[b, h], Kn[b, h], Vn[b, h], p.causal, p.k_smooth, p.q_smooth,
                                     p.sm_scale or None)
        check_close(f"O[{b},{h}]", O[b, h], Or)
        check_lse(f"LSE[{b},{h}]", L[b, h], Lr)
    return O, L


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("k_smooth", [True, False])
def test_fwd_tiny(causal, k_smooth):
    w = synth.WORKLOADS["tiny"]
    Q, K, V, _ = synth.make_inputs(w)
    _fwd_case(Q, K, V, params_for(w, causal=causal, k_smooth=k_smooth))


@pytest.mark.parametrize("N,d,causal", [(64, 64, True), (192, 128, True), (320, 64, False), (576, 128, True),
                                        (1024, 128, False)])
def test_fwd_shapes_ragged_tiles(N, d, causal):
    # N/64 odd, not a multiple of the workgroup's query tile, one block only, ...
    Q, K, V, _ = synth.gaussian_inputs(N, d, sigma_qk=1.5, seed=N + d, heads=3)
    _fwd_case(Q, K, V, binding.SageParams(1, 3, N, d, causal=causal))


@pytest.mark.parametrize("N,d,causal", [(100, 64, True), (100, 64, False), (200, 128, True), (333, 128, False),
                                        (37, 64, False), (1, 64, True), (129, 128, False), (8191, 128, True)])
def test_fwd_partial_last_block(N, d, causal):
    """N that is not a multiple of 64: the last block is partial (its missing rows do not exist)."""
    Q, K, V, _ = synth.gaussian_inputs(N, d, sigma_qk=1.5, seed=2 * N + d, heads=3)
    _fwd_case(Q, K, V, binding.SageParams(1, 3, N, d, causal=causal))


def test_fwd_partial_last_block_q_smoothing_and_no_k_smoothing():
    Q, K, V, _ = synth.gaussian_inputs(300, 128, sigma_qk=1.0, seed=31, heads=2)
    Q = (Q.float() + torch.linspace(-3, 3, 128)).to(torch.bfloat16)
    _fwd_case(Q, K, V, binding.SageParams(1, 2, 300, 128, causal=False, q_smooth=True))
    _fwd_case(Q, K, V, binding.SageParams(1, 2, 300, 128, causal=True, q_smooth=True))
    _fwd_case(Q, K, V, binding.SageParams(1, 2, 300, 128, causal=False, k_smooth=False))


def test_fwd_q_smoothing():
    Q, K, V, _ = synth.gaussian_inputs(512, 128, sigma_qk=1.0, seed=3, heads=2)
    Q = (Q.float() + torch.linspace(-3, 3, 128)).to(torch.bfloat16)
    _fwd_case(Q, K, V, binding.SageParams(1, 2, 512, 128, causal=True, q_smooth=True))
    _fwd_case(Q, K, V, binding.SageParams(1, 2, 512, 128, causal=False, q_smooth=True))


def test_fwd_custom_scale_and_zero_queries():
    Q, K, V, _ = synth.gaussian_inputs(256, 64, seed=9, heads=2)
    _fwd_case(Q, K, V, binding.SageParams(1, 2, 256, 64, causal=True, sm_scale=0.3))
    Z = torch.zeros_like(Q)
    O, L = _fwd_case(Z, K, V, binding.SageParams(1, 2, 256, 64, causal=True))
    assert np.allclose(L[0, 0], np.log(np.arange(1, 257)), atol=1e-5)


def test_fwd_pretrain_shape_sampled_heads():
    w = synth.WORKLOADS["pretrain"]
    Q, K, V, _ = synth.make_inputs(w, heads=[0, 5, 31, 63])
    _fwd_case(Q, K, V, params_for(w, B=4, H=1))


def test_fwd_outlier_shape_with_and_without_k_smoothing():
    w = synth.WORKLOADS["outlier"]
    Q, K, V, _ = synth.make_inputs(w, heads=[3, 20])
    for ks in (True, False):
        _fwd_case(Q, K, V, params_for(w, B=2, H=1, k_smooth=ks))
