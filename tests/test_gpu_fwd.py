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
                                     p.sm_scale or None, bq=p.bq or 64, bkv=p.bkv or 64)
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


NON_SQUARE = [(64, 256, 64, True), (100, 228, 128, True), (192, 64, 64, False), (37, 300, 128, False), (1, 200, 64, False),
              (256, 1024, 128, True), (448, 64, 128, False)]


def non_square_inputs(Nq, Nk, d, seed, heads=3, q_offset=False):
    """Q, dO of Nq rows and K, V of Nk rows from the Gaussian recipe (two draws, so the values of one do
    not depend on the length of the other)."""
    Q, _, _, dO = synth.gaussian_inputs(Nq, d, sigma_qk=1.5, seed=seed, heads=heads)
    _, K, V, _ = synth.gaussian_inputs(Nk, d, sigma_qk=1.5, seed=seed + 1, heads=heads)
    if q_offset:
        Q = (Q.float() + torch.linspace(-3, 3, d)).to(torch.bfloat16)
    return Q, K, V, dO


@pytest.mark.parametrize("Nq,Nk,d,causal", NON_SQUARE)
def test_fwd_non_square(Nq, Nk, d, causal):
    """Q of N_q rows against K, V of N_kv rows; under the mask the last query sits on the last key."""
    Q, K, V, _ = non_square_inputs(Nq, Nk, d, seed=3 * Nq + Nk)
    _fwd_case(Q, K, V, binding.SageParams(1, 3, Nq, d, causal=causal, Nkv=Nk))


def test_fwd_non_square_q_smoothing_and_token_major():
    Q, K, V, _ = non_square_inputs(128, 320, 128, seed=41, heads=4, q_offset=True)
    _fwd_case(Q, K, V, binding.SageParams(1, 4, 128, 128, causal=True, q_smooth=True, Nkv=320))
    _fwd_case(Q, K, V, binding.SageParams(1, 4, 128, 128, causal=False, q_smooth=True, Nkv=320))
    # [B, N, H, d] tensors of the two lengths give the bits of the [B, H, N, d] call
    p = binding.SageParams(2, 2, 128, 128, causal=True, Nkv=320)
    pt = binding.SageParams(2, 2, 128, 128, causal=True, Nkv=320, token_major=True)
    Qd, Kd, Vd = (t.reshape(2, 2, t.shape[2], 128).cuda() for t in (Q, K, V))
    O, L = binding.sagebwd_fwd(Qd, Kd, Vd, p)
    tm = lambda t: t.permute(0, 2, 1, 3).contiguous()
    Ot, Lt = binding.sagebwd_fwd(tm(Qd), tm(Kd), tm(Vd), pt)
    torch.cuda.synchronize()
    assert torch.equal(tm(O), Ot) and torch.equal(L, Lt)


BIG_BLOCKS = [(128, 64), (64, 128), (128, 128)]


@pytest.mark.parametrize("bq,bkv", BIG_BLOCKS)
@pytest.mark.parametrize("N,d,causal", [(128, 64, True), (256, 128, True), (320, 64, False), (448, 128, True), (576, 64, True),
                                        (1024, 128, False), (100, 128, True), (333, 64, False), (200, 64, True)])
def test_fwd_numerics_blocks_of_128(bq, bkv, N, d, causal):
    """B_q, B_kv of 128 (Algorithm 1 leaves them free): Q shares a scale per 128 rows, K and V per 128 keys, and
    the per-token quantiser of P~ takes its row max over the 128 keys of a block (the visible ones); odd and
    even tile counts, a partial last block, the diagonal in the first or the second tile of a block."""
    Q, K, V, _ = synth.gaussian_inputs(N, d, sigma_qk=1.5, seed=N + d + bq, heads=3)
    _fwd_case(Q, K, V, binding.SageParams(1, 3, N, d, causal=causal, bq=bq, bkv=bkv))


@pytest.mark.parametrize("bq,bkv", BIG_BLOCKS)
def test_fwd_numerics_blocks_of_128_q_smoothing_non_square_unsmoothed(bq, bkv):
    Q, K, V, _ = non_square_inputs(192, 448, 128, seed=77, heads=2, q_offset=True)
    _fwd_case(Q, K, V, binding.SageParams(1, 2, 192, 128, causal=True, q_smooth=True, Nkv=448, bq=bq, bkv=bkv))
    _fwd_case(Q, K, V, binding.SageParams(1, 2, 192, 128, causal=False, q_smooth=True, Nkv=448, bq=bq, bkv=bkv))
    Q, K, V, _ = non_square_inputs(100, 300, 64, seed=78, heads=2)
    _fwd_case(Q, K, V, binding.SageParams(1, 2, 100, 64, causal=False, k_smooth=False, Nkv=300, bq=bq, bkv=bkv))
    # the differences from 64 x 64 are real: the same inputs give other bits
    Qd, Kd, Vd = (t.cuda() for t in (Q, K, V))
    O64, _ = binding.sagebwd_fwd(Qd, Kd, Vd, binding.SageParams(1, 2, 100, 64, causal=False, Nkv=300))
    Ob, _ = binding.sagebwd_fwd(Qd, Kd, Vd, binding.SageParams(1, 2, 100, 64, causal=False, Nkv=300, bq=bq, bkv=bkv))
    assert not torch.equal(O64, Ob)
