"""sagebwd_fwd_static: the forward for callers that cannot allocate (its workspace is a built-in
device array).  Through the C ABI it must return exactly what sagebwd_fwd returns, on two calls in a
row, the second on a smaller problem (the array keeps the first call's contents)."""
import pytest
import torch

from paper_2603_02170_amd import binding, synth

pytestmark = pytest.mark.gpu


def _one(N, d, H, causal, q_smooth, seed):
    Q, K, V, _ = (t.cuda() for t in synth.gaussian_inputs(N, d, sigma_qk=1.5, seed=seed, heads=H))
    if q_smooth:
        Q = (Q.float() + torch.linspace(-2, 2, d, device="cuda")).to(torch.bfloat16)
    p = binding.SageParams(1, H, N, d, causal=causal, q_smooth=q_smooth)
    assert binding.workspace_bytes(p, forward_only=True) <= binding.STATIC_SCRATCH_BYTES
    O_ref, L_ref = binding.sagebwd_fwd(Q, K, V, p)
    O = torch.full_like(O_ref, float("nan"))
    L = torch.full_like(L_ref, float("nan"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    binding.sagebwd_fwd_static(Q, K, V, p, O, L)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before          # nothing went through torch's allocator
    assert torch.equal(O, O_ref) and torch.equal(L, L_ref), (N, d, H, causal, q_smooth)


def test_fwd_static_equals_fwd_on_two_calls_in_a_row_the_second_smaller():
    _one(1000, 128, 6, True, False, seed=201)      # partial last block, 16 blocks
    _one(320, 64, 3, False, False, seed=202)       # smaller, other head dimension, no mask
    _one(448, 128, 2, True, True, seed=203)        # Q-smoothing (bias table in the array)
    _one(64, 64, 1, True, False, seed=204)         # one block


def test_fwd_static_refuses_what_does_not_fit():
    p = binding.SageParams(2, 32, 8192, 128)
    x = torch.zeros(1, device="cuda", dtype=torch.bfloat16)
    import ctypes
    cp = p.c()
    rc = binding.load_library().sagebwd_fwd_static(x.data_ptr(), x.data_ptr(), x.data_ptr(), x.data_ptr(),
                                                   x.data_ptr(), ctypes.byref(cp), None)
    assert rc == -5 and "scratch" in binding.sagebwd_strerror(rc)
