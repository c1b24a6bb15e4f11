"""The autograd wrapper returns the bits of the two direct calls and wires the gradients to Q, K, V."""
import pytest
import torch

from paper_2603_02170_amd import binding, synth
from paper_2603_02170_amd.autograd import sage_attention

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("N,Nk,d,causal,token_major,share", [(192, 192, 64, True, False, False), (100, 228, 128, True, False, True),
                                                             (256, 256, 128, False, True, True), (77, 150, 64, False, True, False)])
def test_autograd_wrapper_gives_the_bits_of_the_direct_calls(N, Nk, d, causal, token_major, share):
    H = 3
    Q, _, _, dO = synth.gaussian_inputs(N, d, sigma_qk=1.5, seed=N + d, heads=H)
    _, K, V, _ = synth.gaussian_inputs(Nk, d, sigma_qk=1.5, seed=N + d + 1, heads=H)
    Q, K, V, dO = (t.cuda() for t in (Q, K, V, dO))
    if token_major:
        Q, K, V, dO = (t.permute(0, 2, 1, 3).contiguous() for t in (Q, K, V, dO))
    p = binding.SageParams(1, H, N, d, causal=causal, token_major=token_major, Nkv=0 if Nk == N else Nk)
    O, L = binding.sagebwd_fwd(Q, K, V, p)
    dQ, dK, dV = binding.sagebwd_bwd(Q, K, V, O, dO, L, p)
    q, k, v = (t.clone().requires_grad_(True) for t in (Q, K, V))
    o, lse = sage_attention(q, k, v, causal=causal, token_major=token_major, share_quantized=share, return_lse=True)
    assert not lse.requires_grad
    o.backward(dO)
    torch.cuda.synchronize()
    assert torch.equal(o.detach(), O) and torch.equal(lse, L)
    assert torch.equal(q.grad, dQ) and torch.equal(k.grad, dK) and torch.equal(v.grad, dV)


def test_autograd_wrapper_in_a_training_step():
    """A projection trained through the INT8 attention: the loss falls (the gradients point downhill)."""
    torch.manual_seed(0)
    B, H, N, d = 1, 2, 128, 64
    x = torch.randn(B, H, N, d, device="cuda")
    target = torch.randn(B, H, N, d, device="cuda")
    W = (torch.eye(d, device="cuda") + 0.05 * torch.randn(d, d, device="cuda")).requires_grad_(True)
    losses = []
    for _ in range(12):
        h = (x @ W).to(torch.bfloat16)
        o = sage_attention(h, h, h, causal=True)
        loss = ((o.float() - target) ** 2).mean()
        loss.backward()
        with torch.no_grad():
            W -= 0.5 * W.grad
            W.grad = None
        losses.append(float(loss.detach()))
    assert losses[-1] < 0.97 * losses[0], losses
