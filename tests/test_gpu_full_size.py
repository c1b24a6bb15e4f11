"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times:
the whole batch runs on the GPU and sampled heads / blocks are compared with the oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_02170_amd import binding, synth
from gpu_common import check_close, check_lse, params_for, to_np

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]


def test_headline_shape_fwd_bwd_sampled_heads():
    """B=2 H=32 N=8192 d=128 causal (the shape the metric is quoted on): full GPU run, two
    heads checked end to end against the oracle."""
    w = synth.WORKLOADS["headline"]
    p = params_for(w)
    Q, K, V, dO = synth.make_inputs(w)
    Qd, Kd, Vd, dOd = (t.cuda() for t in (Q, K, V, dO))
    ws = binding.alloc_workspace(p)
    O, L = binding.sagebwd_fwd(Qd, Kd, Vd, p, ws)
    sample = [(0, 5), (1, 30)]
    On, Ln = {}, {}
    for b, h in sample:
        q, k, v = (to_np(t[b, h]) for t in (Q, K, V))
        On[b, h], Ln[b, h] = oracle.forward_head(q, k, v, causal=True)
        check_close(f"O[{b},{h}]", to_np(O[b, h]), On[b, h])
        check_lse(f"LSE[{b},{h}]", to_np(L[b, h]), Ln[b, h])
    # backward: the GPU gets the oracle's O and L on the sampled heads (its own elsewhere)
    O2, L2 = O.clone(), L.clone()
    for b, h in sample:
        O2[b, h] = torch.from_numpy(On[b, h]).to(torch.bfloat16).cuda()
        L2[b, h] = torch.from_numpy(Ln[b, h]).cuda()
    dQ, dK, dV = binding.sagebwd_bwd(Qd, Kd, Vd, O2, dOd, L2, p, ws)
    torch.cuda.synchronize()
    for b, h in sample:
        q, k, v, do = (to_np(t[b, h]) for t in (Q, K, V, dO))
        rQ, rK, rV = oracle.backward_head(q, k, v, On[b, h], do, Ln[b, h], causal=True)
        check_close(f"dV[{b},{h}]", to_np(dV[b, h]), rV)
        check_close(f"dQ[{b},{h}]", to_np(dQ[b, h]), rQ)
        check_close(f"dK[{b},{h}]", to_np(dK[b, h]), rK)
    # every other head: finite, and the gradients are not all zero
    for t in (O, dQ, dK, dV):
        assert torch.isfinite(t.float()).all()
        assert (t.float().abs().amax(dim=(2, 3)) > 0).all()


def _full_launch_sampled_heads(w, sample, k_smooth=None, blocks=(64, 64)):
    """The whole batch of workload `w` runs on the GPU in its own launch configuration (the
    workgroup-to-head mapping depends on B*H and N); the (b, h) pairs in `sample` are compared end to
    end with the oracle.  The backward is given the oracle's O and L on the sampled heads."""
    bq, bkv = blocks
    p = params_for(w, bq=bq, bkv=bkv) if k_smooth is None else params_for(w, k_smooth=k_smooth, bq=bq, bkv=bkv)
    Q, K, V, dO = synth.make_inputs(w)
    Qd, Kd, Vd, dOd = (t.cuda() for t in (Q, K, V, dO))
    ws = binding.alloc_workspace(p)
    O, L = binding.sagebwd_fwd(Qd, Kd, Vd, p, ws)
    On, Ln = {}, {}
    for b, h in sample:
        q, k, v = (to_np(t[b, h]) for t in (Q, K, V))
        On[b, h], Ln[b, h] = oracle.forward_head(q, k, v, causal=w.causal, k_smooth=p.k_smooth, bq=bq, bkv=bkv)
        check_close(f"O[{b},{h}]", to_np(O[b, h]), On[b, h])
        check_lse(f"LSE[{b},{h}]", to_np(L[b, h]), Ln[b, h])
    O2, L2 = O.clone(), L.clone()
    for b, h in sample:
        O2[b, h] = torch.from_numpy(On[b, h]).to(torch.bfloat16).cuda()
        L2[b, h] = torch.from_numpy(Ln[b, h]).cuda()
    dQ, dK, dV = binding.sagebwd_bwd(Qd, Kd, Vd, O2, dOd, L2, p, ws)
    torch.cuda.synchronize()
    for b, h in sample:
        q, k, v, do = (to_np(t[b, h]) for t in (Q, K, V, dO))
        rQ, rK, rV = oracle.backward_head(q, k, v, On[b, h], do, Ln[b, h], causal=w.causal, k_smooth=p.k_smooth, bq=bq, bkv=bkv)
        check_close(f"dV[{b},{h}]", to_np(dV[b, h]), rV)
        check_close(f"dQ[{b},{h}]", to_np(dQ[b, h]), rQ)
        check_close(f"dK[{b},{h}]", to_np(dK[b, h]), rK)
    for t in (O, dQ, dK, dV):
        assert torch.isfinite(t.float()).all()
        assert (t.float().abs().amax(dim=(2, 3)) > 0).all()


def test_pretrain_shape_full_launch_sampled_heads():
    """B=4 H=16 N=2048 d=128 causal, K-smoothing on (the paper's pre-training shape): 64 heads with
    16 work items each, so every kernel takes four heads of an XCD at a time."""
    _full_launch_sampled_heads(synth.WORKLOADS["pretrain"], [(0, 0), (1, 7), (2, 10), (3, 15)])


@pytest.mark.parametrize("k_smooth", [True, False])
def test_outlier_shape_full_launch_sampled_heads(k_smooth):
    """B=2 H=16 N=4096 d=128 causal, per-channel K bias and amplified Q channels, no QK-norm, with
    K-smoothing on and off: 32 heads (four per XCD), the forward's converting logit path."""
    _full_launch_sampled_heads(synth.WORKLOADS["outlier"], [(0, 3), (1, 12)], k_smooth=k_smooth)


def test_long_context_shape_sampled_blocks():
    """B=1 H=32 N=32768 d=128 non-causal, dO ~ N(0, 1e-2): full GPU run (the backward goes
    through several head groups); on one head the oracle checks sampled Q blocks of O, LSE and dQ
    and sampled KV blocks of dK and dV."""
    w = synth.WORKLOADS["long"]
    p = params_for(w)
    Q, K, V, dO = synth.make_inputs(w)
    Qd, Kd, Vd, dOd = (t.cuda() for t in (Q, K, V, dO))
    ws = binding.alloc_workspace(p)
    O, L = binding.sagebwd_fwd(Qd, Kd, Vd, p, ws)
    torch.cuda.synchronize()
    b, h = 0, 19
    q, k, v, do = (to_np(t[b, h]) for t in (Q, K, V, dO))
    qblocks = [0, 77, 300, 511]
    Or, Lr = oracle.forward_head(q, k, v, causal=False, q_blocks=qblocks)
    Og, Lg = to_np(O[b, h]), to_np(L[b, h])
    rows = np.concatenate([np.arange(64 * i, 64 * i + 64) for i in qblocks])
    check_close("O rows", Og[rows], Or[rows])
    check_lse("LSE rows", Lg[rows], Lr[rows])
    # backward is fed the GPU forward's own O and L on both sides (the oracle needs L for every
    # row of the sampled KV blocks; L itself was checked above on the sampled rows)
    dQ, dK, dV = binding.sagebwd_bwd(Qd, Kd, Vd, O, dOd, L, p, ws)
    torch.cuda.synchronize()
    rQ, _, _ = oracle.backward_head(q, k, v, Og, do, Lg, causal=False, q_blocks=qblocks)
    check_close("dQ rows", to_np(dQ[b, h])[rows], rQ[rows])
    kvblocks = [3, 410]
    _, rK, rV = oracle.backward_head(q, k, v, Og, do, Lg, causal=False, kv_blocks=kvblocks)
    krows = np.concatenate([np.arange(64 * i, 64 * i + 64) for i in kvblocks])
    check_close("dK rows", to_np(dK[b, h])[krows], rK[krows])
    check_close("dV rows", to_np(dV[b, h])[krows], rV[krows])
    for t in (O, dQ, dK, dV):
        assert torch.isfinite(t.float()).all()


@pytest.mark.parametrize("name", ["headline_d64", "headline_qsmooth"])
def test_headline_variants_sampled_blocks(name):
    """The headline shape at the paper's other head dimension (d = 64: three forward workgroups
    per CU) and with Q-smoothing on (bias table, staged bias rows, dK bias branch): full GPU run in
    the benchmark's launch configuration; on one head the oracle checks sampled Q blocks of O, LSE,
    dQ and sampled KV blocks of dK, dV (first, interior and last blocks of the causal triangle)."""
    w = synth.WORKLOADS[name]
    p = params_for(w)
    Q, K, V, dO = synth.make_inputs(w)
    Qd, Kd, Vd, dOd = (t.cuda() for t in (Q, K, V, dO))
    ws = binding.alloc_workspace(p)
    O, L = binding.sagebwd_fwd(Qd, Kd, Vd, p, ws)
    torch.cuda.synchronize()
    b, h = 1, 7
    q, k, v, do = (to_np(t[b, h]) for t in (Q, K, V, dO))
    kw = dict(causal=True, k_smooth=w.k_smooth, q_smooth=w.q_smooth)
    qblocks = [0, 1, 64, 127]
    Or, Lr = oracle.forward_head(q, k, v, q_blocks=qblocks, **kw)
    Og, Lg = to_np(O[b, h]), to_np(L[b, h])
    rows = np.concatenate([np.arange(64 * i, 64 * i + 64) for i in qblocks])
    check_close("O rows", Og[rows], Or[rows])
    check_lse("LSE rows", Lg[rows], Lr[rows])
    # the backward is fed the GPU forward's own O and L on both sides (L was checked above)
    dQ, dK, dV = binding.sagebwd_bwd(Qd, Kd, Vd, O, dOd, L, p, ws)
    torch.cuda.synchronize()
    rQ, _, _ = oracle.backward_head(q, k, v, Og, do, Lg, q_blocks=qblocks, **kw)
    check_close("dQ rows", to_np(dQ[b, h])[rows], rQ[rows])
    kvblocks = [0, 63, 126, 127]
    _, rK, rV = oracle.backward_head(q, k, v, Og, do, Lg, kv_blocks=kvblocks, **kw)
    krows = np.concatenate([np.arange(64 * i, 64 * i + 64) for i in kvblocks])
    check_close("dK rows", to_np(dK[b, h])[krows], rK[krows])
    check_close("dV rows", to_np(dV[b, h])[krows], rV[krows])
    for t in (O, dQ, dK, dV):
        assert torch.isfinite(t.float()).all()


def test_very_long_causal_sequence_sampled_blocks():
    """B=1 H=1 N=65536 d=128 causal: 1024 blocks per head, the psi(dS) scratch of the one head is
    4 GiB (half of the default budget) and tile indices pass 2^20; sampled Q blocks of O, LSE, dQ and
    sampled KV blocks of dK, dV against the oracle."""
    w = synth.Workload("very_long", 7, 1, 1, 65536, 128, True)
    p = params_for(w)
    Q, K, V, dO = synth.make_inputs(w)
    Qd, Kd, Vd, dOd = (t.cuda() for t in (Q, K, V, dO))
    ws = binding.alloc_workspace(p)
    O, L = binding.sagebwd_fwd(Qd, Kd, Vd, p, ws)
    torch.cuda.synchronize()
    q, k, v, do = (to_np(t[0, 0]) for t in (Q, K, V, dO))
    qblocks = [0, 513, 1023]
    Or, Lr = oracle.forward_head(q, k, v, causal=True, q_blocks=qblocks)
    Og, Lg = to_np(O[0, 0]), to_np(L[0, 0])
    rows = np.concatenate([np.arange(64 * i, 64 * i + 64) for i in qblocks])
    check_close("O rows", Og[rows], Or[rows])
    check_lse("LSE rows", Lg[rows], Lr[rows])
    dQ, dK, dV = binding.sagebwd_bwd(Qd, Kd, Vd, O, dOd, L, p, ws)
    torch.cuda.synchronize()
    rQ, _, _ = oracle.backward_head(q, k, v, Og, do, Lg, causal=True, q_blocks=qblocks)
    check_close("dQ rows", to_np(dQ[0, 0])[rows], rQ[rows])
    kvblocks = [0, 700, 1023]
    _, rK, rV = oracle.backward_head(q, k, v, Og, do, Lg, causal=True, kv_blocks=kvblocks)
    krows = np.concatenate([np.arange(64 * i, 64 * i + 64) for i in kvblocks])
    check_close("dK rows", to_np(dK[0, 0])[krows], rK[krows])
    check_close("dV rows", to_np(dV[0, 0])[krows], rV[krows])
    for t in (O, dQ, dK, dV):
        assert torch.isfinite(t.float()).all()


@pytest.mark.parametrize("blocks", [(128, 128), (128, 64), (64, 128)])
def test_headline_shape_numerics_blocks_of_128_sampled_head(blocks):
    """The headline shape with B_q, B_kv of 128, in the launch configuration `bench.py --blocks` times: one
    head end to end against the oracle run with the same block sizes."""
    _full_launch_sampled_heads(synth.WORKLOADS["headline"], [(1, 17)], blocks=blocks)
