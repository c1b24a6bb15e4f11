"""GPU parity of the fused backward against the CPU oracle (through the C ABI).

The oracle's backward is fed the oracle's own forward outputs (O, L); the GPU backward
is fed the same arrays, so the comparison isolates the backward."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_02170_amd import binding, synth
from gpu_common import check_close, params_for, to_np

pytestmark = pytest.mark.gpu


def dQ_shape_ok(Q, K, p):
    return Q.shape[2] == p.N and K.shape[2] == p.kv_len


def _bwd_case(Q, K, V, dO, p, heads=None):
    Qn, Kn, Vn, dOn = (to_np(t) for t in (Q, K, V, dO))
    B, H = Q.shape[:2]
    assert dQ_shape_ok(Q, K, p)
    On = np.zeros_like(Qn)
    Ln = np.zeros(Qn.shape[:3], np.float32)
    todo = [(b, h) for b in range(B) for h in range(H)] if heads is None else heads
    for b, h in todo:
        On[b, h], Ln[b, h] = oracle.forward_head(Qn[b, h], Kn[b, h], Vn[b, h], p.causal, p.k_smooth, p.q_smooth,
                                                 p.sm_scale or None, bq=p.bq or 64, bkv=p.bkv or 64)
    Od = torch.from_numpy(On).to(torch.bfloat16).cuda()
    Ld = torch.from_numpy(Ln).cuda()
    dQ, dK, dV = binding.sagebwd_bwd(Q.cuda(), K.cuda(), V.cuda(), Od, dO.cuda(), Ld, p)
    torch.cuda.synchronize()
    dQ, dK, dV = to_np(dQ), to_np(dK), to_np(dV)
    for b, h in todo:
        rQ, rK, rV = oracle.backward_head(Qn[b, h], Kn[b, h], Vn[b, h], On[b, h], dOn[b, h], Ln[b, h], p.causal,
                                          p.k_smooth, p.q_smooth, p.sm_scale or None, bq=p.bq or 64, bkv=p.bkv or 64)
        check_close(f"dV[{b},{h}]", dV[b, h], rV)
        check_close(f"dQ[{b},{h}]", dQ[b, h], rQ)
        check_close(f"dK[{b},{h}]", dK[b, h], rK)


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("k_smooth", [True, False])
def test_bwd_tiny(causal, k_smooth):
    w = synth.WORKLOADS["tiny"]
    Q, K, V, dO = synth.make_inputs(w)
    _bwd_case(Q, K, V, dO, params_for(w, causal=causal, k_smooth=k_smooth))


@pytest.mark.parametrize("N,d,causal", [(64, 64, True), (192, 128, True), (320, 64, False), (576, 128, True),
                                        (1024, 128, False)])
def test_bwd_shapes_ragged_tiles(N, d, causal):
    Q, K, V, dO = synth.gaussian_inputs(N, d, sigma_qk=1.5, seed=N + d, heads=3)
    _bwd_case(Q, K, V, dO, binding.SageParams(1, 3, N, d, causal=causal))


@pytest.mark.parametrize("N,d,causal", [(100, 64, True), (100, 64, False), (200, 128, True), (333, 128, False),
                                        (37, 64, False), (65, 64, True), (129, 128, False), (1000, 128, True)])
def test_bwd_partial_last_block(N, d, causal):
    """N that is not a multiple of 64: no gradient reaches rows that do not exist, and the keys
    that do not exist are masked in every tile of the last KV block."""
    Q, K, V, dO = synth.gaussian_inputs(N, d, sigma_qk=1.5, seed=2 * N + d, heads=3)
    _bwd_case(Q, K, V, dO, binding.SageParams(1, 3, N, d, causal=causal))


def test_bwd_partial_last_block_q_smoothing_and_no_k_smoothing():
    Q, K, V, dO = synth.gaussian_inputs(300, 128, sigma_qk=1.0, seed=31, heads=2)
    Q = (Q.float() + torch.linspace(-3, 3, 128)).to(torch.bfloat16)
    _bwd_case(Q, K, V, dO, binding.SageParams(1, 2, 300, 128, causal=False, q_smooth=True))
    _bwd_case(Q, K, V, dO, binding.SageParams(1, 2, 300, 128, causal=True, q_smooth=True))
    _bwd_case(Q, K, V, dO, binding.SageParams(1, 2, 300, 128, causal=False, k_smooth=False))


def test_bwd_q_smoothing():
    Q, K, V, dO = synth.gaussian_inputs(512, 128, sigma_qk=1.0, seed=3, heads=2)
    Q = (Q.float() + torch.linspace(-3, 3, 128)).to(torch.bfloat16)
    _bwd_case(Q, K, V, dO, binding.SageParams(1, 2, 512, 128, causal=True, q_smooth=True))
    _bwd_case(Q, K, V, dO, binding.SageParams(1, 2, 512, 64 * 2, causal=False, q_smooth=True))


def test_bwd_small_upstream_gradient_and_custom_scale():
    Q, K, V, dO = synth.gaussian_inputs(256, 64, seed=9, heads=2)
    dO = (dO.float() * 1e-3).to(torch.bfloat16)
    _bwd_case(Q, K, V, dO, binding.SageParams(1, 2, 256, 64, causal=True, sm_scale=0.3))


def test_bwd_pretrain_shape_sampled_heads():
    w = synth.WORKLOADS["pretrain"]
    Q, K, V, dO = synth.make_inputs(w, heads=[0, 31, 63])
    _bwd_case(Q, K, V, dO, params_for(w, B=3, H=1))


def test_bwd_outlier_shape_with_and_without_k_smoothing():
    w = synth.WORKLOADS["outlier"]
    Q, K, V, dO = synth.make_inputs(w, heads=[3])
    for ks in (True, False):
        _bwd_case(Q, K, V, dO, params_for(w, B=1, H=1, k_smooth=ks))


def test_bwd_head_groups_share_the_ds_scratch():
    # a scratch budget of two heads' worth of dS forces the 5 heads through 3 groups
    Q, K, V, dO = synth.gaussian_inputs(256, 64, seed=21, heads=5)
    _bwd_case(Q, K, V, dO, binding.SageParams(1, 5, 256, 64, causal=True, scratch_budget=2 * 256 * (256 + 192)))


def test_bwd_q_smoothing_head_dim_64_odd_block_count():
    # d = 64 with Q-smoothing; 5 blocks, so the last workgroup has an idle second group
    Q, K, V, dO = synth.gaussian_inputs(320, 64, sigma_qk=1.0, seed=5, heads=2)
    Q = (Q.float() + torch.linspace(-2, 2, 64)).to(torch.bfloat16)
    _bwd_case(Q, K, V, dO, binding.SageParams(1, 2, 320, 64, causal=True, q_smooth=True))


def test_bwd_zero_upstream_gradient_gives_zero_gradients():
    # dO = 0: delta = 0, every dS tile is all-zero (scale 0, codes 0), all three gradients vanish
    Q, K, V, dO = synth.gaussian_inputs(256, 128, seed=11, heads=1)
    Z = torch.zeros_like(dO)
    O, L = binding.sagebwd_fwd(Q.cuda(), K.cuda(), V.cuda(), binding.SageParams(1, 1, 256, 128, causal=True))
    dQ, dK, dV = binding.sagebwd_bwd(Q.cuda(), K.cuda(), V.cuda(), O, Z.cuda(), L,
                                     binding.SageParams(1, 1, 256, 128, causal=True))
    torch.cuda.synchronize()
    for name, g in (("dQ", dQ), ("dK", dK), ("dV", dV)):
        assert torch.count_nonzero(g).item() == 0, name


def test_bwd_two_steady_intervals_only():
    # N = 256 non-causal: 4 tile rows, the shortest loop that reaches the branch-free interval
    Q, K, V, dO = synth.gaussian_inputs(256, 128, seed=13, heads=2)
    _bwd_case(Q, K, V, dO, binding.SageParams(1, 2, 256, 128, causal=False))


@pytest.mark.parametrize("N,d,causal,q_smooth", [(320, 64, True, False), (100, 128, False, False), (256, 128, True, True)])
def test_token_major_layout_gives_the_same_bits(N, d, causal, q_smooth):
    """[B, N, H, d] tensors (token-major): forward and backward must return exactly what the
    [B, H, N, d] call returns on the same values (the same kernels run on dense workspace copies),
    which the other tests hold to the oracle."""
    Q, K, V, dO = synth.gaussian_inputs(N, d, sigma_qk=1.5, seed=7 * N + d, heads=6)      # [1, 6, N, d]
    Q, K, V, dO = (t.reshape(2, 3, N, d).cuda() for t in (Q, K, V, dO))
    p = binding.SageParams(2, 3, N, d, causal=causal, q_smooth=q_smooth)
    pt = binding.SageParams(2, 3, N, d, causal=causal, q_smooth=q_smooth, token_major=True)
    O, L = binding.sagebwd_fwd(Q, K, V, p)
    dQ, dK, dV = binding.sagebwd_bwd(Q, K, V, O, dO, L, p)
    tm = lambda t: t.permute(0, 2, 1, 3).contiguous()
    Ot, Lt = binding.sagebwd_fwd(tm(Q), tm(K), tm(V), pt)
    dQt, dKt, dVt = binding.sagebwd_bwd(tm(Q), tm(K), tm(V), Ot, tm(dO), Lt, pt)
    torch.cuda.synchronize()
    assert Ot.shape == (2, N, 3, d) and Lt.shape == (2, 3, N)
    assert torch.equal(tm(O), Ot) and torch.equal(L, Lt)
    for a, b, name in ((dQ, dQt, "dQ"), (dK, dKt, "dK"), (dV, dVt, "dV")):
        assert torch.equal(tm(a), b), name


@pytest.mark.parametrize("N,d,causal", [(128, 64, True), (256, 128, False), (200, 128, True)])
def test_in_loop_quantiser_of_ds_within_one_step_of_the_oracle(N, d, causal):
    """psi(dS) is decided inside the kernel from P = exp2(..) of the hardware, so its codes cannot be
    bit-exact; read back from the scratch they must sit within one quantisation step of the oracle's
    codes, agree on almost all entries, and carry the same tile scales."""
    Q, K, V, dO = synth.gaussian_inputs(N, d, sigma_qk=1.0, seed=5 * N + d, heads=2)
    p = binding.SageParams(1, 2, N, d, causal=causal)
    Qn, Kn, Vn, dOn = (to_np(t) for t in (Q, K, V, dO))
    ws = binding.alloc_workspace(p)
    On = np.zeros_like(Qn)
    Ln = np.zeros(Qn.shape[:3], np.float32)
    for h in range(2):
        On[0, h], Ln[0, h] = oracle.forward_head(Qn[0, h], Kn[0, h], Vn[0, h], causal)
    Od, Ld = torch.from_numpy(On).to(torch.bfloat16).cuda(), torch.from_numpy(Ln).cuda()
    binding.sagebwd_bwd(Q.cuda(), K.cuda(), V.cuda(), Od, dO.cuda(), Ld, p, ws)
    for h in range(2):
        inter = {}
        oracle.backward_head(Qn[0, h], Kn[0, h], Vn[0, h], On[0, h], dOn[0, h], Ln[0, h], causal, intermediates=inter)
        ds, sc = binding.sagebwd_export_ds(p, ws, h)
        torch.cuda.synchronize()
        ds, sc = ds.cpu().numpy().astype(np.int32), sc.cpu().numpy()
        ref, rsc = inter["dSh"].astype(np.int32), inter["sdS"]
        assert np.allclose(sc, rsc, rtol=5e-6, atol=0), np.abs(sc / np.where(rsc > 0, rsc, 1) - 1).max()
        diff = np.abs(ds - ref)
        assert diff.max() <= 1, diff.max()
        assert (diff == 0).mean() > 0.999, (diff == 0).mean()    # (measured: every code equal, scales within 6e-7)


def test_side_stream_gives_the_same_bits():
    """Every kernel is enqueued on the caller's stream: a forward + backward on a side stream (with
    unrelated work on the default stream) returns exactly what the default-stream call returns."""
    Q, K, V, dO = (t.cuda() for t in synth.gaussian_inputs(384, 128, sigma_qk=1.0, seed=77, heads=4))
    p = binding.SageParams(1, 4, 384, 128, causal=True)
    O, L = binding.sagebwd_fwd(Q, K, V, p)
    ref = binding.sagebwd_bwd(Q, K, V, O, dO, L, p)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    busy = torch.randn(4096, 4096, device="cuda")
    with torch.cuda.stream(side):
        O2, L2 = binding.sagebwd_fwd(Q, K, V, p)
        got = binding.sagebwd_bwd(Q, K, V, O2, dO, L2, p)
    for _ in range(4):
        busy = busy @ busy * 1e-4            # default-stream work running beside it
    side.synchronize()
    torch.cuda.synchronize()
    assert torch.equal(O, O2) and torch.equal(L, L2)
    for a, b in zip(ref, got):
        assert torch.equal(a, b)


def test_backward_is_deterministic_and_needs_nothing_from_an_old_workspace():
    """dQ comes from stored tiles and a second kernel, not from atomics: two calls return the same
    bits, also when the workspace was overwritten in between (the backward re-runs its pre-pass and
    relies on nothing a previous call left there) and when the scratch budget forces head groups."""
    Q, K, V, dO = (t.cuda() for t in synth.gaussian_inputs(448, 128, sigma_qk=1.0, seed=78, heads=5))
    p = binding.SageParams(1, 5, 448, 128, causal=True, q_smooth=True)
    ws = binding.alloc_workspace(p)
    O, L = binding.sagebwd_fwd(Q, K, V, p, ws)
    a = [t.clone() for t in binding.sagebwd_bwd(Q, K, V, O, dO, L, p, ws)]
    ws.fill_(0x5A)
    b = [t.clone() for t in binding.sagebwd_bwd(Q, K, V, O, dO, L, p, ws)]
    pg = binding.SageParams(1, 5, 448, 128, causal=True, q_smooth=True, scratch_budget=2 * 448 * (448 + 192))   # two heads at a time
    c = binding.sagebwd_bwd(Q, K, V, O, dO, L, pg, binding.alloc_workspace(pg))
    torch.cuda.synchronize()
    for x, y, z in zip(a, b, c):
        assert torch.equal(x, y) and torch.equal(x, z)


@pytest.mark.parametrize("N,d,causal,q_smooth,k_smooth", [(448, 128, True, False, True), (300, 64, False, True, True),
                                                         (1024, 128, True, True, False)])
def test_backward_sharing_the_forwards_quantised_operands_gives_the_same_bits(N, d, causal, q_smooth, k_smooth):
    """SAGEBWD_FLAG_SHARE_QUANTIZED: the forward leaves psi(Q), psi(K) in both operand layouts and the
    backward forms only the dO part of its pre-pass (Algorithm 2 takes the quantised Q, K from the
    forward).  O, LSE and all three gradients must equal the default calls bit for bit."""
    Q, K, V, dO = (t.cuda() for t in synth.gaussian_inputs(N, d, sigma_qk=1.5, seed=300 + N, heads=5))
    if q_smooth:
        Q = (Q.float() + torch.linspace(-2, 2, d, device="cuda")).to(torch.bfloat16)
    kw = dict(causal=causal, q_smooth=q_smooth, k_smooth=k_smooth)
    p = binding.SageParams(1, 5, N, d, **kw)
    ps = binding.SageParams(1, 5, N, d, share_quantized=True, **kw)
    O, L = binding.sagebwd_fwd(Q, K, V, p)
    ref = binding.sagebwd_bwd(Q, K, V, O, dO, L, p)
    ws = binding.alloc_workspace(ps)
    ws.fill_(0x5A)
    Os, Ls = binding.sagebwd_fwd(Q, K, V, ps, ws)
    got = binding.sagebwd_bwd(Q, K, V, Os, dO, Ls, ps, ws)
    torch.cuda.synchronize()
    assert torch.equal(O, Os) and torch.equal(L, Ls)
    for a, b, name in zip(ref, got, ("dQ", "dK", "dV")):
        assert torch.equal(a, b), name


def test_graph_capture_and_replay():
    """The entry points allocate nothing and only launch kernels on the caller's stream, so a
    forward + backward can be captured in a graph; every replay (with new inputs copied into the
    captured buffers, and eager work between the replays) must equal the eager result."""
    N, d, H = 320, 128, 3
    p = binding.SageParams(1, H, N, d, causal=True)
    ws = binding.alloc_workspace(p)
    bufs = [torch.zeros(1, H, N, d, dtype=torch.bfloat16, device="cuda") for _ in range(4)]
    Qb, Kb, Vb, dOb = bufs
    O = torch.empty_like(Qb); L = torch.empty(1, H, N, dtype=torch.float32, device="cuda")
    dQ, dK, dV = (torch.empty_like(Qb) for _ in range(3))
    first = synth.gaussian_inputs(N, d, sigma_qk=1.0, seed=90, heads=H)
    for b, t in zip(bufs, first):
        b.copy_(t)
    # warm-up on the capture stream, then capture
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        binding.sagebwd_fwd(Qb, Kb, Vb, p, ws, O, L)
        binding.sagebwd_bwd(Qb, Kb, Vb, O, dOb, L, p, ws, dQ, dK, dV)
    torch.cuda.current_stream().wait_stream(s)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        binding.sagebwd_fwd(Qb, Kb, Vb, p, ws, O, L)
        binding.sagebwd_bwd(Qb, Kb, Vb, O, dOb, L, p, ws, dQ, dK, dV)
    for seed in (91, 92, 93):
        ins = [t.cuda() for t in synth.gaussian_inputs(N, d, sigma_qk=1.0, seed=seed, heads=H)]
        for b, t in zip(bufs, ins):
            b.copy_(t)
        g.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (O, L, dQ, dK, dV)]
        # the same step eagerly, with its own buffers
        Oe, Le = binding.sagebwd_fwd(*ins[:3], p)
        ge = binding.sagebwd_bwd(ins[0], ins[1], ins[2], Oe, ins[3], Le, p)
        torch.cuda.synchronize()
        for a, b in zip(got, (Oe, Le) + tuple(ge)):
            assert torch.equal(a, b), seed


@pytest.mark.parametrize("heads,N,d", [(8, 512, 64), (16, 512, 64), (24, 512, 64), (48, 512, 64), (11, 512, 64),
                                       (32, 1024, 128), (64, 2048, 128), (32, 4096, 128)])
def test_workgroup_to_head_mappings_give_the_same_bits(heads, N, d):
    """The order in which workgroups take (head, work item) pairs depends on the head count and the
    sequence length (sets of 4, 2 or 1 heads per XCD, or the dense layout; 32 heads of N <= 4096 and 64
    heads of N = 2048 at d = 128 are the sets of four that the pre-training and outlier shapes launch
    with); whatever the order, every head must get exactly the result it gets when it is run alone."""
    Q, K, V, dO = (t.cuda() for t in synth.gaussian_inputs(N, d, sigma_qk=1.0, seed=100 + heads, heads=heads))
    p = binding.SageParams(1, heads, N, d, causal=True)
    O, L = binding.sagebwd_fwd(Q, K, V, p)
    dQ, dK, dV = binding.sagebwd_bwd(Q, K, V, O, dO, L, p)
    p1 = binding.SageParams(1, 1, N, d, causal=True)
    for h in sorted({0, 1, heads // 2, heads - 2, heads - 1}):
        sl = slice(h, h + 1)
        q, k, v, do = (t[:, sl].contiguous() for t in (Q, K, V, dO))
        O1, L1 = binding.sagebwd_fwd(q, k, v, p1)
        g1 = binding.sagebwd_bwd(q, k, v, O1, do, L1, p1)
        torch.cuda.synchronize()
        assert torch.equal(O1, O[:, sl]) and torch.equal(L1, L[:, sl]), h
        for a, b in zip(g1, (dQ, dK, dV)):
            assert torch.equal(a, b[:, sl]), h


@pytest.mark.parametrize("Nq,Nk,d,causal", [(64, 256, 64, True), (100, 228, 128, True), (192, 64, 64, False), (37, 300, 128, False),
                                            (1, 200, 64, False), (256, 1024, 128, True), (448, 64, 128, False), (320, 384, 128, True)])
def test_bwd_non_square(Nq, Nk, d, causal):
    """Q, dO of N_q rows against K, V of N_kv rows: dQ has N_q rows, dK and dV have N_kv; under the mask
    the last query sits on the last key (the diagonal tile of Q block i is KV block i + (N_kv - N_q) / 64)."""
    from test_gpu_fwd import non_square_inputs
    Q, K, V, dO = non_square_inputs(Nq, Nk, d, seed=5 * Nq + Nk)
    _bwd_case(Q, K, V, dO, binding.SageParams(1, 3, Nq, d, causal=causal, Nkv=Nk))


def test_bwd_non_square_q_smoothing_sharing_and_head_groups():
    from test_gpu_fwd import non_square_inputs
    Q, K, V, dO = non_square_inputs(128, 320, 128, seed=43, heads=4, q_offset=True)
    _bwd_case(Q, K, V, dO, binding.SageParams(1, 4, 128, 128, causal=True, q_smooth=True, Nkv=320))
    _bwd_case(Q, K, V, dO, binding.SageParams(1, 4, 128, 128, causal=False, q_smooth=True, Nkv=320))
    # two heads of dS scratch at a time; and the backward taking psi(Q), psi(K) from the forward
    _bwd_case(Q, K, V, dO, binding.SageParams(1, 4, 128, 128, causal=True, Nkv=320, scratch_budget=2 * 128 * (320 + 192)))
    Qd, Kd, Vd, dOd = (t.cuda() for t in (Q, K, V, dO))
    p = binding.SageParams(1, 4, 128, 128, causal=True, Nkv=320)
    ps = binding.SageParams(1, 4, 128, 128, causal=True, Nkv=320, share_quantized=True)
    O, L = binding.sagebwd_fwd(Qd, Kd, Vd, p)
    ref = binding.sagebwd_bwd(Qd, Kd, Vd, O, dOd, L, p)
    ws = binding.alloc_workspace(ps)
    Os, Ls = binding.sagebwd_fwd(Qd, Kd, Vd, ps, ws)
    got = binding.sagebwd_bwd(Qd, Kd, Vd, Os, dOd, Ls, ps, ws)
    torch.cuda.synchronize()
    assert torch.equal(O, Os) and torch.equal(L, Ls)
    for a, b in zip(ref, got):
        assert torch.equal(a, b)


BIG_BLOCKS = [(128, 64), (64, 128), (128, 128)]


@pytest.mark.parametrize("bq,bkv", BIG_BLOCKS)
@pytest.mark.parametrize("N,d,causal", [(128, 64, True), (256, 128, True), (320, 64, False), (448, 128, True), (576, 64, True),
                                        (640, 128, False), (100, 128, True), (333, 64, False), (200, 64, True)])
def test_bwd_numerics_blocks_of_128(bq, bkv, N, d, causal):
    """B_q, B_kv of 128: psi(P) and psi(dS) share one scale per B_q x B_kv block (the maxima over up to four of the
    kernel's tiles, those on or below the diagonal), psi(dO) and psi(Q) one per B_q rows, psi(K) one per B_kv."""
    Q, K, V, dO = synth.gaussian_inputs(N, d, sigma_qk=1.5, seed=N + d + bkv, heads=3)
    _bwd_case(Q, K, V, dO, binding.SageParams(1, 3, N, d, causal=causal, bq=bq, bkv=bkv))


@pytest.mark.parametrize("bq,bkv", BIG_BLOCKS)
def test_bwd_numerics_blocks_of_128_q_smoothing_non_square_head_groups(bq, bkv):
    from test_gpu_fwd import non_square_inputs
    Q, K, V, dO = non_square_inputs(192, 448, 128, seed=79, heads=4, q_offset=True)
    _bwd_case(Q, K, V, dO, binding.SageParams(1, 4, 192, 128, causal=True, q_smooth=True, Nkv=448, bq=bq, bkv=bkv))
    _bwd_case(Q, K, V, dO, binding.SageParams(1, 4, 192, 128, causal=False, q_smooth=True, Nkv=448, bq=bq, bkv=bkv,
                                              scratch_budget=2 * 192 * (448 + 192)))
    Q, K, V, dO = non_square_inputs(100, 300, 64, seed=80, heads=2)
    _bwd_case(Q, K, V, dO, binding.SageParams(1, 2, 100, 64, causal=False, k_smooth=False, Nkv=300, bq=bq, bkv=bkv))


@pytest.mark.parametrize("bq,bkv", BIG_BLOCKS)
def test_bwd_numerics_blocks_of_128_stored_ds_codes_and_scales(bq, bkv):
    """The stored psi(dS): one scale per numerics block (stored once per 64 x 64 tile), codes within one step
    of the oracle's."""
    N, d = 256, 64
    Q, K, V, dO = synth.gaussian_inputs(N, d, sigma_qk=1.5, seed=91, heads=1)
    p = binding.SageParams(1, 1, N, d, causal=True, bq=bq, bkv=bkv)
    Qn, Kn, Vn, dOn = (to_np(t)[0, 0] for t in (Q, K, V, dO))
    On, Ln = oracle.forward_head(Qn, Kn, Vn, True, bq=bq, bkv=bkv)
    inter = {}
    oracle.backward_head(Qn, Kn, Vn, On, dOn, Ln, True, intermediates=inter, bq=bq, bkv=bkv)
    ws = binding.alloc_workspace(p)
    Od = torch.from_numpy(On)[None, None].to(torch.bfloat16).cuda()
    Ld = torch.from_numpy(Ln)[None, None].cuda()
    binding.sagebwd_bwd(Q.cuda(), K.cuda(), V.cuda(), Od, dO.cuda(), Ld, p, ws)
    ds, sc = binding.sagebwd_export_ds(p, ws, 0)
    torch.cuda.synchronize()
    ds, sc = ds.cpu().numpy().astype(np.int32), sc.cpu().numpy()
    # every 64 x 64 tile of a numerics block on or below the diagonal carries the block's scale
    ref, rsc = inter["dSh"].astype(np.int32), inter["sdS"]
    nb = N // 64
    for i in range(nb):
        for j in range(i + 1):
            want = rsc[i // (bq // 64), j // (bkv // 64)]
            assert abs(sc[i, j] / want - 1) < 5e-6, (i, j, sc[i, j], want)
    assert ref.shape == ds.shape
    diff = np.abs(ds - ref)
    assert diff.max() <= 1, diff.max()
    assert (diff == 0).mean() > 0.999, (diff == 0).mean()
