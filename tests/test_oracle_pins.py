"""Pins for the CPU oracle: each test checks it against something other than
itself -- the exact (unquantised) attention and its finite-difference
gradients, closed forms, invariants stated in the paper, the values the paper
prints in its Table 1, an independently written tiled formulation and a
brute-force scalar transcription."""
import math
import os

import numpy as np
import pytest

import oracle
from oracle import tiled_form
from fpa_ref import cos_sim, fpa_backward, fpa_forward, rel_l2

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _bf(x):
    return oracle.round_to_bf16(x)


def _rand(N, d, sigma=1.0, seed=0, qk_norm=False):
    rng = np.random.default_rng(seed)
    Q = rng.standard_normal((N, d)) * sigma
    K = rng.standard_normal((N, d)) * sigma
    V = rng.standard_normal((N, d))
    dO = rng.standard_normal((N, d))
    if qk_norm:
        Q /= np.sqrt((Q ** 2).mean(1, keepdims=True) + 1e-6)
        K /= np.sqrt((K ** 2).mean(1, keepdims=True) + 1e-6)
    return _bf(Q), _bf(K), _bf(V), _bf(dO)


# ------------------------------------------------------------------ helpers
def test_round_to_bf16_matches_definition():
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: ties go to the even mantissa (1.0)
    assert oracle.round_to_bf16(np.float32(1 + 2 ** -8)) == np.float32(1.0)
    assert oracle.round_to_bf16(np.float32(1 + 2 ** -7 + 2 ** -8)) == np.float32(1 + 2 ** -6)
    assert oracle.round_to_bf16(np.float32(1 + 2 ** -8 + 2 ** -20)) == np.float32(1 + 2 ** -7)
    torch = pytest.importorskip("torch")
    x = np.random.default_rng(1).standard_normal(10000).astype(np.float32) * 37
    ref = torch.from_numpy(x).to(torch.bfloat16).float().numpy()
    assert np.array_equal(oracle.round_to_bf16(x), ref)


def test_qk_norm_closed_forms():
    """RMS normalisation (Sec. 4, QK-norm): a row of equal values maps to +-gamma / sqrt(1 + eps / v^2),
    a scaled row gives the same result (eps = 0), the mean square of the output is 1 (unit gain) up to
    the bf16 rounding, and torch's own rms_norm agrees to one bf16 step."""
    d = 64
    g = np.linspace(0.5, 2.0, d).astype(np.float32)
    X = np.full((3, d), 4.0, dtype=np.float32)
    X[1] = -0.5
    X[2, ::2] = -4.0
    y = oracle.qk_norm(X, g, eps=0.0)
    assert np.array_equal(y[0], _bf(g)) and np.array_equal(y[1], _bf(-g)) and np.array_equal(np.abs(y[2]), _bf(g))
    y = oracle.qk_norm(X, g, eps=1e-6)
    assert np.array_equal(y[1], _bf((-np.float32(1 / np.sqrt(0.25 + 1e-6)) * np.float32(0.5)) * g))
    rng = np.random.default_rng(90)
    Z = _bf(rng.standard_normal((200, d)) * 3)
    a, b = oracle.qk_norm(Z, g, eps=0.0), oracle.qk_norm(_bf(Z * 4), g, eps=0.0)     # x4 is exact in bf16
    assert np.array_equal(a, b)
    u = oracle.qk_norm(Z, np.ones(d), eps=0.0).astype(np.float64)
    assert np.abs((u ** 2).mean(axis=1) - 1).max() < 2 ** -7
    torch = pytest.importorskip("torch")
    ref = torch.nn.functional.rms_norm(torch.from_numpy(Z), (d,), torch.from_numpy(g), eps=1e-6).to(torch.bfloat16).float().numpy()
    got = oracle.qk_norm(Z, g, eps=1e-6)
    assert np.abs(got - ref).max() <= np.abs(ref).max() * 2 ** -7 and (got == ref).mean() > 0.99


# ------------------------------------------------------------- the quantiser
def test_quantiser_bound_and_extremes():
    # Sec. 3 "Quantization": |x - delta*q| <= delta/2 and the absmax element maps to +-127
    rng = np.random.default_rng(2)
    X = _bf(rng.standard_normal((256, 64)) * 3)
    q, s = oracle.quantize_blocks(X)
    assert q.dtype == np.int8 and s.dtype == np.float32 and s.shape == (4,)
    for b in range(4):
        xb = X[64 * b:64 * b + 64].astype(np.float64)
        qb = q[64 * b:64 * b + 64].astype(np.float64)
        a = np.abs(xb).max()
        assert math.isclose(float(s[b]), a / 127, rel_tol=1e-6)
        assert np.abs(xb - float(s[b]) * qb).max() <= float(s[b]) * (0.5 + 1e-4)
        i = np.unravel_index(np.abs(xb).argmax(), xb.shape)
        assert abs(qb[i]) == 127
        assert np.abs(qb).max() == 127


def test_quantiser_exact_roundtrip_on_grid():
    # values k * 2^e with |k| <= 127 and a +-127 present are represented exactly
    rng = np.random.default_rng(3)
    k = rng.integers(-127, 128, size=(128, 32))
    k[5, 7] = 127
    k[70, 3] = -127
    for e in (-6, 0, 3):
        X = (k * 2.0 ** e).astype(np.float32)
        q, s = oracle.quantize_blocks(X)
        assert np.array_equal(q.astype(np.int64), k)
        assert np.all(s == np.float32(2.0 ** e))
        assert np.array_equal(q.astype(np.float32) * np.repeat(s, 64)[:, None], X)


def test_quantiser_ties_round_to_even_and_zero_block():
    X = np.zeros((128, 4), dtype=np.float32)
    X[0, 0] = 127.0
    X[1, 0] = 0.5      # tie -> 0
    X[2, 0] = 1.5      # tie -> 2
    X[3, 0] = 2.5      # tie -> 2
    X[4, 0] = -3.5     # tie -> -4
    q, s = oracle.quantize_blocks(X)
    assert list(q[:5, 0]) == [127, 0, 2, 2, -4]
    assert s[0] == 1.0 and s[1] == 0.0 and not q[64:].any()


def test_key_mean_and_prepass_layout():
    rng = np.random.default_rng(4)
    Q, K, V, _ = _rand(128, 16, seed=4)
    K = _bf(K + 3.0)
    pp = oracle.prepass_head(Q, K, V, True, True)
    assert np.allclose(pp["muK"], K.mean(0), atol=1e-6)
    assert np.allclose(pp["muQ"][1], Q[64:].mean(0), atol=1e-6)
    # smoothing removes the channel offset before psi: scale is set by the centred data
    assert float(pp["sK"].max()) < float(np.abs(K).max()) / 127 * 0.8
    pp0 = oracle.prepass_head(Q, K, V, False, False)
    assert not pp0["muK"].any() and not pp0["muQ"].any()
    assert np.array_equal(pp0["Kh"], oracle.quantize_blocks(K)[0])


# ------------------------------------------- against exact attention (FPA)
@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("N,d", [(128, 64), (256, 128)])
def test_oracle_close_to_exact_attention(N, d, causal):
    """The method approximates O = softmax(QK^T/sqrt d) V and its gradients
    (Sec. 3) up to INT8 noise; a dropped scale, a transposed operand or a wrong
    sign in any of the seven matmuls leaves these bounds by a wide margin."""
    Q, K, V, dO = _rand(N, d, seed=10 + N + causal, qk_norm=True)
    sc = 1 / math.sqrt(d)
    O, L = oracle.forward_head(Q, K, V, causal=causal)
    dQ, dK, dV = oracle.backward_head(Q, K, V, O, dO, L, causal=causal)
    ref = fpa_backward(Q, K, V, dO, causal, sc)
    for name, got in (("O", O), ("dQ", dQ), ("dK", dK), ("dV", dV)):
        assert cos_sim(got, ref[name]) > 0.998, name
        assert rel_l2(got, ref[name]) < 0.07, name
    # L lives in the K-smoothed frame: L_true = L + sm_scale * Q mu_K  (row-shift invariance, Sec. 3)
    shift = sc * (Q.astype(np.float64) @ oracle.key_mean(K).astype(np.float64))
    assert np.abs(L + shift - ref["L"]).max() < 0.05


def test_exact_attention_gradients_by_finite_differences():
    """Validates the FPA helper itself (so the pin above is not circular):
    central differences of loss = sum(O o dO)."""
    Q, K, V, dO = _rand(64, 8, seed=5)
    Q, K, V, dO = (x.astype(np.float64) for x in (Q, K, V, dO))
    sc = 1 / math.sqrt(8)
    ref = fpa_backward(Q, K, V, dO, True, sc)
    rng = np.random.default_rng(6)
    eps = 1e-5
    for name, X in (("dQ", Q), ("dK", K), ("dV", V)):
        for _ in range(6):
            i, c = rng.integers(0, 64), rng.integers(0, 8)
            Xp, Xm = X.copy(), X.copy()
            Xp[i, c] += eps
            Xm[i, c] -= eps
            args_p = {"dQ": (Xp, K, V), "dK": (Q, Xp, V), "dV": (Q, K, Xp)}[name]
            args_m = {"dQ": (Xm, K, V), "dK": (Q, Xm, V), "dV": (Q, K, Xm)}[name]
            fp = (fpa_forward(*args_p, True, sc)[0] * dO).sum()
            fm = (fpa_forward(*args_m, True, sc)[0] * dO).sum()
            assert math.isclose((fp - fm) / (2 * eps), ref[name][i, c], rel_tol=1e-5, abs_tol=1e-8)


def test_oracle_gradients_vs_finite_differences_of_exact_attention():
    """Oracle gradients against finite differences of the exact loss directly
    (no analytic formula in between), on a tiny causal problem."""
    Q, K, V, dO = _rand(64, 16, seed=7, qk_norm=True)
    sc = 1 / math.sqrt(16)
    O, L = oracle.forward_head(Q, K, V, causal=True)
    dQ, dK, dV = oracle.backward_head(Q, K, V, O, dO, L, causal=True, return_raw=True)
    Q64, K64, V64, dO64 = (x.astype(np.float64) for x in (Q, K, V, dO))

    def loss(q, k, v):
        return (fpa_forward(q, k, v, True, sc)[0] * dO64).sum()

    eps = 1e-5
    fd = {n: np.zeros((64, 16)) for n in ("dQ", "dK", "dV")}
    for i in range(64):
        for c in range(16):
            for name, idx in (("dQ", 0), ("dK", 1), ("dV", 2)):
                a = [Q64.copy(), K64.copy(), V64.copy()]
                b = [Q64.copy(), K64.copy(), V64.copy()]
                a[idx][i, c] += eps
                b[idx][i, c] -= eps
                fd[name][i, c] = (loss(*a) - loss(*b)) / (2 * eps)
    for name, got in (("dQ", dQ), ("dK", dK), ("dV", dV)):
        assert cos_sim(got, fd[name]) > 0.998, name
        assert rel_l2(got, fd[name]) < 0.07, name


# ----------------------------------------------------- the paper's Table 1
def test_table1_sigma_sweep_matches_printed_values():
    """Paper Table 1 (Sec. 4, QK standard deviation study).  The table does not
    state its shape; N=1024, d=64, non-causal, K-smoothing on, averaged over four
    seeds, reproduces the rows sigma >= 3 to within a few percent.  At sigma = 1
    the oracle's gradient error is about 2.5x the printed one (O still agrees);
    that row is held to a looser band."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "table1_qk_sigma.txt")) if l.strip() and not l.startswith("#")]
    N, d = 1024, 64
    names = ("O", "dQ", "dK", "dV")
    for row in rows:
        sigma = float(row[0])
        paper = dict(zip(names, [(float(row[1 + 2 * i]), float(row[2 + 2 * i])) for i in range(4)]))
        acc = {n: [] for n in names}
        for s in range(4):
            Q, K, V, dO = _rand(N, d, sigma=sigma, seed=100 + 10 * int(sigma) + s)
            O, L = oracle.forward_head(Q, K, V, causal=False)
            dQ, dK, dV = oracle.backward_head(Q, K, V, O, dO, L, causal=False)
            ref = fpa_backward(Q, K, V, dO, False, 1 / math.sqrt(d))
            for name, got in zip(names, (O, dQ, dK, dV)):
                acc[name].append((cos_sim(got, ref[name]), rel_l2(got, ref[name])))
        for name in names:
            c, e = np.mean(acc[name], axis=0)
            pc, pe = paper[name]
            if sigma == 1:
                if name == "O":
                    assert abs(e - pe) < 0.25 * pe and c > 0.9997
                else:
                    assert pe * 0.8 < e < pe * 3.2 and c > 0.998
            else:
                band = 0.15 if sigma < 8 or name in ("O", "dV") else 0.2
                assert abs(e - pe) < band * pe, (sigma, name, e, pe)
                assert abs(c - pc) < max(0.001, 0.25 * (1 - pc)), (sigma, name, c, pc)


# ------------------------------------------------------------- invariants
def test_k_smoothing_softmax_invariance():
    # softmax(Q (K - 1 mu^T)^T) = softmax(Q K^T): checked on the exact attention,
    # then on the oracle: a constant added to every key leaves Kh, sK, O unchanged.
    Q, K, V, dO = _rand(128, 32, seed=8)
    mu = oracle.key_mean(K).astype(np.float64)
    O1, L1, _ = fpa_forward(Q, K, V, True, 0.2)
    O2, L2, _ = fpa_forward(Q, K.astype(np.float64) - mu, V, True, 0.2)
    assert np.allclose(O1, O2, atol=1e-12)
    assert np.allclose(L1, L2 + 0.2 * (Q.astype(np.float64) @ mu), atol=1e-10)
    # shift by a bf16-exact constant that keeps K bf16-representable: integers on an integer grid
    Ki = np.round(K * 8).astype(np.float32)
    shift = np.arange(32, dtype=np.float32)
    a = oracle.forward_head(Q, Ki, V, causal=True, sm_scale=0.01)
    b = oracle.forward_head(Q, Ki + shift, V, causal=True, sm_scale=0.01)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    # without smoothing the shift changes the quantised keys
    c = oracle.prepass_head(Q, Ki + shift, V, k_smooth=False)
    assert not np.array_equal(c["Kh"], oracle.prepass_head(Q, Ki, V, k_smooth=False)["Kh"])


def test_ds_rows_sum_to_zero_and_rms_bound():
    """Ablation section: each row of dS sums to 0 (so dS K = dS K^sm); App. B:
    RMS(dS) <= max_i ||dP_i - delta_i||_inf / sqrt(N).  Checked on the oracle's
    own unquantised intermediates, with delta from its unrounded O."""
    N, d = 256, 32
    Q, K, V, dO = _rand(N, d, seed=9)
    Ob, L, Oraw, Lraw = oracle.forward_head(Q, K, V, causal=False, return_raw=True)
    inter = {}
    oracle.backward_head(Q, K, V, Oraw, dO, Lraw, causal=False, intermediates=inter)
    P, dP, dS = inter["P"], inter["dP"], inter["dS"]
    # rows of P sum to 1 up to the per-token quantisation of P~ in the forward's O only -> exact here
    assert np.abs(P.sum(1) - 1).max() < 1e-6          # L is stored in float32
    # delta uses the INT8 forward output, so rows of dS sum to ~0 up to that noise
    assert np.abs(dS.sum(1)).max() < 0.05 * np.abs(dS).sum(1).max()
    delta = oracle.delta_rows(dO, Oraw)
    bound = np.abs(dP - delta[:, None]).max() / math.sqrt(N)
    rms = math.sqrt((dS ** 2).mean())
    assert rms <= bound
    # with the exact delta the row sums vanish to rounding, and dS K = dS K^sm
    ref = fpa_backward(Q, K, V, dO, False, 1 / math.sqrt(d))
    assert np.abs(ref["dS"].sum(1)).max() < 1e-12
    Ksm = K.astype(np.float64) - K.astype(np.float64).mean(0)
    assert np.allclose(ref["dS"] @ K, ref["dS"] @ Ksm, atol=1e-10)


def test_q_smoothing_decomposition():
    """Sec. 3 decomposition and the dK bias branch of the ablation section:
    with Q-smoothing the oracle still approximates exact attention, and
    dK = dS^T Q^sm + (dS^T 1) mu_Q^T holds exactly for the exact dS."""
    N, d = 256, 64
    Q, K, V, dO = _rand(N, d, seed=11)
    Q = _bf(Q + np.linspace(-2, 2, d)[None, :])      # channel offsets that Q-smoothing removes
    sc = 1 / math.sqrt(d)
    ref = fpa_backward(Q, K, V, dO, True, sc)
    muQ = np.repeat(oracle.block_mean(Q).astype(np.float64), 64, axis=0)
    Qsm = Q.astype(np.float64) - muQ
    dK_center = ref["dS"].T @ Qsm * sc
    dK_bias = np.zeros_like(dK_center)
    for I in range(N // 64):
        sl = slice(64 * I, 64 * I + 64)
        dK_bias += np.outer(ref["dS"][sl].sum(0), muQ[64 * I]) * sc
    assert np.allclose(dK_center + dK_bias, ref["dK"], atol=1e-10)
    O, L = oracle.forward_head(Q, K, V, causal=True, q_smooth=True)
    dQ, dK, dV = oracle.backward_head(Q, K, V, O, dO, L, causal=True, q_smooth=True)
    for name, got in (("O", O), ("dQ", dQ), ("dK", dK), ("dV", dV)):
        assert cos_sim(got, ref[name]) > 0.998, name
        assert rel_l2(got, ref[name]) < 0.07, name
    # dropping the bias branch would be visible: the centred branch alone is far off
    assert rel_l2(dK_center, ref["dK"]) > 0.2


# ----------------------------------------------------------- closed forms
@pytest.mark.parametrize("causal", [True, False])
def test_zero_queries_closed_form(causal):
    """Q = 0 => S = 0, every P^ = 127, O_i = mean of the dequantised visible V
    rows, L_i = log(#visible keys)."""
    N, d = 192, 16
    _, K, V, _ = _rand(N, d, seed=12)
    Q = np.zeros((N, d), dtype=np.float32)
    O, L, Oraw, Lraw = oracle.forward_head(Q, K, V, causal=causal, return_raw=True)
    Vh, sV = oracle.quantize_blocks(V)
    Vdq = Vh.astype(np.float64) * np.repeat(sV.astype(np.float64), 64)[:, None]
    for i in (0, 1, 63, 64, 100, 191):
        nvis = i + 1 if causal else N
        assert math.isclose(Lraw[i], math.log(nvis), abs_tol=1e-12)
        assert np.allclose(Oraw[i], Vdq[:nvis].mean(0), atol=1e-12)
    assert np.array_equal(O, oracle.round_to_bf16(Oraw))


def test_one_hot_limit():
    """One logit far above the rest in every row => O_i = s_V * V^[argmax]."""
    N, d = 128, 16
    rng = np.random.default_rng(13)
    V = _bf(rng.standard_normal((N, d)))
    # orthogonal one-hot codes: query i matches key perm[i] only
    perm = rng.permutation(N)
    K = np.zeros((N, N), dtype=np.float32)
    K[np.arange(N), np.arange(N)] = 1.0
    Q = np.zeros((N, N), dtype=np.float32)
    Q[np.arange(N), perm] = 1.0
    Vp = np.zeros((N, N), dtype=np.float32)
    Vp[:, :d] = V
    O, L, Oraw, _ = oracle.forward_head(Q, K, Vp, causal=False, k_smooth=False, sm_scale=200.0, return_raw=True)
    Vh, sV = oracle.quantize_blocks(Vp)
    Vdq = Vh.astype(np.float64) * np.repeat(sV.astype(np.float64), 64)[:, None]
    assert np.allclose(Oraw, Vdq[perm], atol=1e-12)


# ------------------------------------------ two formulations, brute force
@pytest.mark.parametrize("bq,bkv", [(64, 64), (128, 64), (128, 128), (64, 128)])
@pytest.mark.parametrize("causal,q_smooth", [(True, False), (False, False), (True, True), (False, True)])
def test_non_tiled_oracle_equals_tiled_formulation(causal, q_smooth, bq, bkv):
    """oracle/tiled_form.py shares no code with the oracle (own smoothing, own psi, own delta,
    online softmax, KV-outer backward): the two must agree.  Covers the Q-smoothing bias of the
    logits and the dK bias branch, and the block sizes Algorithm 1 leaves free."""
    N, d = 256, 32
    Q, K, V, dO = _rand(N, d, seed=14 + bq + 2 * bkv, qk_norm=True)
    if q_smooth:
        Q = _bf(Q + np.linspace(-1.5, 1.5, d)[None, :])
    kw = dict(causal=causal, q_smooth=q_smooth, bq=bq, bkv=bkv)
    Ob, L, Oraw, Lraw = oracle.forward_head(Q, K, V, return_raw=True, **kw)
    O2, L2 = tiled_form.forward_tiled(Q, K, V, **kw)
    assert np.abs(Lraw - L2).max() < 1e-12
    # P~/s_P against 127*exp(S - rowmax): identical up to a handful of rounding-boundary codes
    assert rel_l2(O2, Oraw) < 2e-4
    dQ, dK, dV = oracle.backward_head(Q, K, V, Ob, dO, L, return_raw=True, **kw)
    dQ2, dK2, dV2 = tiled_form.backward_tiled(Q, K, V, Ob, dO, L, **kw)
    for a, b in ((dQ, dQ2), (dK, dK2), (dV, dV2)):
        assert np.allclose(a, b, rtol=1e-10, atol=1e-12)


def test_tiled_formulation_has_its_own_prepass():
    """The second formulation imports nothing from the oracle (so that agreement means two
    implementations), and its smoothing and quantiser give the oracle's bits."""
    import ast
    import inspect
    tree = ast.parse(inspect.getsource(tiled_form))
    mods = [n.module or "" for n in ast.walk(tree) if isinstance(n, ast.ImportFrom)] + \
           [a.name for n in ast.walk(tree) if isinstance(n, ast.Import) for a in n.names]
    assert all("oracle" not in m and not m.startswith(".") and m != "" for m in mods), mods
    Q, K, V, _ = _rand(256, 32, seed=21)
    Q = _bf(Q + 0.7)
    K = _bf(K - 2.0)
    pre = tiled_form._Prepared(Q, K, V, True, True, 128, 64)
    pp = oracle.prepass_head(Q, K, V, True, True, 128, 64)
    assert np.array_equal(pre.mu_k, pp["muK"]) and np.array_equal(np.stack(pre.mu_q), pp["muQ"])
    for mine, codes, scales in ((pre.q_codes, "Qh", "sQ"), (pre.k_codes, "Kh", "sK"), (pre.v_codes, "Vh", "sV")):
        assert np.array_equal(np.concatenate(mine), pp[codes].astype(np.float64))
    assert np.array_equal(np.array(pre.q_scale), pp["sQ"]) and np.array_equal(np.array(pre.k_scale), pp["sK"])


def test_kv_block_permutation_invariance():
    """Non-causal: permuting whole KV blocks (with K-smoothing the mean is
    unchanged) permutes nothing in O and L except float summation order."""
    N, d = 256, 32
    Q, K, V, _ = _rand(N, d, seed=15)
    perm = np.concatenate([np.arange(64 * b, 64 * b + 64) for b in (2, 0, 3, 1)])
    a = oracle.forward_head(Q, K, V, causal=False, return_raw=True)
    b = oracle.forward_head(Q, K[perm], V[perm], causal=False, return_raw=True)
    assert np.allclose(a[2], b[2], rtol=1e-12, atol=1e-14)
    assert np.allclose(a[3], b[3], rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("causal,q_smooth", [(True, False), (False, False), (True, True), (False, True)])
def test_brute_force_scalar_transcription(causal, q_smooth):
    """Every step re-done with Python scalars on a 128 x 8 problem: K-smoothing, optional
    Q-smoothing (block means, the mu_Qi K^sm bias of the logits, the (dS^T 1) mu_Q^T branch of dK:
    Sec. 3 decomposition and the dK_bias equation of the ablation section), with and without the
    causal mask."""
    N, d = 128, 8
    Q, K, V, dO = _rand(N, d, seed=16 + 2 * causal + q_smooth)
    if q_smooth:
        Q = _bf(Q + np.linspace(-2, 2, d)[None, :])
    sc = 1 / math.sqrt(d)
    f32 = np.float32
    nb = N // 64
    muK = [f32(sum(float(K[n, c]) for n in range(N)) / N) for c in range(d)]
    Ksm = [[f32(K[n, c] - muK[c]) for c in range(d)] for n in range(N)]
    muQ = [[f32(sum(float(Q[n, c]) for n in range(64 * b, 64 * b + 64)) / 64) if q_smooth else f32(0) for c in range(d)]
           for b in range(nb)]
    Qsm = [[f32(Q[n, c] - muQ[n // 64][c]) if q_smooth else Q[n, c] for c in range(d)] for n in range(N)]
    vis = (lambda i, k: k <= i) if causal else (lambda i, k: True)

    def psi(rows):
        a = max(abs(float(x)) for r in rows for x in r)
        a = f32(a)
        r_ = f32(127.0) / a
        q = [[int(np.rint(f32(f32(x) * r_))) for x in r] for r in rows]
        return q, f32(a / f32(127.0))

    Qh, sQ, Kh, sK, Vh, sV, dOh, sdO = [], [], [], [], [], [], [], []
    for b in range(nb):
        for lst, sl, src in ((Qh, sQ, Qsm), (Kh, sK, Ksm), (Vh, sV, V), (dOh, sdO, dO)):
            q, s = psi([list(src[n]) for n in range(64 * b, 64 * b + 64)])
            lst.extend(q)
            sl.append(s)

    def logit(i, k):
        s = sum(Qh[i][c] * Kh[k][c] for c in range(d)) * float(sQ[i // 64]) * float(sK[k // 64]) * sc
        if q_smooth:
            s += sc * sum(float(muQ[i // 64][c]) * float(Ksm[k][c]) for c in range(d))
        return s

    S = [[logit(i, k) if vis(i, k) else -math.inf for k in range(N)] for i in range(N)]
    O = np.zeros((N, d))
    Lr = np.zeros(N)
    for i in range(N):
        m = max(S[i])
        l = sum(math.exp(s - m) for s in S[i])
        Lr[i] = m + math.log(l)
        for j in range(nb):
            ks = range(64 * j, 64 * j + 64)
            if not any(vis(i, k) for k in ks):
                continue
            M = max(S[i][k] for k in ks)
            ph = [int(np.rint(f32(f32(math.exp(S[i][k] - M)) * f32(127.0)))) for k in ks]
            w = math.exp(M - m) / 127.0 * float(sV[j]) / l
            for c in range(d):
                O[i, c] += w * sum(ph[t] * Vh[64 * j + t][c] for t in range(64))
    kw = dict(causal=causal, q_smooth=q_smooth)
    Ob, L, Oraw, Lraw = oracle.forward_head(Q, K, V, return_raw=True, **kw)
    assert np.allclose(Oraw, O, rtol=1e-11, atol=1e-13) and np.allclose(Lraw, Lr, atol=1e-12)
    # backward
    delta = [sum(float(dO[i, c]) * float(Ob[i, c]) for c in range(d)) for i in range(N)]
    dQ = np.zeros((N, d)); dK = np.zeros((N, d)); dV = np.zeros((N, d))
    for I in range(nb):
        for J in range(nb):
            if causal and J > I:
                continue
            P = [[math.exp(S[i][k] - float(L[i])) if vis(i, k) else 0.0 for k in range(64 * J, 64 * J + 64)]
                 for i in range(64 * I, 64 * I + 64)]
            dS = [[P[a][b] * (sum(float(dO[64 * I + a, c]) * float(V[64 * J + b, c]) for c in range(d)) - delta[64 * I + a])
                   for b in range(64)] for a in range(64)]
            Ph, sP = psi(P)
            dSh, sdS = psi(dS)
            for b in range(64):
                col = sum(dS[a][b] for a in range(64))
                for c in range(d):
                    dV[64 * J + b, c] += float(sP) * float(sdO[I]) * sum(Ph[a][b] * dOh[64 * I + a][c] for a in range(64))
                    dK[64 * J + b, c] += sc * float(sdS) * float(sQ[I]) * sum(dSh[a][b] * Qh[64 * I + a][c] for a in range(64))
                    if q_smooth:
                        dK[64 * J + b, c] += sc * col * float(muQ[I][c])
            for a in range(64):
                for c in range(d):
                    dQ[64 * I + a, c] += sc * float(sdS) * float(sK[J]) * sum(dSh[a][b] * Kh[64 * J + b][c] for b in range(64))
    g = oracle.backward_head(Q, K, V, Ob, dO, L, return_raw=True, **kw)
    for a, b in zip(g, (dQ, dK, dV)):
        assert np.allclose(a, b, rtol=1e-9, atol=1e-12)
    if q_smooth:
        # the bias terms are not negligible here: without them the comparison above would fail
        g0 = oracle.backward_head(Q, K, V, Ob, dO, L, return_raw=True, causal=causal, q_smooth=False)
        assert rel_l2(g0[1], dK) > 1e-3


# ------------------------------------------- block sampling (used by the full-size GPU tests)
@pytest.mark.parametrize("bq,bkv", [(64, 64), (128, 64)])
@pytest.mark.parametrize("causal,q_smooth", [(True, False), (False, False), (True, True), (False, True)])
def test_sampled_blocks_equal_the_full_run(causal, q_smooth, bq, bkv):
    """forward_head(q_blocks=) and backward_head(q_blocks= / kv_blocks=) restrict the work to some
    blocks; the rows they claim to complete must be the rows of the full run (N = 512: several
    blocks on either side of every sampled one, so a wrong column offset or key index shows)."""
    N, d = 512, 32
    Q, K, V, dO = _rand(N, d, seed=60 + causal + 2 * q_smooth, qk_norm=True)
    if q_smooth:
        Q = _bf(Q + np.linspace(-1, 1, d)[None, :])
    kw = dict(causal=causal, q_smooth=q_smooth, bq=bq, bkv=bkv)
    Ob, L, Oraw, Lraw = oracle.forward_head(Q, K, V, return_raw=True, **kw)
    qb = [0, 2, N // bq - 1]
    rows = np.concatenate([np.arange(bq * i, bq * i + bq) for i in qb])
    other = np.setdiff1d(np.arange(N), rows)
    Os, Ls, Osr, Lsr = oracle.forward_head(Q, K, V, return_raw=True, q_blocks=qb, **kw)
    assert np.abs(Osr[rows] - Oraw[rows]).max() <= 1e-12 and np.abs(Lsr[rows] - Lraw[rows]).max() <= 1e-12
    assert np.array_equal(Os[rows], Ob[rows]) and not Osr[other].any()
    full = oracle.backward_head(Q, K, V, Ob, dO, L, return_raw=True, **kw)
    part = oracle.backward_head(Q, K, V, Ob, dO, L, return_raw=True, q_blocks=qb, **kw)
    assert np.abs(part[0][rows] - full[0][rows]).max() <= 1e-12 * max(1.0, np.abs(full[0]).max())
    assert not part[0][other].any()
    kb = [1, 3, N // bkv - 2]
    krows = np.concatenate([np.arange(bkv * j, bkv * j + bkv) for j in kb])
    kother = np.setdiff1d(np.arange(N), krows)
    part = oracle.backward_head(Q, K, V, Ob, dO, L, return_raw=True, kv_blocks=kb, **kw)
    for x, y in ((part[1], full[1]), (part[2], full[2])):
        assert np.abs(x[krows] - y[krows]).max() <= 1e-12 * max(1.0, np.abs(y).max())
        assert not x[kother].any()
    # both at once: only the tiles in (q_blocks x kv_blocks) are visited; dV of a sampled KV block
    # then holds exactly the share of the sampled Q blocks
    both = oracle.backward_head(Q, K, V, Ob, dO, L, return_raw=True, q_blocks=qb, kv_blocks=kb, **kw)
    inter = {}
    oracle.backward_head(Q, K, V, Ob, dO, L, intermediates=inter, **kw)
    share = np.zeros((N, d))
    dOh, sdO = oracle.quantize_blocks(dO, bq)
    for I in qb:
        for J in kb:
            P = inter["P"][bq * I:bq * I + bq, bkv * J:bkv * J + bkv]
            a = np.float32(np.abs(P.astype(np.float32)).max())
            if a > 0:
                Ph = np.rint((P.astype(np.float32) * (np.float32(127) / a)).astype(np.float32)).astype(np.float64)
                share[bkv * J:bkv * J + bkv] += float(np.float32(a / np.float32(127))) * float(sdO[I]) * (Ph.T @ dOh[bq * I:bq * I + bq].astype(np.float64))
    assert np.allclose(both[2], share, rtol=1e-10, atol=1e-13)


def test_sampling_pin_catches_a_wrong_column_offset(monkeypatch):
    """The pin above is sharp: an oracle whose sampled-KV path reads the wrong keys (planted here on
    the CPU: the key index list shifted by one block) disagrees with the full run."""
    N, d = 512, 32
    Q, K, V, dO = _rand(N, d, seed=61, qk_norm=True)
    Ob, L = oracle.forward_head(Q, K, V, causal=False)
    full = oracle.backward_head(Q, K, V, Ob, dO, L, causal=False, return_raw=True)
    from oracle import sage_oracle
    good = sage_oracle._logits_block

    def shifted(pp, i0, n_keys, sm_scale, q_smooth, key_idx=None):
        if key_idx is not None:
            key_idx = (np.asarray(key_idx) + 64) % n_keys
        return good(pp, i0, n_keys, sm_scale, q_smooth, key_idx)

    monkeypatch.setattr(sage_oracle, "_logits_block", shifted)
    bad = oracle.backward_head(Q, K, V, Ob, dO, L, causal=False, return_raw=True, kv_blocks=[1, 3])
    krows = np.concatenate([np.arange(64 * j, 64 * j + 64) for j in (1, 3)])
    assert np.abs(bad[1][krows] - full[1][krows]).max() > 1e-3 * np.abs(full[1]).max()


# ------------------------------------------- non-square attention (N_q != N_kv)
@pytest.mark.parametrize("Nq,Nk,causal", [(64, 256, True), (100, 228, True), (192, 64, False), (37, 300, False), (1, 200, False)])
def test_non_square_close_to_exact_attention(Nq, Nk, causal):
    """Q of N_q rows against K, V of N_kv rows (cross attention, chunked prefill, decoding): the oracle
    still approximates exact attention; under the mask the last query sees every key."""
    d = 64
    rng = np.random.default_rng(80 + Nq + Nk)
    Q, dO = (_bf(rng.standard_normal((Nq, d))) for _ in range(2))
    K, V = (_bf(rng.standard_normal((Nk, d))) for _ in range(2))
    sc = 1 / math.sqrt(d)
    O, L = oracle.forward_head(Q, K, V, causal=causal)
    dQ, dK, dV = oracle.backward_head(Q, K, V, O, dO, L, causal=causal)
    assert O.shape == dQ.shape == (Nq, d) and L.shape == (Nq,) and dK.shape == dV.shape == (Nk, d)
    ref = fpa_backward(Q, K, V, dO, causal, sc)
    for name, got in (("O", O), ("dQ", dQ), ("dK", dK), ("dV", dV)):
        assert cos_sim(got, ref[name]) > 0.997, name
        assert rel_l2(got, ref[name]) < 0.08, name
    shift = sc * (Q.astype(np.float64) @ oracle.key_mean(K).astype(np.float64))
    assert np.abs(L + shift - ref["L"]).max() < 0.05


@pytest.mark.parametrize("q_smooth", [False, True])
def test_non_square_reduces_to_the_square_oracle(q_smooth):
    """Rows of the attention matrix are independent given K and V, so a block-aligned subset of the
    queries must give exactly the rows the square problem gives: the first rows without the mask, the
    last rows with it (last query on last key).  The backward agrees as well when the upstream gradient
    of the other rows is zero (their psi(dO) blocks are all-zero blocks, which contribute nothing)."""
    N, d = 320, 32
    Q, K, V, dO = _rand(N, d, seed=85, qk_norm=True)
    if q_smooth:
        Q = _bf(Q + np.linspace(-1, 1, d)[None, :])
    for causal, rows in ((False, slice(0, 128)), (False, slice(0, 64)), (True, slice(192, 320)), (True, slice(256, 320))):
        kw = dict(causal=causal, q_smooth=q_smooth)
        Ob, L, Oraw, Lraw = oracle.forward_head(Q, K, V, return_raw=True, **kw)
        Os, Ls, Osr, Lsr = oracle.forward_head(Q[rows], K, V, return_raw=True, **kw)
        assert np.array_equal(Osr, Oraw[rows]) and np.array_equal(Lsr, Lraw[rows])
        dOz = np.zeros_like(dO)
        dOz[rows] = dO[rows]
        full = oracle.backward_head(Q, K, V, Ob, dOz, L, return_raw=True, **kw)
        part = oracle.backward_head(Q[rows], K, V, Ob[rows], dO[rows], L[rows], return_raw=True, **kw)
        assert np.array_equal(part[0], full[0][rows])
        assert np.allclose(part[1], full[1], rtol=1e-12, atol=1e-15) and np.allclose(part[2], full[2], rtol=1e-12, atol=1e-15)
        assert not np.delete(full[0], np.arange(N)[rows], axis=0).any()


@pytest.mark.parametrize("causal", [True, False])
def test_non_square_zero_queries_closed_form_and_tiled_formulation(causal):
    Nq, Nk, d = 128, 320, 16
    rng = np.random.default_rng(86)
    K, V = (_bf(rng.standard_normal((Nk, d))) for _ in range(2))
    Z = np.zeros((Nq, d), dtype=np.float32)
    _, _, Oraw, Lraw = oracle.forward_head(Z, K, V, causal=causal, return_raw=True)
    Vh, sV = oracle.quantize_blocks(V)
    Vdq = Vh.astype(np.float64) * np.repeat(sV.astype(np.float64), 64)[:, None]
    for i in (0, 63, 64, 127):
        nvis = i + 1 + (Nk - Nq) if causal else Nk
        assert math.isclose(Lraw[i], math.log(nvis), abs_tol=1e-12)
        assert np.allclose(Oraw[i], Vdq[:nvis].mean(0), atol=1e-12)
    Q, dO = (_bf(rng.standard_normal((Nq, d))) for _ in range(2))
    Ob, L, Oraw, Lraw = oracle.forward_head(Q, K, V, causal=causal, return_raw=True)
    O2, L2 = tiled_form.forward_tiled(Q, K, V, causal=causal)
    assert np.abs(Lraw - L2).max() < 1e-12 and rel_l2(O2, Oraw) < 2e-4
    g = oracle.backward_head(Q, K, V, Ob, dO, L, causal=causal, return_raw=True)
    g2 = tiled_form.backward_tiled(Q, K, V, Ob, dO, L, causal=causal)
    for a, b in zip(g, g2):
        assert np.allclose(a, b, rtol=1e-10, atol=1e-12)


# ------------------------------------------- other numerics block sizes (Algorithm 1 leaves B_q, B_kv free)
@pytest.mark.parametrize("bq,bkv", [(128, 64), (128, 128), (64, 128)])
def test_larger_blocks_quantiser_and_prepass(bq, bkv):
    rng = np.random.default_rng(70)
    X = _bf(rng.standard_normal((256, 16)) * 2)
    q, s = oracle.quantize_blocks(X, bq)
    assert s.shape == (256 // bq,)
    for b in range(256 // bq):
        xb = X[bq * b:bq * b + bq].astype(np.float64)
        assert s[b] == np.float32(np.float32(np.abs(xb).max()) / np.float32(127))
        assert np.abs(q[bq * b:bq * b + bq]).max() == 127
        assert np.abs(xb - float(s[b]) * q[bq * b:bq * b + bq]).max() <= float(s[b]) * (0.5 + 1e-4)
    Q, K, V, _ = _rand(256, 16, seed=71)
    pp = oracle.prepass_head(Q, K, V, True, True, bq, bkv)
    assert pp["sQ"].shape == (256 // bq,) and pp["sK"].shape == (256 // bkv,) and pp["muQ"].shape == (256 // bq, 16)
    assert np.allclose(pp["muQ"][1], Q[bq:2 * bq].mean(0), atol=1e-6)
    # a scale shared by more rows is the maximum of the 64-row scales
    s64 = oracle.quantize_blocks(K - pp["muK"], 64)[1]
    assert np.array_equal(pp["sK"], s64.reshape(-1, bkv // 64).max(axis=1))


@pytest.mark.parametrize("bq,bkv", [(128, 64), (128, 128), (64, 128)])
@pytest.mark.parametrize("causal", [True, False])
def test_larger_blocks_close_to_exact_attention_and_closed_forms(bq, bkv, causal):
    N, d = 256, 64
    Q, K, V, dO = _rand(N, d, seed=72 + causal, qk_norm=True)
    sc = 1 / math.sqrt(d)
    O, L = oracle.forward_head(Q, K, V, causal=causal, bq=bq, bkv=bkv)
    dQ, dK, dV = oracle.backward_head(Q, K, V, O, dO, L, causal=causal, bq=bq, bkv=bkv)
    ref = fpa_backward(Q, K, V, dO, causal, sc)
    for name, got in (("O", O), ("dQ", dQ), ("dK", dK), ("dV", dV)):
        assert cos_sim(got, ref[name]) > 0.997, name
        assert rel_l2(got, ref[name]) < 0.08, name
    # Q = 0: every P^ = 127 and O_i is the mean of the dequantised visible V rows, whatever the blocks
    Z = np.zeros_like(Q)
    _, _, Oraw, Lraw = oracle.forward_head(Z, K, V, causal=causal, bq=bq, bkv=bkv, return_raw=True)
    Vh, sV = oracle.quantize_blocks(V, bkv)
    Vdq = Vh.astype(np.float64) * np.repeat(sV.astype(np.float64), bkv)[:, None]
    for i in (0, 63, 64, 127, 128, 255):
        nvis = i + 1 if causal else N
        assert math.isclose(Lraw[i], math.log(nvis), abs_tol=1e-12)
        assert np.allclose(Oraw[i], Vdq[:nvis].mean(0), atol=1e-12)
    # a partial last block with the larger blocks: N = 200 rounds up to 256
    Q2, K2, V2, dO2 = _rand(200, d, seed=74, qk_norm=True)
    O2, L2 = oracle.forward_head(Q2, K2, V2, causal=causal, bq=bq, bkv=bkv)
    g2 = oracle.backward_head(Q2, K2, V2, O2, dO2, L2, causal=causal, bq=bq, bkv=bkv)
    ref2 = fpa_backward(Q2, K2, V2, dO2, causal, sc)
    for name, got in zip(("O", "dQ", "dK", "dV"), (O2,) + g2):
        assert got.shape == (200, d) and rel_l2(got, ref2[name]) < 0.08, name


# ------------------------------------------- sequence lengths that are not a multiple of 64
@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("N,d", [(100, 64), (37, 64), (200, 128)])
def test_partial_last_block_close_to_exact_attention(N, d, causal):
    """A partial last block (its missing rows do not exist) still approximates exact attention
    on the N tokens that do: a missing key mask, a mean or an absmax taken over appended rows,
    or gradients leaking into them would leave these bounds."""
    Q, K, V, dO = _rand(N, d, seed=40 + N + causal, qk_norm=True)
    sc = 1 / math.sqrt(d)
    O, L = oracle.forward_head(Q, K, V, causal=causal)
    dQ, dK, dV = oracle.backward_head(Q, K, V, O, dO, L, causal=causal)
    assert O.shape == (N, d) and L.shape == (N,) and dQ.shape == dK.shape == dV.shape == (N, d)
    ref = fpa_backward(Q, K, V, dO, causal, sc)
    for name, got in (("O", O), ("dQ", dQ), ("dK", dK), ("dV", dV)):
        assert cos_sim(got, ref[name]) > 0.998, name
        assert rel_l2(got, ref[name]) < 0.07, name
    shift = sc * (Q.astype(np.float64) @ oracle.key_mean(K).astype(np.float64))
    assert np.abs(L + shift - ref["L"]).max() < 0.05


@pytest.mark.parametrize("causal", [True, False])
def test_partial_last_block_zero_queries_closed_form(causal):
    """Q = 0 with N = 150: L_i = log(#visible keys that exist) and O_i is the mean of the
    dequantised V rows over exactly those keys (the scale of the partial block comes from its
    22 rows alone)."""
    N, d = 150, 16
    _, K, V, _ = _rand(N, d, seed=41)
    Q = np.zeros((N, d), dtype=np.float32)
    O, L, Oraw, Lraw = oracle.forward_head(Q, K, V, causal=causal, return_raw=True)
    Vh, sV = oracle.quantize_blocks(oracle.pad_rows(V, 192))
    assert sV[2] == np.float32(np.abs(V[128:]).max()) / np.float32(127.0)
    Vdq = (Vh.astype(np.float64) * np.repeat(sV.astype(np.float64), 64)[:, None])[:N]
    for i in (0, 63, 64, 127, 128, 149):
        nvis = i + 1 if causal else N
        assert math.isclose(Lraw[i], math.log(nvis), abs_tol=1e-12)
        assert np.allclose(Oraw[i], Vdq[:nvis].mean(0), atol=1e-12)


def test_partial_last_block_means_and_prefix_property():
    """mu_K runs over the N tokens that exist, mu_Q of the partial block over its own rows; and
    under the causal mask (K-smoothing off, so that nothing couples the rows) the first 64 query
    rows of an N = 100 problem equal those of the N = 64 problem on the same leading tokens."""
    N, d = 100, 32
    Q, K, V, dO = _rand(N, d, seed=42)
    pp = oracle.prepass_head(Q, K, V, True, True)
    assert np.array_equal(pp["muK"], (K.astype(np.float64).sum(0) / 100.0).astype(np.float32))
    assert np.array_equal(pp["muQ"][1], (Q[64:].astype(np.float64).sum(0) / 36.0).astype(np.float32))
    assert not pp["Kh"][100:].any() and not pp["Qh"][100:].any() and not pp["Vh"][100:].any()
    O, L = oracle.forward_head(Q, K, V, causal=True, k_smooth=False)
    O64, L64 = oracle.forward_head(Q[:64], K[:64], V[:64], causal=True, k_smooth=False)
    assert np.array_equal(O[:64], O64) and np.array_equal(L[:64], L64)


def test_intermediate_error_ordering_follows_the_paper():
    """The paper's trace of intermediate tensors (Sec. 5 "Tracing intermediate tensor error", its
    Table 2) on a trained layer cannot be reproduced without the checkpoint, but its structure can:
    dP is exact (both operands stay unquantised), dS is the least accurate intermediate, and the
    gradients downstream of dS (dQ, dK) are less accurate than O and dV.  Gaussian Q, K of standard
    deviation 5 put the errors in the range the table shows (rel-l2 of dS about 0.2)."""
    N, d, sc = 512, 64, 1 / math.sqrt(64)
    err = {k: [] for k in ("P", "dP", "dS", "O", "dQ", "dK", "dV")}
    for seed in (50, 51):
        Q, K, V, dO = _rand(N, d, sigma=5.0, seed=seed)
        O, L = oracle.forward_head(Q, K, V, causal=False)
        inter = {}
        dQ, dK, dV = oracle.backward_head(Q, K, V, O, dO, L, causal=False, intermediates=inter)
        ref = fpa_backward(Q, K, V, dO, False, sc)
        got = dict(P=inter["P"], dP=inter["dP"], dS=inter["dS"], O=O, dQ=dQ, dK=dK, dV=dV)
        for k in err:
            err[k].append(rel_l2(got[k], ref[k]))
    e = {k: float(np.mean(v)) for k, v in err.items()}
    assert e["dP"] < 1e-12                                   # unquantised matmul of the caller's values
    assert e["dS"] > e["P"] and e["dS"] > 0.05               # dS: the bottleneck
    assert min(e["dQ"], e["dK"]) > max(e["O"], e["dV"])      # what follows dS suffers most
    assert 0.05 < e["dS"] < 0.6 and e["O"] < 0.15
