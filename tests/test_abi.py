"""Host-side checks of the C-ABI library: it loads, exports every symbol the header
declares, and rejects bad arguments before touching the GPU (no compute calls)."""
import ctypes
import os
import re

import pytest

from paper_2603_02170_amd import binding
from paper_2603_02170_amd.binding import SageParams

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.lib_path()):
        from paper_2603_02170_amd import build
        build.build(verbose=False)
    return binding.load_library()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "sagebwd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sagebwd_[a-z_]+)\s*\(", text)))


def test_exports_every_declared_symbol(lib):
    names = _declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_strerror(lib):
    assert binding.sagebwd_strerror(0) == "ok"
    assert "multiple of 64" not in binding.sagebwd_strerror(-2)     # any N >= 1 is accepted
    for code in (-1, -2, -3, -4, -5):
        assert binding.sagebwd_strerror(code) not in ("ok", "unknown status")
    assert binding.sagebwd_strerror(-99) == "unknown status"


def test_workspace_bytes_and_shape_validation(lib):
    p = SageParams(2, 32, 8192, 128)
    n = binding.workspace_bytes(p)
    elems = 2 * 32 * 8192 * 128
    assert n >= 6 * elems + 64 * 8192 * 8192   # six INT8 operand tensors + the INT8 dS scratch
    assert n < 7 * elems + 64 * 8192 * 8192 + (64 << 20)
    # the forward alone needs three INT8 operand tensors and no dS scratch; sharing the quantised
    # Q, K with the backward adds their two transposed layouts to the forward's part
    nf = binding.workspace_bytes(p, forward_only=True)
    assert 3 * elems <= nf < 3 * elems + (16 << 20)
    ps = SageParams(2, 32, 8192, 128, share_quantized=True)
    assert binding.workspace_bytes(ps) == n
    assert 5 * elems <= binding.workspace_bytes(ps, forward_only=True) < 5 * elems + (16 << 20)
    # a smaller scratch budget shrinks the backward's need (heads run in groups), never below one head
    assert binding.workspace_bytes(SageParams(2, 32, 8192, 128, scratch_budget=1 << 30)) < 6 * elems + (1 << 30) + (64 << 20)
    assert binding.workspace_bytes(SageParams(2, 32, 8192, 128, scratch_budget=1)) >= 6 * elems + 8192 * 8192
    # the dS scratch is capped at 8 GiB by default: larger problems run in groups of heads
    assert binding.workspace_bytes(SageParams(1, 32, 32768, 128, causal=False)) < (8 << 30) + 7 * 32 * 32768 * 128 + (64 << 20)
    assert binding.workspace_bytes(SageParams(2, 32, 8192, 128, q_smooth=True)) > n
    # more keys than queries: the K-like tensors and the dS scratch grow, the Q-like ones do not
    sq, rect = SageParams(1, 4, 1024, 128), SageParams(1, 4, 1024, 128, Nkv=4096)
    grow = binding.workspace_bytes(rect) - binding.workspace_bytes(sq)
    assert 3 * 4 * 3072 * 128 + 4 * 1024 * 3072 <= grow < 3 * 4 * 3072 * 128 + 4 * 1024 * 3072 + (1 << 20)
    assert binding.workspace_bytes(SageParams(1, 4, 1024, 128, Nkv=1024)) == binding.workspace_bytes(sq)
    # N that is not a multiple of 64: the workspace is laid out for N rounded up to the block
    assert binding.workspace_bytes(SageParams(1, 1, 100, 64)) == binding.workspace_bytes(SageParams(1, 1, 128, 64))
    assert binding.workspace_bytes(SageParams(1, 1, 128, 64, bq=64, bkv=64)) == binding.workspace_bytes(SageParams(1, 1, 128, 64))
    # numerics blocks of 128 rows are served from the same buffers (scales are stored once per 64-row block)
    assert binding.workspace_bytes(SageParams(1, 1, 128, 64, bq=128, bkv=128), forward_only=True) == \
        binding.workspace_bytes(SageParams(1, 1, 128, 64), forward_only=True)
    for bad in (SageParams(1, 1, 128, 96), SageParams(1, 1, 64, 256), SageParams(1, 1, (1 << 30) + 64, 64),
                SageParams(1, 1, 128, 64, bq=256), SageParams(1, 1, 128, 64, bq=96), SageParams(1, 1, 128, 64, bkv=32)):
        with pytest.raises(binding.SageError) as e:
            binding.workspace_bytes(bad)
        assert e.value.status == -2
    for bad in (SageParams(0, 1, 128, 64), SageParams(1, -1, 128, 64), SageParams(1, 1, 128, 64, sm_scale=-1.0),
                SageParams(1, 1, 128, 64, bq=-64)):
        with pytest.raises(binding.SageError) as e:
            binding.workspace_bytes(bad)
        assert e.value.status == -1


def test_entry_points_reject_bad_arguments_on_the_host(lib):
    cp = SageParams(1, 2, 128, 64).c()
    null = ctypes.c_void_p(None)
    one = ctypes.c_void_p(256)   # never dereferenced: validation fails first
    assert lib.sagebwd_fwd(null, one, one, one, one, ctypes.byref(cp), one, 1 << 30, null) == -1
    assert lib.sagebwd_fwd(one, one, one, one, one, ctypes.byref(cp), one, 16, null) == -3
    assert lib.sagebwd_bwd(one, one, one, one, one, one, one, one, null, ctypes.byref(cp), one, 1 << 30, null) == -1
    assert lib.sagebwd_quantize(one, one, one, null, one, ctypes.byref(cp), one, 1 << 30, null) == -1
    assert lib.sagebwd_export_quantized(ctypes.byref(cp), one, 1 << 30, 7, one, one, null) == -1
    assert lib.sagebwd_fwd(one, one, one, one, one, None, one, 1 << 30, null) == -1
    bad = SageParams(1, 2, 128, 64).c()
    bad.smooth = 8
    assert lib.sagebwd_fwd(one, one, one, one, one, ctypes.byref(bad), one, 1 << 30, null) == -1
    bad = SageParams(1, 2, 128, 64).c()
    bad.flags = 2
    assert lib.sagebwd_fwd(one, one, one, one, one, ctypes.byref(bad), one, 1 << 30, null) == -1
    bad = SageParams(1, 2, 128, 64).c()
    bad.Nkv = -64
    assert lib.sagebwd_fwd(one, one, one, one, one, ctypes.byref(bad), one, 1 << 30, null) == -1
    # QK-norm fused into the pre-pass: both gains with the flag, none without it, eps >= 0
    c = SageParams(1, 2, 128, 64).c()
    c.flags = binding.FLAG_QK_NORM
    assert lib.sagebwd_fwd(one, one, one, one, one, ctypes.byref(c), one, 16, null) == -1
    c.qk_gamma_q, c.qk_gamma_k = 256, 256
    assert lib.sagebwd_fwd(one, one, one, one, one, ctypes.byref(c), one, 16, null) == -3
    c.qk_norm_eps = -1.0
    assert lib.sagebwd_fwd(one, one, one, one, one, ctypes.byref(c), one, 16, null) == -1
    c = SageParams(1, 2, 128, 64).c()
    c.qk_gamma_k = 256
    assert lib.sagebwd_fwd(one, one, one, one, one, ctypes.byref(c), one, 16, null) == -1
    # N_q != N_kv: under the mask the keys must be at least as many and differ by whole blocks
    for nkv, causal, want in ((64, True, -2), (200, True, -2), (192, True, -3), (64, False, -3), (1000, False, -3)):
        c = SageParams(1, 2, 128, 64, causal=causal, Nkv=nkv).c()
        assert lib.sagebwd_fwd(one, one, one, one, one, ctypes.byref(c), one, 16, null) == want, (nkv, causal)
    # the forward accepts its own (smaller) workspace size, the backward does not
    fwd_only = binding.workspace_bytes(SageParams(1, 2, 128, 64), forward_only=True)
    assert fwd_only < binding.workspace_bytes(SageParams(1, 2, 128, 64))
    assert lib.sagebwd_fwd(one, one, one, one, one, ctypes.byref(cp), one, fwd_only - 1, null) == -3
    assert lib.sagebwd_bwd(one, one, one, one, one, one, one, one, one, ctypes.byref(cp), one, fwd_only, null) == -3
    # the no-allocation forward: too large a problem and the sharing flag are refused on the host
    big = SageParams(2, 32, 8192, 128).c()
    assert lib.sagebwd_fwd_static(one, one, one, one, one, ctypes.byref(big), null) == -5
    sh = SageParams(1, 2, 128, 64, share_quantized=True).c()
    assert lib.sagebwd_fwd_static(one, one, one, one, one, ctypes.byref(sh), null) == -1
    assert lib.sagebwd_fwd_static(null, one, one, one, one, ctypes.byref(cp), null) == -1
    bad = SageParams(1, 2, 128, 64).c()
    bad.layout = 2
    assert lib.sagebwd_fwd(one, one, one, one, one, ctypes.byref(bad), one, 1 << 30, null) == -1
    tot, cnt = ctypes.c_double(0), ctypes.c_int(0)
    assert lib.sagebwd_read_timing(99, ctypes.byref(tot), ctypes.byref(cnt)) == -1
    assert lib.sagebwd_set_timing(32) == -1 and lib.sagebwd_set_timing(-1) == -1 and lib.sagebwd_set_timing(0) == 0


def test_probes_reject_bad_arguments_on_the_host(lib):
    ms, ops = ctypes.c_double(0), ctypes.c_double(0)
    fake = ctypes.c_void_p(4096)       # never dereferenced: every call below fails its argument check first
    INVALID = -1
    assert lib.sagebwd_probe_mfma(4, 16, 1, fake, None, ctypes.byref(ms), ctypes.byref(ops)) == INVALID     # unknown kind
    assert lib.sagebwd_probe_mfma(0, 0, 1, fake, None, ctypes.byref(ms), ctypes.byref(ops)) == INVALID      # no iterations
    assert lib.sagebwd_probe_mfma(0, 16, 0, fake, None, ctypes.byref(ms), ctypes.byref(ops)) == INVALID     # no launches
    assert lib.sagebwd_probe_mfma(0, 16, 1, None, None, ctypes.byref(ms), ctypes.byref(ops)) == INVALID     # no sink
    assert lib.sagebwd_probe_mfma(0, 16, 1, fake, None, None, ctypes.byref(ops)) == INVALID
    assert lib.sagebwd_probe_stream(0, fake, None, 4096, 1, fake, None, ctypes.byref(ms)) == INVALID         # copy without dst
    assert lib.sagebwd_probe_stream(1, fake, None, 100, 1, fake, None, ctypes.byref(ms)) == INVALID          # not 16-byte pieces
    assert lib.sagebwd_probe_stream(1, ctypes.c_void_p(4100), None, 4096, 1, fake, None, ctypes.byref(ms)) == INVALID   # misaligned
    assert lib.sagebwd_probe_stream(3, fake, fake, 4096, 1, fake, None, ctypes.byref(ms)) == INVALID
