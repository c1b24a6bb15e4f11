"""Thin ctypes binding of libsagebwd.so: argument marshalling only.

Every step of the path runs in the HIP library; PyTorch is used for device
memory and the current stream.  There is no CPU fallback: if the library is
missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

SMOOTH_K = 1
SMOOTH_Q = 2
FLAG_SHARE_QUANTIZED = 1
FLAG_QK_NORM = 2
LAYOUT_BHND, LAYOUT_BNHD = 0, 1

TENSOR_Q, TENSOR_K, TENSOR_V, TENSOR_DO = 0, 1, 2, 3
KERNEL_PREPASS_FWD, KERNEL_FWD, KERNEL_PREPASS_BWD, KERNEL_BWD, KERNEL_BWD_DQ = range(5)

EXPORTS = (
    "sagebwd_workspace_bytes", "sagebwd_quantize", "sagebwd_export_quantized", "sagebwd_export_stats", "sagebwd_export_ds",
    "sagebwd_fwd", "sagebwd_fwd_static", "sagebwd_bwd", "sagebwd_set_timing", "sagebwd_read_timing",
    "sagebwd_probe_mfma", "sagebwd_probe_stream", "sagebwd_strerror",
)


class _CParams(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("N", ctypes.c_int32), ("d", ctypes.c_int32),
                ("causal", ctypes.c_int32), ("smooth", ctypes.c_int32), ("sm_scale", ctypes.c_float),
                ("layout", ctypes.c_int32), ("bq", ctypes.c_int32), ("bkv", ctypes.c_int32),
                ("flags", ctypes.c_int32), ("Nkv", ctypes.c_int32), ("scratch_budget", ctypes.c_uint64),
                ("qk_gamma_q", ctypes.c_void_p), ("qk_gamma_k", ctypes.c_void_p), ("qk_norm_eps", ctypes.c_float),
                ("reserved", ctypes.c_int32)]


@dataclass
class SageParams:
    B: int
    H: int
    N: int
    d: int
    causal: bool = True
    k_smooth: bool = True
    q_smooth: bool = False
    sm_scale: float = 0.0   # 0 selects 1/sqrt(d)
    token_major: bool = False   # the bf16 tensors are [B, N, H, d] instead of [B, H, N, d]
    share_quantized: bool = False   # the backward takes psi(Q), psi(K) from the forward's workspace
    scratch_budget: int = 0     # bytes of dS scratch the backward holds at once; 0 selects 8 GiB
    bq: int = 0                 # numerics block sizes B_q, B_kv: 0 (= 64), 64 or 128
    bkv: int = 0
    Nkv: int = 0                # rows of K, V, dK, dV; 0 selects N
    qk_gamma_q: object = None   # QK-norm fused into the pre-pass: float32 cuda tensors [d] (both or neither);
    qk_gamma_k: object = None   # the caller keeps them alive while calls are in flight
    qk_norm_eps: float = 1e-6

    def c(self) -> _CParams:
        return _CParams(self.B, self.H, self.N, self.d, int(self.causal),
                        (SMOOTH_K if self.k_smooth else 0) | (SMOOTH_Q if self.q_smooth else 0),
                        float(self.sm_scale), LAYOUT_BNHD if self.token_major else LAYOUT_BHND,
                        int(self.bq), int(self.bkv),
                        (FLAG_SHARE_QUANTIZED if self.share_quantized else 0) | (FLAG_QK_NORM if self.qk_gamma_q is not None else 0),
                        int(self.Nkv), int(self.scratch_budget),
                        None if self.qk_gamma_q is None else self._gain(self.qk_gamma_q),
                        None if self.qk_gamma_k is None else self._gain(self.qk_gamma_k),
                        float(self.qk_norm_eps) if self.qk_gamma_q is not None else 0.0, 0)

    def _gain(self, g):
        if g.dtype != torch.float32 or tuple(g.shape) != (self.d,) or not g.is_contiguous() or not g.is_cuda:
            raise ValueError(f"QK-norm gain: need contiguous cuda float32 ({self.d},)")
        return g.data_ptr()

    @property
    def kv_len(self) -> int:
        return self.Nkv or self.N

    def tensor_shape(self, kv: bool = False):
        """Shape of Q, O, dO, dQ (or, with kv, of K, V, dK, dV) as the caller holds them."""
        n = self.kv_len if kv else self.N
        return (self.B, n, self.H, self.d) if self.token_major else (self.B, self.H, n, self.d)


def lib_path() -> str:
    return os.path.join(_HERE, "libsagebwd.so")


def load_library():
    """dlopen the in-tree library (built by paper_2603_02170_amd.build); raises if absent."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} not found: build it with `python -m paper_2603_02170_amd.build` "
                           "(there is no fallback path)")
    lib = ctypes.CDLL(path)
    vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
    pp = ctypes.POINTER(_CParams)
    lib.sagebwd_workspace_bytes.argtypes = [pp, ctypes.POINTER(sz), ctypes.POINTER(sz)]
    lib.sagebwd_quantize.argtypes = [vp, vp, vp, vp, vp, pp, vp, sz, vp]
    lib.sagebwd_export_quantized.argtypes = [pp, vp, sz, i32, vp, vp, vp]
    lib.sagebwd_export_stats.argtypes = [pp, vp, sz, vp, vp, vp, vp]
    lib.sagebwd_export_ds.argtypes = [pp, vp, sz, i32, vp, vp, vp]
    lib.sagebwd_fwd.argtypes = [vp, vp, vp, vp, vp, pp, vp, sz, vp]
    lib.sagebwd_fwd_static.argtypes = [vp, vp, vp, vp, vp, pp, vp]
    lib.sagebwd_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, pp, vp, sz, vp]
    lib.sagebwd_set_timing.argtypes = [i32]
    lib.sagebwd_read_timing.argtypes = [i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i32)]
    dp = ctypes.POINTER(ctypes.c_double)
    lib.sagebwd_probe_mfma.argtypes = [i32, i32, i32, vp, vp, dp, dp]
    lib.sagebwd_probe_stream.argtypes = [i32, vp, vp, sz, i32, vp, vp, dp]
    lib.sagebwd_strerror.argtypes = [i32]
    lib.sagebwd_strerror.restype = ctypes.c_char_p
    for name in EXPORTS:
        if name != "sagebwd_strerror":
            getattr(lib, name).restype = i32
    _LIB = lib
    return lib


def sagebwd_strerror(status: int) -> str:
    return load_library().sagebwd_strerror(int(status)).decode()


class SageError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {sagebwd_strerror(status)} ({status})")


def _check(status: int, where: str):
    if status != 0:
        raise SageError(status, where)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _expect(t, dtype, shape, name):
    if t.dtype != dtype or tuple(t.shape) != tuple(shape) or not t.is_contiguous() or not t.is_cuda:
        raise ValueError(f"{name}: need contiguous cuda {dtype} {tuple(shape)}, got {t.dtype} {tuple(t.shape)}")


def workspace_bytes(p: SageParams, forward_only: bool = False) -> int:
    """Bytes that serve every call (or, with forward_only, sagebwd_fwd alone)."""
    fwd, bwd = ctypes.c_size_t(0), ctypes.c_size_t(0)
    cp = p.c()
    _check(load_library().sagebwd_workspace_bytes(ctypes.byref(cp), ctypes.byref(fwd), ctypes.byref(bwd)),
           "sagebwd_workspace_bytes")
    return int(fwd.value if forward_only else bwd.value)


def alloc_workspace(p: SageParams, device="cuda", forward_only: bool = False):
    return torch.empty(workspace_bytes(p, forward_only), dtype=torch.uint8, device=device)


def sagebwd_quantize(Q, K, V, p: SageParams, workspace, dO=None, O=None):
    shp, kshp = p.tensor_shape(), p.tensor_shape(kv=True)
    _expect(Q, torch.bfloat16, shp, "Q")
    for t, n in ((K, "K"), (V, "V")):
        _expect(t, torch.bfloat16, kshp, n)
    for t, n in ((dO, "dO"), (O, "O")):
        if t is not None:
            _expect(t, torch.bfloat16, shp, n)
    cp = p.c()
    _check(load_library().sagebwd_quantize(_ptr(Q), _ptr(K), _ptr(V), _ptr(dO), _ptr(O), ctypes.byref(cp),
                                           _ptr(workspace), workspace.numel(), _stream()), "sagebwd_quantize")


def padded_rows(N: int) -> int:
    """Rows of the workspace tensors: N rounded up to the 64-row block."""
    return (N + 63) // 64 * 64


def sagebwd_export_quantized(p: SageParams, workspace, which: int):
    """Row-major int8 [B,H,Np,d] codes and float32 [B,H,Np/64] scales of one quantised tensor
    (Np = N rounded up to a multiple of 64; rows N..Np-1 are zero)."""
    Np = padded_rows(p.kv_len if which in (TENSOR_K, TENSOR_V) else p.N)
    q = torch.empty((p.B, p.H, Np, p.d), dtype=torch.int8, device=workspace.device)
    s = torch.empty((p.B, p.H, Np // 64), dtype=torch.float32, device=workspace.device)
    cp = p.c()
    _check(load_library().sagebwd_export_quantized(ctypes.byref(cp), _ptr(workspace), workspace.numel(), which,
                                                   _ptr(q), _ptr(s), _stream()), "sagebwd_export_quantized")
    return q, s


def sagebwd_export_stats(p: SageParams, workspace, want_delta=False):
    dev = workspace.device
    muK = torch.empty((p.B, p.H, p.d), dtype=torch.float32, device=dev)
    Np = padded_rows(p.N)
    muQ = torch.empty((p.B, p.H, Np // 64, p.d), dtype=torch.float32, device=dev) if p.q_smooth else None
    delta = torch.empty((p.B, p.H, Np), dtype=torch.float32, device=dev) if want_delta else None
    cp = p.c()
    _check(load_library().sagebwd_export_stats(ctypes.byref(cp), _ptr(workspace), workspace.numel(), _ptr(muK),
                                               _ptr(muQ), _ptr(delta), _stream()), "sagebwd_export_stats")
    return muK, muQ, delta


def sagebwd_export_ds(p: SageParams, workspace, head: int):
    """psi(dS) of one head after a backward on this workspace: int8 [Np, Np] codes and float32
    [Np/64, Np/64] tile scales."""
    Np, Nkp = padded_rows(p.N), padded_rows(p.kv_len)
    ds = torch.empty((Np, Nkp), dtype=torch.int8, device=workspace.device)
    sc = torch.empty((Np // 64, Nkp // 64), dtype=torch.float32, device=workspace.device)
    cp = p.c()
    _check(load_library().sagebwd_export_ds(ctypes.byref(cp), _ptr(workspace), workspace.numel(), int(head),
                                            _ptr(ds), _ptr(sc), _stream()), "sagebwd_export_ds")
    return ds, sc


def sagebwd_fwd(Q, K, V, p: SageParams, workspace=None, O=None, LSE=None):
    """O, LSE = INT8 attention forward.  Allocates outputs / workspace when not given."""
    shp, kshp = p.tensor_shape(), p.tensor_shape(kv=True)
    lshp = (p.B, p.H, p.N)
    _expect(Q, torch.bfloat16, shp, "Q")
    for t, n in ((K, "K"), (V, "V")):
        _expect(t, torch.bfloat16, kshp, n)
    if workspace is None:
        workspace = alloc_workspace(p, Q.device, forward_only=True)
    if O is None:
        O = torch.empty(shp, dtype=torch.bfloat16, device=Q.device)
    if LSE is None:
        LSE = torch.empty(lshp, dtype=torch.float32, device=Q.device)
    _expect(O, torch.bfloat16, shp, "O")
    _expect(LSE, torch.float32, lshp, "LSE")
    cp = p.c()
    _check(load_library().sagebwd_fwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), ctypes.byref(cp),
                                      _ptr(workspace), workspace.numel(), _stream()), "sagebwd_fwd")
    return O, LSE


STATIC_SCRATCH_BYTES = 32 << 20


def sagebwd_fwd_static(Q, K, V, p: SageParams, O, LSE):
    """The forward on the library's built-in scratch: the call allocates nothing, so the caller
    passes the outputs too."""
    shp, kshp = p.tensor_shape(), p.tensor_shape(kv=True)
    for t, n in ((Q, "Q"), (O, "O")):
        _expect(t, torch.bfloat16, shp, n)
    for t, n in ((K, "K"), (V, "V")):
        _expect(t, torch.bfloat16, kshp, n)
    _expect(LSE, torch.float32, (p.B, p.H, p.N), "LSE")
    cp = p.c()
    _check(load_library().sagebwd_fwd_static(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), ctypes.byref(cp),
                                             _stream()), "sagebwd_fwd_static")
    return O, LSE


def sagebwd_bwd(Q, K, V, O, dO, LSE, p: SageParams, workspace=None, dQ=None, dK=None, dV=None):
    """dQ, dK, dV = INT8 attention backward."""
    shp, kshp = p.tensor_shape(), p.tensor_shape(kv=True)
    for t, n in ((Q, "Q"), (O, "O"), (dO, "dO")):
        _expect(t, torch.bfloat16, shp, n)
    for t, n in ((K, "K"), (V, "V")):
        _expect(t, torch.bfloat16, kshp, n)
    _expect(LSE, torch.float32, (p.B, p.H, p.N), "LSE")
    if workspace is None:
        workspace = alloc_workspace(p, Q.device)
    outs = []
    for t, n, sh in ((dQ, "dQ", shp), (dK, "dK", kshp), (dV, "dV", kshp)):
        if t is None:
            t = torch.empty(sh, dtype=torch.bfloat16, device=Q.device)
        _expect(t, torch.bfloat16, sh, n)
        outs.append(t)
    cp = p.c()
    _check(load_library().sagebwd_bwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(LSE), _ptr(outs[0]),
                                      _ptr(outs[1]), _ptr(outs[2]), ctypes.byref(cp), _ptr(workspace),
                                      workspace.numel(), _stream()), "sagebwd_bwd")
    return tuple(outs)


TIMING_ALL = 31


def set_timing(kernels):
    """kernels: True / False (all / none) or a mask with bit k set for kernel k (KERNEL_*)."""
    mask = (TIMING_ALL if kernels else 0) if isinstance(kernels, bool) else int(kernels)
    _check(load_library().sagebwd_set_timing(mask), "sagebwd_set_timing")


def read_timing(kernel: int):
    ms = ctypes.c_double(0)
    n = ctypes.c_int(0)
    _check(load_library().sagebwd_read_timing(kernel, ctypes.byref(ms), ctypes.byref(n)), "sagebwd_read_timing")
    return float(ms.value), int(n.value)


PROBE_MFMA_INT8, PROBE_MFMA_BF16, PROBE_MFMA_ZERO_OPERANDS = 0, 1, 2
PROBE_STREAM_COPY, PROBE_STREAM_READ = 0, 1


def sagebwd_probe_mfma(kind: int, iters: int = 4096, reps: int = 3, sink=None):
    """(ms per launch, operations per launch) of the dense matrix-instruction probe."""
    sink = torch.zeros(1, dtype=torch.int32, device="cuda") if sink is None else sink
    ms, ops = ctypes.c_double(0), ctypes.c_double(0)
    _check(load_library().sagebwd_probe_mfma(kind, iters, reps, _ptr(sink), _stream(), ctypes.byref(ms), ctypes.byref(ops)),
           "sagebwd_probe_mfma")
    return float(ms.value), float(ops.value)


def sagebwd_probe_stream(kind: int, src, dst=None, reps: int = 3, sink=None):
    """ms per launch of the streaming probe over the bytes of `src` (copied to `dst`, or only read)."""
    sink = torch.zeros(1, dtype=torch.int32, device="cuda") if sink is None else sink
    nbytes = src.numel() * src.element_size()
    ms = ctypes.c_double(0)
    _check(load_library().sagebwd_probe_stream(kind, _ptr(src), _ptr(dst) if dst is not None else None, nbytes, reps,
                                               _ptr(sink), _stream(), ctypes.byref(ms)), "sagebwd_probe_stream")
    return float(ms.value)
