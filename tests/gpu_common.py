"""Shared helpers of the GPU parity tests."""
import json
import os

import numpy as np
import torch

from paper_2603_02170_amd import binding, synth
from paper_2603_02170_amd.binding import SageParams

from fpa_ref import cos_sim, rel_l1

# Tolerance of the floating-point outputs against the oracle, as the task states it: relative L1 and
# cosine over the whole compared tensor.
REL_L1_MAX = 1e-2
COS_MIN = 0.999
# Localised bounds beside it (two whole-tensor norms cannot see one wrong row among thousands):
#   every 64-row block of the compared rows meets the same relative L1 on its own (denominator: the
#   block's own |ref| sum, floored at a tenth of the mean block's so that a block of near-zero
#   gradient is not held to a relative bound on nothing), and no single element is off by more than
#   MAX_ABS_IN_RMS times the RMS of the reference.
BLOCK_REL_L1_MAX = 1e-2
MAX_ABS_IN_RMS = 0.5
# (Measured over every comparison of the suite: worst block 1.8e-3, worst element 0.21 RMS -- one
# psi(dS) code off by a step in a tile of large scale; a wrong element is off by about one RMS.)
# Regression guards: about five times the worst agreement measured on the MI355X over every
# comparison of the suite, per kind of output (whole-tensor relative L1: O 6.8e-4, dQ 3.8e-5,
# dK 2.4e-5, dV 1.3e-4; LSE max-abs 1.7e-4, on the unsmoothed outlier inputs whose logits are in
# the hundreds).  Far inside the stated tolerance; a kernel change that costs accuracy trips them first.
GUARD_REL_L1 = {"O": 3.5e-3, "dQ": 2e-4, "dK": 1.5e-4, "dV": 7e-4}
LSE_MAX_ABS = 8e-4


def params_for(w, B=None, H=None, **kw):
    args = dict(B=w.B if B is None else B, H=w.H if H is None else H, N=w.N, d=w.d, causal=w.causal,
                k_smooth=w.k_smooth, q_smooth=w.q_smooth)
    args.update(kw)
    return SageParams(**args)


def to_np(t):
    return t.detach().float().cpu().numpy()


def _log(record):
    path = os.environ.get("SAGE_PARITY_LOG")
    if path:
        with open(path, "a") as f:
            f.write(json.dumps(record) + "\n")


def check_close(name, got, ref, rel_l1_max=REL_L1_MAX, cos_min=COS_MIN, block=64, guard=True):
    """got, ref: [rows, d] (whole heads or the concatenated rows of sampled 64-row blocks)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, f"{name}: shape {got.shape} vs {ref.shape}"
    assert np.isfinite(got).all(), f"{name}: non-finite values"
    l1, cs = rel_l1(got, ref), cos_sim(got, ref)
    err = np.abs(got - ref)
    rms = float(np.sqrt((ref ** 2).mean()))
    worst_abs = float(err.max()) / rms if rms > 0 else float(err.max())
    # per block of rows (the last one may be partial)
    rows = got.shape[0]
    nb = -(-rows // block)
    e_blk = np.array([err[block * b:block * b + block].sum() for b in range(nb)])
    r_blk = np.array([np.abs(ref[block * b:block * b + block]).sum() for b in range(nb)])
    floor = 0.1 * r_blk.mean() * np.array([min(block, rows - block * b) / block for b in range(nb)])
    blk = e_blk / np.maximum(r_blk, np.maximum(floor, 1e-300))
    worst_blk = float(blk.max())
    kind = name.split("[")[0].split()[0]
    _log(dict(name=name, kind=kind, rows=rows, rel_l1=l1, cos=cs, worst_block_rel_l1=worst_blk, max_abs_in_rms=worst_abs))
    assert l1 <= rel_l1_max and cs >= cos_min, f"{name}: rel-L1 {l1:.3e} cos {cs:.6f}"
    assert worst_blk <= BLOCK_REL_L1_MAX, f"{name}: block {int(blk.argmax())} rel-L1 {worst_blk:.3e}"
    assert worst_abs <= MAX_ABS_IN_RMS, f"{name}: max |err| = {worst_abs:.3e} x RMS(ref)"
    if guard and kind in GUARD_REL_L1:
        assert l1 <= GUARD_REL_L1[kind], f"{name}: rel-L1 {l1:.3e} above the regression guard {GUARD_REL_L1[kind]:.1e}"
    return l1, cs


def check_lse(name, got, ref, max_abs=LSE_MAX_ABS):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert np.isfinite(got).all(), f"{name}: non-finite values"
    e = float(np.abs(got - ref).max())
    _log(dict(name=name, kind="LSE", rows=int(got.size), max_abs=e))
    assert e <= max_abs, f"{name}: max |LSE - ref| = {e:.3e}"
    return e
