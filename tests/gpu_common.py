"""Shared helpers of the GPU parity tests."""
import numpy as np
import torch

from paper_2603_02170_amd import binding, synth
from paper_2603_02170_amd.binding import SageParams

from fpa_ref import cos_sim, rel_l1

# tolerance of the floating-point outputs against the oracle (relative L1, cosine)
REL_L1_MAX = 1e-2
COS_MIN = 0.999


def params_for(w, B=None, H=None, **kw):
    args = dict(B=w.B if B is None else B, H=w.H if H is None else H, N=w.N, d=w.d, causal=w.causal,
                k_smooth=w.k_smooth, q_smooth=w.q_smooth)
    args.update(kw)
    return SageParams(**args)


def to_np(t):
    return t.detach().float().cpu().numpy()


def check_close(name, got, ref, rel_l1_max=REL_L1_MAX, cos_min=COS_MIN):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert np.isfinite(got).all(), f"{name}: non-finite values"
    l1, cs = rel_l1(got, ref), cos_sim(got, ref)
    assert l1 <= rel_l1_max and cs >= cos_min, f"{name}: rel-L1 {l1:.3e} cos {cs:.6f}"
    return l1, cs
