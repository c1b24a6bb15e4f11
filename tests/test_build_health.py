"""The hot kernels must not spill registers inside their loops: a scratch (private memory) access there
is a memory operation whose wait also drains the asynchronous global -> LDS copies in flight, which has
cost the Q-smoothing backward 15 % once.  This compiles the device code to assembly (no GPU needed)
and reads each kernel's register and scratch figures from the code object metadata."""
import os
import re
import subprocess
import tempfile

import pytest

from paper_2603_02170_amd import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def kernels():
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "sagebwd.s")
        cmd = [build.hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-I", os.path.join(ROOT, "include"),
               "-I", os.path.join(ROOT, "paper_2603_02170_amd", "csrc"), "--cuda-device-only", "-S",
               os.path.join(ROOT, "paper_2603_02170_amd", "csrc", "sagebwd_api.hip"), "-o", out]
        res = subprocess.run(cmd, capture_output=True, text=True)
        assert res.returncode == 0, res.stderr[-2000:]
        text = open(out).read()
    info = {}
    for block in text.split(".amdhsa_kernel ")[1:]:
        name = block.split("\n")[0].strip()
        get = lambda key: int(re.search(key + r"\s+(\d+)", block).group(1))
        info[name] = dict(vgpr=get(r"\.amdhsa_next_free_vgpr"), scratch=get(r"\.amdhsa_private_segment_fixed_size"),
                          lds=get(r"\.amdhsa_group_segment_fixed_size"))
    assert not re.search(r"\bv_pk_(fma|mul|add)_f32\b", text), "packed FP32 instructions must stay out of the build"
    return info


def _pick(kernels, stem, *template_bits):
    hits = [v for k, v in kernels.items() if stem in k and all(b in k for b in template_bits)]
    assert hits, (stem, template_bits)
    return hits


def test_backward_kernels_keep_their_loops_free_of_scratch(kernels):
    # sage_bwd_kernel<D, CAUSAL, QSMOOTH>: the instantiations the benchmark workloads run
    # (..., MODE, KV128>: ELi0ELb0E is the 64 x 64 kernel; the instantiations for numerics blocks of 128 may park
    # a few registers, they are not the fast path)
    for bits in (("ILi128ELb1ELb0E",), ("ILi128ELb0ELb0E",), ("ILi128ELb1ELb1E",), ("ILi64ELb1ELb0E",), ("ILi64ELb1ELb1E",)):
        for k in _pick(kernels, "sage_bwd_kernel", *bits, "ELi0ELb0EEEv"):
            assert k["scratch"] == 0 and k["vgpr"] <= 256, (bits, k)
            assert k["lds"] <= 160 * 1024
    for k in _pick(kernels, "sage_bwd_kernel"):
        assert k["scratch"] <= 64 and k["vgpr"] <= 256 and k["lds"] <= 160 * 1024, k
    for k in _pick(kernels, "sage_bwd_dq_kernel"):
        # three workgroups of four waves per CU: 168 registers, a third of the LDS
        assert k["scratch"] == 0 and k["vgpr"] <= 168 and 3 * k["lds"] <= 160 * 1024, k


def test_forward_kernels_fit_their_occupancy(kernels):
    # four-wave workgroups, two per CU at d = 128 (256 registers) and three at d = 64 (168); the few
    # registers kept in scratch are used before and after the tile loop only
    # (the last template argument, Lb0E / Lb1E, selects numerics blocks of 64 / 128 keys; the latter keeps a pair
    # of row maxima more and may park a few more registers)
    for kv128, scratch in (("ELi4ELb0E", 80), ("ELi4ELb1E", 128)):
        for k in _pick(kernels, "sage_fwd_kernel", "ILi128E", kv128):
            assert k["vgpr"] <= 256 and k["scratch"] <= scratch and 2 * k["lds"] <= 160 * 1024, k
        for k in _pick(kernels, "sage_fwd_kernel", "ILi64E", kv128):
            assert k["vgpr"] <= 168 and k["scratch"] <= scratch and 3 * k["lds"] <= 160 * 1024, k
