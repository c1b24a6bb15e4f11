"""Benchmark of the SageBwd hot path on one MI355X.

One step = one forward + one backward of the whole batch (pre-passes included) with the
inputs resident in HBM.  Prints ONE JSON line: fwd+bwd throughput in TOPS (work convention
4*BH*N^2*d forward + 10*BH*N^2*d backward, halved under the causal mask), the roofline
of the dominant kernel measured with HIP events inside the library on the launch stream,
and the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_PEAK_TOPS = 5000.0     # MI355X dense INT8 MFMA peak (published)
HBM_PEAK_GBS = 8000.0       # MI355X HBM3E peak (published)

# HBM bytes per launch at the headline workload.  NOT measured in this run: taken from the committed
# rocprofv3 FETCH_SIZE / WRITE_SIZE runs summarised in profiles/hbm_traffic_headline_fwd_bwd.txt
# (scaled by the copy-kernel calibration stated there).
PROFILED_TRAFFIC_BYTES = {"headline": {"bwd": 3.5082e9, "fwd": 3.382e8, "bwd_dq": 2.656e9}}


def work_ops(w, fwd=True, bwd=True, matmuls=None):
    """Work convention: 2*N^2*d ops per matmul and head (forward two matmuls, backward five),
    halved under the causal mask.  `matmuls` overrides the count (a kernel that runs some of them)."""
    per = 2 * matmuls if matmuls is not None else (4 if fwd else 0) + (10 if bwd else 0)
    ops = per * w.B * w.H * float(w.N) ** 2 * w.d
    return ops * (0.5 if w.causal else 1.0)


def executed_tiles(w):
    """64 x 64 tiles per head that the kernels visit."""
    t = -(-w.N // 64)
    return t * (t + 1) // 2 if w.causal else t * t


def cpu_baseline(w, seconds_hint=20.0):
    """The oracle as it stands, timed on whole heads of the same workload (a bounded sample)."""
    import numpy as np
    import oracle
    from paper_2603_02170_amd import synth
    try:
        from threadpoolctl import threadpool_info
        threads = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        threads = 1
    heads, t_total = 0, 0.0
    while heads < w.B * w.H and (heads == 0 or t_total + t_total / heads < seconds_hint):
        Q, K, V, dO = (t[0, 0].float().numpy() for t in synth.make_inputs(w, heads=[heads]))
        t0 = time.perf_counter()
        O, L = oracle.forward_head(Q, K, V, causal=w.causal, k_smooth=w.k_smooth, q_smooth=w.q_smooth)
        oracle.backward_head(Q, K, V, O, dO, L, causal=w.causal, k_smooth=w.k_smooth, q_smooth=w.q_smooth)
        t_total += time.perf_counter() - t0
        heads += 1
    ops = work_ops(w) / (w.B * w.H) * heads
    return {"value": ops / t_total / 1e12, "unit": "TOPS", "cores": int(threads), "kind": "oracle",
            "sample": f"{heads} of {w.B * w.H} heads of the {w.name} workload, fwd+bwd, {t_total:.1f} s "
                      f"(NumPy float64; whole-workload estimate {t_total / heads * w.B * w.H:.0f} s)"}


def measured_peaks(torch, binding):
    """What this GPU sustains on the resources the rooflines name, from the library's probe kernels: a
    dense loop of the MFMA instruction the kernels use (INT8 32x32x32, bf16 32x32x16), and 16-byte-per-lane
    streams over 1 GiB (copy, and read only).  Context beside the published peaks, measured under the same
    clocks and power limit as the attention kernels; run after the timed region."""
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    out = {}
    zero = binding.PROBE_MFMA_ZERO_OPERANDS
    for name, kind in (("int8_mfma", binding.PROBE_MFMA_INT8), ("bf16_mfma", binding.PROBE_MFMA_BF16),
                       ("int8_mfma_zero_operands", binding.PROBE_MFMA_INT8 | zero),
                       ("bf16_mfma_zero_operands", binding.PROBE_MFMA_BF16 | zero)):
        ms, ops = binding.sagebwd_probe_mfma(kind, iters=4096, reps=3, sink=sink)
        out[name] = {"value": ops / (ms * 1e-3) / 1e12, "unit": "TFLOP/s" if kind & binding.PROBE_MFMA_BF16 else "TOP/s",
                     "ms": ms}
    src = torch.full((1 << 30,), 7, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    ms = binding.sagebwd_probe_stream(binding.PROBE_STREAM_COPY, src, dst, reps=5, sink=sink)
    out["hbm_copy"] = {"value": 2 * (1 << 30) / (ms * 1e-3) / 1e9, "unit": "GB/s", "ms": ms, "note": "1 GiB read + 1 GiB written"}
    ms = binding.sagebwd_probe_stream(binding.PROBE_STREAM_READ, src, None, reps=5, sink=sink)
    out["hbm_read"] = {"value": (1 << 30) / (ms * 1e-3) / 1e9, "unit": "GB/s", "ms": ms, "note": "1 GiB read"}
    del src, dst
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="headline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-share", action="store_true",
                    help="the backward forms psi(Q), psi(K) again instead of taking them from the forward's "
                         "workspace (SAGEBWD_FLAG_SHARE_QUANTIZED off)")
    ap.add_argument("--blocks", default="64x64",
                    help="numerics block sizes B_q x B_kv (64 or 128 each; the headline metric is quoted on 64x64)")
    ap.add_argument("--events-on-dominant-kernel-only", action="store_true",
                    help="inside the timed region bracket only the dominant kernel with events (the default brackets all "
                         "five; an event between two kernels keeps the second from starting until the first has drained, "
                         "about 10 us each: 1 %% of the headline step, 10 %% of the pre-training shape's); the other four "
                         "are then timed in a second, shorter loop")
    ap.add_argument("--token-major", action="store_true",
                    help="hold Q, K, V, O, dO and the gradients as [B, N, H, d] (the default is [B, H, N, d])")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain 1 GiB device copy (known HBM bytes) to calibrate rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters, then exit")
    a = ap.parse_args()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (every head is independent: shard heads over GPUs with no communication); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2603_02170_amd import binding, synth

    if a.copy_calibration:
        torch.cuda.set_device(0)
        src = torch.full((1 << 30,), 7, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": 1 << 30, "copy_bytes_written": 1 << 30, "launches": 3}))
        return

    w = synth.WORKLOADS[a.workload]
    binding.load_library()      # fails loudly if the HIP library is missing
    torch.cuda.set_device(0)
    bq, bkv = (int(x) for x in a.blocks.split("x"))
    p = binding.SageParams(w.B, w.H, w.N, w.d, causal=w.causal, k_smooth=w.k_smooth, q_smooth=w.q_smooth,
                           token_major=a.token_major, share_quantized=not a.no_share, bq=bq, bkv=bkv)
    Q, K, V, dO = (t.cuda() for t in synth.make_inputs(w))
    if a.token_major:
        Q, K, V, dO = (t.permute(0, 2, 1, 3).contiguous() for t in (Q, K, V, dO))
    ws = binding.alloc_workspace(p)
    O = torch.empty_like(Q)
    L = torch.empty((w.B, w.H, w.N), dtype=torch.float32, device="cuda")
    dQ, dK, dV = (torch.empty_like(Q) for _ in range(3))

    def step():
        binding.sagebwd_fwd(Q, K, V, p, ws, O, L)
        binding.sagebwd_bwd(Q, K, V, O, dO, L, p, ws, dQ, dK, dV)

    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    # forward alone (same inputs), for the fwd-only figure: a forward that no backward follows leaves
    # nothing behind for one (no sharing flag)
    pf = binding.SageParams(w.B, w.H, w.N, w.d, causal=w.causal, k_smooth=w.k_smooth, q_smooth=w.q_smooth,
                            token_major=a.token_major, bq=bq, bkv=bkv)
    for _ in range(2):
        binding.sagebwd_fwd(Q, K, V, pf, ws, O, L)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        binding.sagebwd_fwd(Q, K, V, pf, ws, O, L)
    torch.cuda.synchronize()
    fwd_ms = (time.perf_counter() - t0) * 1e3 / a.steps

    # The timed region: K whole steps, with HIP events (inside the library, on the launch stream) around every
    # kernel.  An event between two kernels keeps the second from starting until the first has drained, about
    # 10 us each; --events-on-dominant-kernel-only brackets only the dominant kernel here and the other four
    # in a second, shorter loop that is not part of the timed region (same calls, same buffers).
    binding.set_timing(1 << binding.KERNEL_BWD if a.events_on_dominant_kernel_only else True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / a.steps
    kern = {}
    names = (("prepass_fwd", binding.KERNEL_PREPASS_FWD), ("fwd", binding.KERNEL_FWD),
             ("prepass_bwd", binding.KERNEL_PREPASS_BWD), ("bwd", binding.KERNEL_BWD), ("bwd_dq", binding.KERNEL_BWD_DQ))
    for name, kid in names:
        tot, n = binding.read_timing(kid)
        if n:
            kern[name] = tot / n
    if a.events_on_dominant_kernel_only:
        binding.set_timing(True)
        for _ in range(min(a.steps, 10)):
            step()
        torch.cuda.synchronize()
        for name, kid in names:
            tot, n = binding.read_timing(kid)
            kern.setdefault(name, tot / max(n, 1))
    binding.set_timing(False)
    kern = {k: kern[k] for k in ("prepass_fwd", "fwd", "prepass_bwd", "bwd", "bwd_dq")}

    peaks = measured_peaks(torch, binding)
    tops = work_ops(w) / (ms * 1e-3) / 1e12
    # sage_bwd_kernel runs four of the five backward matmuls (S recompute, dV, dP, dK); the fifth (dQ)
    # runs in sage_bwd_dq_kernel from the staged psi(dS) tiles
    bwd_ops = work_ops(w, matmuls=4)
    fwd_ops = work_ops(w, bwd=False)
    bwd_tops = bwd_ops / (kern["bwd"] * 1e-3) / 1e12
    fwd_tops = fwd_ops / (kern["fwd"] * 1e-3) / 1e12
    elems = w.B * w.H * w.N * w.d
    # pre-pass (forward): read Q, K, V bf16 once each, write three INT8 tensors = 9 B per (token, channel)
    # algorithmic (K's second read, for the mean, is what a cache can serve); sharing adds two more layouts
    pre_fwd_bytes = elems * (3 * 2 + 3 * 1 + (0 if a.no_share else 2))
    # dQ kernel: reads the staged psi(dS) tiles (4 KiB each) and K^ once per head, writes dQ bf16
    dq_bytes = w.B * w.H * (executed_tiles(w) * 4096.0 + w.N * w.d * 3.0)
    traffic = PROFILED_TRAFFIC_BYTES.get(w.name, {})
    out = {
        "metric": f"attention fwd+bwd TOPS and % of INT8 MFMA peak on one MI355X, N={w.N} d={w.d}",
        "value": tops, "unit": "TOPS", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"{w.name}: B={w.B} H={w.H} N={w.N} d={w.d} causal={w.causal} bf16 N(0,1) "
                               f"{'with' if w.qk_norm else 'without'} QK-norm, K-smoothing {'on' if w.k_smooth else 'off'}, "
                               f"Q-smoothing {'on' if w.q_smooth else 'off'}, {bq}x{bkv} blocks"
                               f"{', tensors [B,N,H,d]' if a.token_major else ''}",
                   "work_convention": "fwd 4*BH*N^2*d + bwd 10*BH*N^2*d ops, x0.5 causal",
                   "step": "sagebwd_fwd then sagebwd_bwd on one workspace, pre-passes included; "
                           + ("the backward re-quantises Q and K" if a.no_share else
                              "the backward takes psi(Q), psi(K) from the forward (Algorithm 2's inputs; "
                              "SAGEBWD_FLAG_SHARE_QUANTIZED), every step of the method runs once per step")},
        "pct_of_int8_peak": 100.0 * tops / INT8_PEAK_TOPS,
        "fwd_only": {"ms": fwd_ms, "TOPS": fwd_ops / (fwd_ms * 1e-3) / 1e12,
                     "pct_of_int8_peak": 100.0 * fwd_ops / (fwd_ms * 1e-3) / 1e12 / INT8_PEAK_TOPS},
        "kernel_ms": kern,
        "kernel_ms_note": ("bwd: mean over the timed region's launches (events around that kernel only); the others: mean "
                           "over a second loop of up to 10 steps with every kernel bracketed, outside the timed region")
                          if a.events_on_dominant_kernel_only else
                          "mean HIP-event duration per launch over the timed region, every kernel bracketed",
        "measured_peaks": peaks,
        "pct_of_measured_int8_peak": 100.0 * tops / peaks["int8_mfma"]["value"],
        "roofline": {"bound": "mfma", "kernel": "sage_bwd_kernel", "achieved": bwd_tops, "peak": INT8_PEAK_TOPS,
                     "unit": "TOP/s", "frac": bwd_tops / INT8_PEAK_TOPS,
                     "traffic": traffic.get("bwd"),
                     "frac_of_mixed_roof": bwd_tops / (INT8_PEAK_TOPS * 0.8),
                     "frac_of_measured_peak": bwd_tops / peaks["int8_mfma"]["value"],
                     "note": "algorithmic ops of the four matmuls this kernel runs (8*N^2*d per head, x0.5 causal) "
                             "over its mean HIP-event duration, against the INT8 MFMA peak; one of the four (dP) "
                             "runs on bf16 MFMA at half rate, so the kernel's own mixed roof is 4/5 of that peak "
                             "(frac_of_mixed_roof).  traffic: from profiles/, not measured in this run"},
        "roofline_fwd": {"bound": "mfma", "kernel": "sage_fwd_kernel", "achieved": fwd_tops, "peak": INT8_PEAK_TOPS,
                         "unit": "TOP/s", "frac": fwd_tops / INT8_PEAK_TOPS, "traffic": traffic.get("fwd"),
                         "frac_of_measured_peak": fwd_tops / peaks["int8_mfma"]["value"]},
        "roofline_bwd_dq": {"bound": "hbm", "kernel": "sage_bwd_dq_kernel",
                            "achieved": dq_bytes / (kern["bwd_dq"] * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                            "frac": dq_bytes / (kern["bwd_dq"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
                            "traffic": traffic.get("bwd_dq"),
                            "frac_of_measured_read": dq_bytes / (kern["bwd_dq"] * 1e-3) / 1e9 / peaks["hbm_read"]["value"],
                            "note": "bytes = staged psi(dS) tiles + K^ + dQ; the tiles are this design's staging "
                                    "of dS between the two backward kernels, not traffic the method itself requires"},
        "roofline_prepass": {"bound": "hbm", "kernel": "prepass (forward)",
                             "achieved": pre_fwd_bytes / (kern["prepass_fwd"] * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                             "unit": "GB/s", "frac": pre_fwd_bytes / (kern["prepass_fwd"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
                             "bytes_per_element": pre_fwd_bytes / elems,
                             "frac_of_measured_copy": pre_fwd_bytes / (kern["prepass_fwd"] * 1e-3) / 1e9 / peaks["hbm_copy"]["value"],
                             "note": "K is read twice (mean, then psi); the second read is not counted"},
    }
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
