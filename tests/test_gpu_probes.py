"""The machine probes of the library (dense MFMA loop, streaming copy / read) return figures a
gfx950 can produce: below the published peaks, and far above what a mis-counted launch would give."""
import pytest
import torch

from paper_2603_02170_amd import binding

pytestmark = pytest.mark.gpu


def test_mfma_probes_lie_below_the_published_peaks():
    for kind, peak in ((binding.PROBE_MFMA_INT8, 5000.0), (binding.PROBE_MFMA_BF16, 2500.0)):
        ms, ops = binding.sagebwd_probe_mfma(kind, iters=1024, reps=2)
        rate = ops / (ms * 1e-3) / 1e12
        print(f"mfma probe kind {kind}: {ms:.3f} ms, {rate:.0f} T/s", flush=True)
        assert 0.3 * peak < rate < 1.05 * peak, (kind, ms, rate)
        # twice the iterations take about twice as long (the loop is what is timed, not the launch)
        ms2, ops2 = binding.sagebwd_probe_mfma(kind, iters=2048, reps=2)
        assert ops2 == 2 * ops
        assert 1.6 < ms2 / ms < 2.4, (ms, ms2)


def test_stream_probes_copy_the_data_and_lie_below_the_hbm_peak():
    n = 1 << 30
    src = torch.arange(n // 8, dtype=torch.int64, device="cuda")
    dst = torch.zeros_like(src)
    ms = binding.sagebwd_probe_stream(binding.PROBE_STREAM_COPY, src, dst, reps=2)
    assert torch.equal(src, dst)
    rate = 2 * n / (ms * 1e-3) / 1e9
    print(f"copy probe: {ms:.3f} ms, {rate:.0f} GB/s", flush=True)
    assert 1500.0 < rate < 8000.0, (ms, rate)
    ms = binding.sagebwd_probe_stream(binding.PROBE_STREAM_READ, src, None, reps=2)
    rate = n / (ms * 1e-3) / 1e9
    print(f"read probe: {ms:.3f} ms, {rate:.0f} GB/s", flush=True)
    assert 1500.0 < rate < 8000.0, (ms, rate)
    # a ragged size (not a multiple of the unrolled stride) still copies every piece
    m = (1 << 20) + 48
    a = torch.randint(0, 255, (m,), dtype=torch.uint8, device="cuda")
    b = torch.zeros_like(a)
    binding.sagebwd_probe_stream(binding.PROBE_STREAM_COPY, a, b, reps=1)
    assert torch.equal(a, b)
