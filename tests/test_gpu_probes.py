"""The two measurement aids of the C-ABI: the streaming-read probe and the clock sample.  Neither is part of the
method; the benchmark reports their figures next to the decode step's bandwidth and the training step's
throughput, so they are checked for what they promise: the probe reads (and leaves memory alone), the clock
sample's two counters advance at the rates the header states."""
import pytest
import torch

from paper_2505_24544_amd import binding as bx

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_read_probe_touches_nothing_and_rejects_bad_arguments():
    buf = torch.arange(1 << 20, dtype=torch.int32, device=DEV)
    ref = buf.clone()
    sink = torch.zeros(4, dtype=torch.int32, device=DEV)
    for nbytes in (16, 4096 + 16, buf.numel() * 4):
        bx.beagle_xattn_probe_read(buf, nbytes, 64, sink)
    torch.cuda.synchronize()
    assert torch.equal(buf, ref)
    assert int(sink.abs().sum()) == 0          # the magic XOR value is not hit by this pattern
    with pytest.raises(bx.BeagleError):
        bx.beagle_xattn_probe_read(buf, 0, 64, sink)
    with pytest.raises(bx.BeagleError):
        bx.beagle_xattn_probe_read(buf, 4096, 0, sink)
    with pytest.raises(bx.BeagleError):
        bx.beagle_xattn_probe_read(buf.data_ptr() + 4, 4096, 64, sink)


def test_clock_sample_counters_advance_at_the_stated_rates():
    out = torch.zeros(2, bx.BEAGLE_CLOCK_SLOTS, 2, dtype=torch.int64, device=DEV)
    a = torch.randn(4096, 4096, device=DEV)
    b = a @ a                                     # library set-up happens here, not inside the sampled region:
    torch.cuda.synchronize()                      # while the GPU idles its cycle counters all but stand still
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    bx.beagle_xattn_probe_clock(out[0])
    e0.record()
    for _ in range(20):
        b = a @ b * 1e-3                          # some milliseconds of work on the same stream
    e1.record()
    bx.beagle_xattn_probe_clock(out[1])
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1)
    c = out.cpu().numpy()
    slots = [x for x in range(bx.BEAGLE_CLOCK_SLOTS) if c[0, x, 1] > 0 and c[1, x, 1] > c[0, x, 1]]
    assert len(slots) >= 64, len(slots)           # 1024 workgroups reach most of the 256 compute units, both times
    for x in slots:
        d_cycles, d_real = int(c[1, x, 0] - c[0, x, 0]), int(c[1, x, 1] - c[0, x, 1])
        # the constant-rate clock runs at 100 MHz: its span covers the event-timed region (and little more)
        assert 0.9 * ms <= d_real / 1e5 <= 1.5 * ms + 0.2, (x, d_real, ms)
        # the cycle counter runs at the shader clock: between the chip's idle and boost frequencies
        mhz = d_cycles / d_real * 100.0
        assert 500.0 <= mhz <= 3000.0, (x, mhz)
    with pytest.raises(bx.BeagleError):
        bx.beagle_xattn_probe_clock(out.data_ptr() + 4)
    with pytest.raises(bx.BeagleError):
        bx.beagle_xattn_probe_clock(None)
