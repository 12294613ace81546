"""The ceiling probes run and report plausible rates (they are measurement aids, not part of the
attention path)."""

import pytest
import torch

from paper_2407_17678_amd import binding as B

pytestmark = pytest.mark.gpu


def _time(fn, n=3):
    fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(n):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / n * 1e-3


def test_mfma_probe_rates():
    scratch = torch.empty(max(B.s2_probe_scratch_bytes(), 4 << 20), dtype=torch.uint8, device="cuda")
    rates = []
    for mix in (0, 1):
        flops = [0.0]

        def run():
            flops[0] = B.s2_probe_mfma(mix, 4000, scratch)
        rates.append(flops[0] / _time(run) / 1e12 if _time(run) else 0.0)
    # between a fifth of the published 2.5 PFLOP/s and all of it; vector work beside the MFMAs costs something
    assert 500 < rates[1] <= rates[0] * 1.05 and rates[0] < 2600, rates
    assert torch.isfinite(scratch[:B.s2_probe_scratch_bytes()].view(torch.float32)).all()


def test_read_probe_rate():
    scratch = torch.empty(4 << 20, dtype=torch.uint8, device="cuda")
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_(0, 255)
    gbs = (1 << 30) / _time(lambda: B.s2_probe_read(src, scratch)) / 1e9
    assert 1000 < gbs < 8200, gbs


def test_atomic_add_probe_adds_what_it_says():
    buf = torch.zeros(4 << 20, dtype=torch.float32, device="cuda")   # 16 MiB = 1024 tiles
    added = B.s2_probe_atomic_add(buf)
    torch.cuda.synchronize()
    assert float(buf.double().sum().item()) * 4 == added   # every add is 1.0f on a 4-byte element
