"""The matrix-core rate probe (a measurement aid): it runs, and what it reports is physically sensible."""
import pytest
import torch

import paper_2509_15763_amd as u

pytestmark = pytest.mark.gpu


def test_probe_reports_a_sensible_rate_and_clock():
    ones = torch.ones(16384, dtype=torch.bfloat16, device="cuda")
    rnd = torch.randn(16384, generator=torch.Generator().manual_seed(0)).to(torch.bfloat16).cuda()
    tf1, mhz1 = u.probe_mfma_rate(ones, blocks=256, iters=20000)
    tf2, mhz2 = u.probe_mfma_rate(rnd, blocks=256, iters=20000)
    print("constant operands", tf1, mhz1, "random operands", tf2, mhz2, flush=True)
    for tf, mhz in ((tf1, mhz1), (tf2, mhz2)):
        assert 500.0 < tf < 2600.0          # no more than the published peak of 2.5 PFLOP/s (plus timing slack)
        assert 800.0 < mhz < 2500.0
        # 1024 SIMDs, one 32x32x16 MFMA (32768 flops) per 32 cycles each: no faster than that at the clock it held
        assert tf <= 1024 * 32768 / 32 * mhz * 1e-6 * 1.05
