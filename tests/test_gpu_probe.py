"""The register-only MFMA rate probe (measurement aid): it runs, ends, and reports a rate inside what
the chip can do: above a fifth of the published bf16 peak, not more than a clock-boost margin above it, and pseudo-random operands
no faster than smooth ones (the clock under matrix load falls with operand toggling)."""
import pytest
import torch

from paper_2512_12131_amd import binding as B

pytestmark = pytest.mark.gpu
PEAK = 2500.0


def test_mfma_probe_reports_a_plausible_rate():
    torch.cuda.set_device(0)
    print("mfma probe: smooth, then pseudo-random operands", flush=True)
    smooth = B.lr_mfma_probe(False, 4000, 10)
    rnd = B.lr_mfma_probe(True, 4000, 10)
    print(f"smooth {smooth:.0f} TFLOP/s, pseudo-random {rnd:.0f} TFLOP/s", flush=True)
    assert 0.2 * PEAK < rnd <= 1.03 * smooth
    assert smooth <= 1.10 * PEAK   # 2.4 GHz is the published clock; a box may hold a little more on smooth operands
