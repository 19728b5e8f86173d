"""The matrix-core rate probe returns sane figures: positive, below the published peak, and not faster with random
operands than with zeros (the chip throttles under switching load, never the other way round)."""
from __future__ import annotations

import pytest

from paper_2502_16982_amd import binding

pytestmark = pytest.mark.gpu


def test_mfma_probe_reports_plausible_rates():
    zeros = binding.muon_probe_mfma_rate(False, iters=8000)
    rand = binding.muon_probe_mfma_rate(True, iters=8000)
    for r in (zeros, rand):
        assert 100.0 < r["tflops"] < 2600.0
        assert 300.0 < r["clock_mhz"] < 2600.0
    assert rand["tflops"] <= zeros["tflops"] * 1.05


def test_mfma_probe_rejects_bad_arguments():
    with pytest.raises(binding.MuonError):
        binding.muon_probe_mfma_rate(True, iters=0)
