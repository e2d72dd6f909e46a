"""The benchmark's measurement aids return plausible figures (they are context for the roofline fractions)."""
import pytest
import torch

from paper_2604_05426_amd import binding as ml

pytestmark = pytest.mark.gpu


def test_calibration_kernels_report_plausible_rates():
    dev = torch.device("cuda:0")
    scratch = torch.zeros(4096, dtype=torch.uint8, device=dev)
    buf = torch.zeros(64 << 20, dtype=torch.uint8, device=dev)
    zeros = ml.multi_lora_calib_mfma(False, scratch)
    rand = ml.multi_lora_calib_mfma(True, scratch)
    read = ml.multi_lora_calib_read(buf, buf.numel(), scratch)
    # dense bf16 MFMA peak is 2.5 PFLOP/s, HBM peak 8 TB/s (a 64 MiB buffer is served by the Infinity Cache)
    assert 500.0 < rand <= zeros * 1.05 and zeros < 2600.0
    assert 1000.0 < read < 20000.0
    assert torch.count_nonzero(scratch).item() == 0
    with pytest.raises(ml.MultiLoraError):
        ml.multi_lora_calib_read(buf, 1024, scratch)
