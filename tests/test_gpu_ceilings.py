"""The measured-ceiling helper on the GPU: its rates must be physically plausible."""
import pytest
import torch

import paper_1211_5590_amd as rnn


@pytest.mark.gpu
def test_measured_ceilings_are_plausible_for_this_chip():
    """The saturating kernels must land at or a little around the published peaks (the clock may sit a few
    per cent above nominal) and not absurdly far under them."""
    scratch = torch.empty(1 << 28, dtype=torch.float32, device="cuda")   # 1 GiB
    c = rnn.rnn_measure_ceilings(scratch)
    torch.cuda.synchronize()
    assert 2000.0 < c["hbm_copy_GBps"] <= 8000.0 * 1.05
    assert c["hbm_copy_GBps"] * 0.8 < c["hbm_read_GBps"] <= 8000.0 * 1.05
    assert 60.0 < c["mfma_f32_TFLOPs"] <= 157.3 * 1.10
    assert 1000.0 < c["mfma_bf16_TFLOPs"] <= 2500.0 * 1.10
    assert 0.3 * 256 * 128 * 2.4 < c["lds_read_GBps"] <= 256 * 256 * 2.4 * 1.10
