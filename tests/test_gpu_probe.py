"""The benchmark's probe of what plain kernels reach on the GPU: runs, and lands where an MI355X can land."""
import pytest
import torch

import paper_2501_07145_amd as rfsf

pytestmark = pytest.mark.gpu


def test_probe_peaks_are_plausible():
    scratch = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")        # four times the last-level cache
    p = rfsf.rfsf_ts_probe_peaks(scratch)
    print(p)
    for key in ("read_gbs", "write_gbs", "write_nt_gbs", "copy_gbs"):
        assert 1500.0 < p[key] < 8000.0, (key, p[key])                       # below the published 8 TB/s, above a third of it
    assert 100.0 < p["mfma_f32_tflops"] < 157.3 * 1.02                       # the issue loop comes close to the fp32 matrix peak
    assert 50.0 < p["valu_f32_tflops"] < 157.3 * 1.02
