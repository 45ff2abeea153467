"""The diagnostic call that measures what the device sustains: it runs, stays inside its buffer
(the buffer's neighbours keep their contents) and reports rates of a plausible order."""
import pytest

from paper_2406_17808_amd import binding as B

pytestmark = pytest.mark.gpu


def test_measured_ceilings_are_sane():
    import torch
    nbytes = 1 << 30
    guard = 1 << 20
    buf = torch.full((nbytes + 2 * guard,), 7, dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    c = B.cascade_measure_ceilings(buf.data_ptr() + guard, nbytes, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert bool((buf[:guard] == 7).all()) and bool((buf[-guard:] == 7).all())
    assert c["compute_units"] > 0 and c["core_clock_mhz"] > 0
    for key in ("read_gb_s", "read_regions_gb_s", "read_with_stores_gb_s", "two_pass_read_gb_s", "copy_gb_s"):
        assert 500.0 < c[key] < 8000.0 * 1.05, (key, c[key])          # HBM3E of one MI355X: 8 TB/s
    assert 100.0 < c["mfma_bf16_tflops"] < 2500.0 * 1.05
    # a write stream next to the reads never makes the reads faster (5 % for run-to-run noise)
    assert c["read_with_stores_gb_s"] < 1.05 * c["read_regions_gb_s"]


def test_measured_ceilings_reject_bad_arguments():
    import torch
    buf = torch.empty(1 << 20, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(B.CascadeError):
        B.cascade_measure_ceilings(buf.data_ptr(), 1 << 20)       # below 1 GiB
    with pytest.raises(B.CascadeError):
        B.cascade_measure_ceilings(0, 1 << 30)
