"""The benchmark aid lococo_measure_peaks on a real GPU."""
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_measured_peaks_are_plausible():
    """A bare MFMA loop and a plain copy on this GPU land below the published peaks (2.5 PFLOP/s
    bf16, 8 TB/s) and within reach of them; bad arguments are refused."""
    from paper_2406_05317_amd import binding as lb
    scratch = torch.empty(2 << 30, dtype=torch.uint8, device="cuda")
    tf, gbs = lb.lococo_measure_peaks(scratch)
    print(f"bare MFMA loop {tf:.0f} TFLOP/s, copy {gbs:.0f} GB/s")
    assert 800.0 < tf < 2600.0, tf
    assert 1000.0 < gbs < 8200.0, gbs
    with pytest.raises(lb.LococoError) as e:
        lb.lococo_measure_peaks(scratch[:1 << 20])
    assert e.value.status == lb.LOCOCO_EINVAL
    with pytest.raises(lb.LococoError) as e:
        lb.lococo_measure_peaks(scratch[1:(64 << 20) + 1])
    assert e.value.status == lb.LOCOCO_EINVAL
