"""The library's measured-peak microbenchmarks return plausible figures for an MI355X."""
import pytest

pytestmark = pytest.mark.gpu


def test_measured_peaks_are_plausible():
    import torch
    assert torch.cuda.is_available()
    from paper_2502_00021_amd import pxr
    pk = pxr.measure_peaks()
    # 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz = 39.3 T lane-operations/s is the ceiling for unpacked VALU work
    assert 15.0 < pk["fma_tlaneops"] <= 40.0, pk
    assert 15.0 < pk["imad_tlaneops"] <= 40.0, pk
    assert 1500.0 < pk["copy_gbs"] <= 8000.0, pk
    assert 1500.0 < pk["write_gbs"] <= 8000.0 and 1500.0 < pk["read_gbs"] <= 8000.0, pk
    assert pk["read_gbs"] > 0.9 * pk["write_gbs"]
