"""The render kernel's two arithmetic shortcuts equal the plain forms for every float (exhaustive, on the device)."""
import pytest

pytestmark = pytest.mark.gpu


def test_short_reciprocal_and_floor_convert_are_exact_everywhere():
    import torch
    assert torch.cuda.is_available()
    from paper_2502_00021_amd import pxr
    r = pxr.selftest_arithmetic()
    # every float in [2^-100, 2^100]: 200 binades of 2^23 values, plus the upper end point
    assert r["recip_checked"] == 200 * 2 ** 23 + 1, r
    # every pattern that is not NaN: 2^32 - 2 * (2^23 - 1)
    assert r["floor_checked"] == 2 ** 32 - 2 * (2 ** 23 - 1), r
    assert r["recip_mismatches"] == 0 and r["floor_mismatches"] == 0, r
