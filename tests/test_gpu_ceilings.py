"""The measured-ceiling diagnostics (what plain kernels reach on the box) return sane figures.
No parity content: nothing of the sweep runs in them."""
import pytest

from paper_2605_18856_amd import bsse

pytestmark = pytest.mark.gpu


def test_plain_ceilings_are_below_the_vendor_peaks_and_not_far_below():
    c = bsse.bsse_ceilings()
    assert 3000.0 < c["stream_read_GBs"] < 8000.0
    assert 1200.0 < c["mfma_bf16_TFLOPs"] < 2600.0
    assert 80.0 < c["mfma_f32_TFLOPs"] < 160.0
    assert 0.2 < c["empty_launch_us"] < 50.0


def test_mixed_ceiling_falls_with_the_vector_share():
    alone = bsse.bsse_mixed_ceiling(32, 0)
    light = bsse.bsse_mixed_ceiling(32, 96)
    heavy = bsse.bsse_mixed_ceiling(32, 312)
    heavier = bsse.bsse_mixed_ceiling(32, 960)
    assert 1200.0 < alone < 2600.0
    assert heavier < heavy < light <= alone * 1.05
    # 960 vector instructions of 4 cycles for two wavefronts per SIMD bound the rate by themselves
    assert heavier < 0.4 * alone
    with pytest.raises(bsse.BsseError):
        bsse.bsse_mixed_ceiling(30, 312)
