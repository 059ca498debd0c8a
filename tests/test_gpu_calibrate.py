"""The two calibration calls give plausible figures for an MI355X (bounded by its published peaks)."""
import pytest

pytestmark = pytest.mark.gpu


def test_mfma_loop_and_copy_rates_are_below_the_published_peaks():
    import paper_2211_12281_amd as kge
    kge.load()
    tf = kge.calibrate_mfma(2048)
    assert 300.0 < tf <= 2500.0 * 1.02, tf         # dense bf16 peak 2.5 PFLOP/s
    tv = kge.calibrate_mfma(2048, varied=True)     # the same loop on operands that toggle bits: never faster by more than noise
    assert 300.0 < tv <= tf * 1.05, (tv, tf)
    gbs = kge.calibrate_copy(1 << 28)
    assert 1000.0 < gbs <= 8000.0 * 1.02, gbs      # HBM3E peak 8 TB/s
