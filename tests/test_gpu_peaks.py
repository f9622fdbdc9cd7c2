"""The measurement library (libcodecomp_peaks.so) on the GPU: its figures are physically sensible and ordered the way
the design document reads them.  Loose bounds: these are measurements, not results."""
import pytest

pytestmark = pytest.mark.gpu


def test_peaks_are_sensible():
    from paper_2604_10235_amd import peaks
    try:
        peaks.measure()                       # first call: set-up and clocks
        m = peaks.measure()
    finally:
        peaks.release()
    assert m["compute_units"] >= 1 and m["mix_waves_per_simd"] == 2
    assert 200.0 < m["mfma_bf16_tflops"] < 2600.0            # below the published dense bf16 peak
    assert 1e12 < m["exp_per_s"] < m["fma_per_s"] < 2e14      # an exponential costs several fused multiply-adds
    assert 1e12 < m["mix_logits_per_s"] < 2e13
    # the mix cannot beat the MFMA alone (32 cycles per MFMA and SIMD) and is no worse than MFMA + VALU work in turn
    assert 32.0 <= m["mix_cycles_per_mfma"] < 80.0
    assert 500.0 < m["read_gb_per_s"] < 8000.0 and 500.0 < m["copy_gb_per_s"] < 8000.0


def test_pass_model_rows():
    from paper_2604_10235_amd import peaks
    try:
        rows = peaks.measure_pass_model()
    finally:
        peaks.release()
    assert len(rows) >= 8 and rows[0]["features"] == "LDS ring + barrier"
    for r in rows:
        assert 5e11 < r["logits_per_s"] < 2e13 and 500 < r["clock_mhz"] < 3000 and 32.0 <= r["cycles_per_mfma"] < 150.0, r
        streams = "loads" in r["features"]
        assert (r["hbm_gb_per_s"] > 100.0) == streams and (r["tiles_ahead"] > 0) == streams, r
