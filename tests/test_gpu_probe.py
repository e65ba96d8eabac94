"""The matrix-instruction rate probe runs and reports figures that make sense (it is a measurement helper: the
numbers themselves belong to the bench)."""
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tr():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2603_21365_amd import tide_route
    tide_route.load_library()
    return tide_route


def test_mfma_probe_reports_a_plausible_rate(tr):
    for waves in (4, 8):
        for zero in (False, True):
            r = tr.mfma_probe(waves, 64, 3, zero)
            # 32 cycles per instruction when a wave issues back to back (two waves of a SIMD run one after the other
            # rather than in turns, so a wave sees little more than that in its own loop either way)
            assert 30.0 <= r["cycles_per_instruction_and_wave"] <= 80.0, r
            assert 0.5 <= r["clock_ghz"] <= 2.6, r
            assert 300.0 <= r["tflops"] <= 2600.0, r          # never above the nominal 2.5 PFLOP/s
