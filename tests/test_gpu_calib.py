"""GPU: the matrix-core calibration loops run, report their flop count and reject bad arguments."""
import pytest
import torch

from paper_2405_07719_amd import calib

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mode", [0, 1])
def test_calib_mfma_runs_and_counts_flop(usp, mode):
    sink = torch.full((calib.USP_CALIB_SINK_BYTES // 4,), float("nan"), dtype=torch.float32, device="cuda")
    flop = calib.usp_calib_mfma(mode, 11, sink)          # odd: rounded down to 10 steps
    torch.cuda.synchronize()
    assert flop == 256 * 8 * 10 * 32 * 2 * 32 * 32 * 16
    assert bool(torch.isfinite(sink).all())            # every thread of every workgroup stored its sum


def test_calib_mfma_rejects_bad_arguments(usp):
    sink = torch.empty(calib.USP_CALIB_SINK_BYTES, dtype=torch.uint8, device="cuda")
    small = torch.empty(1024, dtype=torch.uint8, device="cuda")
    with pytest.raises(usp.UspError) as e:
        calib.usp_calib_mfma(0, 10, small)
    assert e.value.status == 5
    with pytest.raises(usp.UspError):
        calib.usp_calib_mfma(2, 10, sink)
    with pytest.raises(usp.UspError):
        calib.usp_calib_mfma(0, 1, sink)
