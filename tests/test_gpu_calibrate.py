"""The two calibration kernels of the benchmark run, are timed by the profiling hook and report their work."""
import pytest
import torch

from paper_2506_19830_amd import binding as B

pytestmark = pytest.mark.gpu


def test_calibration_kernels_run_and_are_timed():
    sink = torch.zeros(64 * 512, dtype=torch.float32, device="cuda")
    word = torch.zeros(4, dtype=torch.int32, device="cuda")
    src = torch.ones((64 << 20) + 48, dtype=torch.uint8, device="cuda")[:(64 << 20) + 16]   # a ragged tail of pieces
    B.la_profile_reset()
    B.la_profile_select(["calib_mfma", "calib_read"], 1)
    B.la_profile_enable(True)
    flops = B.la_calibrate_mfma(64, 100, sink)
    nbytes = B.la_calibrate_read(src, word)
    torch.cuda.synchronize()
    B.la_profile_enable(False)
    prof = B.la_profile_collect()
    B.la_profile_select(None, 1)
    B.la_profile_reset()
    assert flops == 64 * 8 * 4 * 100 * 2 * 32 * 32 * 16
    assert nbytes == (64 << 20) + 16
    assert prof["calib_mfma"][0] == 1 and prof["calib_mfma"][1] > 0
    assert prof["calib_read"][0] == 1 and prof["calib_read"][1] > 0
    assert torch.isfinite(sink).all() and (sink != 0).any()        # the accumulators were written out
    assert int(word[0]) == 0                                       # the read kernel stores nothing on its real path
    with pytest.raises(ValueError):
        B.la_calibrate_mfma(65, 10, sink)                          # sink too small for 65 workgroups
    with pytest.raises(B.LaError):
        B.la_calibrate_read(src[1:17], word)                       # not 16-byte aligned
