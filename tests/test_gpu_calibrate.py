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
    sink.zero_()
    assert B.la_calibrate_mfma(64, 100, sink, data=True) == flops     # the loop on pseudo-random operands
    torch.cuda.synchronize()
    assert torch.isfinite(sink).all() and (sink != 0).any()
    with pytest.raises(B.LaError):
        B.la_calibrate_mfma(64, 101, sink, data=True)              # an odd number of rounds
    with pytest.raises(ValueError):
        B.la_calibrate_mfma(65, 10, sink)                          # sink too small for 65 workgroups
    with pytest.raises(B.LaError):
        B.la_calibrate_read(src[1:17], word)                       # not 16-byte aligned


def test_device_exponential_of_the_accept_path_is_accurate():
    """The fp64 exponential the resampling kernels use (their own routine) against numpy's over the range they meet:
    within two units in the last place for normal results, exact zero far below the range, denormal results to an
    absolute 1e-320."""
    import numpy as np
    rng = np.random.default_rng(5)
    y = np.concatenate([-rng.random(400_000) * 40.0,                  # the bulk of a row: masses down to e^-40
                        -rng.random(200_000) * 700.0,                 # the whole normal range
                        -np.logspace(-18, 0, 20_000),                 # next to 0
                        np.array([0.0, -0.0, -1e-300, -708.3, -745.0, -750.0, -1e4, -1e300, -np.inf]),
                        -(np.arange(2000) + 0.5) * np.log(2.0),       # half-way points of the argument reduction
                        -700.0 - rng.random(10_000) * 45.0])          # into the denormals
    dev = torch.from_numpy(y).cuda()
    out = torch.full_like(dev, float("nan"))
    B.la_selftest_exp64(dev, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    with np.errstate(under="ignore"):
        ref = np.exp(y)
    assert np.isfinite(got).all() and (got >= 0).all()
    normal = ref >= 2.3e-308
    ulp = np.spacing(ref[normal])
    assert (np.abs(got[normal] - ref[normal]) <= 2 * ulp).all(), float((np.abs(got[normal] - ref[normal]) / ulp).max())
    assert (np.abs(got[~normal] - ref[~normal]) <= 1e-320).all()
    assert (got[y <= -750.0] == 0.0).all() and got[y == 0.0].tolist() == [1.0, 1.0]
    with pytest.raises(B.LaError):
        B.la_selftest_exp64(None, out)
