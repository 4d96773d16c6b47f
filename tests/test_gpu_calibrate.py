"""lcn_calibrate: the part's ceilings measured in place (what the roofline
fractions are read against; no part of the method)."""
import pytest

pytestmark = pytest.mark.gpu


def test_measured_ceilings_are_plausible():
    import torch
    import paper_2107_06876_amd as lcn
    buf = torch.empty(512 << 20, dtype=torch.uint8, device="cuda:0")
    copy = lcn.lcn_calibrate(lcn.CAL_COPY_GBS, buf)
    read = lcn.lcn_calibrate(lcn.CAL_READ_GBS, buf)
    bf16 = lcn.lcn_calibrate(lcn.CAL_MFMA_BF16_TFLOPS, buf)
    f64 = lcn.lcn_calibrate(lcn.CAL_MFMA_F64_TFLOPS, buf)
    launch = lcn.lcn_calibrate(lcn.CAL_LAUNCH_US, buf)
    print("copy %.0f GB/s, read %.0f GB/s, bf16 %.0f TFLOP/s, fp64 %.1f TFLOP/s, empty launch %.2f us"
          % (copy, read, bf16, f64, launch), flush=True)
    # nothing can beat the published peaks (8 TB/s, 2.5 PFLOP/s, 78.6 TFLOP/s); a tenth of them is the least to expect
    assert 800.0 < copy < 8000.0 * 1.05 and 800.0 < read < 8000.0 * 1.05
    assert 250.0 < bf16 < 2500.0 * 1.05 and 7.8 < f64 < 78.6 * 1.05
    assert 0.5 < launch < 50.0


def test_calibrate_rejects_a_workspace_that_is_too_small_or_misaligned():
    import torch
    import paper_2107_06876_amd as lcn
    small = torch.empty(1 << 20, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(lcn.LcnError) as err:
        lcn.lcn_calibrate(lcn.CAL_COPY_GBS, small)
    assert err.value.status == lcn.binding.ERR_INVALID_ARG
    big = torch.empty((64 << 20) + 256, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(lcn.LcnError) as err:
        lcn.lcn_calibrate(lcn.CAL_READ_GBS, big[1:])
    assert err.value.status == lcn.binding.ERR_INVALID_ARG
    with pytest.raises(lcn.LcnError) as err:
        lcn.lcn_calibrate(7, big)
    assert err.value.status == lcn.binding.ERR_INVALID_ARG
