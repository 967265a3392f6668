"""Calibration kernels of the library (measurement support): they must move / count what they say."""
import pytest

import paper_2405_05118_amd as mdh
from paper_2405_05118_amd import binding as B
from paper_2405_05118_amd import workloads as W

torch = pytest.importorskip("torch")


@pytest.mark.gpu
def test_copy_and_read():
    n = 3 * 1024 * 1024 + 64  # not a multiple of the grid size
    src = W.device_uniform(W.SEED_BASE + 90, 1, (n,), 0.0, 1.0)
    dst = torch.zeros_like(src)
    mdh.mdh_calib_copy(src, dst)
    out = torch.full((B.MDH_CALIB_STREAM_LANES + 64,), float("nan"), dtype=torch.float32, device="cuda")
    mdh.mdh_calib_read(src, out)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    # every element is read exactly once: the partial sums add up to the sum of the buffer
    want = float(src.double().sum())
    assert abs(float(out[: B.MDH_CALIB_STREAM_LANES].double().sum()) - want) <= 1e-6 * want
    assert torch.isnan(out[B.MDH_CALIB_STREAM_LANES:]).all()  # nothing written beyond the documented size


@pytest.mark.gpu
def test_mfma_and_valu_counts():
    out = torch.empty(B.MDH_CALIB_BLOCKS * 256, dtype=torch.float32, device="cuda")
    flop = mdh.mdh_calib_mfma(out, 8)
    torch.cuda.synchronize()
    assert flop == B.MDH_CALIB_BLOCKS * 4 * 8 * 16 * 4096
    # lane (m, k-half) x (n, k-half): a = (lane & 7)/8, b = (lane & 3)/4 summed over k in {0,1};
    # the value only has to be finite and identical for all workgroups
    assert torch.isfinite(out).all()
    assert torch.equal(out[:256], out[-256:])
    outi = torch.empty(B.MDH_CALIB_BLOCKS * 256, dtype=torch.int32, device="cuda")
    ops = mdh.mdh_calib_valu(outi, 4)
    torch.cuda.synchronize()
    assert ops == B.MDH_CALIB_BLOCKS * 256 * 4 * 64
    with pytest.raises(mdh.MdhError):
        mdh.mdh_calib_mfma(out, 0)
