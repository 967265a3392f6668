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


@pytest.mark.gpu
def test_valu_kinds_count_and_compute():
    import numpy as np

    outi = torch.empty(B.MDH_CALIB_BLOCKS * 256, dtype=torch.int32, device="cuda")
    clk = torch.zeros(2, dtype=torch.int64, device="cuda")
    for kind in (B.MDH_CALIB_KIND_XOR_MAX, B.MDH_CALIB_KIND_CMP_SELECT, B.MDH_CALIB_KIND_ADD3, B.MDH_CALIB_KIND_FMA_F32,
                 B.MDH_CALIB_KIND_ADD_VGPR):
        ops = mdh.mdh_calib_valu_kind(kind, outi, 64, None, clk)
        torch.cuda.synchronize()
        assert ops == B.MDH_CALIB_BLOCKS * 256 * 64 * 64
        c = clk.cpu().numpy()
        assert c[0] > 0 and c[1] > 0
    hz = mdh.mdh_calib_realtime_hz()
    assert hz > 0
    # the instruction-mix loop really evaluates the max-with-index reduction it is modelled on: redo it
    # on the host for the 256 lanes of a workgroup (every workgroup computes the same)
    rng = np.random.default_rng(11)
    w = np.concatenate([rng.integers(1, 1000, 8), rng.integers(-1000, 0, 8), rng.integers(0, 16, 256 * 2 * 8)]).astype(np.int32)
    iters = 200
    ops = mdh.mdh_calib_valu_kind(B.MDH_CALIB_KIND_PRL_MIX, outi, iters, torch.from_numpy(w).cuda(), clk)
    torch.cuda.synchronize()
    assert ops == B.MDH_CALIB_BLOCKS * 256 * iters * 48
    ar = w[16:].reshape(256, 2, 8).astype(np.int64)
    dw = (w[:8].astype(np.int64) - w[8:16].astype(np.int64))
    base = int(w[8:16].astype(np.int64).sum())
    bs = np.full((256, 2), -2**31, dtype=np.int64)
    bi = np.full((256, 2), 2**31 - 1, dtype=np.int64)
    s = 12345
    for b in range(iters):
        br = np.empty(8, dtype=np.int64)
        for f in range(8):
            s = (s * 5 + 1) & 0xFFFFFFFF
            br[f] = (s >> 9) & 15
        sc = base + ((ar == br) * dw).sum(axis=2)
        take = sc > bs
        bs = np.where(take, sc, bs)
        bi = np.where(take, b, bi)
    want = (bs[:, 0] ^ bi[:, 0] ^ bs[:, 1] ^ bi[:, 1]).astype(np.int64)
    want = ((want + 2**31) % 2**32 - 2**31).astype(np.int32)
    got = outi.cpu().numpy().reshape(-1, 256)
    assert np.array_equal(got[0], want) and np.array_equal(got[-1], want)
    # the loop built from the fast instruction kinds computes the same reduction (scores exact in fp32),
    # reported per block of four made-up records
    blocks = 50
    ops = mdh.mdh_calib_valu_kind(B.MDH_CALIB_KIND_PRL_FAST_MIX, outi, blocks, torch.from_numpy(w).cuda(), clk)
    torch.cuda.synchronize()
    assert ops == B.MDH_CALIB_BLOCKS * 256 * blocks * 203
    agree = int(w[:8].astype(np.int64).sum())
    ndw = (w[8:16].astype(np.int64) - w[:8].astype(np.int64))
    best = np.full((256, 2), -2**62, dtype=np.int64)
    blk = np.zeros((256, 2), dtype=np.int64)
    s = 12345
    for bb in range(blocks):
        top = np.full((256, 2), -2**62, dtype=np.int64)
        for u in range(4):
            br = np.empty(8, dtype=np.int64)
            for f in range(8):
                s = (s * 5 + 1) & 0xFFFFFFFF
                br[f] = (s >> 9) & 15
            top = np.maximum(top, agree + ((ar != br) * ndw).sum(axis=2))
        take = top > best
        blk = np.where(take, bb, blk)
        best = np.maximum(best, top)
    want = (best[:, 0] ^ blk[:, 0] ^ best[:, 1] ^ blk[:, 1])
    want = ((want + 2**31) % 2**32 - 2**31).astype(np.int32)
    got = outi.cpu().numpy().reshape(-1, 256)
    assert np.array_equal(got[0], want) and np.array_equal(got[-1], want)
    ghz = clk.cpu().numpy()[0] / clk.cpu().numpy()[1] * hz / 1e9
    assert 0.3 < ghz < 4.0, ghz
    with pytest.raises(mdh.MdhError):
        mdh.mdh_calib_valu_kind(7, outi, 4)
