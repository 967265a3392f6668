"""MCC_Capsule (ten dimensions; MCC on 4 x 4 matrices): host planner and GPU parity against the
oracle, element by element at small shapes and at the paper's first-layer shapes."""
import numpy as np
import pytest

import oracle
import paper_2405_05118_amd as mdh
from paper_2405_05118_amd import binding as B
from paper_2405_05118_amd import workloads as W

TOL = 1e-4

RESNET50 = dict(H=230, W=230, C=3, K=64, R=7, S=7, stride=(2, 2))
MOBILENET = dict(H=225, W=225, C=3, K=32, R=3, S=3, stride=(2, 2))
VGG16 = dict(H=224, W=224, C=3, K=64, R=3, S=3, stride=(1, 1))


def sizes_of(N, H, Wd, C, K, R, S, stride):
    P, Q = (H - R) // stride[0] + 1, (Wd - S) // stride[1] + 1
    return (N, P, Q, K, C, R, S, stride[0], stride[1])


def test_planner_ten_dimensions():
    for net in (RESNET50, MOBILENET, VGG16):
        s = sizes_of(16, net["H"], net["W"], net["C"], net["K"], net["R"], net["S"], net["stride"])
        p = mdh.mdh_default_params(mdh.MDH_MCC_CAPSULE, s)
        assert p.D == 10
        ext = (s[0], s[1], s[2], s[3], 4, 4, s[4], s[5], s[6], 4)
        for d in range(10):
            e = p.extent(d)
            assert e >= ext[d] if p.ragged else e == ext[d]
        assert [p.extent(d) for d in (4, 5, 9)] == [4, 4, 4]
        assert mdh.mdh_validate_params(mdh.MDH_MCC_CAPSULE, s, p) == 0
        n = mdh.mdh_num_candidates(mdh.MDH_MCC_CAPSULE, s)
        assert n >= 1
        for i in range(n):
            assert mdh.mdh_validate_params(mdh.MDH_MCC_CAPSULE, s, mdh.mdh_candidate(mdh.MDH_MCC_CAPSULE, s, i)) == 0
    # many input channels: the filter slice does not fit in LDS
    s = sizes_of(1, 38, 38, 64, 128, 7, 7, (1, 1))
    with pytest.raises(mdh.MdhError) as e:
        mdh.mdh_default_params(mdh.MDH_MCC_CAPSULE, s)
    assert e.value.status == 4


torch = pytest.importorskip("torch")


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def inputs(N, H, Wd, C, K, R, S, seed):
    x = W.normal(seed, 1, (N, H, Wd, C, 4, 4))
    f = W.normal(seed, 2, (K, R, S, C, 4, 4))
    return x, f


def run(x, f, stride, p):
    N, H, Wd = x.shape[:3]
    K, R, S = f.shape[:3]
    P, Q = (H - R) // stride[0] + 1, (Wd - S) // stride[1] + 1
    out = torch.full((N, P, Q, K, 4, 4), float("nan"), dtype=torch.float32, device="cuda")
    mdh.mdh_mcc_capsule(dev(x), dev(f), out, stride, p)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64)


SMALL = [
    # N, H, W, C, K, R, S, stride
    (1, 12, 21, 3, 8, 7, 7, (2, 2)),
    (2, 9, 12, 3, 32, 3, 3, (2, 2)),
    (1, 8, 19, 3, 70, 3, 3, (1, 1)),
    (2, 5, 9, 1, 5, 2, 3, (1, 2)),
    (1, 7, 8, 2, 16, 1, 1, (1, 1)),
    (1, 6, 30, 4, 12, 5, 2, (3, 1)),
]


@pytest.mark.gpu
@pytest.mark.parametrize("case", SMALL)
def test_small_all_candidates(case):
    N, H, Wd, C, K, R, S, stride = case
    x, f = inputs(N, H, Wd, C, K, R, S, W.SEED_BASE + 97)
    ref, refabs = oracle.mcc_capsule(x, f, stride, with_abs=True)
    s = sizes_of(N, H, Wd, C, K, R, S, stride)
    cands = [None] + [mdh.mdh_candidate(mdh.MDH_MCC_CAPSULE, s, i) for i in range(mdh.mdh_num_candidates(mdh.MDH_MCC_CAPSULE, s))]
    for p in cands:
        got = run(x, f, stride, p)
        assert np.all(np.isfinite(got)), "output not fully overwritten"
        err = float(np.max(np.abs(got - ref) / np.where(refabs > 0, refabs, 1.0)))
        assert err <= TOL, (case, p and p.table())


@pytest.mark.gpu
def test_identity_matrices_and_ones():
    # identity 4x4 filter matrices at one tap: a shifted copy of the input blocks, exactly
    x = W.normal(W.SEED_BASE + 98, 1, (1, 9, 11, 3, 4, 4))
    f = np.zeros((8, 3, 3, 3, 4, 4), np.float32)
    f[5, 2, 1, 2] = np.eye(4)
    got = run(x, f, (1, 1), None)
    assert np.array_equal(got[0, :, :, 5], x[0, 2:9, 1:10, 2].astype(np.float64))
    assert np.all(got[0, :, :, :5] == 0)
    ones = run(np.ones((1, 7, 8, 3, 4, 4), np.float32), np.ones((8, 3, 3, 3, 4, 4), np.float32), (1, 1), None)
    assert np.all(ones == 3 * 3 * 3 * 4)


@pytest.mark.gpu
@pytest.mark.parametrize("net,N", [(RESNET50, 2), (MOBILENET, 2), (VGG16, 1), (RESNET50, 16)])  # the last: as timed by bench.py
def test_paper_shapes_whole_output(net, N):
    # every output element (one image at a time) against the fp64 oracle
    x, f = inputs(N, net["H"], net["W"], net["C"], net["K"], net["R"], net["S"], W.SEED_BASE + 99)
    got = run(x, f, net["stride"], None)
    _, P, Q, K = got.shape[:4]
    assert np.all(np.isfinite(got))
    for n in range(N):
        ref, refabs = oracle.mcc_capsule(x[n:n + 1], f, net["stride"], with_abs=True)
        err = np.abs(got[n] - ref[0]) / refabs[0]
        for pos in ((0, 0, 0, 0, 0), (P - 1, Q - 1, K - 1, 3, 3), (P - 1, 0, K - 1, 0, 3), (3, 7, 7, 1, 2), (4, 8, 8 % K, 2, 1)):
            assert err[pos] <= TOL, (n, pos)
        assert float(err.max()) <= TOL, (n, np.unravel_index(int(err.argmax()), err.shape))


@pytest.mark.gpu
def test_tune_picks_a_valid_configuration():
    N, H, Wd, C, K, R, S, stride = 1, 21, 40, 3, 16, 3, 3, (2, 2)
    x, f = inputs(N, H, Wd, C, K, R, S, W.SEED_BASE + 96)
    s = sizes_of(N, H, Wd, C, K, R, S, stride)
    out = torch.empty((N, s[1], s[2], K, 4, 4), dtype=torch.float32, device="cuda")
    best, ms = mdh.mdh_tune(mdh.MDH_MCC_CAPSULE, s, [dev(x), dev(f), out], reps=2)
    assert ms > 0 and mdh.mdh_validate_params(mdh.MDH_MCC_CAPSULE, s, best) == 0
    ref, refabs = oracle.mcc_capsule(x, f, stride, with_abs=True)
    assert float(np.max(np.abs(run(x, f, stride, best) - ref) / refabs)) <= TOL
