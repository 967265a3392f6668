"""Multi-channel convolution with few input channels and strides (the first-layer shapes of the
paper's deep-learning study: ResNet-50 N x 230 x 230 x 3 -> 64 channels, 7x7, stride 2; MobileNet
N x 225 x 225 x 3 -> 32 channels, 3x3, stride 2).  The library fuses the reduction dimensions s
and c there; the definition (and the oracle) is unchanged."""
import numpy as np
import pytest

import oracle
import paper_2405_05118_amd as mdh
from paper_2405_05118_amd import binding as B
from paper_2405_05118_amd import workloads as W

TOL = 1e-4

RESNET50 = dict(H=230, W=230, C=3, K=64, R=7, S=7, stride=(2, 2))
MOBILENET = dict(H=225, W=225, C=3, K=32, R=3, S=3, stride=(2, 2))


def sizes_of(N, H, Wd, C, K, R, S, stride):
    P, Q = (H - R) // stride[0] + 1, (Wd - S) // stride[1] + 1
    return (N, P, Q, K, C, R, S, stride[0], stride[1])


def test_default_fuses_s_and_c_for_few_channels():
    for net in (RESNET50, MOBILENET):
        s = sizes_of(16, net["H"], net["W"], net["C"], net["K"], net["R"], net["S"], net["stride"])
        p = mdh.mdh_default_params(mdh.MDH_MCC, s)
        assert p.blk[4] == 1 and p.prt[1][4] == net["C"]  # c walked in single steps inside LDS
        assert p.prt[0][4] == 1  # and not chunked over the HBM layer
        assert mdh.mdh_validate_params(mdh.MDH_MCC, s, p) == 0
        for d in range(7):
            assert p.extent(d) >= s[d] if p.ragged else p.extent(d) == s[d]
    # ResNet's 112 output columns are 7 blocks of 16, not a multiple of 32: no ragged columns
    s = sizes_of(1, 230, 230, 3, 64, 7, 7, (2, 2))
    p = mdh.mdh_default_params(mdh.MDH_MCC, s)
    assert p.blk[2] == 16 and p.extent(2) == 112 and p.prt[B.L_HBM][2] == 1 and p.strided == 0
    # with a batch of 16 the tiles (16 x 16 pixels x 32 channels) are dealt out one at a time to the
    # workgroups resident on the chip (strided = 1: parts of (n, p, q) not owned by position)
    s = sizes_of(16, 230, 230, 3, 64, 7, 7, (2, 2))
    p = mdh.mdh_default_params(mdh.MDH_MCC, s)
    assert p.blk[2] == 16 and p.extent(2) == 112 and p.strided == 1
    assert p.prt[B.L_HBM][2] == 1 and p.prt[B.L_WG][2] == 7 and p.prt[B.L_WG][1] == 7 and p.prt[B.L_WG][3] == 2
    assert mdh.mdh_validate_params(mdh.MDH_MCC, s, p) == 0
    q = p.copy()
    q.prt[B.L_HBM][2], q.prt[B.L_WG][2] = 7, 1  # dealt tiles are single column tiles
    assert mdh.mdh_validate_params(mdh.MDH_MCC, s, q) != 0
    cands = [mdh.mdh_candidate(mdh.MDH_MCC, s, i) for i in range(mdh.mdh_num_candidates(mdh.MDH_MCC, s))]
    assert any(c.blk[2] == 32 and c.extent(2) == 128 for c in cands)
    # the owned variant (a workgroup walks the whole row of 7 tiles with its filter slice resident) stays
    # a candidate, and the default of the 3 x 3 filters (6 steps per tile)
    assert any(c.blk[4] == 1 and c.strided == 0 and c.prt[B.L_HBM][2] == 7 and c.prt[B.L_WG][2] == 1 for c in cands)
    v = mdh.mdh_default_params(mdh.MDH_MCC, sizes_of(16, 226, 226, 3, 64, 3, 3, (1, 1)))
    assert v.blk[4] == 1 and v.strided == 0 and v.prt[B.L_HBM][2] > 1
    # many channels keep the channel-chunked kernel
    p = mdh.mdh_default_params(mdh.MDH_MCC, (16, 224, 224, 128, 64, 7, 7, 1, 1))
    assert p.blk[4] == 2


torch = pytest.importorskip("torch")


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run(x, f, stride, p):
    N, H, Wd, C = x.shape
    K, R, S, _ = f.shape
    P, Q = (H - R) // stride[0] + 1, (Wd - S) // stride[1] + 1
    out = torch.full((N, P, Q, K), float("nan"), dtype=torch.float32, device="cuda")
    n = mdh.mdh_workspace_size(mdh.MDH_MCC, (N, P, Q, K, x.shape[3], R, S, stride[0], stride[1]), p)
    ws = torch.empty(max(n, 4) // 4, dtype=torch.int32, device="cuda") if n else None
    mdh.mdh_mcc(dev(x), dev(f), out, stride, p, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64)


SMALL = [
    # N, H, W, C, K, R, S, stride
    (1, 1, 1, 3, 2, 1, 1, (1, 1)),   # three input elements: fewer than one 16-byte piece
    (1, 1, 4, 1, 3, 1, 2, (1, 1)),   # exactly four
    (2, 2, 1, 1, 1, 2, 1, (1, 1)),
    (2, 37, 37, 3, 64, 7, 7, (2, 2)),
    (1, 21, 40, 3, 32, 3, 3, (2, 2)),
    (2, 12, 19, 1, 5, 3, 2, (1, 1)),
    (1, 30, 30, 4, 70, 5, 5, (1, 2)),
    (1, 9, 70, 8, 130, 1, 1, (1, 1)),
    (3, 10, 11, 2, 33, 2, 3, (3, 1)),
]


@pytest.mark.gpu
@pytest.mark.parametrize("case", SMALL)
def test_small_all_candidates(case):
    N, H, Wd, C, K, R, S, stride = case
    x, f = W.mcc_inputs(W.MccCfg(N, H, Wd, C, K, R, S, stride, W.SEED_BASE + 71))
    ref, refabs = oracle.mcc(x, f, stride, with_abs=True)
    s = sizes_of(N, H, Wd, C, K, R, S, stride)
    cands = [None] + [mdh.mdh_candidate(mdh.MDH_MCC, s, i) for i in range(mdh.mdh_num_candidates(mdh.MDH_MCC, s))]
    if N * H * Wd * C >= 4:  # that kernel reads 16-byte pieces: an input of fewer than four elements has none
        assert any(p is not None and p.blk[4] == 1 for p in cands), "the fused (s,c) kernel is not among the candidates"
    else:
        assert not any(p is not None and p.blk[4] == 1 for p in cands)
    for p in cands:
        got = run(x, f, stride, p)
        assert np.all(np.isfinite(got)), "output not fully overwritten"
        err = float(np.max(np.abs(got - ref) / np.where(refabs > 0, refabs, 1.0)))
        assert err <= TOL, (case, p and p.table(), p and list(p.blk))


@pytest.mark.gpu
def test_dealt_tiles_draw_tickets_and_leave_the_counters_at_zero():
    # more tiles than resident workgroups: all but the first two tiles of a workgroup come from the ticket
    # counter of its filter slice (two slices here, the second ragged).  Every dealt candidate against the
    # oracle and bit for bit against the owned-tile default; calls of other shapes in between and a second
    # round show that every call leaves the counters at zero.
    N, H, Wd, C, K, R, S, stride = 40, 99, 163, 3, 40, 5, 5, (2, 2)
    x, f = W.mcc_inputs(W.MccCfg(N, H, Wd, C, K, R, S, stride, W.SEED_BASE + 74))
    ref, refabs = oracle.mcc(x, f, stride, with_abs=True)
    s = sizes_of(N, H, Wd, C, K, R, S, stride)
    cands = [mdh.mdh_candidate(mdh.MDH_MCC, s, i) for i in range(mdh.mdh_num_candidates(mdh.MDH_MCC, s))]
    dealt = [p for p in cands if p.blk[4] == 1 and p.strided == 1]
    owned = [p for p in cands if p.blk[4] == 1 and p.strided == 0]
    assert len(dealt) >= 6 and owned
    for p in dealt:  # more tiles than a launch keeps resident (at most 4 workgroups per compute unit)
        assert p.prt[B.L_WG][0] * p.prt[B.L_WG][1] * p.prt[B.L_WG][2] * p.prt[B.L_WG][3] > 1024
    base = run(x, f, stride, owned[0])
    assert float(np.max(np.abs(base - ref) / np.where(refabs > 0, refabs, 1.0))) <= TOL
    xs, fs = W.mcc_inputs(W.MccCfg(3, 21, 40, 3, 32, 3, 3, (2, 2), W.SEED_BASE + 75))
    small_ref = run(xs, fs, (2, 2), None)
    for rnd in range(2):
        for p in dealt:
            got = run(x, f, stride, p)
            assert np.array_equal(got, base), (rnd, p.table(), list(p.blk))
            assert np.array_equal(run(xs, fs, (2, 2), None), small_ref)


@pytest.mark.gpu
def test_all_ones_closed_form():
    x = np.ones((1, 23, 39, 3), np.float32)
    f = np.ones((64, 7, 7, 3), np.float32)
    got = run(x, f, (2, 2), None)
    assert got.shape == (1, 9, 17, 64) and np.all(got == 147)


@pytest.mark.gpu
@pytest.mark.parametrize("net,N", [(RESNET50, 16), (RESNET50, 1), (MOBILENET, 16)])
def test_paper_shapes_whole_output(net, N):
    # every output element of the paper's first-layer shapes against the fp64 oracle
    cfg = W.MccCfg(N, net["H"], net["W"], net["C"], net["K"], net["R"], net["S"], net["stride"], W.SEED_BASE + 72)
    x, f = W.mcc_inputs(cfg)
    got = run(x, f, cfg.stride, None)
    _, P, Q, K = got.shape
    assert np.all(np.isfinite(got))
    for n in range(N):
        ref, refabs = oracle.mcc(x[n:n + 1], f, cfg.stride, with_abs=True)
        err = np.abs(got[n] - ref[0]) / refabs[0]
        for pos in ((0, 0, 0), (P - 1, Q - 1, K - 1), (P - 1, 0, K - 1), (7, 15, 31), (8, 16, 32 % K)):
            assert err[pos] <= TOL, (n, pos)
        assert float(err.max()) <= TOL, (n, np.unravel_index(int(err.argmax()), err.shape))


@pytest.mark.gpu
def test_conv2d_is_the_single_channel_special_case():
    # Conv2D = md_hom(*, (++,++,+,+)) over (p,q,r,s): MCC with N = K = C = 1 (the classical variant the
    # paper contrasts MCC with); checked through mdh_mcc and through the generic runtime-compiled path
    Hh, Wd, R, S = 45, 70, 5, 3
    x, f = W.mcc_inputs(W.MccCfg(1, Hh, Wd, 1, 1, R, S, (1, 1), W.SEED_BASE + 73))
    ref, refabs = oracle.mcc(x, f, (1, 1), with_abs=True)
    got = run(x, f, (1, 1), None)
    assert float(np.max(np.abs(got - ref) / refabs)) <= TOL
    P, Q = Hh - R + 1, Wd - S + 1
    d = mdh.custom_desc((P, Q, R, S), (0, 0, 1, 1), ["float", "float"],
                        [(0, "(i0+i2)*%d+(i1+i3)" % Wd), (1, "i2*N3+i3")], "float", 4, "r = a0 * a1;", "r = x + y;", fast_dim=1)
    op = mdh.mdh_custom_create(d)
    out = torch.full((P, Q), float("nan"), dtype=torch.float32, device="cuda")
    n = mdh.mdh_custom_workspace_size(op)
    ws = torch.empty(max(n, 4), dtype=torch.uint8, device="cuda") if n else None
    mdh.mdh_custom_run(op, [dev(x), dev(f)], out, ws)
    torch.cuda.synchronize()
    g2 = out.cpu().numpy().astype(np.float64)
    assert float(np.max(np.abs(g2 - ref[0, :, :, 0]) / refabs[0, :, :, 0])) <= TOL
