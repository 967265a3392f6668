"""GPU parity at the benchmark configurations' full sizes, in the launch configuration
bench.py times (the library's default parameters): sampled outputs the oracle computes
one by one, plus properties that hold at any size."""
import numpy as np
import pytest

import oracle
import paper_2405_05118_amd as mdh
from paper_2405_05118_amd import workloads as W

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL_CONTRACTION = 1e-4
TOL_STENCIL = 1e-6


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def ws_for(inst, sizes):
    n = mdh.mdh_workspace_size(inst, sizes)
    return torch.empty(max(n, 4) // 4, dtype=torch.int32, device="cuda") if n else None


def sample_positions(rng, shape, n, tile_edges=()):
    """Random positions plus the corners and a few tile-edge positions."""
    pos = [tuple(int(rng.integers(0, s)) for s in shape) for _ in range(n)]
    pos += [tuple(0 for _ in shape), tuple(s - 1 for s in shape)]
    for e in tile_edges:
        pos.append(tuple(min(max(x, 0), s - 1) for x, s in zip(e, shape)))
    return np.array(pos, dtype=np.int64)


@pytest.mark.parametrize("name", ["matmul_4096", "matmul_ts"])
def test_matmul_full_size_sampled(name):
    cfg = W.CONFIGS[name]
    A, Bm = W.matmul_inputs(cfg)
    sizes = (cfg.M, cfg.N, cfg.K)
    a, b = dev(A), dev(Bm)
    C = torch.full((cfg.M, cfg.N), float("nan"), dtype=torch.float32, device="cuda")
    mdh.mdh_matmul(a, b, C, None, ws_for(mdh.MDH_MATMUL, sizes))
    torch.cuda.synchronize()
    got = C.cpu().numpy()
    assert np.all(np.isfinite(got))
    rng = np.random.default_rng(1)
    pos = sample_positions(rng, (cfg.M, cfg.N), 2000, [(127, 127), (128, 128), (cfg.M - 129, 63), (255, 64 % cfg.N)])
    ref, refabs = oracle.matmul_at(A, Bm, pos[:, 0], pos[:, 1])
    err = np.abs(got[pos[:, 0], pos[:, 1]].astype(np.float64) - ref) / refabs
    assert err.max() <= TOL_CONTRACTION
    # property at any size: column sums.  1^T C = (1^T A) B, evaluated in fp64 on the host
    colsum = got.astype(np.float64).sum(axis=0)
    want = A.astype(np.float64).sum(axis=0) @ Bm.astype(np.float64)
    scale = np.abs(A.astype(np.float64)).sum(axis=0) @ np.abs(Bm.astype(np.float64))
    assert np.max(np.abs(colsum - want) / scale) <= TOL_CONTRACTION


def test_matmul_ts_split_and_unsplit_agree():
    cfg = W.CONFIGS["matmul_ts"]
    sizes = (cfg.M, cfg.N, cfg.K)
    A, Bm = W.matmul_inputs(cfg)
    a, b = dev(A), dev(Bm)
    outs = []
    seen = set()
    for i in range(mdh.mdh_num_candidates(mdh.MDH_MATMUL, sizes)):
        p = mdh.mdh_candidate(mdh.MDH_MATMUL, sizes, i)
        S = p.prt[3][2]
        if S in seen or S not in (1, 2, 8):
            continue
        seen.add(S)
        n = mdh.mdh_workspace_size(mdh.MDH_MATMUL, sizes, p)
        ws = torch.empty(max(n, 4) // 4, dtype=torch.int32, device="cuda") if n else None
        C = torch.empty((cfg.M, cfg.N), dtype=torch.float32, device="cuda")
        mdh.mdh_matmul(a, b, C, p, ws)
        torch.cuda.synchronize()
        outs.append((S, C.cpu().numpy().astype(np.float64)))
        del ws
    assert len(outs) >= 2 and any(S > 1 for S, _ in outs), "the split-k path was not exercised"
    rng = np.random.default_rng(2)
    pos = sample_positions(rng, (cfg.M, cfg.N), 500)
    ref, refabs = oracle.matmul_at(A, Bm, pos[:, 0], pos[:, 1])
    for S, got in outs:
        err = np.abs(got[pos[:, 0], pos[:, 1]] - ref) / refabs
        assert err.max() <= TOL_CONTRACTION, S


def test_jacobi_full_size():
    cfg = W.CONFIGS["jacobi3d_512"]
    x = W.stencil_inputs(cfg)
    out = torch.full((cfg.nx, cfg.ny, cfg.nz), float("nan"), dtype=torch.float32, device="cuda")
    mdh.mdh_stencil(dev(x), out, cfg.c0, cfg.c1)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    del out
    ref = oracle.jacobi3d(x, cfg.c0, cfg.c1)  # the full oracle takes well under a second
    err = np.abs(got.astype(np.float64) - ref) / np.where(ref != 0, ref, 1.0)
    assert float(err.max()) <= TOL_STENCIL


def test_mcc_full_size_sampled():
    cfg = W.CONFIGS["mcc_resnet"]
    x, f = W.mcc_inputs(cfg)
    P = (cfg.H - cfg.R) // cfg.stride[0] + 1
    Q = (cfg.W - cfg.S) // cfg.stride[1] + 1
    out = torch.full((cfg.N, P, Q, cfg.K), float("nan"), dtype=torch.float32, device="cuda")
    sizes = (cfg.N, P, Q, cfg.K, cfg.C, cfg.R, cfg.S, cfg.stride[0], cfg.stride[1])
    mdh.mdh_mcc(dev(x), dev(f), out, cfg.stride, None, ws_for(mdh.MDH_MCC, sizes))
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    del out
    assert np.all(np.isfinite(got))
    rng = np.random.default_rng(3)
    pos = sample_positions(rng, (cfg.N, P, Q, cfg.K), 3000, [(0, 3, 31, 63), (5, 4, 32, 64), (15, 223, 0, 127), (7, 100, 223, 0)])
    ref, refabs = oracle.mcc_at(x, f, pos, cfg.stride)
    err = np.abs(got[tuple(pos.T)].astype(np.float64) - ref) / refabs
    assert err.max() <= TOL_CONTRACTION
    # property at any size: summing the output over k equals convolving with the k-summed filter
    fsum = f.astype(np.float64).sum(axis=0, keepdims=True).astype(np.float32)
    refs, refsabs = oracle.mcc_at(x, fsum, np.concatenate([pos[:200, :3], np.zeros((200, 1), np.int64)], 1), cfg.stride)
    gsum = got[tuple(pos[:200, :3].T)].astype(np.float64).sum(axis=-1)
    assert np.max(np.abs(gsum - refs) / (refsabs * cfg.K)) <= TOL_CONTRACTION


def test_custom_reduce_full_size_sampled():
    cfg = W.CONFIGS["prl_2p16_2p18"]
    A, Bt, wp, wm = W.prl_inputs(cfg)
    sizes = (cfg.nA, cfg.nB, cfg.nF)
    s = torch.full((cfg.nA,), -1, dtype=torch.int32, device="cuda")
    i = torch.full((cfg.nA,), -1, dtype=torch.int32, device="cuda")
    mdh.mdh_custom_reduce(dev(A), dev(Bt), dev(wp), dev(wm), s, i, None, ws_for(mdh.MDH_CUSTOM_REDUCE, sizes))
    torch.cuda.synchronize()
    gs, gi = s.cpu().numpy(), i.cpu().numpy()
    rng = np.random.default_rng(4)
    rows = np.unique(np.concatenate([rng.integers(0, cfg.nA, 300), [0, 63, 64, 127, 128, cfg.nA - 1]]))
    rs, ri = oracle.custom_reduce_rows(A, Bt, wp, wm, rows)
    assert np.array_equal(gs[rows], rs) and np.array_equal(gi[rows], ri)
    # properties for every a: the reported index is in range and really scores the reported
    # score (vectorised numpy over all a), and no record of a random subset of B beats it
    assert gi.min() >= 0 and gi.max() < cfg.nB
    d = (wp.astype(np.int64) - wm.astype(np.int64))
    sc = ((A == Bt[gi]) * d + wm.astype(np.int64)).sum(axis=1)
    assert np.array_equal(sc, gs.astype(np.int64))
    sub = rng.integers(0, cfg.nB, 64)
    for b in sub:
        sb = ((A == Bt[b]) * d + wm.astype(np.int64)).sum(axis=1)
        assert np.all((sb < gs) | ((sb == gs) & (gi <= b)))
