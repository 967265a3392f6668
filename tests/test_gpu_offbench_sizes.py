"""Library defaults at sizes other than the benchmark ones, where the planner takes a different
(de/re)-composition: other MFMA pixel blocks and a split channel dimension for small images,
ragged MatMul extents with 64 x 64 tiles, a deep split of k, narrow stencil grids, rows of a
thousand elements in the scan.  Sampled against the oracle (or the whole output where the oracle
is fast enough)."""
import numpy as np
import pytest

import oracle
import paper_2405_05118_amd as mdh
from paper_2405_05118_amd import binding as B
from paper_2405_05118_amd import workloads as W

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 1e-4


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def ws_for(inst, sizes):
    n = mdh.mdh_workspace_size(inst, sizes)
    return torch.empty(max(n, 4) // 4, dtype=torch.int32, device="cuda") if n else None


@pytest.mark.parametrize("case", [
    # N, H, W, C, K, R, S, stride, expected (blk[p], blk[q]), channel parts > 1
    (16, 9, 9, 512, 512, 3, 3, 1, (4, 8), True),
    (16, 16, 16, 256, 256, 3, 3, 1, (2, 16), True),
    (16, 58, 58, 64, 64, 3, 3, 1, (4, 8), False),
    (8, 114, 114, 32, 64, 3, 3, 1, (2, 16), False),
    (3, 30, 30, 200, 70, 3, 3, 2, None, True),
])
def test_mcc_defaults_on_small_images(case):
    N, H, Wd, C, K, R, S, st, blk, split = case
    cfg = W.MccCfg(N, H, Wd, C, K, R, S, (st, st), W.SEED_BASE + 95)
    x, f = W.mcc_inputs(cfg)
    P, Q = (H - R) // st + 1, (Wd - S) // st + 1
    sizes = (N, P, Q, K, C, R, S, st, st)
    p = mdh.mdh_default_params(mdh.MDH_MCC, sizes)
    if blk is not None:
        assert (p.blk[1], p.blk[2]) == blk
    assert (p.prt[B.L_WG][4] > 1) == split
    out = torch.full((N, P, Q, K), float("nan"), dtype=torch.float32, device="cuda")
    mdh.mdh_mcc(dev(x), dev(f), out, (st, st), None, ws_for(mdh.MDH_MCC, sizes))
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.all(np.isfinite(got))
    rng = np.random.default_rng(5)
    pos = np.array([[rng.integers(0, N), rng.integers(0, P), rng.integers(0, Q), rng.integers(0, K)] for _ in range(1500)]
                   + [[0, 0, 0, 0], [N - 1, P - 1, Q - 1, K - 1], [0, P - 1, 0, K - 1], [N - 1, 0, Q - 1, 0]], dtype=np.int64)
    ref, refabs = oracle.mcc_at(x, f, pos, (st, st))
    assert float(np.max(np.abs(got[tuple(pos.T)].astype(np.float64) - ref) / refabs)) <= TOL


@pytest.mark.parametrize("shape", [(3000, 3000, 1000), (1000, 1000, 1000), (64, 64, 1 << 20), (4096, 200, 4100)])
def test_matmul_defaults_on_ragged_and_deep_shapes(shape):
    M, N, K = shape
    A = W.uniform(W.SEED_BASE + 96, 1, (M, K), -1, 1)
    Bm = W.uniform(W.SEED_BASE + 96, 2, (K, N), -1, 1)
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    mdh.mdh_matmul(dev(A), dev(Bm), C, None, ws_for(mdh.MDH_MATMUL, shape))
    torch.cuda.synchronize()
    got = C.cpu().numpy()
    assert np.all(np.isfinite(got))
    rng = np.random.default_rng(6)
    i = np.concatenate([rng.integers(0, M, 800), [0, M - 1, M - 1, 0, min(M - 1, 127), min(M - 1, 128)]])
    j = np.concatenate([rng.integers(0, N, 800), [0, N - 1, 0, N - 1, min(N - 1, 63), min(N - 1, 64)]])
    ref, refabs = oracle.matmul_at(A, Bm, i, j)
    assert float(np.max(np.abs(got[i, j].astype(np.float64) - ref) / refabs)) <= TOL


@pytest.mark.parametrize("shape", [(200, 260, 64), (64, 300, 128), (130, 130, 100)])
def test_stencil_defaults_on_narrow_grids(shape):
    cfg = W.StencilCfg(*shape, 0.5, float(np.float32(1.0 / 12.0)), W.SEED_BASE + 97)
    x = W.stencil_inputs(cfg)
    p = mdh.mdh_default_params(mdh.MDH_STENCIL, shape)
    assert p.prt[B.L_LANE][2] < 64
    out = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    mdh.mdh_stencil(dev(x), out, cfg.c0, cfg.c1)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    ref = oracle.jacobi3d(x, cfg.c0, cfg.c1)
    assert float(np.max(np.abs(got - ref) / np.where(ref != 0, np.abs(ref), 1.0))) <= 1e-6


@pytest.mark.parametrize("shape", [(5000, 1000), (3000, 1536), (6000, 700)])
def test_scan_defaults_on_rows_of_about_a_thousand(shape):
    R, n = shape
    X = W.uniform(W.SEED_BASE + 98, 1, (R, n), -1, 1)
    out = torch.full((R, n), float("nan"), dtype=torch.float32, device="cuda")
    mdh.mdh_scan(dev(X), out, None, ws_for(mdh.MDH_SCAN, (R, n)))
    torch.cuda.synchronize()
    ref, refabs = oracle.scan_rows(X, with_abs=True)
    assert float(np.max(np.abs(out.cpu().numpy().astype(np.float64) - ref) / np.where(refabs > 0, refabs, 1.0))) <= 1e-5


def test_mcc_tune_with_and_without_workspace():
    # with a workspace the search may pick a configuration that splits the channel dimension over
    # workgroups; without one those candidates are skipped and the result needs no workspace
    cfg = W.MccCfg(4, 9, 9, 256, 128, 3, 3, (1, 1), W.SEED_BASE + 99)
    x, f = W.mcc_inputs(cfg)
    sizes = (4, 7, 7, 128, 256, 3, 3, 1, 1)
    out = torch.full((4, 7, 7, 128), float("nan"), dtype=torch.float32, device="cuda")
    ref, refabs = oracle.mcc(x, f, (1, 1), with_abs=True)
    big = torch.empty(8 * out.numel(), dtype=torch.float32, device="cuda")
    for ws in (big, None):
        best, ms = mdh.mdh_tune(mdh.MDH_MCC, sizes, [dev(x), dev(f), out], workspace=ws, reps=2)
        assert ms > 0 and mdh.mdh_validate_params(mdh.MDH_MCC, sizes, best) == 0
        need = mdh.mdh_workspace_size(mdh.MDH_MCC, sizes, best)
        assert need <= (big.numel() * 4 if ws is not None else 0)
        out.fill_(float("nan"))
        mdh.mdh_mcc(dev(x), dev(f), out, (1, 1), best, ws)
        torch.cuda.synchronize()
        assert float(np.max(np.abs(out.cpu().numpy().astype(np.float64) - ref) / refabs)) <= TOL
