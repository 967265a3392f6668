"""GPU parity at the benchmark configurations' full sizes, in the launch configuration
bench.py times (the library's default parameters): EVERY output element is compared with the
fp64 / int32 oracle (scaled error <= 1e-4 for the contractions, relative error <= 1e-6 for the
stencil, bit-exact for the custom reduce); tile corners and edges are asserted by name on top."""
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


def scaled_err(got, ref, refabs):
    """Componentwise-scaled error |gpu - ref| / sum |a*b| of every element (fp64)."""
    return np.abs(got.astype(np.float64) - ref) / refabs


def assert_named(err, positions, tol, what):
    """Tile corners / edges asserted one by one, so that a failure names the position."""
    for pos in positions:
        pos = tuple(min(max(int(x), 0), s - 1) for x, s in zip(pos, err.shape))
        assert err[pos] <= tol, (what, pos, float(err[pos]))


def matmul_edges(M, N):
    # corners, and both sides of the 64 / 128 / 256 tile boundaries and of the XCD band boundary
    e = [(0, 0), (M - 1, N - 1), (0, N - 1), (M - 1, 0)]
    for t in (32, 64, 128, 256, 1024):
        e += [(t - 1, t - 1), (t, t), (M - t - 1, t - 1), (M - t, N - t), (t - 1, N - t)]
    return e


@pytest.mark.parametrize("name", ["matmul_4096", "matmul_ts"])
def test_matmul_full_size_whole_output(name):
    cfg = W.CONFIGS[name]
    A, Bm = W.matmul_inputs(cfg)
    sizes = (cfg.M, cfg.N, cfg.K)
    a, b = dev(A), dev(Bm)
    C = torch.full((cfg.M, cfg.N), float("nan"), dtype=torch.float32, device="cuda")
    mdh.mdh_matmul(a, b, C, None, ws_for(mdh.MDH_MATMUL, sizes))
    torch.cuda.synchronize()
    got = C.cpu().numpy()
    del a, b, C
    assert np.all(np.isfinite(got))
    ref, refabs = oracle.matmul(A, Bm, with_abs=True)  # every element, fp64
    err = scaled_err(got, ref, refabs)
    assert_named(err, matmul_edges(cfg.M, cfg.N), TOL_CONTRACTION, name)
    assert float(err.max()) <= TOL_CONTRACTION, (name, np.unravel_index(int(err.argmax()), err.shape))


def test_matmul_ts_split_and_unsplit_whole_output():
    cfg = W.CONFIGS["matmul_ts"]
    sizes = (cfg.M, cfg.N, cfg.K)
    A, Bm = W.matmul_inputs(cfg)
    a, b = dev(A), dev(Bm)
    outs = []
    seen = set()
    d = mdh.mdh_default_params(mdh.MDH_MATMUL, sizes)
    cands = [mdh.mdh_candidate(mdh.MDH_MATMUL, sizes, i) for i in range(mdh.mdh_num_candidates(mdh.MDH_MATMUL, sizes))]
    # the default's own tile first (split 4 ways it is the configuration of bench.py's split-k line)
    cands.sort(key=lambda p: not all(list(p.prt[l][:3]) == list(d.prt[l][:3]) for l in (1, 2, 4, 5)))
    for p in cands:
        S = p.prt[3][2]
        if S in seen or S not in (1, 2, 4, 8):
            continue
        seen.add(S)
        n = mdh.mdh_workspace_size(mdh.MDH_MATMUL, sizes, p)
        ws = torch.empty(max(n, 4) // 4, dtype=torch.int32, device="cuda") if n else None
        C = torch.full((cfg.M, cfg.N), float("nan"), dtype=torch.float32, device="cuda")
        mdh.mdh_matmul(a, b, C, p, ws)
        torch.cuda.synchronize()
        outs.append((S, C.cpu().numpy()))
        del ws, C
    assert len(outs) >= 3 and any(S == 4 for S, _ in outs), "the split-k path (S = 4 is the bench line) was not exercised"
    ref, refabs = oracle.matmul(A, Bm, with_abs=True)
    for S, got in outs:
        err = scaled_err(got, ref, refabs)
        assert_named(err, matmul_edges(cfg.M, cfg.N), TOL_CONTRACTION, "split k x%d" % S)
        assert float(err.max()) <= TOL_CONTRACTION, (S, np.unravel_index(int(err.argmax()), err.shape))


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


def test_mcc_full_size_whole_output():
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
    # every element, one image at a time (the fp64 reference of one image is 51 MB)
    edges = [(0, 0, 0), (P - 1, Q - 1, cfg.K - 1), (3, 31, 63), (4, 32, 64), (P - 1, 0, cfg.K - 1), (100, Q - 1, 0),
             (7, 63, 31), (8, 64, 32), (P - 4, Q - 32, 96), (P - 5, Q - 33, 95)]
    worst = 0.0
    for n in range(cfg.N):
        ref, refabs = oracle.mcc(x[n:n + 1], f, cfg.stride, with_abs=True)
        err = scaled_err(got[n], ref[0], refabs[0])
        assert_named(err, edges, TOL_CONTRACTION, "image %d" % n)
        worst = max(worst, float(err.max()))
        assert worst <= TOL_CONTRACTION, (n, np.unravel_index(int(err.argmax()), err.shape))


def test_custom_reduce_full_size_whole_output():
    cfg = W.CONFIGS["prl_2p16_2p18"]
    A, Bt, wp, wm = W.prl_inputs(cfg)
    sizes = (cfg.nA, cfg.nB, cfg.nF)
    s = torch.full((cfg.nA,), -1, dtype=torch.int32, device="cuda")
    i = torch.full((cfg.nA,), -1, dtype=torch.int32, device="cuda")
    mdh.mdh_custom_reduce(dev(A), dev(Bt), dev(wp), dev(wm), s, i, None, ws_for(mdh.MDH_CUSTOM_REDUCE, sizes))
    torch.cuda.synchronize()
    gs, gi = s.cpu().numpy(), i.cpu().numpy()
    rs, ri = oracle.custom_reduce(A, Bt, wp, wm)  # all 2^16 records against all 2^18, int32
    for a in (0, 63, 64, 127, 128, cfg.nA - 1):  # lane / wavefront / workgroup boundaries, by name
        assert (gs[a], gi[a]) == (rs[a], ri[a]), a
    assert np.array_equal(gs, rs) and np.array_equal(gi, ri)
