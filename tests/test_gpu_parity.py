"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element
on seeded inputs.  Sizes span several tiles and ragged tails; every candidate tile
configuration is a valid (de/re)-composition and must give the same result.

Tolerances (fp32 products are exact in fp64 and every fp32 accumulation step adds at most 2^-24
relative to the running |sum| <= sum |a*b|: worst case K * 2^-24, typically ~sqrt(K) * 2^-24):
  MatMul / MCC : max |gpu - ref| / sum_k |a*b|  <= 1e-4   (componentwise-scaled error)
  Jacobi-3D    : max |gpu - ref| / ref          <= 1e-6   (all terms non-negative)
  custom reduce: bit-exact (int32)
"""
import numpy as np
import pytest

import oracle
import paper_2405_05118_amd as mdh
from paper_2405_05118_amd import binding as B
from paper_2405_05118_amd import workloads as W

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL_CONTRACTION = 1e-4
TOL_STENCIL = 1e-6


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def workspace(inst, sizes, p):
    n = mdh.mdh_workspace_size(inst, sizes, p)
    return torch.empty(max(n, 4) // 4, dtype=torch.int32, device="cuda") if n else None


def candidates(inst, sizes, limit=None):
    n = mdh.mdh_num_candidates(inst, sizes)
    idx = list(range(n))
    if limit is not None and n > limit:
        step = n / float(limit)
        idx = sorted({int(i * step) for i in range(limit)} | {0})
    return [None] + [mdh.mdh_candidate(inst, sizes, i) for i in idx]


# ------------------------------------------------------------------------------ MatMul


def run_matmul(A, Bm, p):
    M, K = A.shape
    N = Bm.shape[1]
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    ws = workspace(mdh.MDH_MATMUL, (M, N, K), p)
    mdh.mdh_matmul(dev(A), dev(Bm), C, p, ws)
    torch.cuda.synchronize()
    return C.cpu().numpy().astype(np.float64)


def scaled_err(got, ref, refabs):
    den = np.where(refabs > 0, refabs, 1.0)
    return float(np.max(np.abs(got - ref) / den))


@pytest.mark.parametrize("shape", [(256, 256, 256), (300, 200, 100), (129, 65, 33), (64, 64, 8), (1, 1, 1), (70, 260, 1030)])
def test_matmul_small_all_candidates(shape):
    M, N, K = shape
    cfg = W.MatmulCfg(M, N, K, W.SEED_BASE + 11)
    A, Bm = W.matmul_inputs(cfg)
    ref, refabs = oracle.matmul(A, Bm, with_abs=True)
    for p in candidates(mdh.MDH_MATMUL, shape, limit=14):
        got = run_matmul(A, Bm, p)
        assert np.all(np.isfinite(got)), "output not fully overwritten"
        assert scaled_err(got, ref, refabs) <= TOL_CONTRACTION, (shape, p and p.table())


@pytest.mark.parametrize("shape", [(1300, 1100, 96), (2200, 700, 64), (640, 2304, 40)])
def test_matmul_both_loop_orders_of_the_workgroup_layer(shape):
    # more than one band of eight tile rows / tile columns, ragged last band, ragged tiles: the two
    # orders assign the same tiles to other workgroups -- same arithmetic per element, same bits
    M, N, K = shape
    A, Bm = W.matmul_inputs(W.MatmulCfg(M, N, K, W.SEED_BASE + 13))
    ref, refabs = oracle.matmul(A, Bm, with_abs=True)
    wg = B.L_WG * B.MDH_MAX_D
    for tile in ((128, 128), (64, 64)):
        cands = [c for c in candidates(mdh.MDH_MATMUL, shape)[1:]
                 if c.prt[B.L_WAVE][2] == 1 and c.prt[B.L_WG][2] == 1 and c.extent(0) // c.prt[B.L_WG][0] == tile[0]
                 and c.extent(1) // c.prt[B.L_WG][1] == tile[1] and list(c.order[:2]) == [wg + 0, wg + 1]]
        assert cands, tile
        p = cands[0]
        q = p.copy()
        q.order[0], q.order[1] = wg + 1, wg + 0
        assert mdh.mdh_validate_params(mdh.MDH_MATMUL, shape, q) == 0
        got_i, got_j = run_matmul(A, Bm, p), run_matmul(A, Bm, q)
        assert np.all(np.isfinite(got_j))
        assert scaled_err(got_i, ref, refabs) <= TOL_CONTRACTION
        assert np.array_equal(got_i, got_j), (shape, tile)


@pytest.mark.parametrize("shape", [(256, 256, 256), (300, 200, 100), (129, 65, 33), (70, 260, 1030), (33, 47, 17),
                                   (17, 16, 4096), (200, 300, 500), (512, 512, 512)])
def test_matmul_k_on_the_wavefront_layer_every_candidate(shape):
    # #PRT(WAVE, k) > 1: every wavefront owns the whole output tile and a part of k, the wavefront results
    # are added in LDS; all instantiations (16 x 16 x 4 and 32 x 32 x 2 blocks, 2..16 wavefronts, with and
    # without workgroup parts of k on top), ragged edges in every dimension
    M, N, K = shape
    A, Bm = W.matmul_inputs(W.MatmulCfg(M, N, K, W.SEED_BASE + 13))
    ref, refabs = oracle.matmul(A, Bm, with_abs=True)
    ks = [p for p in candidates(mdh.MDH_MATMUL, shape) if p is not None and p.prt[B.L_WAVE][2] > 1]
    if K >= 128:  # a wavefront keeps at least 16 k: short reductions have few or no such candidates
        assert len(ks) >= 6, "the wavefront-layer candidates are missing"
        assert {p.blk[0] for p in ks} == {16, 32}
    for p in ks:
        assert p.in_region[0] == B.MR_VGPR and p.out_region == B.MR_LDS
        got = run_matmul(A, Bm, p)
        assert np.all(np.isfinite(got)), "output not fully overwritten"
        assert scaled_err(got, ref, refabs) <= TOL_CONTRACTION, (shape, p.table())
    d = mdh.mdh_default_params(mdh.MDH_MATMUL, shape)
    if M > 16 and K >= 32:
        assert d.prt[B.L_WAVE][2] > 1, "small outputs default to k on the wavefront layer"


def test_matmul_with_few_rows_takes_the_small_m_kernel():
    # M <= 16 through mdh_matmul: the register-streaming kernel of the batched entry point, same bits
    # (both strip widths of that kernel: 64 columns per wavefront, and 16 per workgroup where those fill
    # the chip and the reduction is short -- the last two shapes)
    for M, N, K in ((16, 1000, 2048), (1, 130, 257), (7, 64, 48), (8, 3512, 40), (16, 4096, 1024)):
        A, Bm = W.matmul_inputs(W.MatmulCfg(M, N, K, W.SEED_BASE + 14))
        d = mdh.mdh_default_params(mdh.MDH_MATMUL, (M, N, K))
        assert d.D == 3 and list(d.blk[:3]) == [16, 16, 4]
        assert d.prt[B.L_VGPR][1] == (1 if N >= 3512 else 4)
        assert mdh.mdh_validate_params(mdh.MDH_MATMUL, (M, N, K), d) == 0
        ref, refabs = oracle.matmul(A, Bm, with_abs=True)
        got = run_matmul(A, Bm, None)
        assert scaled_err(got, ref, refabs) <= TOL_CONTRACTION
        assert np.array_equal(got, run_matmul(A, Bm, d))
        C = torch.full((1, M, N), float("nan"), dtype=torch.float32, device="cuda")
        n = mdh.mdh_workspace_size(mdh.MDH_BMATMUL, (1, M, N, K, 0, 0, 0))
        ws = torch.empty(max(n, 4) // 4, dtype=torch.int32, device="cuda") if n else None
        mdh.mdh_matmul_ex(dev(A[None]), dev(Bm[None]), C, False, False, False, None, ws)
        assert np.array_equal(got, C[0].cpu().numpy().astype(np.float64))


def test_matmul_closed_forms():
    # all-ones gives K in every cell (exact in fp32); identity returns A
    M, N, K = 200, 136, 520
    got = run_matmul(np.ones((M, K), np.float32), np.ones((K, N), np.float32), None)
    assert np.all(got == K)
    A = W.uniform(5, 1, (192, 192), -1, 1)
    assert np.array_equal(run_matmul(A, np.eye(192, dtype=np.float32), None), A.astype(np.float64))


def test_matmul_split_is_deterministic_and_homomorphic():
    shape = (128, 64, 2048)
    A, Bm = W.matmul_inputs(W.MatmulCfg(*shape, W.SEED_BASE + 12))
    ref, refabs = oracle.matmul(A, Bm, with_abs=True)
    split = [p for p in candidates(mdh.MDH_MATMUL, shape) if p is not None and p.prt[B.L_WG][2] > 1]
    assert split, "no split-k candidate for a tall reduction"
    for p in split[:4]:
        g1 = run_matmul(A, Bm, p)
        g2 = run_matmul(A, Bm, p)
        assert np.array_equal(g1, g2)
        assert scaled_err(g1, ref, refabs) <= TOL_CONTRACTION
    # homomorphic property on the GPU path: split k by hand, add the halves
    h = run_matmul(np.ascontiguousarray(A[:, :1000]), Bm[:1000], None) + run_matmul(np.ascontiguousarray(A[:, 1000:]), Bm[1000:], None)
    assert scaled_err(h, ref, refabs) <= TOL_CONTRACTION


# ------------------------------------------------------------------------------ Jacobi-3D


def run_stencil(x, c0, c1, p):
    nx, ny, nz = (s - 2 for s in x.shape)
    out = torch.full((nx, ny, nz), float("nan"), dtype=torch.float32, device="cuda")
    mdh.mdh_stencil(dev(x), out, c0, c1, p)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64)


def rel_err(got, ref):
    den = np.where(ref != 0, np.abs(ref), 1.0)
    return float(np.max(np.abs(got - ref) / den))


@pytest.mark.parametrize("shape", [(64, 64, 64), (37, 29, 70), (5, 8, 512), (16, 24, 520), (3, 1, 1), (40, 17, 1030)])
def test_stencil_small_all_candidates(shape):
    cfg = W.StencilCfg(*shape, 0.5, float(np.float32(1.0 / 12.0)), W.SEED_BASE + 21)
    x = W.stencil_inputs(cfg)
    ref = oracle.jacobi3d(x, cfg.c0, cfg.c1)
    for p in candidates(mdh.MDH_STENCIL, shape, limit=12):
        got = run_stencil(x, cfg.c0, cfg.c1, p)
        assert np.all(np.isfinite(got)), "output not fully overwritten"
        assert rel_err(got, ref) <= TOL_STENCIL, (shape, p and p.table())


@pytest.mark.parametrize("shape", [(33, 200, 40), (70, 130, 100), (20, 64, 128), (9, 70, 64)])
def test_stencil_narrow_grids_every_candidate(shape):
    # nz <= 128: the default tiles have 32 or 16 lanes along k and several lane-rows per wavefront
    cfg = W.StencilCfg(*shape, 0.5, float(np.float32(1.0 / 12.0)), W.SEED_BASE + 22)
    x = W.stencil_inputs(cfg)
    ref = oracle.jacobi3d(x, cfg.c0, cfg.c1)
    d = mdh.mdh_default_params(mdh.MDH_STENCIL, shape)
    assert d.prt[B.L_LANE][2] == (16 if shape[2] <= 64 else 32) and d.prt[B.L_LANE][1] * d.prt[B.L_LANE][2] == 64
    for p in candidates(mdh.MDH_STENCIL, shape):
        got = run_stencil(x, cfg.c0, cfg.c1, p)
        assert np.all(np.isfinite(got)), "output not fully overwritten"
        assert rel_err(got, ref) <= TOL_STENCIL, (shape, p and p.table())


def test_stencil_closed_forms_and_halo_untouched():
    nx, ny, nz = 20, 24, 36
    c0, c1 = 0.5, float(np.float32(1.0 / 12.0))
    const = np.full((nx + 2, ny + 2, nz + 2), 3.0, np.float32)
    assert np.allclose(run_stencil(const, c0, c1, None), 3.0, rtol=3e-7, atol=0)
    # a single 1 lands in exactly seven outputs
    x = np.zeros((nx + 2, ny + 2, nz + 2), np.float32)
    x[5, 9, 17] = 1.0
    got = run_stencil(x, 0.5, 0.125, None)
    want = np.zeros((nx, ny, nz))
    want[4, 8, 16] = 0.5
    for d in ((1, 0, 0), (-1, 0, 0), (0, 1, 0), (0, -1, 0), (0, 0, 1), (0, 0, -1)):
        want[4 + d[0], 8 + d[1], 16 + d[2]] = 0.125
    assert np.array_equal(got, want)
    # inputs are never written
    xin = dev(W.uniform(3, 1, (nx + 2, ny + 2, nz + 2), 0, 1))
    keep = xin.clone()
    out = torch.empty((nx, ny, nz), dtype=torch.float32, device="cuda")
    mdh.mdh_stencil(xin, out, c0, c1)
    torch.cuda.synchronize()
    assert torch.equal(xin, keep)


# ------------------------------------------------------------------------------ MCC


def run_mcc(x, f, stride, p):
    N, H, Wd, C = x.shape
    K, R, S, _ = f.shape
    P, Q = (H - R) // stride[0] + 1, (Wd - S) // stride[1] + 1
    out = torch.full((N, P, Q, K), float("nan"), dtype=torch.float32, device="cuda")
    mdh.mdh_mcc(dev(x), dev(f), out, stride, p, workspace(mdh.MDH_MCC, (N, P, Q, K, C, R, S, stride[0], stride[1]), p))
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64)


MCC_SMALL = [
    # N, H, W, C, K, R, S, stride
    (2, 38, 38, 32, 128, 7, 7, (1, 1)),   # full tiles: P = Q = 32
    (1, 20, 45, 16, 64, 3, 3, (1, 1)),    # ragged q
    (2, 15, 17, 5, 9, 3, 2, (2, 2)),      # strided, ragged everything, C not a multiple of 4
    (1, 9, 9, 3, 4, 1, 1, (1, 1)),        # 1x1 filter
    (3, 1, 1, 40, 7, 1, 1, (1, 1)),       # reduces to a matmul
    (2, 16, 16, 24, 40, 3, 3, (1, 1)),    # 14 x 14 outputs: blocks of 2 x 16 and 4 x 8 pixels pay off
    (3, 15, 15, 16, 130, 3, 3, (2, 2)),   # 7 x 7 outputs, strided, ragged channels
    (2, 9, 9, 200, 70, 3, 3, (1, 1)),     # many input channels, few pixels: c split over workgroups
]


@pytest.mark.parametrize("case", MCC_SMALL)
def test_mcc_small_all_candidates(case):
    N, H, Wd, C, K, R, S, stride = case
    cfg = W.MccCfg(N, H, Wd, C, K, R, S, stride, W.SEED_BASE + 31)
    x, f = W.mcc_inputs(cfg)
    ref, refabs = oracle.mcc(x, f, stride, with_abs=True)
    P, Q = ref.shape[1:3]
    sizes = (N, P, Q, K, C, R, S, stride[0], stride[1])
    for p in candidates(mdh.MDH_MCC, sizes):
        got = run_mcc(x, f, stride, p)
        assert np.all(np.isfinite(got)), "output not fully overwritten"
        assert scaled_err(got, ref, refabs) <= TOL_CONTRACTION, (case, p and p.table())


def test_mcc_closed_forms():
    x = np.ones((1, 12, 40, 16), np.float32)
    f = np.ones((32, 5, 5, 16), np.float32)
    assert np.all(run_mcc(x, f, (1, 1), None) == 16 * 25)
    x = W.normal(9, 1, (1, 10, 40, 8))
    f = np.zeros((4, 3, 4, 8), np.float32)
    f[1, 2, 3, 5] = 1.0  # output channel 1 = input channel 5 shifted by (2,3)
    got = run_mcc(x, f, (1, 1), None)
    assert np.array_equal(got[..., 1], x[:, 2:10, 3:40, 5].astype(np.float64))
    assert np.all(got[..., 0] == 0)


# ------------------------------------------------------------------------------ custom reduce


def run_prl(A, Bt, wp, wm, p):
    nA, nF = A.shape
    s = torch.full((nA,), -12345, dtype=torch.int32, device="cuda")
    i = torch.full((nA,), -12345, dtype=torch.int32, device="cuda")
    ws = workspace(mdh.MDH_CUSTOM_REDUCE, (nA, Bt.shape[0], nF), p)
    mdh.mdh_custom_reduce(dev(A), dev(Bt), dev(wp), dev(wm), s, i, p, ws)
    torch.cuda.synchronize()
    return s.cpu().numpy(), i.cpu().numpy()


@pytest.mark.parametrize("shape", [(1000, 3000, 8), (1, 1, 8), (130, 5, 8), (777, 1234, 5), (300, 900, 12), (64, 4097, 16), (513, 700, 1)])
def test_custom_reduce_small_all_candidates(shape):
    nA, nB, nF = shape
    A, Bt, wp, wm = W.prl_inputs(W.PrlCfg(nA, nB, nF, W.SEED_BASE + 41))
    rs, ri = oracle.custom_reduce(A, Bt, wp, wm)
    for p in candidates(mdh.MDH_CUSTOM_REDUCE, shape, limit=16):
        s, i = run_prl(A, Bt, wp, wm, p)
        assert np.array_equal(s, rs) and np.array_equal(i, ri), (shape, p and p.table())


def test_custom_reduce_ties_and_extreme_weights():
    # tiny alphabets: most records tie -> the smallest index must win on every path
    rng = np.random.default_rng(7)
    A = rng.integers(0, 2, (500, 8)).astype(np.int32)
    Bt = rng.integers(0, 2, (2500, 8)).astype(np.int32)
    wp = rng.integers(1, 4, 8).astype(np.int32)
    wm = rng.integers(-3, 1, 8).astype(np.int32)
    rs, ri = oracle.custom_reduce(A, Bt, wp, wm)
    for p in candidates(mdh.MDH_CUSTOM_REDUCE, (500, 2500, 8), limit=16):
        s, i = run_prl(A, Bt, wp, wm, p)
        assert np.array_equal(s, rs) and np.array_equal(i, ri)
    # equal weights: every b ties, index 0 everywhere
    w = np.full(8, 9, np.int32)
    s, i = run_prl(A, Bt, w, w, None)
    assert np.all(s == 72) and np.all(i == 0)
    # weights near the int32 range whose sums still fit
    big = np.array([2**27] * 8, np.int32)
    s, i = run_prl(A, Bt, big, -big, None)
    rs, ri = oracle.custom_reduce(A, Bt, big, -big)
    assert np.array_equal(s, rs) and np.array_equal(i, ri)
    # the smallest score there is: one field whose weight is INT_MIN either way, so every pair scores
    # INT_MIN and the first index must be reported (no neutral element stands in for a real pair)
    lo = np.array([-2**31], np.int32)
    A1 = rng.integers(0, 3, (300, 1)).astype(np.int32)
    B1 = rng.integers(0, 3, (1500, 1)).astype(np.int32)
    rs, ri = oracle.custom_reduce(A1, B1, lo, lo)
    assert np.all(rs == -2**31) and np.all(ri == 0)
    for p in candidates(mdh.MDH_CUSTOM_REDUCE, (300, 1500, 1), limit=8):
        s, i = run_prl(A1, B1, lo, lo, p)
        assert np.array_equal(s, rs) and np.array_equal(i, ri)


# ------------------------------------------------------------------------------ edge cases


def test_empty_and_error_paths_on_device():
    z = torch.empty((0, 5), dtype=torch.float32, device="cuda")
    b = torch.empty((5, 7), dtype=torch.float32, device="cuda")
    c = torch.empty((0, 7), dtype=torch.float32, device="cuda")
    mdh.mdh_matmul(z, b, c)  # empty ++ dimension: nothing to do, no error
    x = torch.zeros((2, 6, 6), dtype=torch.float32, device="cuda")
    o = torch.empty((0, 4, 4), dtype=torch.float32, device="cuda")
    mdh.mdh_stencil(x, o, 0.5, 0.1)
    # a non-dividing explicit configuration is refused and leaves the output untouched
    s = (256, 256, 256)
    p = mdh.mdh_default_params(mdh.MDH_MATMUL, s)
    p.prt[B.L_WG][0] += 1
    A = torch.ones((256, 256), dtype=torch.float32, device="cuda")
    C = torch.full((256, 256), 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(mdh.MdhError) as e:
        mdh.mdh_matmul(A, A, C, p)
    assert e.value.status == 3
    torch.cuda.synchronize()
    assert torch.all(C == 7.0)


def test_tune_returns_a_valid_configuration():
    shape = (256, 256, 256)
    A, Bm = W.matmul_inputs(W.MatmulCfg(*shape, W.SEED_BASE + 1))
    a, b = dev(A), dev(Bm)
    c = torch.empty((256, 256), dtype=torch.float32, device="cuda")
    ws = torch.empty(16 * 256 * 256, dtype=torch.float32, device="cuda")
    best, ms = mdh.mdh_tune(mdh.MDH_MATMUL, shape, [a, b, c], workspace=ws, reps=2)
    assert ms > 0 and mdh.mdh_validate_params(mdh.MDH_MATMUL, shape, best) == 0
    ref, refabs = oracle.matmul(A, Bm, with_abs=True)
    assert scaled_err(run_matmul(A, Bm, best), ref, refabs) <= TOL_CONTRACTION
