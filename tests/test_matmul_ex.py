"""bMatMul and MatMul^T (batched MatMul with transposed views): same md_hom as MatMul, one
more concatenation dimension, other index functions.  The reference is the MatMul oracle
applied to the arrays the transposed views describe; that reading of the views is itself pinned
against the generic evaluator with the paper's index functions."""
import itertools

import numpy as np
import pytest

import oracle
import paper_2405_05118_amd as mdh
from oracle import instances as G
from paper_2405_05118_amd import binding as B
from paper_2405_05118_amd import workloads as W

TOL = 1e-4


def reference(A, Bm, ta, tb, tc):
    """MatMul oracle on the logical operands: A_b (M x K) = stored A_b transposed if ta, etc."""
    outs, outabs = [], []
    for b in range(A.shape[0]):
        a = np.ascontiguousarray(A[b].T) if ta else A[b]
        bb = np.ascontiguousarray(Bm[b].T) if tb else Bm[b]
        c, cabs = oracle.matmul(a, bb, with_abs=True)
        outs.append(c.T if tc else c)
        outabs.append(cabs.T if tc else cabs)
    return np.stack(outs), np.stack(outabs)


def test_transposed_views_against_generic_evaluator():
    rng = np.random.default_rng(5)
    for ta, tb, tc in itertools.product((False, True), repeat=3):
        nb, M, N, K = 2, 3, 4, 5
        A = rng.integers(-4, 5, (nb, K, M) if ta else (nb, M, K)).astype(np.float32)
        Bm = rng.integers(-4, 5, (nb, N, K) if tb else (nb, K, N)).astype(np.float32)
        want = G.bmatmul_t(A.astype(int).tolist(), Bm.astype(int).tolist(), ta, tb, tc)
        got, _ = reference(A, Bm, ta, tb, tc)
        assert np.array_equal(got, np.array(want, dtype=np.float64)), (ta, tb, tc)


HOST_SIZES = [
    (1, 16, 1000, 2048, 0, 0, 0),   # ResNet-50 training MatMul of the paper's low-level example
    (1, 1, 1000, 2048, 0, 0, 0),    # ResNet-50 inference
    (1, 16, 4096, 25088, 0, 0, 0),  # VGG-16 training
    (8, 300, 200, 100, 1, 1, 1),
    (3, 1024, 1024, 1024, 1, 0, 1),
]


@pytest.mark.parametrize("sizes", HOST_SIZES)
def test_planner(sizes):
    inst = mdh.MDH_BMATMUL
    p = mdh.mdh_default_params(inst, sizes)
    assert p.D == 4
    assert (p.in_transposed[0], p.in_transposed[1], p.out_transposed) == sizes[4:]
    for d in range(4):
        e = p.extent(d)
        assert e >= sizes[d] if p.ragged else e == sizes[d]
    n = mdh.mdh_num_candidates(inst, sizes)
    assert n >= 2
    for i in range(n):
        c = mdh.mdh_candidate(inst, sizes, i)
        assert mdh.mdh_validate_params(inst, sizes, c) == 0
    # a configuration written for other views is not the configuration of this call
    q = p.copy()
    q.in_transposed[0] ^= 1
    assert mdh.mdh_validate_params(inst, sizes, q) == 6
    # small M: the default spends workgroups on the reduction dimension
    if sizes[1] <= 16:
        assert p.prt[B.L_WG][3] > 1 and mdh.mdh_workspace_size(inst, sizes, p) == p.prt[B.L_WG][3] * sizes[0] * sizes[1] * sizes[2] * 4


def test_small_m_default_streams_operands_to_registers():
    # M <= 16 without transposed views: 16 x 16 x 4 block, no LDS staging, k parts on wavefronts
    # and workgroups (the paper's point about parallelising the reduction of these shapes)
    for sizes in HOST_SIZES[:3]:
        p = mdh.mdh_default_params(mdh.MDH_BMATMUL, sizes)
        assert list(p.blk[:4]) == [1, 16, 16, 4]
        assert p.in_region[0] == 2 and p.in_region[1] == 2
        assert p.prt[B.L_WAVE][3] > 1
    # B transposed (a weight matrix stored [N][K]): the same kernel, a lane then takes 4 consecutive k of
    # its column for four steps of 16 at once (16 register-layer parts of k instead of 4)
    p = mdh.mdh_default_params(mdh.MDH_BMATMUL, (1, 16, 1000, 8192, 0, 1, 0))
    assert list(p.blk[:4]) == [1, 16, 16, 4] and p.in_transposed[1] == 1 and p.prt[B.L_VGPR][3] == 16
    assert p.prt[B.L_VGPR][2] == 4 and p.prt[B.L_WG][3] > 1
    assert mdh.mdh_validate_params(mdh.MDH_BMATMUL, (1, 16, 1000, 8192, 0, 1, 0), p) == 0
    assert mdh.mdh_validate_params(mdh.MDH_BMATMUL, (1, 16, 1000, 8192, 0, 0, 0), p) == 6
    # a small transposed B, or one with enough columns to fill the chip: strips of ONE block column, all of
    # k inside the workgroup (rounds of 128 k per wavefront), nothing combined between workgroups; the rows
    # of A and B are read as whole runs of k and reach the operand layout through LDS (in_region)
    for sizes in ((1, 16, 1000, 2048, 0, 1, 0), (1, 16, 4096, 25088, 0, 1, 0)):
        p = mdh.mdh_default_params(mdh.MDH_BMATMUL, sizes)
        assert list(p.blk[:4]) == [1, 16, 16, 4] and p.prt[B.L_VGPR][2] == 1 and p.prt[B.L_VGPR][3] == 32
        assert p.prt[B.L_WG][2] == -(-sizes[2] // 16) and p.prt[B.L_WG][3] == 1 and p.prt[B.L_WAVE][3] == 4
        assert p.in_region[0] == B.MR_LDS and p.in_region[1] == B.MR_LDS
        q = p.copy()
        q.in_region[0] = q.in_region[1] = B.MR_VGPR  # four wavefronts only with the staged operands
        assert mdh.mdh_validate_params(mdh.MDH_BMATMUL, sizes, q) != 0
        assert mdh.mdh_workspace_size(mdh.MDH_BMATMUL, sizes, p) == 0
        assert mdh.mdh_validate_params(mdh.MDH_BMATMUL, sizes, p) == 0
        q = p.copy()
        q.prt[B.L_WG][3] = 2  # narrow strips do not split k over workgroups
        assert mdh.mdh_validate_params(mdh.MDH_BMATMUL, sizes, q) != 0
    # the same strips are a candidate for the plain view
    sizes = (1, 16, 1000, 2048, 0, 0, 0)
    narrow = [c for c in (mdh.mdh_candidate(mdh.MDH_BMATMUL, sizes, i) for i in range(mdh.mdh_num_candidates(mdh.MDH_BMATMUL, sizes)))
              if c.blk[1] == 16 and c.prt[B.L_VGPR][2] == 1]
    assert sorted(c.prt[B.L_WAVE][3] for c in narrow) == [8, 16]
    assert all(mdh.mdh_validate_params(mdh.MDH_BMATMUL, sizes, c) == 0 for c in narrow)
    assert all(c.in_region[1] == B.MR_VGPR for c in narrow)  # staging whole runs of k needs B transposed
    q = narrow[0].copy()
    q.in_region[0] = q.in_region[1] = B.MR_LDS
    assert mdh.mdh_validate_params(mdh.MDH_BMATMUL, sizes, q) != 0
    # A or C transposed, or more rows: the LDS-tiled kernel
    for sizes in ((1, 16, 1000, 2048, 1, 0, 0), (1, 16, 1000, 2048, 0, 0, 1), (1, 17, 1000, 2048, 0, 0, 0)):
        p = mdh.mdh_default_params(mdh.MDH_BMATMUL, sizes)
        assert list(p.blk[:4]) == [1, 32, 32, 2]


torch = pytest.importorskip("torch")


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run(A, Bm, ta, tb, tc, p):
    nb = A.shape[0]
    M, K = (A.shape[2], A.shape[1]) if ta else (A.shape[1], A.shape[2])
    N = Bm.shape[1] if tb else Bm.shape[2]
    sizes = (nb, M, N, K, int(ta), int(tb), int(tc))
    C = torch.full((nb, N, M) if tc else (nb, M, N), float("nan"), dtype=torch.float32, device="cuda")
    n = mdh.mdh_workspace_size(mdh.MDH_BMATMUL, sizes, p)
    ws = torch.empty(max(n, 4) // 4, dtype=torch.int32, device="cuda") if n else None
    mdh.mdh_matmul_ex(dev(A), dev(Bm), C, ta, tb, tc, p, ws)
    torch.cuda.synchronize()
    return C.cpu().numpy().astype(np.float64), sizes


@pytest.mark.gpu
@pytest.mark.parametrize("shape", [(1, 128, 128, 64), (3, 70, 45, 33), (2, 16, 200, 300), (1, 1, 130, 257), (5, 33, 31, 8)])
def test_all_views_all_candidates(shape):
    nb, M, N, K = shape
    for ta, tb, tc in itertools.product((False, True), repeat=3):
        A = W.uniform(W.SEED_BASE + 61, 1, (nb, K, M) if ta else (nb, M, K), -1, 1)
        Bm = W.uniform(W.SEED_BASE + 61, 2, (nb, N, K) if tb else (nb, K, N), -1, 1)
        ref, refabs = reference(A, Bm, ta, tb, tc)
        sizes = (nb, M, N, K, int(ta), int(tb), int(tc))
        cands = [None] + [mdh.mdh_candidate(mdh.MDH_BMATMUL, sizes, i) for i in range(mdh.mdh_num_candidates(mdh.MDH_BMATMUL, sizes))]
        for p in cands[:: max(1, len(cands) // 6)]:
            got, _ = run(A, Bm, ta, tb, tc, p)
            assert np.all(np.isfinite(got))
            err = float(np.max(np.abs(got - ref) / np.where(refabs > 0, refabs, 1.0)))
            assert err <= TOL, (shape, ta, tb, tc, p and p.table())


@pytest.mark.gpu
@pytest.mark.parametrize("shape", [(2, 16, 200, 300), (1, 1, 130, 257), (3, 7, 64, 48), (1, 16, 256, 1024),
                                   (1, 12, 70, 1000), (1, 16, 1000, 2048)])
def test_small_m_every_candidate(shape):
    nb, M, N, K = shape
    A = W.uniform(W.SEED_BASE + 63, 1, (nb, M, K), -1, 1)
    Bm = W.uniform(W.SEED_BASE + 63, 2, (nb, K, N), -1, 1)
    ref, refabs = reference(A, Bm, False, False, False)
    sizes = (nb, M, N, K, 0, 0, 0)
    cands = [mdh.mdh_candidate(mdh.MDH_BMATMUL, sizes, i) for i in range(mdh.mdh_num_candidates(mdh.MDH_BMATMUL, sizes))]
    small = [p for p in cands if p.blk[1] == 16]
    assert len(small) >= 5
    for p in small:
        got, _ = run(A, Bm, False, False, False, p)
        assert np.all(np.isfinite(got)), p.table()
        err = float(np.max(np.abs(got - ref) / np.where(refabs > 0, refabs, 1.0)))
        assert err <= TOL, (shape, p.table())


@pytest.mark.gpu
@pytest.mark.parametrize("tb", [False, True])
@pytest.mark.parametrize("shape", [(1, 16, 1000, 2048), (2, 5, 1000, 2085), (2, 5, 77, 100), (1, 16, 16, 128),
                                   (3, 13, 250, 4226), (1, 1, 1, 1), (1, 16, 4096, 1024), (1, 9, 33, 127)])
def test_small_m_narrow_strips(shape, tb):
    # strips of one block column, k over the wavefronts of a workgroup in rounds of 128: whole rounds and
    # a ragged last one, a ragged last strip, fewer than 16 rows, fewer rounds than wavefronts, batches;
    # both views of B, 8 and 16 wavefronts (4 and 8 with the operands staged through LDS); NaN-filled output
    # shows every element is written
    nb, M, N, K = shape
    A = W.uniform(W.SEED_BASE + 68, 1, (nb, M, K), -1, 1)
    Bm = W.uniform(W.SEED_BASE + 68, 2, (nb, N, K) if tb else (nb, K, N), -1, 1)
    ref, refabs = reference(A, Bm, False, tb, False)
    sizes = (nb, M, N, K, 0, int(tb), 0)
    cands = [mdh.mdh_candidate(mdh.MDH_BMATMUL, sizes, i) for i in range(mdh.mdh_num_candidates(mdh.MDH_BMATMUL, sizes))]
    d = mdh.mdh_default_params(mdh.MDH_BMATMUL, sizes)
    narrow = [p for p in [d] + cands if p.blk[1] == 16 and p.prt[B.L_VGPR][2] == 1]
    assert sorted(set(p.prt[B.L_WAVE][3] for p in narrow if p.in_region[1] == B.MR_VGPR)) == [8, 16]
    # B transposed: also the variant that reads whole runs of k and stages both operands through LDS
    assert sorted(set(p.prt[B.L_WAVE][3] for p in narrow if p.in_region[1] == B.MR_LDS)) == ([4, 8] if tb else [])
    for p in narrow:
        assert mdh.mdh_workspace_size(mdh.MDH_BMATMUL, sizes, p) == 0
        got, _ = run(A, Bm, False, tb, False, p)
        assert np.all(np.isfinite(got)), p.table()
        err = float(np.max(np.abs(got - ref) / np.where(refabs > 0, refabs, 1.0)))
        assert err <= TOL, (shape, tb, p.table())
        again, _ = run(A, Bm, False, tb, False, p)
        assert np.array_equal(got, again)


@pytest.mark.gpu
@pytest.mark.parametrize("tb", [False, True])
def test_small_m_one_launch_and_second_kernel_agree_bit_for_bit(tb):
    # a reduction split over workgroups is combined by the last part of a strip to arrive (the default:
    # out_region = device memory) or by a second kernel (out_region = registers): same order, same bits;
    # calls of different shapes in a row share the arrival counters, which every call leaves at zero
    # (the last two shapes split k into 32 and 64 parts: two and four rounds of the combination's loads)
    for rep, (nb, M, N, K) in enumerate(((1, 16, 1000, 2048), (2, 12, 200, 4096), (1, 16, 1000, 2048), (3, 7, 130, 1024),
                                         (1, 5, 100, 16384), (1, 16, 64, 65536))):
        A = W.uniform(W.SEED_BASE + 66 + rep, 1, (nb, M, K), -1, 1)
        Bm = W.uniform(W.SEED_BASE + 66 + rep, 2, (nb, N, K) if tb else (nb, K, N), -1, 1)
        sizes = (nb, M, N, K, 0, int(tb), 0)
        d = mdh.mdh_default_params(mdh.MDH_BMATMUL, sizes)
        if d.prt[B.L_WG][3] == 1:  # the default is the kernel with narrow strips: take the first candidate that splits k
            cands = [mdh.mdh_candidate(mdh.MDH_BMATMUL, sizes, i) for i in range(mdh.mdh_num_candidates(mdh.MDH_BMATMUL, sizes))]
            d = next(c for c in cands if c.blk[1] == 16 and c.prt[B.L_WG][3] > 1 and c.out_region == B.MR_HBM)
        assert d.blk[1] == 16 and d.prt[B.L_WG][3] > 1 and d.out_region == B.MR_HBM, (sizes, d.table())
        if K >= 16384:
            assert d.prt[B.L_WG][3] >= 32, (sizes, d.table())
        second = d.copy()
        second.out_region = B.MR_VGPR
        assert mdh.mdh_validate_params(mdh.MDH_BMATMUL, sizes, second) == 0
        g1, _ = run(A, Bm, False, tb, False, d)
        g2, _ = run(A, Bm, False, tb, False, second)
        g3, _ = run(A, Bm, False, tb, False, d)
        assert np.array_equal(g1, g2) and np.array_equal(g1, g3), sizes
        ref, refabs = reference(A, Bm, False, tb, False)
        assert float(np.max(np.abs(g1 - ref) / refabs)) <= TOL


@pytest.mark.gpu
@pytest.mark.parametrize("views", [(0, 0, 0), (1, 0, 0), (0, 1, 0), (1, 1, 1)])
def test_many_tiles_many_batches(views):
    # more than eight tile rows (banded tile order), a workgroup count divisible by 8 (the XCD-aware
    # order), ragged edges in every dimension, k-tiles of 16 and of 32
    ta, tb, tc = views
    for nb, M, N, K in ((8, 1300, 520, 200), (2, 1100, 260, 1060)):
        A = W.uniform(W.SEED_BASE + 65, 1, (nb, K, M) if ta else (nb, M, K), -1, 1)
        Bm = W.uniform(W.SEED_BASE + 65, 2, (nb, N, K) if tb else (nb, K, N), -1, 1)
        ref, refabs = reference(A, Bm, ta, tb, tc)
        got, _ = run(A, Bm, ta, tb, tc, None)
        assert np.all(np.isfinite(got))
        assert float(np.max(np.abs(got - ref) / refabs)) <= TOL, (nb, M, N, K, views)


@pytest.mark.gpu
@pytest.mark.parametrize("name", ["bmatmul_16x1024", "matmul_t_4096"])
def test_bench_sizes_whole_output(name):
    # every element of every batch entry against the fp64 oracle (bMatMul 16 x 1024^3 and MatMul^T 4096^3
    # as bench.py times them); tile corners asserted by name on top
    cfg = W.CONFIGS[name]
    ta, tb, tc = cfg.trans
    A, Bm = W.bmatmul_inputs(cfg)
    got, _ = run(A, Bm, ta, tb, tc, None)
    assert np.all(np.isfinite(got))
    for b in range(cfg.batch):
        a2 = np.ascontiguousarray(A[b].T) if ta else A[b]
        b2 = np.ascontiguousarray(Bm[b].T) if tb else Bm[b]
        ref, refabs = oracle.matmul(a2, b2, with_abs=True)
        Cb = got[b].T if tc else got[b]
        err = np.abs(Cb - ref) / refabs
        for i, j in ((0, 0), (cfg.M - 1, cfg.N - 1), (127, 127), (128, 128), (127, 128), (cfg.M - 129, 63), (1023, 1024 % cfg.N)):
            assert err[i, j] <= TOL, (name, b, i, j)
        assert float(err.max()) <= TOL, (name, b, np.unravel_index(int(err.argmax()), err.shape))


@pytest.mark.gpu
def test_paper_shapes_small_m():
    # MatMul sizes of the paper's deep-learning study: (M, N, K) = (16, 1000, 2048) and (1, 1000, 2048)
    for M in (16, 1):
        A = W.uniform(W.SEED_BASE + 62, 1, (1, M, 2048), -1, 1)
        Bm = W.uniform(W.SEED_BASE + 62, 2, (1, 2048, 1000), -1, 1)
        ref, refabs = reference(A, Bm, False, False, False)
        got, sizes = run(A, Bm, False, False, False, None)
        assert float(np.max(np.abs(got - ref) / refabs)) <= TOL
        # all-ones closed form through the transposed views
        ones_a = np.ones((1, 2048, M), np.float32)
        ones_b = np.ones((1, 1000, 2048), np.float32)
        got, _ = run(ones_a, ones_b, True, True, True, None)
        assert got.shape == (1, 1000, M) and np.all(got == 2048)


@pytest.mark.gpu
def test_tune_picks_a_valid_configuration():
    sizes = (2, 16, 300, 700, 0, 0, 0)
    A = W.uniform(W.SEED_BASE + 64, 1, (2, 16, 700), -1, 1)
    Bm = W.uniform(W.SEED_BASE + 64, 2, (2, 700, 300), -1, 1)
    C = torch.empty((2, 16, 300), dtype=torch.float32, device="cuda")
    ws = torch.empty(64 * 2 * 16 * 300, dtype=torch.float32, device="cuda")
    best, ms = mdh.mdh_tune(mdh.MDH_BMATMUL, sizes, [dev(A), dev(Bm), C], workspace=ws, reps=2)
    assert ms > 0 and mdh.mdh_validate_params(mdh.MDH_BMATMUL, sizes, best) == 0
    ref, refabs = reference(A, Bm, False, False, False)
    got, _ = run(A, Bm, False, False, False, best)
    assert float(np.max(np.abs(got - ref) / refabs)) <= TOL
