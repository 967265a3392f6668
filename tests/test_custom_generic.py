"""Generic md_hom with runtime-compiled scalar function and combine operator (mdh_custom_*).

Reference: the generic evaluator of oracle/mdhom.py (the paper's definitions of md_hom, ++, pw and
the views, evaluated literally) on small index spaces, and the C oracle / a library routine on
larger ones.  The instances below are those of the paper's example table that the fixed kernels
do not cover (Histo, GenHisto, map, reduce, Jacobi1D) plus Dot, MatVec, MatMul and PRL again, this
time through user-supplied source."""
import ctypes

import numpy as np
import pytest

import oracle
import paper_2405_05118_amd as mdh
from oracle import instances as G
from paper_2405_05118_amd import binding as B
from paper_2405_05118_amd import workloads as W

# ------------------------------------------------------------------ pins of the new oracle instances


def test_histo_oracle_against_bincount():
    rng = np.random.default_rng(11)
    elems = rng.integers(0, 7, 40).tolist()
    bins = list(range(7))
    assert G.histo(elems, bins) == np.bincount(elems, minlength=7).tolist()
    # bins need not be 0..B-1, and a value that never occurs counts 0
    assert G.histo([5, 9, 5, 2], [9, 4, 5]) == [1, 0, 2]
    # GenHisto with max: largest element not above the bin bound (a different f and operator)
    got = G.gen_histo([3, 8, 1, 6], [2, 7, 9], lambda e, b: e if e <= b else -1, max)
    assert got == [1, 6, 8]


def test_jacobi1d_oracle_against_printed_form():
    # w_i = c * (v_i + v_{i+1} + v_{i+2}), N-2 outputs (Section "Introduction")
    x = [1, 4, 9, 16, 25, 36]
    assert G.jacobi1d(x, 2) == [2 * (1 + 4 + 9), 2 * (4 + 9 + 16), 2 * (9 + 16 + 25), 2 * (16 + 25 + 36)]
    assert G.map_f(lambda v: v * v, [1, 2, 3]) == [1, 4, 9]
    assert G.reduce_op(min, [4, 2, 7]) == 2


# ------------------------------------------------------------------ descriptions used below

PRL_PRE = "struct rec { int f[8]; }; struct res { int score; int idx; };"
PRL_F = ("int s = 0; for (int k = 0; k < 8; ++k) s += a0.f[k] == a1.f[k] ? a2.f[k] : a3.f[k];"
         " r.score = s; r.idx = (int)i1;")
PRL_OP = "if (x.score > y.score || (x.score == y.score && x.idx < y.idx)) r = x; else r = y;"


def d_dot(K):
    return mdh.custom_desc((K,), (1,), ["float", "float"], [(0, "i0"), (1, "i0")], "float", 4, "r = a0 * a1;", "r = x + y;")


def d_matvec(M, K):
    return mdh.custom_desc((M, K), (0, 1), ["float", "float"], [(0, "i0*N1+i1"), (1, "i1")], "float", 4,
                           "r = a0 * a1;", "r = x + y;")


def d_matmul(M, N, K, fast=1):
    return mdh.custom_desc((M, N, K), (0, 0, 1), ["float", "float"], [(0, "i0*N2+i2"), (1, "i2*N1+i1")], "float", 4,
                           "r = a0 * a1;", "r = x + y;", fast_dim=fast)


def d_prl(nA, nB):
    return mdh.custom_desc((nA, nB), (0, 1), ["rec"] * 4, [(0, "i0"), (1, "i1"), (2, "0"), (3, "0")], "res", 8,
                           PRL_F, PRL_OP, PRL_PRE, fast_dim=0)


def test_compiled_histo_oracle_pins():
    """The C version of the Histo definition (used for large inputs): against the generic evaluator
    on small inputs, and closed forms (every element in one bin; bins absent from the data;
    duplicate bin values count the same elements; the counts of distinct bins that cover the data
    add up to the number of elements)."""
    import oracle

    rng = np.random.default_rng(5)
    elems = rng.integers(0, 9, size=200).astype(np.int32)
    bins = np.array([3, 0, 8, 8, 11, 5], dtype=np.int32)
    assert oracle.histo(elems, bins).tolist() == G.histo(elems.tolist(), bins.tolist())
    assert oracle.histo(np.full(1000, 4, np.int32), np.array([4, 5], np.int32)).tolist() == [1000, 0]
    assert oracle.histo(np.empty(0, np.int32), np.array([1, 2], np.int32)).tolist() == [0, 0]
    big = rng.integers(0, 256, size=100000).astype(np.int32)
    counts = oracle.histo(big, np.arange(256, dtype=np.int32))
    assert int(counts.sum()) == big.size and counts.dtype == np.int64
    # a planted mistake: comparing with the bin's position instead of its value
    assert oracle.histo(np.array([7, 7, 2], np.int32), np.array([2, 7], np.int32)).tolist() == [1, 2]


def d_histo(nbins, ne):
    return mdh.custom_desc((nbins, ne), (0, 1), ["int", "int"], [(0, "i1"), (1, "i0")], "int", 4,
                           "r = a0 == a1 ? 1 : 0;", "r = x + y;")


def d_jacobi1d(n, c):
    return mdh.custom_desc((n,), (0,), ["float"], [(0, "i0"), (0, "i0+1"), (0, "i0+2")], "float", 4,
                           "r = (float)%r * (a0 + a1 + a2);" % float(c))


# ------------------------------------------------------------------ host side (no GPU)


@pytest.mark.parametrize("desc", [d_dot(1 << 20), d_dot(1000), d_matvec(512, 4096), d_matvec(7, 33),
                                  d_matmul(40, 50, 60), d_prl(1000, 3000), d_histo(256, 100000), d_jacobi1d(5000, 0.5)])
def test_planner_tables(desc):
    p = mdh.mdh_custom_default_params(desc)
    assert p.D == desc.D and list(p.blk[: p.D]) == [1] * p.D  # the paper's full partitioning
    for d in range(p.D):
        e = p.extent(d)
        assert e >= desc.sizes[d] if p.ragged else e == desc.sizes[d]
    assert mdh.mdh_custom_validate_params(desc, p) == 0
    n = mdh.mdh_custom_num_candidates(desc)
    assert n >= 2
    for i in range(n):
        assert mdh.mdh_custom_validate_params(desc, mdh.mdh_custom_candidate(desc, i)) == 0


def test_register_parts_of_concatenation_dimensions():
    # MatMul: A does not depend on j, B not on i: blocking a concatenation dimension in registers
    # re-uses the loaded element; the default blocks, candidates cover 1, 2, 4 and 8 parts
    d = d_matmul(1024, 1024, 1024)
    p = mdh.mdh_custom_default_params(d)
    assert max(p.prt[B.L_VGPR][0], p.prt[B.L_VGPR][1]) == 8 and p.prt[B.L_VGPR][2] == 1  # eight parts on one dimension
    vs = {max(c.prt[B.L_VGPR][:3]) for c in (mdh.mdh_custom_candidate(d, i) for i in range(mdh.mdh_custom_num_candidates(d)))}
    assert {1, 2, 4, 8} <= vs
    src = mdh.mdh_custom_source(mdh.mdh_custom_create(d, p))
    assert "mdh_T acc[8];" in src
    # register parts on a reduced dimension are not a configuration of this kernel
    q = p.copy()
    q.prt[B.L_VGPR][2], q.prt[B.L_HBM][2] = 2, q.prt[B.L_HBM][2] // 2
    assert mdh.mdh_custom_validate_params(d, q) == 6
    # Jacobi1D: every access depends on the only dimension, nothing to re-use -- but four consecutive
    # indices per lane share 16-byte accesses; where the extent is ragged the interior lanes run a
    # copy of the scalar phase and of the stores without clamps and bounds checks
    pj = mdh.mdh_custom_default_params(d_jacobi1d(1 << 20, 0.5))
    assert pj.prt[B.L_VGPR][0] == 4 and pj.prt[B.L_LANE][0] == 256 and not pj.ragged
    src = mdh.mdh_custom_source(mdh.mdh_custom_create(d_jacobi1d(1 << 20, 0.5), pj))
    assert "N0 - 1" not in src and "b0 + 4 <= N0" not in src
    dj = d_jacobi1d((1 << 20) + 3, 0.5)
    pj = mdh.mdh_custom_default_params(dj)
    assert pj.prt[B.L_VGPR][0] == 4 and pj.ragged
    src = mdh.mdh_custom_source(mdh.mdh_custom_create(dj, pj))
    assert src.count("if (b0 + 4 <= N0) {") == 2 and src.count("N0 - 1") == 1
    # too few points for 1024 workgroups of four-index lanes: one index per lane
    assert mdh.mdh_custom_default_params(d_jacobi1d(1 << 16, 0.5)).prt[B.L_VGPR][0] == 1


def test_planner_rejects_bad_tables():
    desc = d_matvec(512, 4096)
    p = mdh.mdh_custom_default_params(desc)
    q = p.copy()
    q.prt[B.L_HBM][1] += 1  # product no longer N_d
    assert mdh.mdh_custom_validate_params(desc, q) == 3
    q = p.copy()
    q.prt[B.L_LDS][1], q.prt[B.L_HBM][1] = q.prt[B.L_HBM][1], 1  # parts on a layer the generic kernel does not stage
    assert mdh.mdh_custom_validate_params(desc, q) == 6
    q = p.copy()
    q.prt[B.L_LANE][0], q.prt[B.L_WG][0] = 2048, 1  # more than 1024 lanes
    q.prt[B.L_HBM][0] = 1
    q.ragged = 1
    assert mdh.mdh_custom_validate_params(desc, q) == 4
    # a workgroup part of the reduced dimension that owns no index
    small = d_matvec(4, 100)
    q = mdh.mdh_custom_default_params(small)
    q.prt[B.L_WG][1], q.prt[B.L_LANE][1], q.prt[B.L_HBM][1], q.ragged = 4, 64, 1, 1
    assert mdh.mdh_custom_validate_params(small, q) == 3


def test_compiles_without_gpu_and_reports_errors():
    op = mdh.mdh_custom_create(d_prl(100, 300))
    src = mdh.mdh_custom_source(op)
    assert "mdh_custom_main" in src and "struct rec" in src and "a0.f[k] == a1.f[k]" in src
    mdh.mdh_custom_destroy(op)
    with pytest.raises(mdh.MdhError) as e:
        mdh.mdh_custom_create(mdh.custom_desc((8,), (1,), ["float"], [(0, "i0")], "float", 4, "r = a0 +;", "r = x + y;"))
    assert e.value.status == 6 and "error" in str(e.value)
    with pytest.raises(mdh.MdhError) as e:  # sizeof(out_type) disagrees with out_elem_bytes
        mdh.mdh_custom_create(mdh.custom_desc((8,), (1,), ["float"], [(0, "i0")], "double", 4, "r = a0;", "r = x + y;"))
    assert "out_elem_bytes" in str(e.value)
    with pytest.raises(mdh.MdhError) as e:  # a reduced dimension needs an operator
        mdh.mdh_custom_create(mdh.custom_desc((8,), (1,), ["float"], [(0, "i0")], "float", 4, "r = a0;"))
    assert e.value.status == 1


# ------------------------------------------------------------------ GPU parity

torch = pytest.importorskip("torch")


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run(desc, inputs, out, params=None):
    op = mdh.mdh_custom_create(desc, params)
    n = mdh.mdh_custom_workspace_size(op)
    ws = torch.empty(max(n, 4), dtype=torch.uint8, device="cuda") if n else None
    mdh.mdh_custom_run(op, inputs, out, ws)
    torch.cuda.synchronize()
    mdh.mdh_custom_destroy(op)
    return out


def all_params(desc):
    return [None] + [mdh.mdh_custom_candidate(desc, i) for i in range(mdh.mdh_custom_num_candidates(desc))]


@pytest.mark.gpu
def test_small_against_generic_evaluator():
    rng = np.random.default_rng(3)
    # MatMul (integers stored as float: exact)
    M, N, K = 5, 7, 9
    A = rng.integers(-4, 5, (M, K)).astype(np.float32)
    Bm = rng.integers(-4, 5, (K, N)).astype(np.float32)
    want = np.array(G.matmul(A.astype(int).tolist(), Bm.astype(int).tolist()), dtype=np.float32)
    for p in all_params(d_matmul(M, N, K)):
        got = run(d_matmul(M, N, K), [dev(A), dev(Bm)], torch.full((M, N), float("nan"), device="cuda"), p)
        assert np.array_equal(got.cpu().numpy(), want)
    # Histo and GenHisto(max)
    elems = rng.integers(0, 6, 50).astype(np.int32)
    bins = np.array([4, 0, 9, 5, 1], np.int32)
    want = G.histo(elems.tolist(), bins.tolist())
    for p in all_params(d_histo(5, 50)):
        got = run(d_histo(5, 50), [dev(elems), dev(bins)], torch.full((5,), -7, dtype=torch.int32, device="cuda"), p)
        assert got.cpu().tolist() == want
    gh = mdh.custom_desc((5, 50), (0, 1), ["int", "int"], [(0, "i1"), (1, "i0")], "int", 4,
                         "r = a0 <= a1 ? a0 : -1;", "r = x > y ? x : y;")
    want = G.gen_histo(elems.tolist(), bins.tolist(), lambda e, b: e if e <= b else -1, max)
    got = run(gh, [dev(elems), dev(bins)], torch.full((5,), -7, dtype=torch.int32, device="cuda"))
    assert got.cpu().tolist() == want
    # PRL through user-defined struct types and operator
    nA, nB = 6, 11
    A8 = rng.integers(0, 3, (nA, 8)).astype(np.int32)
    B8 = rng.integers(0, 3, (nB, 8)).astype(np.int32)
    wp = rng.integers(1, 9, 8).astype(np.int32)
    wm = rng.integers(-9, 1, 8).astype(np.int32)
    sc, ix = G.custom_reduce(A8.tolist(), B8.tolist(), wp.tolist(), wm.tolist())
    for p in all_params(d_prl(nA, nB)):
        got = run(d_prl(nA, nB), [dev(A8), dev(B8), dev(wp), dev(wm)], torch.full((nA, 2), -1, dtype=torch.int32, device="cuda"), p)
        assert got[:, 0].cpu().tolist() == sc and got[:, 1].cpu().tolist() == ix
    # Jacobi1D: three accesses to one buffer; map; reduce(min)
    x = rng.integers(0, 10, 12).astype(np.float32)
    want = G.jacobi1d(x.astype(int).tolist(), 2)
    got = run(d_jacobi1d(10, 2.0), [dev(x)], torch.full((10,), float("nan"), device="cuda"))
    assert got.cpu().tolist() == want
    v = rng.integers(-50, 50, 37).astype(np.int32)
    dm = mdh.custom_desc((37,), (1,), ["int"], [(0, "i0")], "int", 4, "r = a0;", "r = x < y ? x : y;")
    for p in all_params(dm):
        got = run(dm, [dev(v)], torch.full((1,), 99, dtype=torch.int32, device="cuda"), p)
        assert got.item() == G.reduce_op(min, v.tolist())


@pytest.mark.gpu
def test_pure_concatenation_several_indices_per_lane():
    # Jacobi1D with a ragged extent, every candidate (1, 2 and 4 consecutive indices per lane, the
    # interior lanes on the copy without clamps) against the definitional evaluator; integers: exact
    rng = np.random.default_rng(11)
    n = 2051
    x = rng.integers(0, 10, n + 2).astype(np.float32)
    want = G.jacobi1d(x.astype(int).tolist(), 2)
    d = d_jacobi1d(n, 2.0)
    seen = set()
    for p in all_params(d):
        seen.add((p or mdh.mdh_custom_default_params(d)).prt[B.L_VGPR][0])
        got = run(d, [dev(x)], torch.full((n,), float("nan"), device="cuda"), p)
        assert got.cpu().tolist() == want, p and p.table()
    assert {1, 2, 4} <= seen
    # two concatenation dimensions, the fast one ragged: out[i,j] = a[i,j] + b[j]
    from oracle import mdhom as H
    M, N = 3, 601
    a = rng.integers(-9, 10, (M, N)).astype(np.float32)
    b = rng.integers(-9, 10, N).astype(np.float32)
    iv = H.inp_view([[lambda i, j: (i, j)], [lambda i, j: (j,)]])
    h = H.md_hom(lambda t: t[0] + t[1], (H.concat(0), H.concat(1)))
    (o,) = H.out_view([[lambda i, j: (i, j)]])(h(iv([a.astype(int).tolist(), b.astype(int).tolist()], [range(M), range(N)])))
    want = [[o[(i, j)] for j in range(N)] for i in range(M)]
    d2 = mdh.custom_desc((M, N), (0, 0), ["float", "float"], [(0, "i0*N1+i1"), (1, "i1")], "float", 4, "r = a0 + a1;")
    seen = set()
    for p in all_params(d2):
        seen.add((p or mdh.mdh_custom_default_params(d2)).prt[B.L_VGPR][1])
        got = run(d2, [dev(a), dev(b)], torch.full((M, N), float("nan"), device="cuda"), p)
        assert got.cpu().tolist() == want, p and p.table()
    assert {1, 4} <= seen
    # at a size where the default takes four indices per lane, ragged and not: the closed form for
    # x[i] = i, out[i] = 2 * (3i + 3), exact in fp32 below 2^24
    for n in ((1 << 21) + 3, 1 << 21):
        d = d_jacobi1d(n, 2.0)
        assert mdh.mdh_custom_default_params(d).prt[B.L_VGPR][0] == 4
        xs = torch.arange(n + 2, dtype=torch.float32, device="cuda")
        got = run(d, [xs], torch.full((n,), float("nan"), device="cuda"))
        assert np.array_equal(got.cpu().numpy(), (6 * np.arange(n) + 6).astype(np.float32))


@pytest.mark.gpu
def test_transposed_output_view():
    # out_index as a view: C written transposed, (i,j,0) -> C[j,i]
    rng = np.random.default_rng(4)
    M, N, K = 33, 18, 70
    A = rng.integers(-3, 4, (M, K)).astype(np.float32)
    Bm = rng.integers(-3, 4, (K, N)).astype(np.float32)
    d = mdh.custom_desc((M, N, K), (0, 0, 1), ["float", "float"], [(0, "i0*N2+i2"), (1, "i2*N1+i1")], "float", 4,
                        "r = a0 * a1;", "r = x + y;", out_index="i1*N0+i0")
    for p in all_params(d)[:6]:
        got = run(d, [dev(A), dev(Bm)], torch.full((N, M), float("nan"), device="cuda"), p)
        assert np.array_equal(got.cpu().numpy(), (A.astype(np.float64) @ Bm.astype(np.float64)).T.astype(np.float32))


@pytest.mark.gpu
def test_larger_against_c_oracle_every_candidate():
    # Dot and MatVec: tolerance as for the fixed instances (scaled error)
    K = 300007
    x = W.uniform(W.SEED_BASE + 80, 1, (K,), -1, 1)
    y = W.uniform(W.SEED_BASE + 80, 2, (K,), -1, 1)
    ref, scale = oracle.dot(x, y)
    for p in all_params(d_dot(K)):
        got = run(d_dot(K), [dev(x), dev(y)], torch.full((1,), float("nan"), device="cuda"), p)
        assert abs(got.item() - ref) / scale <= 1e-4
    M, Kk = 301, 2050
    A = W.uniform(W.SEED_BASE + 81, 1, (M, Kk), -1, 1)
    xv = W.uniform(W.SEED_BASE + 81, 2, (Kk,), -1, 1)
    ref = oracle.matvec(A, xv)
    scale = np.abs(A.astype(np.float64)) @ np.abs(xv.astype(np.float64))
    for p in all_params(d_matvec(M, Kk)):
        got = run(d_matvec(M, Kk), [dev(A), dev(xv)], torch.full((M,), float("nan"), device="cuda"), p)
        assert float(np.max(np.abs(got.cpu().numpy() - ref) / scale)) <= 1e-4
    # PRL: bit-exact against the C oracle
    cfg = W.PrlCfg(700, 5000, 8, W.SEED_BASE + 82)
    A8, B8, wp, wm = W.prl_inputs(cfg)
    sc, ix = oracle.custom_reduce(A8, B8, wp, wm)
    for p in all_params(d_prl(cfg.nA, cfg.nB)):
        got = run(d_prl(cfg.nA, cfg.nB), [dev(A8), dev(B8), dev(wp), dev(wm)],
                  torch.full((cfg.nA, 2), -1, dtype=torch.int32, device="cuda"), p).cpu().numpy()
        assert np.array_equal(got[:, 0], sc) and np.array_equal(got[:, 1], ix)
    # Histo against the library routine it reduces to
    elems = W.integers(W.SEED_BASE + 83, 1, (200000,), 0, 255).astype(np.int32)
    bins = np.arange(256, dtype=np.int32)
    want = np.bincount(elems, minlength=256)
    for p in all_params(d_histo(256, 200000)):
        got = run(d_histo(256, 200000), [dev(elems), dev(bins)], torch.full((256,), -1, dtype=torch.int32, device="cuda"), p)
        assert np.array_equal(got.cpu().numpy(), want)


@pytest.mark.gpu
def test_handle_is_reusable_and_checks_workspace():
    d = d_matvec(64, 100000)
    op = mdh.mdh_custom_create(d)
    n = mdh.mdh_custom_workspace_size(op)
    assert n > 0  # few rows: the reduced dimension is split over workgroups
    A = W.uniform(W.SEED_BASE + 84, 1, (64, 100000), -1, 1)
    xv = W.uniform(W.SEED_BASE + 84, 2, (100000,), -1, 1)
    out = torch.empty(64, device="cuda")
    with pytest.raises(mdh.MdhError) as e:
        mdh.mdh_custom_run(op, [dev(A), dev(xv)], out, None)
    assert e.value.status == 5
    ws = torch.empty(n, dtype=torch.uint8, device="cuda")
    first = mdh.mdh_custom_run(op, [dev(A), dev(xv)], out, ws).clone()
    second = mdh.mdh_custom_run(op, [dev(A), dev(xv)], out, ws)
    torch.cuda.synchronize()
    assert torch.equal(first, second)  # deterministic: fixed combine order on every level
    ref = oracle.matvec(A, xv)
    scale = np.abs(A.astype(np.float64)) @ np.abs(xv.astype(np.float64))
    assert float(np.max(np.abs(first.cpu().numpy() - ref) / scale)) <= 1e-4


# ------------------------------------------------------------------ prefix-sum dimension (reduce = 2)


def d_scan_rows(R, n, op="r = x + y;", ty="float"):
    return mdh.custom_desc((R, n), (0, 2), [ty], [(0, "i0*N1+i1")], ty, 4, "r = a0;", op)


def d_bottom_box_sums(R, C):
    # md_hom(id, (prefix-sum(+), +)) with the rows read bottom-up through the index function
    return mdh.custom_desc((R, C), (2, 1), ["float"], [(0, "(N0-1-i0)*N1+i1")], "float", 4, "r = a0;", "r = x + y;")


def test_prefix_sum_dimension_is_sequential_in_the_table():
    d = d_scan_rows(64, 3000)
    p = mdh.mdh_custom_default_params(d)
    assert p.prt[B.L_WG][1] == 1 and p.prt[B.L_LANE][1] == 1 and p.prt[B.L_HBM][1] == 3000
    assert mdh.mdh_custom_validate_params(d, p) == 0
    q = p.copy()
    q.prt[B.L_LANE][1], q.prt[B.L_HBM][1] = 4, 750  # lanes on the prefix-sum dimension: not this kernel
    assert mdh.mdh_custom_validate_params(d, q) == 6
    # two prefix-sum dimensions are refused
    with pytest.raises(mdh.MdhError):
        mdh.mdh_custom_default_params(mdh.custom_desc((4, 4), (2, 2), ["int"], [(0, "i0*N1+i1")], "int", 4, "r = a0;", "r = x + y;"))
    assert "have_run" in mdh.mdh_custom_source(mdh.mdh_custom_create(d))


@pytest.mark.gpu
def test_scan_and_mbbs_through_the_generic_path():
    rng = np.random.default_rng(6)
    # scan(+) and scan(max) on integers against the generic evaluator
    v = rng.integers(-9, 10, 41).astype(np.int32)
    for op, f in (("r = x + y;", lambda a, b: a + b), ("r = x > y ? x : y;", max)):
        d = mdh.custom_desc((41,), (2,), ["int"], [(0, "i0")], "int", 4, "r = a0;", op)
        got = run(d, [dev(v)], torch.full((41,), -99, dtype=torch.int32, device="cuda"))
        assert got.cpu().tolist() == G.scan(f, v.tolist())
    # row-wise scan against the generic evaluator (small) and the C oracle (larger), every candidate
    X = rng.integers(-4, 5, (3, 7)).astype(np.float32)
    got = run(d_scan_rows(3, 7), [dev(X)], torch.full((3, 7), float("nan"), device="cuda"))
    assert got.cpu().numpy().tolist() == G.scan_rows(lambda a, b: a + b, X.astype(int).tolist())
    Xl = W.uniform(W.SEED_BASE + 85, 1, (70, 1500), -1, 1)
    ref, refabs = oracle.scan_rows(Xl, with_abs=True)
    for p in all_params(d_scan_rows(70, 1500)):
        got = run(d_scan_rows(70, 1500), [dev(Xl)], torch.full((70, 1500), float("nan"), device="cuda"), p)
        assert float(np.max(np.abs(got.cpu().numpy() - ref) / refabs)) <= 1e-4
    # the md_hom of MBBS: two dimensions, two operators (prefix-sum(+), +)
    M = rng.integers(-5, 6, (6, 9)).astype(np.float32)
    got = run(d_bottom_box_sums(6, 9), [dev(M)], torch.full((6,), float("nan"), device="cuda"))
    assert got.cpu().tolist() == G.bottom_box_sums(M.astype(int).tolist())
    Ml = rng.integers(-5, 6, (300, 500)).astype(np.float32)  # integer sums below 2^24: exact
    want = np.cumsum(Ml[::-1].astype(np.float64).sum(axis=1))
    for p in all_params(d_bottom_box_sums(300, 500)):
        got = run(d_bottom_box_sums(300, 500), [dev(Ml)], torch.full((300,), float("nan"), device="cuda"), p)
        assert np.array_equal(got.cpu().numpy().astype(np.float64), want)
    assert float(want.max()) == max(G.bottom_box_sums(Ml[-3:, :4].astype(int).tolist()) + [float(want.max())])


@pytest.mark.gpu
def test_custom_tune_returns_a_valid_configuration():
    d = d_histo(64, 50000)
    elems = W.integers(W.SEED_BASE + 86, 1, (50000,), 0, 63).astype(np.int32)
    bins = np.arange(64, dtype=np.int32)
    out = torch.empty(64, dtype=torch.int32, device="cuda")
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    best, ms = mdh.mdh_custom_tune(d, [dev(elems), dev(bins)], out, ws, reps=2, max_candidates=6)
    assert ms > 0 and mdh.mdh_custom_validate_params(d, best) == 0
    got = run(d, [dev(elems), dev(bins)], torch.full((64,), -1, dtype=torch.int32, device="cuda"), best)
    assert np.array_equal(got.cpu().numpy(), np.bincount(elems, minlength=64))


@pytest.mark.gpu
def test_high_dimensional_instances_through_the_generic_path():
    # MCC itself, all seven dimensions (n,p,q,k | c,r,s), strided index functions p*sh+r, q*sw+s
    N, Hh, Wd, C, K, R, S, sh, sw = 2, 11, 13, 3, 5, 3, 2, 2, 1
    x, f = W.mcc_inputs(W.MccCfg(N, Hh, Wd, C, K, R, S, (sh, sw), W.SEED_BASE + 87))
    P, Q = (Hh - R) // sh + 1, (Wd - S) // sw + 1
    ref, refabs = oracle.mcc(x, f, (sh, sw), with_abs=True)
    d = mdh.custom_desc((N, P, Q, K, C, R, S), (0, 0, 0, 0, 1, 1, 1), ["float", "float"],
                        [(0, "((i0*%d + (i1*%d+i5))*%d + (i2*%d+i6))*N4 + i4" % (Hh, sh, Wd, sw)),
                         (1, "((i3*N5 + i5)*N6 + i6)*N4 + i4")], "float", 4, "r = a0 * a1;", "r = x + y;", fast_dim=3)
    for p in all_params(d)[:8]:
        got = run(d, [dev(x), dev(f)], torch.full((N, P, Q, K), float("nan"), device="cuda"), p)
        assert float(np.max(np.abs(got.cpu().numpy() - ref) / refabs)) <= 1e-4
    # a tensor contraction with transposed accesses, C[a,b,c] = sum_d A[d,b,a] * B[c,d]
    # (the kind of view the coupled-cluster examples of the paper use)
    na, nb, nc, nd = 6, 5, 7, 9
    rng = np.random.default_rng(12)
    A = rng.integers(-3, 4, (nd, nb, na)).astype(np.float32)
    Bm = rng.integers(-3, 4, (nc, nd)).astype(np.float32)
    want = np.einsum("dba,cd->abc", A.astype(np.float64), Bm.astype(np.float64))
    d = mdh.custom_desc((na, nb, nc, nd), (0, 0, 0, 1), ["float", "float"],
                        [(0, "(i3*N1 + i1)*N0 + i0"), (1, "i2*N3 + i3")], "float", 4, "r = a0 * a1;", "r = x + y;")
    got = run(d, [dev(A), dev(Bm)], torch.full((na, nb, nc), float("nan"), device="cuda"))
    assert np.array_equal(got.cpu().numpy().astype(np.float64), want)
    # reduce with two operators at once: one pass, a pair (sum, max) as the result type
    v = rng.integers(-100, 100, 5000).astype(np.int32)
    d = mdh.custom_desc((5000,), (1,), ["int"], [(0, "i0")], "pr", 8, "r.s = a0; r.m = a0;",
                        "r.s = x.s + y.s; r.m = x.m > y.m ? x.m : y.m;", "struct pr { int s; int m; };")
    got = run(d, [dev(v)], torch.zeros(2, dtype=torch.int32, device="cuda"))
    assert got.cpu().tolist() == [int(v.sum()), int(v.max())]


@pytest.mark.gpu
def test_bench_sizes_against_the_oracle():
    """The two workloads bench.py runs through the generic path, at its sizes, inputs and default
    configuration: Histo 256 bins x 2^24 elements (every bin against the compiled oracle) and the
    custom reduce 2^16 x 2^18 (sampled records against the compiled oracle), bit-exact."""
    nb, ne = 256, 1 << 24
    elems = W.device_integers(W.SEED_BASE + 13, 1, (ne,), 0, nb - 1)
    bins = torch.arange(nb, dtype=torch.int32, device="cuda")
    got = run(d_histo(nb, ne), [elems, bins], torch.full((nb,), -1, dtype=torch.int32, device="cuda"))
    want = oracle.histo(elems.cpu().numpy(), bins.cpu().numpy())
    assert np.array_equal(got.cpu().numpy().astype(np.int64), want) and int(want.sum()) == ne

    cfg = W.CONFIGS["prl_2p16_2p18"]
    alph = W.prl_alphabets(cfg.nF)
    A = torch.stack([W.device_integers(cfg.seed, 1 + 2 * f, (cfg.nA,), 0, a - 1) for f, a in enumerate(alph)], 1).contiguous()
    Bm = torch.stack([W.device_integers(cfg.seed, 2 + 2 * f, (cfg.nB,), 0, a - 1) for f, a in enumerate(alph)], 1).contiguous()
    wp = W.device_integers(cfg.seed, 40, (cfg.nF,), 1, W.PRL_WEIGHT_MAX)
    wm = W.device_integers(cfg.seed, 41, (cfg.nF,), -W.PRL_WEIGHT_MAX, 0)
    got = run(d_prl(cfg.nA, cfg.nB), [A, Bm, wp, wm], torch.full((cfg.nA, 2), -1, dtype=torch.int32, device="cuda")).cpu().numpy()
    rows = np.unique(np.concatenate([np.random.default_rng(11).integers(0, cfg.nA, 500), [0, cfg.nA - 1]])).astype(np.int64)
    sc, ix = oracle.custom_reduce_rows(A.cpu().numpy(), Bm.cpu().numpy(), wp.cpu().numpy(), wm.cpu().numpy(), rows)
    assert np.array_equal(got[rows, 0], sc) and np.array_equal(got[rows, 1], ix)
