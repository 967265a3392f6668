"""Row-wise scan(+) = md_hom(id, (++, prefix-sum(+))): host planner and GPU parity against the
oracle (fp64 inclusive prefix sums of the same fp32 inputs)."""
import numpy as np
import pytest

import oracle
import paper_2405_05118_amd as mdh
from paper_2405_05118_amd import binding as B
from paper_2405_05118_amd import workloads as W

TOL = 1e-5  # |gpu - ref| / prefix sum of |x|; fp32 tree inside a tile, fp64 carries between tiles


@pytest.mark.parametrize("sizes", [(1, 1 << 24), (4096, 4096), (3, 1000), (1, 1), (70000, 17), (0, 5), (5, 0)])
def test_planner(sizes):
    inst = mdh.MDH_SCAN
    p = mdh.mdh_default_params(inst, sizes)
    assert p.D == 2 and list(p.blk[:2]) == [1, 1] and p.strided == 0
    for d in range(2):
        e = p.extent(d)
        assert e >= sizes[d] if p.ragged else e == sizes[d]
    assert mdh.mdh_validate_params(inst, sizes, p) == 0
    for i in range(mdh.mdh_num_candidates(inst, sizes)):
        c = mdh.mdh_candidate(inst, sizes, i)
        assert mdh.mdh_validate_params(inst, sizes, c) == 0
    C = p.prt[B.L_WG][1]

    def want_ws(q):
        c = q.prt[B.L_WG][1]
        if c <= 1:
            return 0
        if q.in_region[0] == B.MR_VGPR:  # single pass: ticket, time-out flag, totals, group sums
            return 8 * (2 + sizes[0] * c + sizes[0] * ((c + 63) // 64))
        return 8 * c * sizes[0]  # three kernels: chunk totals

    assert mdh.mdh_workspace_size(inst, sizes, p) == want_ws(p)
    kinds = set()
    for i in range(mdh.mdh_num_candidates(inst, sizes)):
        c = mdh.mdh_candidate(inst, sizes, i)
        assert mdh.mdh_workspace_size(inst, sizes, c) == want_ws(c)
        if c.prt[B.L_WG][1] > 1:
            kinds.add(int(c.in_region[0]))
    if C > 1:  # both ways of exchanging the chunk totals are in the search space
        assert kinds == {B.MR_HBM, B.MR_VGPR}
        assert p.in_region[0] == B.MR_VGPR and p.prt[B.L_HBM][1] == 1 and p.prt[B.L_VGPR][1] in (4, 8, 16, 32)
    # a long single row is cut into chunks over workgroups, many rows are not
    if sizes == (1, 1 << 24):
        assert C > 1
    if sizes == (4096, 4096):  # a row of two tiles stays in the workgroup's registers
        assert C == 1 and p.prt[B.L_HBM][1] == 1 and p.prt[B.L_VGPR][1] == 8


def test_planner_rejects_empty_chunk():
    sizes = (2, 5000)
    p = mdh.mdh_default_params(mdh.MDH_SCAN, sizes)
    q = p.copy()
    q.prt[B.L_WG][1], q.prt[B.L_HBM][1], q.ragged = 8, 1, 1  # chunks 5..7 start beyond the row
    assert mdh.mdh_validate_params(mdh.MDH_SCAN, sizes, q) == 3
    q = p.copy()
    q.prt[B.L_WAVE][1] = 5  # no such instantiation (and the product changes)
    assert mdh.mdh_validate_params(mdh.MDH_SCAN, sizes, q) != 0
    # the single-pass variant holds a chunk in registers: only 2, 4 or 8 tiles per chunk
    sizes = (1, 1 << 24)
    three = [c for c in cands(sizes)[1:] if c.prt[B.L_WG][1] > 1 and c.in_region[0] == B.MR_HBM and c.prt[B.L_HBM][1] > 8]
    assert three
    q = three[0].copy()
    q.in_region[0] = B.MR_VGPR
    assert mdh.mdh_validate_params(mdh.MDH_SCAN, sizes, q) != 0
    q.in_region[0] = B.MR_LDS  # no such variant
    assert mdh.mdh_validate_params(mdh.MDH_SCAN, sizes, q) != 0


torch = pytest.importorskip("torch")


def run(x, p):
    xs = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    out = torch.full_like(xs, float("nan"))
    sizes = x.shape if x.ndim == 2 else (1, x.size)
    n = mdh.mdh_workspace_size(mdh.MDH_SCAN, sizes, p)
    ws = torch.empty(max(n, 8) // 8, dtype=torch.float64, device="cuda") if n else None
    mdh.mdh_scan(xs, out, p, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64)


def cands(sizes):
    return [None] + [mdh.mdh_candidate(mdh.MDH_SCAN, sizes, i) for i in range(mdh.mdh_num_candidates(mdh.MDH_SCAN, sizes))]


@pytest.mark.gpu
@pytest.mark.parametrize("shape", [(1, 1), (1, 5), (3, 1000), (7, 1024), (2, 1025), (5, 4099), (1, 300007), (33, 20000), (600, 257)])
def test_every_candidate(shape):
    x = W.uniform(W.SEED_BASE + 95, 1, shape, -1, 1)
    ref, refabs = oracle.scan_rows(x, with_abs=True)
    for p in cands(shape):
        got = run(x, p)
        assert np.all(np.isfinite(got)), "output not fully overwritten"
        err = float(np.max(np.abs(got - ref) / refabs))
        assert err <= TOL, (shape, p and p.table(), err)


@pytest.mark.gpu
def test_single_pass_many_chunks():
    """Rows of several hundred chunks: totals travel through groups of 64 chunks and their sums."""
    shape = (2, 2100003)
    x = W.uniform(W.SEED_BASE + 96, 1, shape, -1, 1)
    ref, refabs = oracle.scan_rows(x, with_abs=True)
    seen = 0
    for p in cands(shape):
        if p is None or p.prt[B.L_WG][1] <= 1 or p.in_region[0] != B.MR_VGPR:
            continue
        seen += 1
        first = run(x, p)
        err = float(np.max(np.abs(first - ref) / refabs))
        assert err <= TOL, (p.table(), err)
        assert np.array_equal(first, run(x, p)), "not bit-identical run to run"
    assert seen >= 4
    assert max(p.prt[B.L_WG][1] for p in cands(shape)[1:]) > 128  # more than two groups
    # the workspace afterwards: every chunk was drawn (and every workgroup drew one number past the
    # end), no wait ran into its bound
    p = mdh.mdh_default_params(mdh.MDH_SCAN, shape)
    assert p.in_region[0] == B.MR_VGPR
    xs = torch.from_numpy(x).cuda()
    out = torch.empty_like(xs)
    ws = torch.full((mdh.mdh_workspace_size(mdh.MDH_SCAN, shape, p) // 8,), -7, dtype=torch.int64, device="cuda")
    mdh.mdh_scan(xs, out, p, ws)
    torch.cuda.synchronize()
    words = ws.cpu().numpy()
    chunks = shape[0] * p.prt[B.L_WG][1]
    assert chunks < words[0] <= 2 * chunks and words[1] == 0


@pytest.mark.gpu
def test_exact_on_small_integers_and_ones():
    ones = np.ones((2, 70001), np.float32)
    for p in cands(ones.shape):
        got = run(ones, p)
        assert np.array_equal(got[0], np.arange(1, 70002)) and np.array_equal(got[1], got[0])
    rng = np.random.default_rng(9)
    x = rng.integers(-3, 4, (4, 9000)).astype(np.float32)  # partial sums stay far below 2^24: exact
    assert np.array_equal(run(x, None), np.cumsum(x.astype(np.float64), axis=1))


@pytest.mark.gpu
def test_long_row_and_explicit_chunks():
    n = (1 << 24) + 12345
    x = W.uniform(W.SEED_BASE + 96, 1, (1, n), 0, 1)  # non-negative: the prefix itself is the scale
    ref = oracle.scan_rows(x)
    got = run(x, None)
    assert float(np.max(np.abs(got - ref) / np.maximum(ref, 1e-30))) <= TOL
    # one workgroup walking the whole row (C = 1) must agree with the chunked evaluation
    sizes = (1, n)
    one = [p for p in cands(sizes)[1:] if p.prt[B.L_WG][1] == 1]
    if one:
        assert float(np.max(np.abs(run(x, one[0]) - ref) / np.maximum(ref, 1e-30))) <= TOL
    with pytest.raises(mdh.MdhError) as e:  # chunked configuration without workspace
        mdh.mdh_scan(torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda"))
    assert e.value.status == 5


@pytest.mark.gpu
def test_full_size_row_exact():
    """One row of 2^28 elements, the configuration bench.py times: a 1 at every 16th position keeps
    every partial sum an integer below 2^24, so each order of additions gives the same exact result."""
    n = 1 << 28
    shape = (1, n)
    x = torch.zeros(n, dtype=torch.float32, device="cuda")
    x[::16] = 1.0
    out = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    p = mdh.mdh_default_params(mdh.MDH_SCAN, shape)
    assert p.prt[B.L_WG][1] > 1 and p.in_region[0] == B.MR_VGPR  # chunks over workgroups, single pass
    ws = torch.empty(mdh.mdh_workspace_size(mdh.MDH_SCAN, shape, p) // 8, dtype=torch.int64, device="cuda")
    mdh.mdh_scan(x, out, None, ws)
    torch.cuda.synchronize()
    step = 1 << 24
    for j0 in range(0, n, step):  # expected values chunk by chunk (device memory)
        want = (torch.arange(j0, j0 + step, device="cuda", dtype=torch.int64) // 16 + 1).to(torch.float32)
        assert torch.equal(out[j0:j0 + step], want), j0
    assert int(ws[1].item()) == 0  # no wait ran into its bound
    assert mdh.mdh_scan_timed_out(x, None, ws) is False  # the same word through the library's helper
    ws[1] = 1  # what a kernel whose wait expired leaves behind
    assert mdh.mdh_scan_timed_out(x, None, ws) is True
    # a configuration without waits never reports a time-out, whatever its workspace holds
    assert mdh.mdh_scan_timed_out(torch.empty((8, 4096), device="cuda"), None, None) is False


@pytest.mark.gpu
@pytest.mark.parametrize("shape", [(1, 1 << 28), (65536, 4096)])
def test_full_size_random(shape):
    """The two shapes bench.py times, its inputs, library defaults; the oracle scans a copy of the
    device data and every element is compared (scaled by the prefix sum of |x|)."""
    x = W.device_uniform(W.SEED_BASE + 12, 1, shape, -1.0, 1.0)
    out = torch.full_like(x, float("nan"))
    n = mdh.mdh_workspace_size(mdh.MDH_SCAN, shape)
    ws = torch.empty(max(n, 8) // 8, dtype=torch.float64, device="cuda") if n else None
    mdh.mdh_scan(x, out, None, ws)
    assert not mdh.mdh_scan_timed_out(x, None, ws)
    ref, refabs = oracle.scan_rows(x.cpu().numpy(), with_abs=True)
    got = out.cpu().numpy()
    del x, out
    worst = 0.0
    rows = ref.shape[0]
    for r0 in range(0, rows, 4096):  # in slabs: the whole difference would double the memory
        for c0 in range(0, ref.shape[1], 1 << 24):
            sl = (slice(r0, r0 + 4096), slice(c0, c0 + (1 << 24)))
            worst = max(worst, float(np.max(np.abs(got[sl] - ref[sl]) / refabs[sl])))
    assert worst <= TOL, worst


@pytest.mark.gpu
def test_tune_picks_a_valid_configuration():
    shape = (4, 200000)
    x = W.uniform(W.SEED_BASE + 97, 1, shape, -1, 1)
    xs = torch.from_numpy(x).cuda()
    out = torch.empty_like(xs)
    ws = torch.empty(1 << 16, dtype=torch.float64, device="cuda")
    best, ms = mdh.mdh_tune(mdh.MDH_SCAN, shape, [xs, out], workspace=ws, reps=2)
    assert ms > 0 and mdh.mdh_validate_params(mdh.MDH_SCAN, shape, best) == 0
    ref, refabs = oracle.scan_rows(x, with_abs=True)
    assert float(np.max(np.abs(run(x, best) - ref) / refabs)) <= TOL
