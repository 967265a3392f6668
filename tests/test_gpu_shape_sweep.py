"""Seeded sweep of small, ragged shapes through every device entry point of the library, against the
oracle: the library default and two randomly drawn candidates per shape.  Outputs sit between guard
words, so a store outside the output shows as a changed guard; NaN-filled outputs show that every
element is written.  Extents are log-uniform: 1, a few, and a few tiles all occur."""
import numpy as np
import pytest

import oracle
import paper_2405_05118_amd as mdh
from paper_2405_05118_amd import workloads as W

torch = pytest.importorskip("torch")

GUARD = 1024
COUNT = 30
TOL = 1e-4


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def guarded(shape, dtype=torch.float32):
    n = int(np.prod(shape))
    is_f = dtype == torch.float32
    buf = torch.full((n + 2 * GUARD,), float("nan") if is_f else -77, dtype=dtype, device="cuda")
    buf[:GUARD] = 12345
    buf[GUARD + n:] = 12345
    return buf, buf[GUARD:GUARD + n].view(*shape)


def guards_ok(buf, n):
    return bool((buf[:GUARD] == 12345).all() and (buf[GUARD + n:] == 12345).all())


def wsp(inst, sizes, p):
    n = mdh.mdh_workspace_size(inst, sizes, p)
    return torch.empty(max(n, 8) // 4, dtype=torch.int32, device="cuda") if n else None


def check(case, got, ref, refabs, tol=TOL):
    got = got.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got)), (case, "output not fully written")
    if got.size:
        err = float(np.max(np.abs(got - ref) / np.where(refabs > 0, refabs, 1.0)))
        assert err <= tol, (case, err)


class Draw:
    def __init__(self, name):
        self.rng = np.random.default_rng(sum(map(ord, name)) + 7)

    def ri(self, lo, hi):
        return int(np.clip(np.exp(self.rng.uniform(np.log(lo), np.log(hi + 1))), lo, hi))

    def bit(self):
        return int(self.rng.integers(2))

    def params(self, inst, sizes):
        """None (the library default) and up to two other candidates."""
        nc = mdh.mdh_num_candidates(inst, sizes)
        out = [None]
        if nc > 1:
            for i in self.rng.choice(np.arange(1, nc), size=min(2, nc - 1), replace=False):
                out.append(mdh.mdh_candidate(inst, sizes, int(i)))
        return out


@pytest.mark.gpu
def test_matmul_shapes():
    d = Draw("matmul")
    for it in range(COUNT):
        M, N, K = d.ri(1, 700), d.ri(1, 700), d.ri(1, 3000)
        A, Bm = W.uniform(it, 1, (M, K), -1, 1), W.uniform(it, 2, (K, N), -1, 1)
        ref, refabs = oracle.matmul(A, Bm, with_abs=True)
        for p in d.params(mdh.MDH_MATMUL, (M, N, K)):
            buf, C = guarded((M, N))
            mdh.mdh_matmul(dev(A), dev(Bm), C, p, wsp(mdh.MDH_MATMUL, (M, N, K), p))
            torch.cuda.synchronize()
            check(((M, N, K), p and p.table()), C, ref, refabs)
            assert guards_ok(buf, M * N), ((M, N, K), p and p.table())


@pytest.mark.gpu
def test_batched_and_transposed_matmul_shapes():
    d = Draw("bmatmul")
    for it in range(2 * COUNT):
        small = it % 2 == 0  # every other case has at most 16 rows: the register-streaming kernels
        nb, M, N, K = d.ri(1, 5), (d.ri(1, 16) if small else d.ri(1, 300)), d.ri(1, 900), d.ri(1, 5000)
        ta, tb, tc = (0, d.bit(), 0) if small else (d.bit(), d.bit(), d.bit())
        sizes = (nb, M, N, K, ta, tb, tc)
        A = W.uniform(it, 1, (nb, K, M) if ta else (nb, M, K), -1, 1)
        Bm = W.uniform(it, 2, (nb, N, K) if tb else (nb, K, N), -1, 1)
        A64 = A.astype(np.float64).transpose(0, 2, 1) if ta else A.astype(np.float64)
        B64 = Bm.astype(np.float64).transpose(0, 2, 1) if tb else Bm.astype(np.float64)
        ref, refabs = A64 @ B64, np.abs(A64) @ np.abs(B64)  # the definition, through numpy's fp64 matmul
        if tc:
            ref, refabs = ref.transpose(0, 2, 1), refabs.transpose(0, 2, 1)
        for p in d.params(mdh.MDH_BMATMUL, sizes):
            buf, C = guarded((nb, N, M) if tc else (nb, M, N))
            mdh.mdh_matmul_ex(dev(A), dev(Bm), C, bool(ta), bool(tb), bool(tc), p, wsp(mdh.MDH_BMATMUL, sizes, p))
            torch.cuda.synchronize()
            check((sizes, p and p.table()), C, ref, refabs)
            assert guards_ok(buf, nb * M * N), (sizes, p and p.table())


def conv_geometry(d, max_p, max_q):
    R, S, sh, sw = d.ri(1, 7), d.ri(1, 7), d.ri(1, 3), d.ri(1, 3)
    N, P, Q = d.ri(1, 5), d.ri(1, max_p), d.ri(1, max_q)
    # the input may have rows and columns that no output pixel reaches
    H, Wd = (P - 1) * sh + R + int(d.rng.integers(sh)), (Q - 1) * sw + S + int(d.rng.integers(sw))
    return N, P, Q, H, Wd, R, S, sh, sw


@pytest.mark.gpu
@pytest.mark.parametrize("few_channels", [False, True])
def test_mcc_shapes(few_channels):
    d = Draw("mccflat" if few_channels else "mcc")
    for it in range(COUNT):
        N, P, Q, H, Wd, R, S, sh, sw = conv_geometry(d, 40, 40)
        C, K = (d.ri(1, 8) if few_channels else d.ri(9, 150)), d.ri(1, 140)
        sizes = (N, P, Q, K, C, R, S, sh, sw)
        x, f = W.mcc_inputs(W.MccCfg(N, H, Wd, C, K, R, S, (sh, sw), it))
        ref, refabs = oracle.mcc(x, f, (sh, sw), with_abs=True)
        for p in d.params(mdh.MDH_MCC, sizes):
            buf, out = guarded((N, P, Q, K))
            mdh.mdh_mcc(dev(x), dev(f), out, (sh, sw), p, wsp(mdh.MDH_MCC, sizes, p))
            torch.cuda.synchronize()
            check((sizes, (H, Wd), p and p.table()), out, ref, refabs)
            assert guards_ok(buf, N * P * Q * K), (sizes, p and p.table())


@pytest.mark.gpu
def test_capsule_shapes():
    d = Draw("capsule")
    ran = 0
    for it in range(COUNT):
        N, P, Q, H, Wd, R, S, sh, sw = conv_geometry(d, 14, 20)
        C, K = d.ri(1, 4), d.ri(1, 40)
        sizes = (N, P, Q, K, C, R, S, sh, sw)
        try:
            ps = d.params(mdh.MDH_MCC_CAPSULE, sizes)
        except mdh.MdhError as e:  # the filter slice does not fit in LDS: no configuration
            assert e.status == 4, sizes
            continue
        x, f = W.normal(it, 1, (N, H, Wd, C, 4, 4)), W.normal(it, 2, (K, R, S, C, 4, 4))
        ref, refabs = oracle.mcc_capsule(x, f, (sh, sw), with_abs=True)
        for p in ps:
            buf, out = guarded((N, P, Q, K, 4, 4))
            mdh.mdh_mcc_capsule(dev(x), dev(f), out, (sh, sw), p)
            torch.cuda.synchronize()
            check((sizes, (H, Wd), p and p.table()), out, ref, refabs)
            assert guards_ok(buf, N * P * Q * K * 16), (sizes, p and p.table())
        ran += 1
    assert ran >= COUNT // 2


@pytest.mark.gpu
def test_stencil_shapes():
    d = Draw("stencil")
    for it in range(COUNT):
        sizes = (d.ri(1, 70), d.ri(1, 70), d.ri(1, 300))
        x = W.uniform(it, 1, tuple(n + 2 for n in sizes), -1, 1)
        ref = oracle.jacobi3d(x, 0.3, 0.1)
        for p in d.params(mdh.MDH_STENCIL, sizes):
            buf, out = guarded(sizes)
            mdh.mdh_stencil(dev(x), out, 0.3, 0.1, p)
            torch.cuda.synchronize()
            check((sizes, p and p.table()), out, ref, np.ones_like(ref), 1e-5)
            assert guards_ok(buf, int(np.prod(sizes))), (sizes, p and p.table())


@pytest.mark.gpu
def test_custom_reduce_shapes():
    d = Draw("prl")
    for it in range(COUNT):
        nA, nB, nF = d.ri(1, 3000), d.ri(1, 5000), d.ri(1, 8)
        A, Bm, wa, wd = W.prl_inputs(W.PrlCfg(nA, nB, nF, it))
        rs, rb = oracle.custom_reduce(A, Bm, wa, wd)
        for p in d.params(mdh.MDH_CUSTOM_REDUCE, (nA, nB, nF)):
            b1, sc = guarded((nA,), torch.int32)
            b2, ix = guarded((nA,), torch.int32)
            mdh.mdh_custom_reduce(dev(A), dev(Bm), dev(wa), dev(wd), sc, ix, p, wsp(mdh.MDH_CUSTOM_REDUCE, (nA, nB, nF), p))
            torch.cuda.synchronize()
            assert np.array_equal(sc.cpu().numpy(), rs) and np.array_equal(ix.cpu().numpy(), rb), ((nA, nB, nF), p and p.table())
            assert guards_ok(b1, nA) and guards_ok(b2, nA)


@pytest.mark.gpu
def test_dot_and_matvec_shapes():
    d = Draw("dot")
    for it in range(COUNT):
        K = d.ri(1, 3000000)
        x, y = W.uniform(it, 1, (K,), -1, 1), W.uniform(it, 2, (K,), -1, 1)
        ref, refabs = oracle.dot(x, y)
        for p in d.params(mdh.MDH_DOT, (K,)):
            buf, out = guarded((1,))
            mdh.mdh_dot(dev(x), dev(y), out, p, wsp(mdh.MDH_DOT, (K,), p))
            torch.cuda.synchronize()
            check((K, p and p.table()), out, np.array([ref]), np.array([refabs]))
            assert guards_ok(buf, 1)
    d = Draw("matvec")
    for it in range(COUNT):
        M, K = d.ri(1, 3000), d.ri(1, 6000)
        A, x = W.uniform(it, 1, (M, K), -1, 1), W.uniform(it, 2, (K,), -1, 1)
        ref, refabs = oracle.matvec(A, x, with_abs=True)
        for p in d.params(mdh.MDH_MATVEC, (M, K)):
            buf, y = guarded((M,))
            mdh.mdh_matvec(dev(A), dev(x), y, p, wsp(mdh.MDH_MATVEC, (M, K), p))
            torch.cuda.synchronize()
            check(((M, K), p and p.table()), y, ref, refabs)
            assert guards_ok(buf, M)


@pytest.mark.gpu
def test_scan_shapes():
    d = Draw("scan")
    for it in range(COUNT):
        R, n = (d.ri(1, 3000), d.ri(1, 3000)) if it % 2 else (d.ri(1, 4), d.ri(1, 3000000))
        X = W.uniform(it, 1, (R, n), -1, 1)
        ref, refabs = oracle.scan_rows(X, with_abs=True)
        for p in d.params(mdh.MDH_SCAN, (R, n)):
            buf, out = guarded((R, n))
            ws = wsp(mdh.MDH_SCAN, (R, n), p)
            mdh.mdh_scan(dev(X), out, p, ws)
            torch.cuda.synchronize()
            assert not mdh.mdh_scan_timed_out(dev(X), p, ws)
            check(((R, n), p and p.table()), out, ref, refabs)
            assert guards_ok(buf, R * n)
