"""Pins for the nested-loop C oracle (oracle/mdh_oracle.c): brute force against the
generic from-the-definition evaluator, closed forms, special cases that reduce to
each other or to a library routine, and the homomorphic split property.  CPU only.

A plausible mistake (dropped term, wrong sign/index, transposed operand, wrong
tie-break) fails at least one test here; tests/test_oracle_mutants.py checks that
claim by planting such mistakes in a Python copy of the loops."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import instances as G

rng = np.random.default_rng(20240511)


def _small_ints(shape, lo=-4, hi=5):
    return rng.integers(lo, hi, size=shape).astype(np.float32)


# --------------------------------------------------------------------------- MatMul


def test_matmul_bruteforce_vs_generic():
    A, B = _small_ints((5, 3)), _small_ints((3, 4))
    want = G.matmul([[int(v) for v in r] for r in A], [[int(v) for v in r] for r in B])
    got, gabs = oracle.matmul(A, B, with_abs=True)
    assert np.array_equal(got, np.array(want, dtype=np.float64))
    assert np.array_equal(gabs, np.abs(A.astype(np.float64)) @ np.abs(B.astype(np.float64)))


def test_matmul_all_ones_gives_K():
    for (M, N, K) in ((3, 2, 7), (17, 9, 300)):
        C = oracle.matmul(np.ones((M, K), np.float32), np.ones((K, N), np.float32))
        assert np.all(C == K)


def test_matmul_identity_and_transposition_sensitivity():
    A = rng.standard_normal((6, 6)).astype(np.float32)
    assert np.array_equal(oracle.matmul(A, np.eye(6, dtype=np.float32)), A.astype(np.float64))
    assert np.array_equal(oracle.matmul(np.eye(6, dtype=np.float32), A), A.astype(np.float64))
    # a unit matrix E_pq picks row/column: (E_pq A)[p,:] = A[q,:]  (fails if A or B is transposed)
    E = np.zeros((6, 6), np.float32)
    E[1, 4] = 1
    got = oracle.matmul(E, A)
    want = np.zeros((6, 6))
    want[1, :] = A[4, :]
    assert np.array_equal(got, want)


def test_matmul_matches_library_routine():
    A = rng.uniform(-1, 1, (37, 53)).astype(np.float32)
    B = rng.uniform(-1, 1, (53, 29)).astype(np.float32)
    want = A.astype(np.float64) @ B.astype(np.float64)
    assert np.allclose(oracle.matmul(A, B), want, rtol=0, atol=1e-12)


def test_matmul_split_property():
    A = rng.uniform(-1, 1, (12, 20)).astype(np.float32)
    B = rng.uniform(-1, 1, (20, 10)).astype(np.float32)
    whole = oracle.matmul(A, B)
    # split i and j: concatenation of the halves, exactly
    assert np.array_equal(np.vstack([oracle.matmul(A[:5], B), oracle.matmul(A[5:], B)]), whole)
    assert np.array_equal(np.hstack([oracle.matmul(A, B[:, :3]), oracle.matmul(A, B[:, 3:])]), whole)
    # split k: point-wise sum of the halves (fp64 rounding only)
    parts = oracle.matmul(A[:, :7], B[:7]) + oracle.matmul(A[:, 7:], B[7:])
    assert np.allclose(parts, whole, rtol=0, atol=1e-13)


def test_matmul_at_equals_full():
    A = rng.uniform(-1, 1, (9, 31)).astype(np.float32)
    B = rng.uniform(-1, 1, (31, 8)).astype(np.float32)
    full, fabs = oracle.matmul(A, B, with_abs=True)
    is_, js = np.array([0, 8, 3, 3]), np.array([0, 7, 2, 5])
    v, va = oracle.matmul_at(A, B, is_, js)
    assert np.array_equal(v, full[is_, js]) and np.array_equal(va, fabs[is_, js])


# --------------------------------------------------------------------------- Jacobi-3D


def test_jacobi_bruteforce_vs_generic():
    x = rng.integers(0, 9, size=(5, 6, 7)).astype(np.float32)
    c0, c1 = 0.5, 0.25  # exactly representable: integer inputs give exact results
    want = G.jacobi3d([[[Fraction(int(v)) for v in r] for r in p] for p in x], Fraction(1, 2), Fraction(1, 4))
    got = oracle.jacobi3d(x, c0, c1)
    assert got.shape == (3, 4, 5)
    assert np.array_equal(got, np.array([[[float(v) for v in r] for r in p] for p in want]))


def test_jacobi_each_neighbour_has_its_own_place():
    # a single 1 in the input shows up in exactly seven outputs with the right weights
    nx, ny, nz = 4, 5, 6
    x = np.zeros((nx + 2, ny + 2, nz + 2), np.float32)
    x[2, 3, 4] = 1.0
    out = oracle.jacobi3d(x, 0.5, 0.125)
    want = np.zeros((nx, ny, nz))
    want[1, 2, 3] = 0.5
    for d in ((1, 0, 0), (-1, 0, 0), (0, 1, 0), (0, -1, 0), (0, 0, 1), (0, 0, -1)):
        want[1 + d[0], 2 + d[1], 3 + d[2]] = 0.125
    assert np.array_equal(out, want)


def test_jacobi_constant_and_linear_fields_are_fixed_points():
    c0, c1 = np.float32(0.5), np.float32(1.0 / 12.0)
    nx, ny, nz = 6, 7, 8
    const = np.full((nx + 2, ny + 2, nz + 2), 3.0, np.float32)
    out = oracle.jacobi3d(const, c0, c1)
    # c0 + 6*c1 differs from 1 only by the rounding of float(1/12)
    assert np.allclose(out, 3.0, rtol=2e-7, atol=0)
    i, j, k = np.meshgrid(np.arange(nx + 2), np.arange(ny + 2), np.arange(nz + 2), indexing="ij")
    lin = (2 * i - 3 * j + 5 * k + 7).astype(np.float32)
    out = oracle.jacobi3d(lin, c0, c1)
    centre = lin[1:-1, 1:-1, 1:-1].astype(np.float64)
    scale = float(c0) + 6 * float(c1)
    assert np.allclose(out, centre * scale, rtol=1e-15, atol=1e-12)


def test_jacobi_matches_array_slicing():
    x = rng.uniform(0, 1, (9, 8, 11)).astype(np.float32)
    c0, c1 = np.float32(0.5), np.float32(1.0 / 12.0)
    d = x.astype(np.float64)
    want = float(c0) * d[1:-1, 1:-1, 1:-1] + float(c1) * (
        d[:-2, 1:-1, 1:-1] + d[2:, 1:-1, 1:-1] + d[1:-1, :-2, 1:-1] + d[1:-1, 2:, 1:-1] + d[1:-1, 1:-1, :-2] + d[1:-1, 1:-1, 2:]
    )
    assert np.allclose(oracle.jacobi3d(x, c0, c1), want, rtol=0, atol=1e-15)


def test_jacobi_split_property():
    x = rng.uniform(0, 1, (8, 9, 10)).astype(np.float32)
    whole = oracle.jacobi3d(x, 0.5, 0.0833)
    # halves read overlapping halos of the same buffer; results concatenate exactly
    for axis, cut in ((0, 2), (1, 4), (2, 5)):
        lo = [slice(None)] * 3
        hi = [slice(None)] * 3
        lo[axis] = slice(0, cut + 2)
        hi[axis] = slice(cut, None)
        got = np.concatenate([oracle.jacobi3d(x[tuple(lo)], 0.5, 0.0833), oracle.jacobi3d(x[tuple(hi)], 0.5, 0.0833)], axis=axis)
        assert np.array_equal(got, whole)


# --------------------------------------------------------------------------- MCC


def test_mcc_bruteforce_vs_generic():
    for stride in ((1, 1), (2, 1)):
        x = _small_ints((2, 5, 4, 3))
        f = _small_ints((2, 3, 2, 3))
        want = G.mcc(x.astype(int).tolist(), f.astype(int).tolist(), stride)
        got = oracle.mcc(x, f, stride)
        assert np.array_equal(got, np.array(want, dtype=np.float64))


def test_mcc_all_ones_gives_CRS():
    x = np.ones((2, 9, 8, 5), np.float32)
    f = np.ones((3, 4, 3, 5), np.float32)
    out, oabs = oracle.mcc(x, f, with_abs=True)
    assert out.shape == (2, 6, 6, 3)
    assert np.all(out == 5 * 4 * 3) and np.all(oabs == 60)


def test_mcc_delta_filter_is_a_shifted_channel_copy():
    x = rng.standard_normal((2, 8, 9, 4)).astype(np.float32)
    f = np.zeros((3, 3, 4, 4), np.float32)
    f[1, 2, 3, 1] = 1.0  # output channel 1 <- input channel 1 shifted by (r,s) = (2,3)
    out = oracle.mcc(x, f)
    P, Q = 6, 6
    assert np.array_equal(out[..., 1], x[:, 2 : 2 + P, 3 : 3 + Q, 1].astype(np.float64))
    assert np.all(out[..., 0] == 0) and np.all(out[..., 2] == 0)


def test_mcc_reduces_to_matmul_for_1x1():
    # R=S=1, H=W=1: out[n,0,0,k] = sum_c in[n,c]*filt[k,c]  = (X F^T)[n,k]
    X = rng.uniform(-1, 1, (7, 13)).astype(np.float32)
    F = rng.uniform(-1, 1, (5, 13)).astype(np.float32)
    out = oracle.mcc(X.reshape(7, 1, 1, 13), F.reshape(5, 1, 1, 13))
    assert np.allclose(out.reshape(7, 5), oracle.matmul(X, np.ascontiguousarray(F.T)), rtol=0, atol=1e-14)


def test_mcc_stride_subsamples_the_unit_stride_result():
    x = rng.standard_normal((1, 11, 12, 3)).astype(np.float32)
    f = rng.standard_normal((2, 3, 2, 3)).astype(np.float32)
    full = oracle.mcc(x, f, (1, 1))
    assert np.array_equal(oracle.mcc(x, f, (2, 3)), full[:, ::2, ::3, :][:, : (11 - 3) // 2 + 1, : (12 - 2) // 3 + 1])


def test_mcc_split_property():
    x = rng.standard_normal((2, 7, 8, 6)).astype(np.float32)
    f = rng.standard_normal((4, 3, 3, 6)).astype(np.float32)
    whole = oracle.mcc(x, f)
    # ++ dims: n, k (plain slices); p (overlapping input rows)
    assert np.array_equal(np.concatenate([oracle.mcc(x[:1], f), oracle.mcc(x[1:], f)], 0), whole)
    assert np.array_equal(np.concatenate([oracle.mcc(x, f[:1]), oracle.mcc(x, f[1:])], 3), whole)
    assert np.array_equal(np.concatenate([oracle.mcc(x[:, :5], f), oracle.mcc(x[:, 3:], f)], 1), whole)
    # + dims: c, r, s
    c = oracle.mcc(np.ascontiguousarray(x[..., :2]), np.ascontiguousarray(f[..., :2])) + oracle.mcc(
        np.ascontiguousarray(x[..., 2:]), np.ascontiguousarray(f[..., 2:]))
    assert np.allclose(c, whole, rtol=0, atol=1e-13)
    r = oracle.mcc(x[:, :6], f[:, :2]) + oracle.mcc(x[:, 2:], f[:, 2:])
    assert np.allclose(r, whole, rtol=0, atol=1e-13)
    s = oracle.mcc(x[:, :, :6], f[:, :, :1]) + oracle.mcc(x[:, :, 1:], f[:, :, 1:])
    assert np.allclose(s, whole, rtol=0, atol=1e-13)


def test_mcc_at_equals_full():
    x = rng.standard_normal((2, 6, 7, 3)).astype(np.float32)
    f = rng.standard_normal((3, 2, 3, 3)).astype(np.float32)
    full, fabs = oracle.mcc(x, f, with_abs=True)
    idx = np.array([[0, 0, 0, 0], [1, 4, 4, 2], [1, 2, 3, 1]])
    v, va = oracle.mcc_at(x, f, idx)
    assert np.array_equal(v, full[tuple(idx.T)]) and np.array_equal(va, fabs[tuple(idx.T)])


# --------------------------------------------------------------------------- custom reduce


def _records(n, nF, alph=3):
    return rng.integers(0, alph, size=(n, nF)).astype(np.int32)


def test_custom_reduce_bruteforce_vs_generic():
    for (nA, nB, nF) in ((6, 8, 3), (8, 5, 8), (1, 1, 2)):
        A, B = _records(nA, nF), _records(nB, nF)
        wp = rng.integers(1, 10, nF).astype(np.int32)
        wm = rng.integers(-10, 1, nF).astype(np.int32)
        s, i = oracle.custom_reduce(A, B, wp, wm)
        gs, gi = G.custom_reduce(A.tolist(), B.tolist(), wp.tolist(), wm.tolist())
        assert s.tolist() == gs and i.tolist() == gi


def test_custom_reduce_equal_weights_pin_the_tie_break():
    # agree == disagree weight: every b scores nF*w -> the smallest index wins
    A, B = _records(9, 4, alph=50), _records(30, 4, alph=50)
    w = np.full(4, 7, np.int32)
    s, i = oracle.custom_reduce(A, B, w, w)
    assert np.all(s == 28) and np.all(i == 0)


def test_custom_reduce_finds_embedded_copies_first_position():
    nF = 5
    A = np.arange(20 * nF, dtype=np.int32).reshape(20, nF)  # all records distinct in every field
    B = -1 - _records(64, nF, alph=1000)  # negative: never equal to a field of A
    pos = rng.permutation(64)[:20]
    B[pos] = A
    dup = (pos[3] + 1) % 64
    while dup in pos:
        dup = (dup + 1) % 64
    B[dup] = A[3]  # a second copy of record 3
    wp = rng.integers(1, 100, nF).astype(np.int32)
    wm = rng.integers(-100, 0, nF).astype(np.int32)
    s, i = oracle.custom_reduce(A, B, wp, wm)
    assert np.all(s == wp.sum())
    want = pos.copy()
    want[3] = min(pos[3], dup)
    assert np.array_equal(i, want)


def test_custom_reduce_score_formula_by_hand():
    A = np.array([[1, 2, 3]], np.int32)
    B = np.array([[1, 0, 0], [1, 2, 0], [0, 2, 3], [9, 9, 9]], np.int32)
    wp = np.array([10, 20, 40], np.int32)
    wm = np.array([-1, -2, -4], np.int32)
    # scores: 10-2-4=4 ; 10+20-4=26 ; -1+20+40=59 ; -7
    s, i = oracle.custom_reduce(A, B, wp, wm)
    assert (s[0], i[0]) == (59, 2)
    s, i = oracle.custom_reduce(A, B[:2], wp, wm)
    assert (s[0], i[0]) == (26, 1)
    s, i = oracle.custom_reduce(A, B[3:], wp, wm)
    assert (s[0], i[0]) == (-7, 0)


def test_custom_reduce_split_property_and_rows():
    A, B = _records(40, 8, alph=2), _records(90, 8, alph=2)  # tiny alphabet: many ties
    wp = rng.integers(1, 5, 8).astype(np.int32)
    wm = rng.integers(-5, 1, 8).astype(np.int32)
    s, i = oracle.custom_reduce(A, B, wp, wm)
    for cut in (1, 37, 89):
        s1, i1 = oracle.custom_reduce(A, B[:cut], wp, wm)
        s2, i2 = oracle.custom_reduce(A, B[cut:], wp, wm)
        cs, ci = oracle.maxidx_combine(s1, i1, s2, i2 + cut)
        assert np.array_equal(cs, s) and np.array_equal(ci, i)
        # the operator is commutative
        cs, ci = oracle.maxidx_combine(s2, i2 + cut, s1, i1)
        assert np.array_equal(cs, s) and np.array_equal(ci, i)
    # ++ dimension: splitting A concatenates
    sa, ia = oracle.custom_reduce(A[:13], B, wp, wm)
    assert np.array_equal(sa, s[:13]) and np.array_equal(ia, i[:13])
    rows = np.array([39, 0, 7])
    sr, ir = oracle.custom_reduce_rows(A, B, wp, wm, rows)
    assert np.array_equal(sr, s[rows]) and np.array_equal(ir, i[rows])


def test_custom_reduce_permuting_B_only_moves_indices():
    A, B = _records(25, 6, alph=4), _records(70, 6, alph=4)
    wp = rng.integers(1, 50, 6).astype(np.int32)
    wm = rng.integers(-50, 1, 6).astype(np.int32)
    s, i = oracle.custom_reduce(A, B, wp, wm)
    perm = rng.permutation(70)
    s2, i2 = oracle.custom_reduce(A, B[perm], wp, wm)
    assert np.array_equal(s, s2)
    # the winner under the permutation scores the same as the original winner, and the
    # original index is the smallest among all records with that score
    scores = ((A[:, None, :] == B[None, :, :]) * (wp - wm) + wm).sum(-1)
    assert np.array_equal(scores.max(1), s)
    assert np.array_equal(scores.argmax(1), i)  # numpy's argmax returns the first maximum
    assert np.array_equal(scores[np.arange(25), perm[i2]], s)


# --------------------------------------------------------------------------- Dot / MatVec


def test_dot_and_matvec_bruteforce_vs_generic():
    x, y = _small_ints((7,)), _small_ints((7,))
    d, dabs = oracle.dot(x, y)
    assert d == G.dot([int(v) for v in x], [int(v) for v in y])
    assert dabs == float(np.abs(x.astype(np.float64) * y).sum())
    A = _small_ints((4, 7))
    got, gabs = oracle.matvec(A, x, with_abs=True)
    assert got.tolist() == G.matvec([[int(v) for v in r] for r in A], [int(v) for v in x])
    assert np.array_equal(gabs, np.abs(A.astype(np.float64)) @ np.abs(x.astype(np.float64)))


def test_dot_and_matvec_closed_forms_and_reductions_to_matmul():
    K = 1000
    ones = np.ones(K, np.float32)
    assert oracle.dot(ones, ones)[0] == K
    ramp = np.arange(K, dtype=np.float32)
    assert oracle.dot(ramp, ones)[0] == K * (K - 1) / 2
    # a unit vector picks a column of A (fails if A is read transposed)
    A = rng.uniform(-1, 1, (9, 13)).astype(np.float32)
    e = np.zeros(13, np.float32)
    e[5] = 1
    assert np.array_equal(oracle.matvec(A, e), A[:, 5].astype(np.float64))
    # MatVec is MatMul with N = 1, Dot is MatVec with M = 1
    x = rng.uniform(-1, 1, 13).astype(np.float32)
    assert np.array_equal(oracle.matvec(A, x), oracle.matmul(A, x.reshape(13, 1)).ravel())
    assert oracle.dot(A[2], x)[0] == oracle.matvec(A[2:3], x)[0]
    assert np.allclose(oracle.matvec(A, x), A.astype(np.float64) @ x.astype(np.float64), rtol=0, atol=1e-14)


def test_dot_and_matvec_split_property():
    A = rng.uniform(-1, 1, (6, 40)).astype(np.float32)
    x = rng.uniform(-1, 1, 40).astype(np.float32)
    whole = oracle.matvec(A, x)
    assert np.array_equal(np.concatenate([oracle.matvec(A[:2], x), oracle.matvec(A[2:], x)]), whole)
    parts = oracle.matvec(np.ascontiguousarray(A[:, :17]), x[:17]) + oracle.matvec(np.ascontiguousarray(A[:, 17:]), x[17:])
    assert np.allclose(parts, whole, rtol=0, atol=1e-14)
    d = oracle.dot(A[0], x)[0]
    assert abs(oracle.dot(A[0, :9], x[:9])[0] + oracle.dot(A[0, 9:], x[9:])[0] - d) <= 1e-14
