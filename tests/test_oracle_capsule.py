"""Pins of the MCC_Capsule oracle (reading of the missing example table: MCC whose scalars are
MI x MK and MK x MJ matrices; Appendix "Data Characteristics used in Deep Neural Networks")."""
import numpy as np

import oracle
from oracle import instances as G


def rnd(shape, seed):
    return np.random.default_rng(seed).integers(-3, 4, shape).astype(np.float32)


def test_reduces_to_mcc_for_1x1_matrices():
    x, f = rnd((2, 9, 8, 3, 1, 1), 1), rnd((5, 3, 2, 3, 1, 1), 2)
    got = oracle.mcc_capsule(x, f, (2, 1))
    want = oracle.mcc(x[..., 0, 0], f[..., 0, 0], (2, 1))
    assert np.array_equal(got[..., 0, 0], want)


def test_single_tap_is_a_matrix_product():
    # N=P=Q=K=C=R=S=1: out = in (MI x MK) @ filt (MK x MJ)
    a, b = rnd((1, 1, 1, 1, 4, 4), 3), rnd((1, 1, 1, 1, 4, 4), 4)
    got = oracle.mcc_capsule(a, b)[0, 0, 0, 0]
    assert np.array_equal(got, a.reshape(4, 4).astype(np.float64) @ b.reshape(4, 4).astype(np.float64))
    # not symmetric in the two matrices: a transposed operand would be caught
    assert not np.array_equal(got, (b.reshape(4, 4).astype(np.float64) @ a.reshape(4, 4).astype(np.float64)))
    # rectangular matrices: MI=2, MK=3, MJ=5
    a, b = rnd((1, 1, 1, 1, 2, 3), 5), rnd((1, 1, 1, 1, 3, 5), 6)
    assert np.array_equal(oracle.mcc_capsule(a, b)[0, 0, 0, 0], a.reshape(2, 3).astype(np.float64) @ b.reshape(3, 5))


def test_identity_filter_matrices_shift_and_copy():
    # filter = identity matrix at tap (r0,s0), channel c0 -> out[n,p,q,k] = in[n,p+r0,q+s0,c0] (a 4x4 block)
    x = rnd((1, 6, 7, 2, 4, 4), 7)
    f = np.zeros((1, 3, 3, 2, 4, 4), np.float32)
    f[0, 1, 2, 1] = np.eye(4)
    got = oracle.mcc_capsule(x, f)
    assert np.array_equal(got[0, :, :, 0], x[0, 1:5, 2:7, 1].astype(np.float64))


def test_all_ones_and_abs():
    x, f = np.ones((1, 5, 5, 3, 4, 4), np.float32), np.ones((2, 3, 3, 3, 4, 4), np.float32)
    got, gabs = oracle.mcc_capsule(x, f, with_abs=True)
    assert np.all(got == 3 * 3 * 3 * 4) and np.array_equal(got, gabs)
    xs, fs = rnd((1, 4, 4, 2, 4, 4), 8), rnd((2, 2, 2, 2, 4, 4), 9)
    _, gabs = oracle.mcc_capsule(xs, fs, with_abs=True)
    assert np.array_equal(gabs, oracle.mcc_capsule(np.abs(xs), np.abs(fs)))


def test_against_generic_evaluator_and_sampled_form():
    x, f = rnd((1, 4, 5, 2, 2, 3), 10), rnd((2, 2, 3, 2, 3, 2), 11)
    want = np.array(G.mcc_capsule(x.astype(int).tolist(), f.astype(int).tolist(), (2, 1)), dtype=np.float64)
    got = oracle.mcc_capsule(x, f, (2, 1))
    assert got.shape == want.shape == (1, 2, 3, 2, 2, 2) and np.array_equal(got, want)
    idx = np.array([[0, 1, 2, 1, 1, 0], [0, 0, 0, 0, 0, 1]], np.int64)
    at, _ = oracle.mcc_capsule_at(x, f, idx, (2, 1))
    assert np.array_equal(at, got[tuple(idx.T)])


def test_homomorphic_splits():
    x, f = rnd((2, 6, 6, 3, 4, 4), 12), rnd((3, 3, 3, 3, 4, 4), 13)
    whole = oracle.mcc_capsule(x, f)
    # ++ over k: concatenation of the halves; + over c: sum of the halves
    assert np.array_equal(np.concatenate([oracle.mcc_capsule(x, f[:1]), oracle.mcc_capsule(x, f[1:])], axis=3), whole)
    assert np.array_equal(oracle.mcc_capsule(x[:, :, :, :1], f[:, :, :, :1]) + oracle.mcc_capsule(x[:, :, :, 1:], f[:, :, :, 1:]), whole)
    # + over mk: split the inner matrix dimension
    assert np.array_equal(oracle.mcc_capsule(x[..., :1], f[..., :1, :]) + oracle.mcc_capsule(x[..., 1:], f[..., 1:, :]), whole)
