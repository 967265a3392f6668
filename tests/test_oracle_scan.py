"""Pins of the prefix-sum combine operator and the scan oracles (Appendix, Example "Prefix-Sum";
Section "Examples", Subfigure 8)."""
import itertools
from fractions import Fraction

import numpy as np

import oracle
from oracle import instances as G
from oracle import mdhom as H


def test_operator_on_the_definition():
    # P = {0,1}, Q = {2,3}: the left part is unchanged (Q has no index <= i), the right part gets
    # the left part's value at max(P) = 1
    a1 = H.MDA([(0, 1)], {(0,): 10, (1,): 30})
    a2 = H.MDA([(2, 3)], {(2,): 5, (3,): 12})
    got = H.prefix_sum(0, lambda x, y: x + y)(a1, a2)
    assert got.index_sets == [(0, 1, 2, 3)] or tuple(got.index_sets) == ((0, 1, 2, 3),)
    assert [got[(i,)] for i in range(4)] == [10, 30, 35, 42]
    # interleaved index sets: every index takes the nearest index below it of the other operand
    a1 = H.MDA([(0, 2)], {(0,): 1, (2,): 4})  # scans over {0,2}
    a2 = H.MDA([(1, 3)], {(1,): 10, (3,): 110})  # scans over {1,3}
    got = H.prefix_sum(0, lambda x, y: x + y)(a1, a2)
    assert [got[(i,)] for i in range(4)] == [1, 11, 14, 114]
    # index set function is id (the dimension is kept), unlike point-wise combination
    assert H.prefix_sum(0, min).index_set_function((3, 1)) == (1, 3)


def test_scan_is_the_inclusive_prefix_sum():
    x = [3, -1, 4, 1, -5, 9, 2, -6]
    assert G.scan(lambda a, b: a + b, x) == list(itertools.accumulate(x))
    assert G.scan(max, x) == list(itertools.accumulate(x, max))
    # a non-commutative check would be invalid; exact rationals instead of floats
    xs = [Fraction(1, k + 1) for k in range(7)]
    assert G.scan(lambda a, b: a + b, xs) == list(itertools.accumulate(xs))
    X = [[1, 2, 3], [10, 20, 30]]
    assert G.scan_rows(lambda a, b: a + b, X) == [[1, 3, 6], [10, 30, 60]]


def test_homomorphic_property_of_scan():
    # scan(P ++ Q) = prefix-sum(scan(P), scan(Q)) for a split at any cut (Definition
    # "Multi-Dimensional Homomorphism")
    x = [2, 7, 1, 8, 2, 8, 1]
    add = lambda a, b: a + b
    whole = G.scan(add, x)
    for cut in range(1, len(x)):
        left = H.MDA([tuple(range(cut))], {(i,): v for i, v in enumerate(G.scan(add, x[:cut]))})
        right = H.MDA([tuple(range(cut, len(x)))], {(cut + i,): v for i, v in enumerate(G.scan(add, x[cut:]))})
        both = H.prefix_sum(0, add)(left, right)
        assert [both[(i,)] for i in range(len(x))] == whole


def test_bottom_box_sums():
    X = [[1, 2], [3, 4], [5, 6]]
    # bottom row, bottom two rows, all rows
    assert G.bottom_box_sums(X) == [11, 18, 21]
    assert max(G.bottom_box_sums([[5, -9], [-2, 1], [3, -1]])) == 2  # boxes: 2, 1, -3


def test_c_oracle_scan_rows():
    rng = np.random.default_rng(21)
    X = rng.integers(-5, 6, (4, 37)).astype(np.float32)
    got, gabs = oracle.scan_rows(X, with_abs=True)
    assert np.array_equal(got, np.cumsum(X.astype(np.float64), axis=1))  # small integers: exact
    assert np.array_equal(gabs, np.cumsum(np.abs(X.astype(np.float64)), axis=1))
    want = G.scan_rows(lambda a, b: a + b, X.astype(int).tolist())
    assert got.tolist() == want
    ones = np.ones((2, 1000), np.float32)
    assert np.array_equal(oracle.scan_rows(ones)[1], np.arange(1, 1001))
    Xf = rng.standard_normal((3, 5000)).astype(np.float32)
    assert np.allclose(oracle.scan_rows(Xf), np.cumsum(Xf.astype(np.float64), axis=1), rtol=0, atol=1e-9)
