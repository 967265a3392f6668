"""Pins for the generic md_hom evaluator (oracle/mdhom.py): values the paper
prints and hand-computable cases.  CPU only."""
from fractions import Fraction

import pytest

from oracle import mdhom as H


def _blocks(lines):
    out, cur = [], []
    for ln in lines:
        if ln == "":
            if cur:
                out.append(cur)
                cur = []
        else:
            cur.append([int(t) for t in ln.split()])
    if cur:
        out.append(cur)
    return out


def test_concat_worked_example(golden):
    # Section "Combine Operators": 3x3 ++ 3x2 in the second dimension = 3x5
    left, right, want = _blocks(golden("concat_3x3_3x2.txt"))
    a1 = H.MDA.from_nested(left)
    a2 = H.MDA.from_nested(right, offsets=(0, 3))
    got = H.concat(1)(a1, a2)
    assert got.size == (3, 5)
    assert got == H.MDA.from_nested(want)
    # the operands commute: ++ is defined through the index sets, not the order
    assert H.concat(1)(a2, a1) == got


def test_concat_undefined_case():
    # same passage: 3x3 ++ 2x2 matches in no dimension -> undefined
    a1 = H.MDA.from_nested([[1, 2, 3], [4, 5, 6], [7, 8, 9]])
    a2 = H.MDA.from_nested([[11, 12], [13, 14]], offsets=(0, 3))
    with pytest.raises(ValueError):
        H.concat(1)(a1, a2)
    with pytest.raises(ValueError):
        H.concat(0)(a1, a2)
    # overlapping index sets are not disjoint -> undefined as well
    with pytest.raises(ValueError):
        H.concat(1)(a1, a1)


def test_mda_example_parts(golden):
    # Section "Multi-Dimensional Arrays": a on {0,1}x{0,1,2,3} and its five parts
    a = H.MDA.from_nested([[10, 11, 12, 13], [20, 21, 22, 23]])
    parts = {}
    for ln in golden("mda_example_parts.txt"):
        if not ln:
            continue
        name, i1, i2 = [t.strip() for t in ln.split(";")]
        parts[name] = a.restrict([[int(t) for t in i1.split()], [int(t) for t in i2.split()]])
    assert H.concat(0)(parts["a11"], parts["a12"]) == a
    assert H.concat(1)(H.concat(1)(parts["a21"], parts["a22"]), parts["a23"]) == a
    assert parts["a22"].size == (2, 1) and parts["a11"].size == (1, 4)


def test_pointwise_collapses_dimension():
    # Example "Point-Wise Combination": index-set function 0_f, result lives on {0}
    a1 = H.MDA([[0, 1], [0]], {(0, 0): 3, (1, 0): 4})
    a2 = H.MDA([[0, 1], [0]], {(0, 0): 10, (1, 0): 20})
    r = H.pointwise(1, lambda x, y: x + y)(a1, a2)
    assert r.index_sets == ((0, 1), (0,))
    assert r.data == {(0, 0): 13, (1, 0): 24}
    bad = H.MDA([[0, 1], [5]], {(0, 5): 1, (1, 5): 2})
    with pytest.raises(ValueError):
        H.pointwise(1, lambda x, y: x + y)(a1, bad)


def test_map_is_all_concat():
    # Example "Function Mapping": map(f) = md_hom(f, (++,...,++)) keeps the index sets
    a = H.MDA.from_nested([[1, 2, 3], [4, 5, 6]])
    r = H.md_hom(lambda x: x * x, (H.concat(0), H.concat(1)))(a)
    assert r == H.MDA.from_nested([[1, 4, 9], [16, 25, 36]])


def test_reduce_is_all_pointwise():
    # Example "Reduction": red(+) = md_hom(id, (pw(+),...,pw(+))) -> singleton at (0,..,0)
    a = H.MDA.from_nested([[1, 2, 3], [4, 5, 6]])
    add = lambda x, y: x + y
    r = H.md_hom(lambda x: x, (H.pointwise(0, add), H.pointwise(1, add)))(a)
    assert r.index_sets == ((0,), (0,)) and r[(0, 0)] == 21
    # a non-commutative but associative operator exposes the iteration order (ascending)
    cat = lambda x, y: x + y
    s = H.MDA.from_nested(["a", "b", "c", "d"])
    assert H.md_hom(lambda x: x, (H.pointwise(0, cat),))(s)[(0,)] == "abcd"


def test_matvec_mixed_operators():
    # Figure "matrix-vector multiplication": md_hom(*, (++, +)) with views
    # (i,k)->M[i,k], (i,k)->v[k]; output view (i,0)->w[i]
    M = [[1, 2, 3], [4, 5, 6]]
    v = [7, 8, 9]
    iv = H.inp_view([[lambda i, k: (i, k)], [lambda i, k: (k,)]])
    h = H.md_hom(lambda t: t[0] * t[1], (H.concat(0), H.pointwise(1, lambda x, y: x + y)))
    (w,) = H.out_view([[lambda i, k: (i,)]])(h(iv([M, v], [range(2), range(3)])))
    assert w == {(0,): 50, (1,): 122}


def test_double_reduction_output_view():
    # Section "Output views", example Double Reduction: one pass, two operators, the
    # pair is written to two scalar buffers via index functions (0)->()
    vals = [2, 3, 4]
    iv = H.inp_view([[lambda i: (i,)]])
    op = lambda x, y: (x[0] + y[0], x[1] * y[1])
    h = H.md_hom(lambda t: (t[0], t[0]), (H.pointwise(0, op),))
    o1, o2 = H.out_view([[lambda i: ()], [lambda i: ()]])(h(iv([vals], [range(3)])))
    assert o1 == {(): 9} and o2 == {(): 24}


def test_jacobi1d_view_sizes():
    # Example "Input View -- Jacobi1D": a 512-vector gives an MDA of size 510, and the
    # buffer size rule N = 1 + max index recovers 512 from the accesses
    fns = [[lambda i: (i + 0,), lambda i: (i + 1,), lambda i: (i + 2,)]]
    assert H.buf_sizes(fns, [range(510)]) == [(512,)]
    v = list(range(512))
    a = H.inp_view(fns)([v], [range(510)])
    assert a.size == (510,) and a[(0,)] == (0, 1, 2) and a[(509,)] == (509, 510, 511)


def test_matmul_buf_sizes():
    fns = [[lambda i, j, k: (i, k)], [lambda i, j, k: (k, j)]]
    assert H.buf_sizes(fns, [range(3), range(5), range(4)]) == [(3, 4), (4, 5)]


def test_homomorphic_property_matvec():
    # Definition "Multi-Dimensional Homomorphism": h(a1 ++_d a2) = h(a1) op_d h(a2)
    add = lambda x, y: x + y
    ops = (H.concat(0), H.pointwise(1, add))
    h = H.md_hom(lambda t: t[0] * t[1], ops)
    a = H.MDA.from_nested([[(i + 1, k + 2) for k in range(4)] for i in range(3)])
    whole = h(a)
    for d, cut in ((0, 1), (0, 2), (1, 1), (1, 3)):
        lo = [range(3), range(4)]
        hi = [range(3), range(4)]
        lo[d] = range(0, cut)
        hi[d] = range(cut, a.size[d])
        assert ops[d](h(a.restrict(lo)), h(a.restrict(hi))) == whole


def test_operator_order_is_irrelevant_for_valid_mixes():
    # Lemma (well-definedness for mixes of ++ and pw(+)): permuting the nesting of the
    # iterated operators gives the same function.  Evaluate with dims swapped.
    add = lambda x, y: x + y
    f = lambda t: Fraction(t[0]) * t[1]
    a = H.MDA.from_nested([[(i + 1, 3 * k - i) for k in range(4)] for i in range(3)])
    r1 = H.md_hom(f, (H.concat(0), H.pointwise(1, add)))(a)
    at = H.MDA([a.index_sets[1], a.index_sets[0]], {(k, i): v for (i, k), v in a.data.items()})
    r2 = H.md_hom(f, (H.pointwise(0, add), H.concat(1)))(at)
    assert {(i, 0): v for (_, i), v in r2.data.items()} == r1.data


def test_partitioning_worked_example(golden):
    # Appendix Definition "MDA Partitioning" on the MatVec 512x4096 example
    rows = [ln for ln in golden("matvec_partitioning.txt") if ln]
    for ln in rows:
        _, N, P = [t.strip() for t in ln.split(";")]
        N, P = int(N), [int(t) for t in P.split()]
        prod = 1
        for x in P:
            prod *= x
        assert prod == N  # full partitioning: every part is a single element
        assert H.part_offset(N, P, [0] * len(P)) == (0, 1)
        assert H.part_offset(N, P, [x - 1 for x in P]) == (N - 1, 1)
    # dimension 1: part (1,3,5) starts at 1*256 + 3*32 + 5*1
    assert H.part_offset(512, [2, 8, 32], [1, 3, 5]) == (357, 1)
    # coarser: only the first two layers -> parts of 32 elements
    assert H.part_offset(512, [2, 8], [1, 3]) == (352, 32)
    # the parts of a partitioning tile the index set exactly once
    seen = []
    for p1 in range(2):
        for p2 in range(4):
            os_, ps = H.part_offset(64, [2, 4], [p1, p2])
            seen += list(range(os_, os_ + ps))
    assert seen == list(range(64))
    with pytest.raises(ValueError):
        H.part_offset(10, [4], [0])


def test_tvm_layers_multiply_to_sizes(golden):
    # the multi-layer partitioning of the ResNet-50 MatMul example is a full partitioning
    for ln in golden("tvm_matmul_resnet50_layers.txt"):
        if not ln:
            continue
        _, N, P = [t.strip() for t in ln.split(";")]
        prod = 1
        for x in P.split():
            prod *= int(x)
        assert prod == int(N)
