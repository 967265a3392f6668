"""Generic md_hom evaluator, straight from the definitions -- TEST INFRASTRUCTURE.

Only tests, the smoke check and the bench's cpu_baseline leg may import this
package; it shares no code with the HIP path and must stay obviously correct
rather than fast (pure Python, for tiny index spaces only).

What is modelled, each following the paper's definition of the same name:

* ``MDA``            -- Definition "Multi-Dimensional Array": a function from a
                        product of finite index sets to scalars.
* ``concat``         -- Example "Concatenation": combine operator ++ in dimension d,
                        index-set function id.
* ``pointwise``      -- Example "Point-Wise Combination": pw(op) in dimension d,
                        index-set function 0_f (the dimension collapses to {0}).
* ``md_hom``         -- Definition "Higher-Order Function md_hom": the iterated
                        combine  op_1_{i_1} ... op_D_{i_D} f(a[i_1..i_D]).
* ``inp_view``       -- Definition "Input View" via index functions.
* ``out_view``       -- Definition "Output View" via index functions.
* ``part_offset``    -- Appendix Definition "MDA Partitioning": offset/size of
                        a part of the uniform multi-layer partitioning.

Parity status: pinned by tests/test_oracle_generic.py against the values the
paper prints (the 3x3 ++ 3x2 example, the MDA example with its five parts, the
MatVec 512x4096 partitioning) and against hand-computable map / reduce /
double-reduction cases.
"""
from __future__ import annotations

import itertools
from typing import Callable, Dict, Sequence, Tuple

Index = Tuple[int, ...]


class MDA:
    """A D-dimensional array: index_sets[d] is the sorted tuple I_d, data maps every
    index tuple of I_1 x ... x I_D to a scalar."""

    def __init__(self, index_sets: Sequence[Sequence[int]], data: Dict[Index, object]):
        self.index_sets = tuple(tuple(sorted(s)) for s in index_sets)
        for s in self.index_sets:
            if len(set(s)) != len(s) or any(i < 0 for i in s):
                raise ValueError("index sets are finite sets of natural numbers")
        expect = set(itertools.product(*self.index_sets))
        if set(data.keys()) != expect:
            raise ValueError("an MDA is total on the product of its index sets")
        self.data = dict(data)

    @property
    def D(self) -> int:
        return len(self.index_sets)

    @property
    def size(self) -> Tuple[int, ...]:
        return tuple(len(s) for s in self.index_sets)

    def __getitem__(self, idx: Index):
        return self.data[tuple(idx)]

    def restrict(self, subsets: Sequence[Sequence[int]]) -> "MDA":
        """a|_{J_1 x ... x J_D} for J_d a subset of I_d."""
        for J, I in zip(subsets, self.index_sets):
            if not set(J) <= set(I):
                raise ValueError("restriction to a non-subset")
        keys = itertools.product(*[tuple(sorted(J)) for J in subsets])
        return MDA(subsets, {k: self.data[k] for k in keys})

    def __eq__(self, other) -> bool:
        return (
            isinstance(other, MDA)
            and self.index_sets == other.index_sets
            and self.data == other.data
        )

    @staticmethod
    def from_nested(rows, offsets: Sequence[int] | None = None) -> "MDA":
        """Build from nested lists (tuples are scalar values, e.g. pairs); index
        sets are [off_d, off_d + N_d)."""
        shape = []
        r = rows
        while isinstance(r, list):
            shape.append(len(r))
            r = r[0] if len(r) else None
        offsets = tuple(offsets) if offsets is not None else (0,) * len(shape)
        data = {}
        for idx in itertools.product(*[range(n) for n in shape]):
            v = rows
            for i in idx:
                v = v[i]
            data[tuple(i + o for i, o in zip(idx, offsets))] = v
        return MDA([range(o, o + n) for n, o in zip(shape, offsets)], data)


def _check_other_dims(a1: MDA, a2: MDA, d: int) -> None:
    if a1.D != a2.D:
        raise ValueError("combine operator: dimensionalities differ")
    for e in range(a1.D):
        if e != d and a1.index_sets[e] != a2.index_sets[e]:
            raise ValueError(
                "combine operator undefined: index sets must coincide in every "
                "dimension except the one combined"
            )


def concat(d: int) -> Callable[[MDA, MDA], MDA]:
    """++ in (0-based) dimension d; P and Q must be disjoint."""

    def op(a1: MDA, a2: MDA) -> MDA:
        _check_other_dims(a1, a2, d)
        P, Q = set(a1.index_sets[d]), set(a2.index_sets[d])
        if P & Q:
            raise ValueError("concatenation needs disjoint index sets")
        sets = list(a1.index_sets)
        sets[d] = tuple(sorted(P | Q))
        data = {}
        for idx in itertools.product(*sets):
            data[idx] = a1.data[idx] if idx[d] in P else a2.data[idx]
        return MDA(sets, data)

    op.index_set_function = lambda I: tuple(sorted(I))  # id
    op.is_concat = True
    return op


def pointwise(d: int, oplus: Callable) -> Callable[[MDA, MDA], MDA]:
    """pw(oplus) in dimension d: both operands have index set {0} in d."""

    def op(a1: MDA, a2: MDA) -> MDA:
        _check_other_dims(a1, a2, d)
        if a1.index_sets[d] != (0,) or a2.index_sets[d] != (0,):
            raise ValueError("point-wise combination operates on index set {0}")
        return MDA(a1.index_sets, {idx: oplus(a1.data[idx], a2.data[idx]) for idx in a1.data})

    op.index_set_function = lambda I: (0,)  # 0_f
    op.is_concat = False
    return op


def prefix_sum(d: int, oplus: Callable) -> Callable[[MDA, MDA], MDA]:
    """The prefix-sum combine operator in dimension d (Appendix, Example "Prefix-Sum"): index set
    function id; with P, Q the disjoint index sets of the operands in d,

        result[.., i, ..] = a1[.., i, ..]          (+) a2[.., max_{<=i}(Q), ..]   for i in P
        result[.., i, ..] = a1[.., max_{<=i}(P), ..] (+) a2[.., i, ..]            for i in Q

    where max_{<=i}(S) is the largest index of S not above i.  Reading of the case the paper leaves
    open: if S has no index <= i the term is absent and the other operand's value is taken alone
    (so that folding singletons in ascending order gives the inclusive scan)."""

    def below(S, i):
        c = [s for s in S if s <= i]
        return max(c) if c else None

    def op(a1: MDA, a2: MDA) -> MDA:
        _check_other_dims(a1, a2, d)
        P, Q = tuple(a1.index_sets[d]), tuple(a2.index_sets[d])
        if set(P) & set(Q):
            raise ValueError("prefix-sum needs disjoint index sets")
        sets = list(a1.index_sets)
        sets[d] = tuple(sorted(set(P) | set(Q)))
        data = {}
        for idx in itertools.product(*sets):
            i = idx[d]
            if i in P:
                j = below(Q, i)
                left = a1.data[idx]
                data[idx] = left if j is None else oplus(left, a2.data[idx[:d] + (j,) + idx[d + 1:]])
            else:
                j = below(P, i)
                right = a2.data[idx]
                data[idx] = right if j is None else oplus(a1.data[idx[:d] + (j,) + idx[d + 1:]], right)
        return MDA(sets, data)

    op.index_set_function = lambda I: tuple(sorted(I))  # id
    op.is_concat = False
    return op


def md_hom(f: Callable, ops: Sequence[Callable], use_mda_indices: bool = False):
    """md_hom(f, (op_1..op_D)): returns the function a -> op_1_{i_1 in I_1} ...
    op_D_{i_D in I_D} f_vec(a restricted to the single point (i_1..i_D)).

    With use_mda_indices the scalar function also receives the index tuple
    (the USE_MDA_INDICES variant)."""
    D = len(ops)

    def f_vec(a: MDA, point: Index) -> MDA:
        # singleton in, singleton out; output index sets are isf_d({i_d})
        out_sets = [ops[d].index_set_function((point[d],)) for d in range(D)]
        x = a.data[point]
        y = f(x, point) if use_mda_indices else f(x)
        (key,) = itertools.product(*out_sets)
        return MDA(out_sets, {key: y})

    def h(a: MDA) -> MDA:
        if a.D != D:
            raise ValueError("md_hom: dimensionality mismatch")
        if D == 0:
            raise ValueError("D = 0 is the scalar function itself")

        def level(d: int, prefix: Index) -> MDA:
            # op_d iterated over i_d in I_d (ascending), applied to the inner levels
            acc = None
            for i in a.index_sets[d]:
                part = f_vec(a, prefix + (i,)) if d == D - 1 else level(d + 1, prefix + (i,))
                acc = part if acc is None else ops[d](acc, part)
            if acc is None:
                raise ValueError("empty index set: the iterated combine has no value")
            return acc

        return level(0, ())

    return h


def inp_view(index_functions: Sequence[Sequence[Callable[..., Index]]]):
    """index_functions[b][a](i_1..i_D) -> index into BUF b.  Returns a function
    (bufs, index_sets) -> MDA whose element at (i_1..i_D) is the tuple
    (bufs[b][idx_{b,a}(i_1..i_D)])_{b,a}.  BUFs are dicts or nested lists."""

    def get(buf, idx: Index):
        v = buf
        for i in idx:
            v = v[i]
        return v

    def iv(bufs, index_sets) -> MDA:
        data = {}
        for point in itertools.product(*[tuple(sorted(s)) for s in index_sets]):
            data[point] = tuple(
                get(bufs[b], fn(*point)) for b, fns in enumerate(index_functions) for fn in fns
            )
        return MDA(index_sets, data)

    return iv


def buf_sizes(index_functions, index_sets):
    """BUF extents implied by the accesses: N^b_d = 1 + max over all accesses of the
    d-th component of idx_{b,a}(i_1..i_D)."""
    sizes = []
    for fns in index_functions:
        mx = None
        for point in itertools.product(*[tuple(sorted(s)) for s in index_sets]):
            for fn in fns:
                t = fn(*point)
                mx = list(t) if mx is None else [max(m, x) for m, x in zip(mx, t)]
        sizes.append(tuple(m + 1 for m in mx))
    return sizes


def out_view(index_functions: Sequence[Sequence[Callable[..., Index]]]):
    """index_functions[b][a](i_1..i_D) -> index into output BUF b, for the a-th
    component of the MDA's (tuple-valued) elements.  Returns mda -> list of dicts
    {buf index: value}; cells never written stay absent (the paper's bottom)."""

    def ov(mda: MDA):
        bufs = [dict() for _ in index_functions]
        comp = 0
        for b, fns in enumerate(index_functions):
            for fn in fns:
                for point, val in mda.data.items():
                    v = val[comp] if isinstance(val, tuple) else val
                    key = tuple(fn(*point))
                    if key in bufs[b] and bufs[b][key] != v:
                        raise ValueError("output view is not a function (conflicting writes)")
                    bufs[b][key] = v
                comp += 1
        return bufs

    return ov


def part_offset(N: int, P: Sequence[int], p: Sequence[int]) -> Tuple[int, int]:
    """(OS, PS) of part p = (p^1..p^L) of the uniform L-layer partitioning of an
    index set of N elements into P = (P^1..P^L) parts per layer:
    OS = sum_l p^l * N / (P^1*...*P^l),  PS = N / (P^1*...*P^L)."""
    prod = 1
    os_ = 0
    for Pl, pl in zip(P, p):
        if not 0 <= pl < Pl:
            raise ValueError("part index out of range")
        prod *= Pl
        if N % prod:
            raise ValueError("the product of part counts must divide N")
        os_ += pl * (N // prod)
    return os_, N // prod
