"""The four md_hom instances written in the paper's high-level form

        out_view( md_hom(f, (op_1..op_D)) ( inp_view(bufs) ) )

with the generic evaluator of ``mdhom.py`` -- TEST INFRASTRUCTURE.  Pure Python,
exact arithmetic where the inputs allow it (ints / Fractions), for index spaces
of a few hundred points.  These are the brute-force cross-check of the nested
loops in ``mdh_oracle.c``: same definition, evaluated through a different
mechanism (iterated combine operators on MDAs instead of loop nests).
"""
from __future__ import annotations

from . import mdhom as H


def _add(x, y):
    return x + y


def dot(x, y):
    """md_hom(*, (+)) over (k); output view (0)->() (a scalar)."""
    iv = H.inp_view([[lambda k: (k,)], [lambda k: (k,)]])
    h = H.md_hom(lambda t: t[0] * t[1], (H.pointwise(0, _add),))
    (o,) = H.out_view([[lambda k: ()]])(h(iv([x, y], [range(len(x))])))
    return o[()]


def matvec(A, x):
    """md_hom(*, (++,+)) over (i,k); views (i,k)->A[i,k], (i,k)->x[k]; (i,0)->y[i]."""
    M, K = len(A), len(x)
    iv = H.inp_view([[lambda i, k: (i, k)], [lambda i, k: (k,)]])
    h = H.md_hom(lambda t: t[0] * t[1], (H.concat(0), H.pointwise(1, _add)))
    (y,) = H.out_view([[lambda i, k: (i,)]])(h(iv([A, x], [range(M), range(K)])))
    return [y[(i,)] for i in range(M)]


def matmul(A, B):
    """md_hom(*, (++,++,+)); views (i,j,k)->A[i,k], (i,j,k)->B[k,j]; (i,j,0)->C[i,j]
    (Section "Examples", Subfigure 1).  A, B nested lists; returns nested list C."""
    M, K, N = len(A), len(A[0]), len(B[0])
    iv = H.inp_view([[lambda i, j, k: (i, k)], [lambda i, j, k: (k, j)]])
    h = H.md_hom(lambda ab: ab[0] * ab[1], (H.concat(0), H.concat(1), H.pointwise(2, _add)))
    ov = H.out_view([[lambda i, j, k: (i, j)]])
    (c,) = ov(h(iv([A, B], [range(M), range(N), range(K)])))
    return [[c[(i, j)] for j in range(N)] for i in range(M)]


def bmatmul_t(A, B, trans_a=False, trans_b=False, trans_c=False):
    """bMatMul = md_hom(*, (++,++,++,+)) over (b,i,j,k) with the transposed views of
    MatMul^T: (b,i,j,k)->A[b,k,i] if trans_a else A[b,i,k]; B[b,j,k] if trans_b else B[b,k,j];
    output (b,i,j,0)->C[b,j,i] if trans_c else C[b,i,j]  (Section "Examples", Subfigure 1,
    routines 4 and 5).  A, B nested lists with the batch as first index."""
    nb = len(A)
    M = len(A[0][0]) if trans_a else len(A[0])
    K = len(A[0]) if trans_a else len(A[0][0])
    N = len(B[0]) if trans_b else len(B[0][0])
    ia = (lambda b, i, j, k: (b, k, i)) if trans_a else (lambda b, i, j, k: (b, i, k))
    ib = (lambda b, i, j, k: (b, j, k)) if trans_b else (lambda b, i, j, k: (b, k, j))
    ic = (lambda b, i, j, k: (b, j, i)) if trans_c else (lambda b, i, j, k: (b, i, j))
    iv = H.inp_view([[ia], [ib]])
    h = H.md_hom(lambda t: t[0] * t[1], (H.concat(0), H.concat(1), H.concat(2), H.pointwise(3, _add)))
    (c,) = H.out_view([[ic]])(h(iv([A, B], [range(nb), range(M), range(N), range(K)])))
    rows, cols = (N, M) if trans_c else (M, N)
    return [[[c[(b, r, q)] for q in range(cols)] for r in range(rows)] for b in range(nb)]


def jacobi3d(x, c0, c1):
    """md_hom(J_3D, (++,++,++)); the input view reads the one buffer seven times
    with offset index functions; output view (i,j,k)->(i,j,k)."""
    nx, ny, nz = len(x) - 2, len(x[0]) - 2, len(x[0][0]) - 2
    iv = H.inp_view(
        [
            [
                lambda i, j, k: (i + 1, j + 1, k + 1),
                lambda i, j, k: (i + 0, j + 1, k + 1),
                lambda i, j, k: (i + 2, j + 1, k + 1),
                lambda i, j, k: (i + 1, j + 0, k + 1),
                lambda i, j, k: (i + 1, j + 2, k + 1),
                lambda i, j, k: (i + 1, j + 1, k + 0),
                lambda i, j, k: (i + 1, j + 1, k + 2),
            ]
        ]
    )

    def J3D(t):
        return c0 * t[0] + c1 * (t[1] + t[2] + t[3] + t[4] + t[5] + t[6])

    h = H.md_hom(J3D, (H.concat(0), H.concat(1), H.concat(2)))
    ov = H.out_view([[lambda i, j, k: (i, j, k)]])
    (o,) = ov(h(iv([x], [range(nx), range(ny), range(nz)])))
    return [[[o[(i, j, k)] for k in range(nz)] for j in range(ny)] for i in range(nx)]


def mcc(x, filt, stride=(1, 1)):
    """7-dimensional md_hom(*, (++,++,++,++,+,+,+)) over (n,p,q,k,c,r,s); index
    functions p*sh+r and q*sw+s (Section "Examples", Subfigure 2)."""
    N, Hh, W, C = len(x), len(x[0]), len(x[0][0]), len(x[0][0][0])
    K, R, S = len(filt), len(filt[0]), len(filt[0][0])
    sh, sw = stride
    P, Q = (Hh - R) // sh + 1, (W - S) // sw + 1
    iv = H.inp_view(
        [
            [lambda n, p, q, k, c, r, s: (n, p * sh + r, q * sw + s, c)],
            [lambda n, p, q, k, c, r, s: (k, r, s, c)],
        ]
    )
    ops = (
        H.concat(0),
        H.concat(1),
        H.concat(2),
        H.concat(3),
        H.pointwise(4, _add),
        H.pointwise(5, _add),
        H.pointwise(6, _add),
    )
    h = H.md_hom(lambda t: t[0] * t[1], ops)
    ov = H.out_view([[lambda n, p, q, k, c, r, s: (n, p, q, k)]])
    (o,) = ov(h(iv([x, filt], [range(N), range(P), range(Q), range(K), range(C), range(R), range(S)])))
    return [[[[o[(n, p, q, k)] for k in range(K)] for q in range(Q)] for p in range(P)] for n in range(N)]


def max_idx(u, v):
    """The user-defined combine operator on (score, index) pairs."""
    (s1, b1), (s2, b2) = u, v
    if s1 > s2:
        return (s1, b1)
    if s2 > s1:
        return (s2, b2)
    return (s1, min(b1, b2))


def custom_reduce(A, B, w_agree, w_disagree):
    """md_hom(wght, (++, pw(max_idx))) over (a,b) with an index-carrying scalar
    function (USE_MDA_INDICES variant); output view writes the pair's two
    components to two buffers at (a)."""
    nA, nB, nF = len(A), len(B), len(w_agree)
    iv = H.inp_view([[lambda a, b: (a,)], [lambda a, b: (b,)]])

    def wght(t, point):
        ra, rb = t
        s = 0
        for f in range(nF):
            s += w_agree[f] if ra[f] == rb[f] else w_disagree[f]
        return (s, point[1])

    h = H.md_hom(wght, (H.concat(0), H.pointwise(1, max_idx)), use_mda_indices=True)
    ov = H.out_view([[lambda a, b: (a,)], [lambda a, b: (a,)]])
    sc, ix = ov(h(iv([A, B], [range(nA), range(nB)])))
    return [sc[(a,)] for a in range(nA)], [ix[(a,)] for a in range(nA)]


def histo(elems, bins):
    """Histo = md_hom(f_Histo, (++, +)) over (b, e): f_Histo(e, b) = 1 iff the element equals the
    bin value, else 0 (Section "Examples", Subfigures 4-6: the standard histogram as the instance
    of GenHisto with + and f_Histo); output view (b,0)->out[b]."""
    return gen_histo(elems, bins, lambda e, b: 1 if e == b else 0, _add)


def gen_histo(elems, bins, f, oplus):
    """GenHisto: user-defined scalar function f(element, bin) and associative, commutative
    operator oplus over the element dimension (same passage)."""
    nb, ne = len(bins), len(elems)
    iv = H.inp_view([[lambda b, e: (e,)], [lambda b, e: (b,)]])
    h = H.md_hom(lambda t: f(t[0], t[1]), (H.concat(0), H.pointwise(1, oplus)))
    (o,) = H.out_view([[lambda b, e: (b,)]])(h(iv([elems, bins], [range(nb), range(ne)])))
    return [o[(b,)] for b in range(nb)]


def jacobi1d(x, c):
    """Jacobi1D = md_hom(J_1D, (++)) over (i), J_1D = c * (v_i + v_{i+1} + v_{i+2}): the one
    buffer is read three times with index functions i, i+1, i+2 (Section "Introduction", running
    stencil example; Example on input views with several accesses); output (i)->(i), N-2 cells."""
    n = len(x) - 2
    iv = H.inp_view([[lambda i: (i,), lambda i: (i + 1,), lambda i: (i + 2,)]])
    h = H.md_hom(lambda t: c * (t[0] + t[1] + t[2]), (H.concat(0),))
    (o,) = H.out_view([[lambda i: (i,)]])(h(iv([x], [range(n)])))
    return [o[(i,)] for i in range(n)]


def map_f(f, x):
    """map(f) = md_hom(f, (++)) (Appendix example "map")."""
    iv = H.inp_view([[lambda i: (i,)]])
    h = H.md_hom(lambda t: f(t[0]), (H.concat(0),))
    (o,) = H.out_view([[lambda i: (i,)]])(h(iv([x], [range(len(x))])))
    return [o[(i,)] for i in range(len(x))]


def reduce_op(oplus, x):
    """reduce(oplus) = md_hom(id, (pw(oplus))) (Appendix example "reduce")."""
    iv = H.inp_view([[lambda i: (i,)]])
    h = H.md_hom(lambda t: t[0], (H.pointwise(0, oplus),))
    (o,) = H.out_view([[lambda i: ()]])(h(iv([x], [range(len(x))])))
    return o[()]


def scan(oplus, x):
    """scan(oplus) = md_hom(id, (prefix-sum(oplus))) over (i) (Section "Examples", Subfigure 8;
    Appendix, Example "Prefix-Sum"); output view (i)->(i)."""
    iv = H.inp_view([[lambda i: (i,)]])
    h = H.md_hom(lambda t: t[0], (H.prefix_sum(0, oplus),))
    (o,) = H.out_view([[lambda i: (i,)]])(h(iv([x], [range(len(x))])))
    return [o[(i,)] for i in range(len(x))]


def scan_rows(oplus, X):
    """Row-wise scan: md_hom(id, (++, prefix-sum(oplus))) over (i, j)."""
    R, n = len(X), len(X[0])
    iv = H.inp_view([[lambda i, j: (i, j)]])
    h = H.md_hom(lambda t: t[0], (H.concat(0), H.prefix_sum(1, oplus)))
    (o,) = H.out_view([[lambda i, j: (i, j)]])(h(iv([X], [range(R), range(n)])))
    return [[o[(i, j)] for j in range(n)] for i in range(R)]


def bottom_box_sums(X):
    """The md_hom of MBBS: md_hom(id, (prefix-sum(+), +)) over (i, j) with the input view reading
    the rows bottom-up, (i,j)->X[R-1-i, j]: element i is the sum of the bottom i+1 rows (all
    columns).  Two different operators on the two dimensions (Section "Experimental Results": the
    remark on several reduction dimensions with different combine operators).  The maximum over i
    that gives the Maximum Bottom Box Sum itself is a reduce(max) on this result.
    Reading of the missing figure -- parity unpinned against the paper."""
    R, C = len(X), len(X[0])
    iv = H.inp_view([[lambda i, j: (R - 1 - i, j)]])
    h = H.md_hom(lambda t: t[0], (H.prefix_sum(0, _add), H.pointwise(1, _add)))
    (o,) = H.out_view([[lambda i, j: (i,)]])(h(iv([X], [range(R), range(C)])))
    return [o[(i,)] for i in range(R)]


def mcc_capsule(x, filt, stride=(1, 1)):
    """MCC_Capsule as a 10-dimensional md_hom(*, (++ x6, + x4)) over (n,p,q,k,mi,mj,c,r,s,mk) with
    views in[n,p*sh+r,q*sw+s,c,mi,mk] and filt[k,r,s,c,mk,mj] (Section "Examples", Subfigure 2;
    reading of the missing figure: MCC on MI x MK / MK x MJ matrices)."""
    N, Hh, W, C, MI, MK = len(x), len(x[0]), len(x[0][0]), len(x[0][0][0]), len(x[0][0][0][0]), len(x[0][0][0][0][0])
    K, R, S, MJ = len(filt), len(filt[0]), len(filt[0][0]), len(filt[0][0][0][0][0])
    sh, sw = stride
    P, Q = (Hh - R) // sh + 1, (W - S) // sw + 1
    iv = H.inp_view(
        [
            [lambda n, p, q, k, mi, mj, c, r, s, mk: (n, p * sh + r, q * sw + s, c, mi, mk)],
            [lambda n, p, q, k, mi, mj, c, r, s, mk: (k, r, s, c, mk, mj)],
        ]
    )
    ops = tuple(H.concat(d) for d in range(6)) + tuple(H.pointwise(d, _add) for d in range(6, 10))
    h = H.md_hom(lambda t: t[0] * t[1], ops)
    ov = H.out_view([[lambda n, p, q, k, mi, mj, c, r, s, mk: (n, p, q, k, mi, mj)]])
    sets = [range(N), range(P), range(Q), range(K), range(MI), range(MJ), range(C), range(R), range(S), range(MK)]
    (o,) = ov(h(iv([x, filt], sets)))
    return [[[[[[o[(n, p, q, k, a, b)] for b in range(MJ)] for a in range(MI)] for k in range(K)] for q in range(Q)]
             for p in range(P)] for n in range(N)]
