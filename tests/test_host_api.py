"""Host-side logic of libmdh (no GPU, no compute calls): the library loads, exports every
symbol include/mdh.h declares, and the planner enforces the paper's constraints."""
import ctypes
import os
import re

import pytest

import paper_2405_05118_amd as mdh
from paper_2405_05118_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

OK, E_NULL, E_SIZE, E_NOTDIV, E_RES, E_WS, E_UNSUP, E_LAUNCH, E_STATIC = range(9)

CASES = [
    (mdh.MDH_MATMUL, (256, 256, 256)),
    (mdh.MDH_MATMUL, (4096, 4096, 4096)),
    (mdh.MDH_MATMUL, (65536, 64, 4096)),
    (mdh.MDH_MATMUL, (300, 200, 100)),
    (mdh.MDH_STENCIL, (512, 512, 512)),
    (mdh.MDH_STENCIL, (37, 29, 70)),
    (mdh.MDH_MCC, (16, 224, 224, 128, 64, 7, 7, 1, 1)),
    (mdh.MDH_MCC, (2, 14, 14, 40, 12, 3, 3, 2, 2)),
    (mdh.MDH_CUSTOM_REDUCE, (1 << 16, 1 << 18, 8)),
    (mdh.MDH_CUSTOM_REDUCE, (1000, 3000, 5)),
]


def test_every_declared_symbol_is_exported():
    text = open(os.path.join(ROOT, "include", "mdh.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(mdh_[a-z_]+)\s*\(", text))
    assert declared, "no declarations found in the header"
    L = mdh.lib()
    for name in sorted(declared):
        assert hasattr(L, name), "libmdh.so does not export " + name
    assert declared == set(B.EXPORTS)


def test_struct_layout_matches_header():
    # 4 + 6*10*4 + 10*4 + 60 + 3 + 4 + 1 + 4 + 1 + 3 = 360
    assert ctypes.sizeof(mdh.TileParams) == 360
    assert mdh.mdh_version() == "0.1"
    assert "NULL" in mdh.mdh_strerror(E_NULL)


def test_part_offset_worked_example(golden):
    # Appendix Definition "MDA Partitioning" on the MatVec 512 x 4096 example
    for ln in golden("matvec_partitioning.txt"):
        if not ln:
            continue
        _, N, P = [t.strip() for t in ln.split(";")]
        N, P = int(N), [int(t) for t in P.split()]
        assert mdh.mdh_part_offset(N, P, [0] * len(P)) == (0, 1)
        assert mdh.mdh_part_offset(N, P, [x - 1 for x in P]) == (N - 1, 1)
    assert mdh.mdh_part_offset(512, [2, 8, 32], [1, 3, 5]) == (357, 1)
    assert mdh.mdh_part_offset(4096, [4, 16], [3, 15]) == (4032, 64)
    with pytest.raises(mdh.MdhError) as e:
        mdh.mdh_part_offset(10, [4], [0])
    assert e.value.status == E_NOTDIV
    with pytest.raises(mdh.MdhError) as e:
        mdh.mdh_part_offset(16, [4], [4])
    assert e.value.status == E_SIZE


def test_tvm_layering_is_expressible(golden):
    # a real schedule's part counts multiply to the sizes; our offset formula walks it
    for ln in golden("tvm_matmul_resnet50_layers.txt"):
        if not ln:
            continue
        _, N, P = [t.strip() for t in ln.split(";")]
        N, P = int(N), [int(t) for t in P.split()]
        assert mdh.mdh_part_offset(N, P, [x - 1 for x in P]) == (N - 1, 1)


@pytest.mark.parametrize("inst,sizes", CASES)
def test_default_params_satisfy_the_constraints(inst, sizes):
    p = mdh.mdh_default_params(inst, sizes)
    D = p.D
    assert D == {0: 3, 1: 3, 2: 7, 3: 2}[inst]
    for d in range(D):
        e = p.extent(d)
        if p.ragged:
            assert e >= sizes[d]
        else:
            assert e == sizes[d]  # algorithmic constraint of parameter 0
    lanes = 1
    for d in range(D):
        lanes *= p.prt[B.L_WAVE][d] * p.prt[B.L_LANE][d]
    assert lanes <= 1024  # model constraint: lanes per workgroup
    # the order is a permutation of all (layer, dim) pairs
    used = sorted(p.order[i] for i in range(6 * D))
    assert used == sorted(l * B.MDH_MAX_D + d for l in range(6) for d in range(D))
    assert mdh.mdh_validate_params(inst, sizes, p) == OK


@pytest.mark.parametrize("inst,sizes", CASES)
def test_all_candidates_are_valid(inst, sizes):
    n = mdh.mdh_num_candidates(inst, sizes)
    assert n >= 1
    first = mdh.mdh_candidate(inst, sizes, 0)
    default = mdh.mdh_default_params(inst, sizes)
    assert bytes(first) == bytes(default)
    for i in range(n):
        p = mdh.mdh_candidate(inst, sizes, i)
        assert mdh.mdh_validate_params(inst, sizes, p) == OK
    with pytest.raises(mdh.MdhError):
        mdh.mdh_candidate(inst, sizes, n)


def test_non_dividing_tiles_are_rejected():
    s = (4096, 4096, 4096)
    p = mdh.mdh_default_params(mdh.MDH_MATMUL, s)
    q = p.copy()
    q.prt[B.L_WG][0] += 1  # product no longer equals M
    assert mdh.mdh_validate_params(mdh.MDH_MATMUL, s, q) == E_NOTDIV
    q = p.copy()
    q.prt[B.L_HBM][2] //= 2  # covers only half of K
    assert mdh.mdh_validate_params(mdh.MDH_MATMUL, s, q) == E_NOTDIV
    q = p.copy()
    q.prt[B.L_LDS][2] = 0
    assert mdh.mdh_validate_params(mdh.MDH_MATMUL, s, q) == E_NOTDIV
    # ragged sizes need the explicit extension flag
    s2 = (300, 200, 100)
    r = mdh.mdh_default_params(mdh.MDH_MATMUL, s2)
    assert r.ragged == 1
    r.ragged = 0
    assert mdh.mdh_validate_params(mdh.MDH_MATMUL, s2, r) == E_NOTDIV


def test_resource_and_support_limits():
    s = (512, 512, 512)
    p = mdh.mdh_default_params(mdh.MDH_STENCIL, s)
    q = p.copy()
    q.prt[B.L_WAVE][1] = 16  # 16 lane-rows x 128 lanes = 2048 lanes per workgroup
    q.prt[B.L_WG][1] = 512 // (16 * q.prt[B.L_VGPR][1])
    assert mdh.mdh_validate_params(mdh.MDH_STENCIL, s, q) == E_RES
    q = p.copy()
    q.prt[B.L_VGPR][1] = 1  # valid partitioning, but no kernel keeps 1 row per lane
    q.prt[B.L_WG][1] = 512 // q.prt[B.L_WAVE][1]
    assert mdh.mdh_validate_params(mdh.MDH_STENCIL, s, q) == E_UNSUP
    q = p.copy()
    q.order[0], q.order[1] = q.order[1], q.order[0]  # another loop order
    assert mdh.mdh_validate_params(mdh.MDH_STENCIL, s, q) == E_UNSUP


def test_matmul_loop_order_of_the_workgroup_layer_is_a_choice():
    # parameter D1: (WG,i),(WG,j) = bands of tile rows (default), (WG,j),(WG,i) = bands of tile columns;
    # both run on the LDS-tiled kernel, every other permutation has no instantiation
    s = (4096, 4096, 4096)
    p = mdh.mdh_default_params(mdh.MDH_MATMUL, s)
    wg = B.L_WG * B.MDH_MAX_D
    assert list(p.order[:3]) == [wg + 0, wg + 1, wg + 2]
    q = p.copy()
    q.order[0], q.order[1] = wg + 1, wg + 0
    assert mdh.mdh_validate_params(mdh.MDH_MATMUL, s, q) == 0
    cands = [mdh.mdh_candidate(mdh.MDH_MATMUL, s, i) for i in range(mdh.mdh_num_candidates(mdh.MDH_MATMUL, s))]
    assert any(list(c.order[:3]) == [wg + 1, wg + 0, wg + 2] and c.table() == p.table() for c in cands)
    q = p.copy()
    q.order[0], q.order[2] = wg + 2, wg + 0  # k outermost
    assert mdh.mdh_validate_params(mdh.MDH_MATMUL, s, q) == E_UNSUP
    q = p.copy()
    q.order[3], q.order[4] = q.order[4], q.order[3]  # the memory layer: one order only
    assert mdh.mdh_validate_params(mdh.MDH_MATMUL, s, q) == E_UNSUP
    # a single row or column of tiles: nothing to choose, no such candidate
    s = (65536, 64, 4096)
    cands = [mdh.mdh_candidate(mdh.MDH_MATMUL, s, i) for i in range(mdh.mdh_num_candidates(mdh.MDH_MATMUL, s))]
    assert all(list(c.order[:2]) == [wg + 0, wg + 1] for c in cands)


def test_workspace_only_for_split_reductions():
    s = (65536, 64, 4096)
    for i in range(mdh.mdh_num_candidates(mdh.MDH_MATMUL, s)):
        p = mdh.mdh_candidate(mdh.MDH_MATMUL, s, i)
        S = p.prt[B.L_WG][2]
        want = S * s[0] * s[1] * 4 if S > 1 else 0
        assert mdh.mdh_workspace_size(mdh.MDH_MATMUL, s, p) == want
    assert mdh.mdh_workspace_size(mdh.MDH_STENCIL, (64, 64, 64)) == 0
    s = (1 << 16, 1 << 18, 8)
    p = mdh.mdh_default_params(mdh.MDH_CUSTOM_REDUCE, s)
    S = p.prt[B.L_WG][1]
    assert S > 1 and mdh.mdh_workspace_size(mdh.MDH_CUSTOM_REDUCE, s, p) == S * s[0] * 2 * 4


def test_size_errors_before_any_launch():
    L = mdh.lib()
    null = None
    # K = 0: the reduction dimension has no neutral element to return
    assert L.mdh_matmul(4, 4, 0, null, null, null, null, null, 0, null) == E_SIZE
    assert L.mdh_matmul(-1, 4, 4, null, null, null, null, null, 0, null) == E_SIZE
    assert L.mdh_matmul(4, 4, 4, null, null, null, null, null, 0, null) == E_NULL
    assert L.mdh_matmul(0, 4, 4, null, null, null, null, null, 0, null) == OK  # empty ++ dimension
    assert L.mdh_stencil(0, 8, 8, null, null, 0.5, 0.1, null, null) == OK
    assert L.mdh_stencil(8, 8, 8, null, null, 0.5, 0.1, null, null) == E_NULL
    assert L.mdh_stencil(2000, 2000, 2000, null, null, 0.5, 0.1, null, null) == E_SIZE
    assert L.mdh_custom_reduce(8, 0, 8, null, null, null, null, null, null, null, null, 0, null) == E_SIZE
    assert L.mdh_custom_reduce(8, 8, 17, null, null, null, null, null, null, null, null, 0, null) == E_SIZE
    assert L.mdh_custom_reduce(0, 8, 8, null, null, null, null, null, null, null, null, 0, null) == OK
    assert L.mdh_mcc(1, 6, 6, 4, 4, 7, 7, 1, 1, null, null, null, null, null, 0, null) == E_SIZE  # H < R
    assert L.mdh_mcc(1, 8, 8, 4, 4, 3, 3, 0, 1, null, null, null, null, null, 0, null) == E_SIZE  # stride 0
    assert L.mdh_mcc(0, 8, 8, 4, 4, 3, 3, 1, 1, null, null, null, null, null, 0, null) == OK
    # a split reduction without workspace is refused, nothing is launched
    s = (65536, 64, 4096)
    p = None
    for i in range(mdh.mdh_num_candidates(mdh.MDH_MATMUL, s)):
        c = mdh.mdh_candidate(mdh.MDH_MATMUL, s, i)
        if c.prt[B.L_WG][2] > 1:
            p = c
            break
    assert p is not None
    one = ctypes.c_void_p(16)  # non-NULL dummy addresses: the call must stop at the workspace check
    assert L.mdh_matmul(*s, one, one, one, ctypes.byref(p), null, 0, null) == E_WS


def test_size_errors_of_the_later_entry_points():
    L = mdh.lib()
    null = None
    one = ctypes.c_void_p(16)
    # Dot / MatVec: the reduction dimension may not be empty
    assert L.mdh_dot(0, null, null, null, null, null, 0, null) == E_SIZE
    assert L.mdh_dot(8, null, null, null, null, null, 0, null) == E_NULL
    assert L.mdh_matvec(4, 0, null, null, null, null, null, 0, null) == E_SIZE
    assert L.mdh_matvec(0, 4, null, null, null, null, null, 0, null) == OK
    # bMatMul: empty batch is an empty call, K = 0 and more than 65535 batch entries are size errors
    assert L.mdh_matmul_ex(0, 4, 4, 4, null, 0, null, 0, null, 0, null, null, 0, null) == OK
    assert L.mdh_matmul_ex(2, 4, 4, 0, null, 0, null, 0, null, 0, null, null, 0, null) == E_SIZE
    assert L.mdh_matmul_ex(70000, 4, 4, 4, null, 0, null, 0, null, 0, null, null, 0, null) == E_SIZE
    assert L.mdh_matmul_ex(2, 4, 4, 4, null, 0, null, 0, null, 0, null, null, 0, null) == E_NULL
    # small M splits the reduction: without workspace the call stops before any launch
    assert L.mdh_matmul_ex(1, 16, 1000, 2048, one, 0, one, 0, one, 0, null, null, 0, null) == E_WS
    # scan: empty rows / empty row length are empty calls; a chunked long row needs its workspace
    assert L.mdh_scan(0, 8, null, null, null, null, 0, null) == OK
    assert L.mdh_scan(8, 0, null, null, null, null, 0, null) == OK
    assert L.mdh_scan(-1, 8, null, null, null, null, 0, null) == E_SIZE
    assert L.mdh_scan(2, 8, null, null, null, null, 0, null) == E_NULL
    assert L.mdh_scan(1, 1 << 24, one, one, null, null, 0, null) == E_WS
    assert L.mdh_scan(1, 1 << 24, one, one, null, ctypes.c_void_p(20), 1 << 30, null) == E_WS  # misaligned workspace
    assert L.mdh_scan(1 << 20, 1 << 20, one, one, null, null, 0, null) == E_SIZE  # more than 2^31-1 elements
    flag = ctypes.c_int32(7)
    assert L.mdh_scan_timed_out(8, 4096, null, null, null, ctypes.byref(flag)) == OK and flag.value == 0  # no waits
    assert L.mdh_scan_timed_out(1, 1 << 24, null, null, null, ctypes.byref(flag)) == E_WS  # single pass: needs the workspace
    assert L.mdh_scan_timed_out(1, 1 << 24, null, null, null, null) == E_NULL
    # MCC_Capsule: as MCC, plus the LDS limit on the filter slice
    assert L.mdh_mcc_capsule(1, 6, 6, 3, 8, 7, 7, 1, 1, null, null, null, null, null) == E_SIZE  # H < R
    assert L.mdh_mcc_capsule(0, 8, 8, 3, 8, 3, 3, 1, 1, null, null, null, null, null) == OK
    assert L.mdh_mcc_capsule(1, 8, 8, 3, 8, 3, 3, 1, 1, null, null, null, null, null) == E_NULL
    assert L.mdh_mcc_capsule(1, 38, 38, 64, 8, 7, 7, 1, 1, one, one, one, null, null) == E_RES
    # the entry point without allocations: same checks, plus the limit of the static scratch array
    assert L.mdh_custom_reduce_static(8, 0, 8, one, one, one, one, one, one, null, null) == E_SIZE
    assert L.mdh_custom_reduce_static(0, 8, 8, null, null, null, null, null, null, null, null) == OK
    assert L.mdh_custom_reduce_static(8, 8, 8, null, one, one, one, one, one, null, null) == E_NULL
    assert L.mdh_custom_reduce_static((1 << 17) + 128, 1 << 18, 8, one, one, one, one, one, one, null, null) == E_STATIC  # S = 16
    assert L.mdh_static_scratch_bytes() == 16 << 20
    assert "static" in mdh.mdh_strerror(E_STATIC)
    # calibration kernels
    assert L.mdh_calib_copy(one, one, 24, null) == E_SIZE  # not a multiple of 16 bytes
    assert L.mdh_calib_copy(null, one, 32, null) == E_NULL
    assert L.mdh_calib_mfma(null, 8, null, null) == E_NULL
    assert L.mdh_calib_valu_kind(0, null, null, 8, null, null, null) == E_NULL
    assert L.mdh_calib_valu_kind(3, one, null, 8, null, null, null) == E_NULL  # the mix needs its weights
    assert L.mdh_calib_valu_kind(0, one, null, 0, null, null, null) == E_SIZE
    # generic path: description limits
    d = mdh.custom_desc((8,), (1,), ["float"], [(0, "i0")], "float", 4, "r = a0;", "r = x + y;")
    d.D = 0
    assert L.mdh_custom_default_params(ctypes.byref(d), ctypes.byref(mdh.TileParams())) == E_SIZE
    d.D = 1
    d.sizes[0] = 0  # an empty index set has no value under md_hom without a neutral element
    assert L.mdh_custom_default_params(ctypes.byref(d), ctypes.byref(mdh.TileParams())) == E_SIZE
    d.sizes[0] = 8
    d.acc_buf[0] = 3  # no such input buffer
    assert L.mdh_custom_default_params(ctypes.byref(d), ctypes.byref(mdh.TileParams())) == E_SIZE
    assert mdh.mdh_custom_workspace_size(mdh.CustomOp(None, "")) == 0


def test_mcc_defaults_and_candidates_validate_for_any_channel_count():
    # the reduction dimension c is split over workgroups in whole channel chunks: whatever the channel
    # count, no part of the default or of a candidate may be left without channels
    for C in list(range(9, 600, 13)) + [16, 32, 64, 128, 200, 256, 512, 1000, 2048]:
        for (N, P, Q, K) in ((2, 7, 7, 70), (1, 28, 28, 128), (16, 14, 14, 256), (3, 5, 9, 33)):
            sizes = (N, P, Q, K, C, 3, 3, 1, 1)
            p = mdh.mdh_default_params(mdh.MDH_MCC, sizes)
            assert mdh.mdh_validate_params(mdh.MDH_MCC, sizes, p) == 0, sizes
            S = p.prt[3][4]
            assert (mdh.mdh_workspace_size(mdh.MDH_MCC, sizes, p) == (S * N * P * Q * K * 4 if S > 1 else 0)), sizes
            for i in range(mdh.mdh_num_candidates(mdh.MDH_MCC, sizes)):
                assert mdh.mdh_validate_params(mdh.MDH_MCC, sizes, mdh.mdh_candidate(mdh.MDH_MCC, sizes, i)) == 0, (sizes, i)
    # a split that would leave a part empty is rejected: 200 channels in 8 parts of whole 16-channel chunks
    sizes = (2, 7, 7, 70, 200, 3, 3, 1, 1)
    p = mdh.mdh_default_params(mdh.MDH_MCC, sizes)
    assert p.prt[3][4] == 4
    q = p.copy()
    q.prt[3][4], q.prt[0][4] = 8, 2
    assert mdh.mdh_validate_params(mdh.MDH_MCC, sizes, q) == 3


def test_planner_over_a_seeded_sweep_of_sizes():
    # ~1300 seeded random shapes over every instance: the default configuration exists and validates, its
    # parts cover the sizes (exactly unless it says ragged), every candidate validates, and the workspace
    # size is defined for each of them.  Host only; the sizes are log-uniform so that tiny, ragged and
    # large extents all occur.
    import numpy as np

    rng = np.random.default_rng(20240511)

    def ri(lo, hi):
        return int(np.clip(np.exp(rng.uniform(np.log(lo), np.log(hi + 1))), lo, hi))

    def shapes():
        for _ in range(120):
            yield mdh.MDH_MATMUL, (ri(1, 5000), ri(1, 5000), ri(1, 9000)), None
            tr = [int(rng.integers(2)) for _ in range(3)]
            yield mdh.MDH_BMATMUL, (ri(1, 20), ri(1, 600), ri(1, 5000), ri(1, 30000), *tr), None
            yield mdh.MDH_BMATMUL, (ri(1, 4), ri(1, 16), ri(1, 9000), ri(1, 70000), 0, int(rng.integers(2)), 0), None
            yield mdh.MDH_STENCIL, (ri(1, 600), ri(1, 600), ri(1, 600)), None
            R, S = ri(1, 7), ri(1, 7)
            yield mdh.MDH_MCC, (ri(1, 32), ri(1, 120), ri(1, 120), ri(1, 300), ri(1, 600), R, S, ri(1, 3), ri(1, 3)), None
            yield mdh.MDH_MCC, (ri(1, 32), ri(1, 120), ri(1, 120), ri(1, 130), ri(1, 8), R, S, ri(1, 3), ri(1, 3)), None
            c = (ri(1, 16), ri(1, 60), ri(1, 60), ri(1, 70), ri(1, 4), R, S, ri(1, 2), ri(1, 2))
            yield mdh.MDH_MCC_CAPSULE, c, (c[0], c[1], c[2], c[3], 4, 4, c[4], c[5], c[6], 4)
            yield mdh.MDH_CUSTOM_REDUCE, (ri(1, 100000), ri(1, 300000), ri(1, 8)), None
            yield mdh.MDH_DOT, (ri(1, 1 << 28),), None
            yield mdh.MDH_MATVEC, (ri(1, 40000), ri(1, 40000)), None
            yield mdh.MDH_SCAN, (ri(1, 100000), ri(1, 1 << 20)), None

    n_checked = 0
    for inst, sizes, ext in shapes():
        try:
            p = mdh.mdh_default_params(inst, sizes)
        except mdh.MdhError as e:
            # the capsule kernel keeps its filter slice in LDS: large filters have no configuration
            assert inst == mdh.MDH_MCC_CAPSULE and e.status == E_RES, (inst, sizes, e.status)
            continue
        assert mdh.mdh_validate_params(inst, sizes, p) == OK, (inst, sizes)
        ext = ext or sizes
        for d in range(p.D):
            e = p.extent(d)
            assert (e >= ext[d]) if p.ragged else (e == ext[d]), (inst, sizes, d, e)
        for i in range(mdh.mdh_num_candidates(inst, sizes)):
            c = mdh.mdh_candidate(inst, sizes, i)
            assert mdh.mdh_validate_params(inst, sizes, c) == OK, (inst, sizes, i)
            assert mdh.mdh_workspace_size(inst, sizes, c) >= 0
        n_checked += 1
    assert n_checked > 1200
