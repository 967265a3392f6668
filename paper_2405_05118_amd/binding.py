"""ctypes binding of libmdh.so: argument marshalling only.

Device buffers are torch tensors on ``cuda`` (ROCm); their ``data_ptr()`` and the
current torch stream's handle are what crosses the C ABI.  Every step of the
computation runs inside the library's kernels.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmdh.so")

MDH_MATMUL, MDH_STENCIL, MDH_MCC, MDH_CUSTOM_REDUCE, MDH_DOT, MDH_MATVEC, MDH_BMATMUL, MDH_SCAN, MDH_MCC_CAPSULE = 0, 1, 2, 3, 4, 5, 6, 7, 8
MDH_NUM_LAYERS, MDH_MAX_D = 6, 10
L_HBM, L_LDS, L_VGPR, L_WG, L_WAVE, L_LANE = range(6)
MR_HBM, MR_LDS, MR_VGPR = range(3)  # memory regions of in_region / out_region

EXPORTS = (
    "mdh_strerror", "mdh_version", "mdh_part_offset", "mdh_default_params", "mdh_validate_params",
    "mdh_workspace_size", "mdh_matmul", "mdh_stencil", "mdh_mcc", "mdh_custom_reduce", "mdh_tune",
    "mdh_num_candidates", "mdh_candidate", "mdh_last_launch_error", "mdh_dot", "mdh_matvec",
    "mdh_matmul_ex", "mdh_scan", "mdh_mcc_capsule", "mdh_calib_copy", "mdh_calib_read", "mdh_calib_mfma", "mdh_calib_valu",
    "mdh_custom_default_params", "mdh_custom_validate_params", "mdh_custom_num_candidates", "mdh_custom_candidate",
    "mdh_custom_create", "mdh_custom_source", "mdh_custom_workspace_size", "mdh_custom_run", "mdh_custom_destroy",
    "mdh_custom_tune", "mdh_calib_valu_kind", "mdh_calib_realtime_hz", "mdh_custom_reduce_static",
    "mdh_static_scratch_bytes", "mdh_scan_timed_out",
)
MDH_CUSTOM_MAX_IN, MDH_CUSTOM_MAX_ACC = 4, 8
MDH_CALIB_BLOCKS = 2048
MDH_CALIB_STREAM_LANES = 256 * 512
(MDH_CALIB_KIND_XOR_MAX, MDH_CALIB_KIND_CMP_SELECT, MDH_CALIB_KIND_ADD3, MDH_CALIB_KIND_PRL_MIX, MDH_CALIB_KIND_FMA_F32,
 MDH_CALIB_KIND_ADD_VGPR, MDH_CALIB_KIND_PRL_FAST_MIX) = range(7)
MDH_CALIB_MIX_WEIGHTS = 16 + 256 * 2 * 8


class TileParams(ctypes.Structure):
    """Mirror of ``mdh_tile_params`` (include/mdh.h)."""

    _fields_ = [
        ("D", ctypes.c_int32),
        ("prt", (ctypes.c_int32 * MDH_MAX_D) * MDH_NUM_LAYERS),
        ("blk", ctypes.c_int32 * MDH_MAX_D),
        ("order", ctypes.c_uint8 * (MDH_NUM_LAYERS * MDH_MAX_D)),
        ("strided", ctypes.c_uint8),
        ("lane_fast_dim", ctypes.c_uint8),
        ("ragged", ctypes.c_uint8),
        ("in_region", ctypes.c_uint8 * 4),
        ("out_region", ctypes.c_uint8),
        ("in_transposed", ctypes.c_uint8 * 4),
        ("out_transposed", ctypes.c_uint8),
        ("reserved", ctypes.c_uint8 * 3),
    ]

    def copy(self) -> "TileParams":
        c = TileParams()
        ctypes.memmove(ctypes.byref(c), ctypes.byref(self), ctypes.sizeof(TileParams))
        return c

    def extent(self, d: int) -> int:
        e = self.blk[d]
        for l in range(MDH_NUM_LAYERS):
            e *= self.prt[l][d]
        return e

    def table(self):
        return [[self.prt[l][d] for d in range(self.D)] for l in range(MDH_NUM_LAYERS)]


class MdhError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = "%s: %s (status %d)" % (where, mdh_strerror(status), status)
        if status == 7:
            msg += " [" + lib().mdh_last_launch_error().decode() + "]"
        super().__init__(msg)


_lib = None


def lib() -> ctypes.CDLL:
    """Load libmdh.so (built in-tree by ``build.py``).  No fallback: raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libmdh.so is not built: run `python -m paper_2405_05118_amd.build` "
                "(or __graft_entry__.build()); there is no CPU fallback"
            )
        # torch ships its own copy of the HIP runtime; it has to be the first one the process
        # loads so that libmdh.so binds to the runtime that owns torch's device memory and streams
        # (loaded the other way round, launches fail with "no ROCm-capable device")
        import torch  # noqa: F401

        L = ctypes.CDLL(LIB_PATH)
        i64, i32, vp, sz, f32 = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float
        pp = ctypes.POINTER(TileParams)
        p64 = ctypes.POINTER(i64)
        L.mdh_strerror.restype = ctypes.c_char_p
        L.mdh_strerror.argtypes = [ctypes.c_int]
        L.mdh_version.restype = ctypes.c_char_p
        L.mdh_last_launch_error.restype = ctypes.c_char_p
        L.mdh_part_offset.argtypes = [i64, i32, ctypes.POINTER(i32), ctypes.POINTER(i32), p64, p64]
        L.mdh_default_params.argtypes = [ctypes.c_int, p64, pp]
        L.mdh_validate_params.argtypes = [ctypes.c_int, p64, pp]
        L.mdh_workspace_size.restype = sz
        L.mdh_workspace_size.argtypes = [ctypes.c_int, p64, pp]
        L.mdh_matmul.argtypes = [i64, i64, i64, vp, vp, vp, pp, vp, sz, vp]
        L.mdh_stencil.argtypes = [i64, i64, i64, vp, vp, f32, f32, pp, vp]
        L.mdh_mcc.argtypes = [i64] * 9 + [vp, vp, vp, pp, vp, sz, vp]
        L.mdh_custom_reduce.argtypes = [i64, i64, i32, vp, vp, vp, vp, vp, vp, pp, vp, sz, vp]
        L.mdh_matmul_ex.argtypes = [i64, i64, i64, i64, vp, i32, vp, i32, vp, i32, pp, vp, sz, vp]
        L.mdh_custom_reduce_static.argtypes = [i64, i64, i32, vp, vp, vp, vp, vp, vp, pp, vp]
        L.mdh_static_scratch_bytes.restype = sz
        L.mdh_static_scratch_bytes.argtypes = []
        L.mdh_dot.argtypes = [i64, vp, vp, vp, pp, vp, sz, vp]
        L.mdh_scan.argtypes = [i64, i64, vp, vp, pp, vp, sz, vp]
        L.mdh_scan_timed_out.argtypes = [i64, i64, pp, vp, vp, ctypes.POINTER(i32)]
        L.mdh_mcc_capsule.argtypes = [i64] * 9 + [vp, vp, vp, pp, vp]
        L.mdh_matvec.argtypes = [i64, i64, vp, vp, vp, pp, vp, sz, vp]
        L.mdh_tune.argtypes = [ctypes.c_int, p64, ctypes.POINTER(vp), ctypes.POINTER(f32), vp, sz, vp, i32, pp,
                               ctypes.POINTER(f32)]
        dp = ctypes.POINTER(CustomDesc)
        L.mdh_custom_default_params.argtypes = [dp, pp]
        L.mdh_custom_validate_params.argtypes = [dp, pp]
        L.mdh_custom_num_candidates.restype = i32
        L.mdh_custom_num_candidates.argtypes = [dp]
        L.mdh_custom_candidate.argtypes = [dp, i32, pp]
        L.mdh_custom_create.argtypes = [dp, pp, ctypes.POINTER(vp), ctypes.c_char_p, sz]
        L.mdh_custom_source.restype = ctypes.c_char_p
        L.mdh_custom_source.argtypes = [vp]
        L.mdh_custom_workspace_size.restype = sz
        L.mdh_custom_workspace_size.argtypes = [vp]
        L.mdh_custom_run.argtypes = [vp, ctypes.POINTER(vp), vp, vp, sz, vp]
        L.mdh_custom_tune.argtypes = [dp, ctypes.POINTER(vp), vp, vp, sz, vp, i32, i32, pp, ctypes.POINTER(f32)]
        L.mdh_custom_destroy.restype = None
        L.mdh_custom_destroy.argtypes = [vp]
        L.mdh_calib_copy.argtypes = [vp, vp, i64, vp]
        L.mdh_calib_read.argtypes = [vp, i64, vp, vp]
        L.mdh_calib_mfma.argtypes = [vp, i32, p64, vp]
        L.mdh_calib_valu.argtypes = [vp, i32, p64, vp]
        L.mdh_calib_valu_kind.argtypes = [i32, vp, vp, i32, p64, vp, vp]
        L.mdh_calib_realtime_hz.restype = i64
        L.mdh_calib_realtime_hz.argtypes = []
        L.mdh_num_candidates.restype = i32
        L.mdh_num_candidates.argtypes = [ctypes.c_int, p64]
        L.mdh_candidate.argtypes = [ctypes.c_int, p64, i32, pp]
        _lib = L
    return _lib


def _sizes(sizes: Sequence[int]):
    return (ctypes.c_int64 * len(sizes))(*[int(s) for s in sizes])


def _pref(p: Optional[TileParams]):
    return ctypes.byref(p) if p is not None else None


def _check(st: int, where: str):
    if st != 0:
        raise MdhError(st, where)


_raw_stream = None


def _stream() -> int:
    """Handle of torch's current stream on the current device.  torch's C entry point for it is several
    times cheaper than building a torch.cuda.Stream object per call, which matters for kernels of a few
    microseconds; the portable form is the fallback."""
    global _raw_stream
    import torch

    if _raw_stream is None:
        f = getattr(torch._C, "_cuda_getCurrentRawStream", None)
        _raw_stream = f if f is not None else False
    if _raw_stream:
        return int(_raw_stream(torch.cuda.current_device()))
    return int(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype, name):
    import torch

    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError("%s must be a contiguous %s tensor on the GPU" % (name, dtype))
    return ctypes.c_void_p(t.data_ptr())


def _ws(ws):
    if ws is None:
        return None, 0
    return ctypes.c_void_p(ws.data_ptr()), ws.numel() * ws.element_size()


# ------------------------------------------------------------------ host-only helpers


def mdh_strerror(status: int) -> str:
    return lib().mdh_strerror(int(status)).decode()


def mdh_version() -> str:
    return lib().mdh_version().decode()


def mdh_part_offset(N: int, P: Sequence[int], p: Sequence[int]):
    L = len(P)
    os_, ps = ctypes.c_int64(), ctypes.c_int64()
    st = lib().mdh_part_offset(int(N), L, (ctypes.c_int32 * L)(*P), (ctypes.c_int32 * L)(*p), ctypes.byref(os_), ctypes.byref(ps))
    _check(st, "mdh_part_offset")
    return os_.value, ps.value


def mdh_default_params(inst: int, sizes: Sequence[int]) -> TileParams:
    p = TileParams()
    _check(lib().mdh_default_params(inst, _sizes(sizes), ctypes.byref(p)), "mdh_default_params")
    return p


def mdh_validate_params(inst: int, sizes: Sequence[int], p: TileParams) -> int:
    return int(lib().mdh_validate_params(inst, _sizes(sizes), ctypes.byref(p)))


def mdh_workspace_size(inst: int, sizes: Sequence[int], p: Optional[TileParams] = None) -> int:
    return int(lib().mdh_workspace_size(inst, _sizes(sizes), _pref(p)))


def mdh_num_candidates(inst: int, sizes: Sequence[int]) -> int:
    return int(lib().mdh_num_candidates(inst, _sizes(sizes)))


def mdh_candidate(inst: int, sizes: Sequence[int], idx: int) -> TileParams:
    p = TileParams()
    _check(lib().mdh_candidate(inst, _sizes(sizes), idx, ctypes.byref(p)), "mdh_candidate")
    return p


# ------------------------------------------------------------------ device entry points


def mdh_matmul(A, B, C, params: Optional[TileParams] = None, workspace=None):
    import torch

    M, K = A.shape
    K2, N = B.shape
    assert K == K2 and tuple(C.shape) == (M, N)
    wp, wb = _ws(workspace)
    st = lib().mdh_matmul(M, N, K, _dev(A, torch.float32, "A"), _dev(B, torch.float32, "B"), _dev(C, torch.float32, "C"),
                          _pref(params), wp, wb, ctypes.c_void_p(_stream()))
    _check(st, "mdh_matmul")
    return C


def mdh_stencil(x, out, c0: float, c1: float, params: Optional[TileParams] = None):
    import torch

    nx, ny, nz = (s - 2 for s in x.shape)
    assert tuple(out.shape) == (nx, ny, nz)
    st = lib().mdh_stencil(nx, ny, nz, _dev(x, torch.float32, "in"), _dev(out, torch.float32, "out"), float(c0), float(c1),
                           _pref(params), ctypes.c_void_p(_stream()))
    _check(st, "mdh_stencil")
    return out


def mdh_mcc(x, filt, out, stride=(1, 1), params: Optional[TileParams] = None, workspace=None):
    import torch

    N, H, W, C = x.shape
    K, R, S, C2 = filt.shape
    assert C == C2
    sh, sw = stride
    P, Q = (H - R) // sh + 1, (W - S) // sw + 1
    assert tuple(out.shape) == (N, P, Q, K)
    wp, wb = _ws(workspace)
    st = lib().mdh_mcc(N, H, W, C, K, R, S, sh, sw, _dev(x, torch.float32, "in"), _dev(filt, torch.float32, "filt"),
                       _dev(out, torch.float32, "out"), _pref(params), wp, wb, ctypes.c_void_p(_stream()))
    _check(st, "mdh_mcc")
    return out


def mdh_custom_reduce(A, B, w_agree, w_disagree, out_score, out_index, params: Optional[TileParams] = None,
                      workspace=None):
    import torch

    nA, nF = A.shape
    nB, nF2 = B.shape
    assert nF == nF2 == w_agree.numel() == w_disagree.numel()
    assert out_score.numel() == nA and out_index.numel() == nA
    i32 = torch.int32
    wp, wb = _ws(workspace)
    st = lib().mdh_custom_reduce(nA, nB, nF, _dev(A, i32, "A"), _dev(B, i32, "B"), _dev(w_agree, i32, "w_agree"),
                                 _dev(w_disagree, i32, "w_disagree"), _dev(out_score, i32, "out_score"),
                                 _dev(out_index, i32, "out_index"), _pref(params), wp, wb, ctypes.c_void_p(_stream()))
    _check(st, "mdh_custom_reduce")
    return out_score, out_index


def mdh_custom_reduce_static(A, B, w_agree, w_disagree, out_score, out_index, params: Optional[TileParams] = None):
    """mdh_custom_reduce without a workspace: split-reduction partial results go to the library's static array."""
    import torch

    nA, nF = A.shape
    nB, nF2 = B.shape
    assert nF == nF2 == w_agree.numel() == w_disagree.numel()
    assert out_score.numel() == nA and out_index.numel() == nA
    i32 = torch.int32
    st = lib().mdh_custom_reduce_static(nA, nB, nF, _dev(A, i32, "A"), _dev(B, i32, "B"), _dev(w_agree, i32, "w_agree"),
                                        _dev(w_disagree, i32, "w_disagree"), _dev(out_score, i32, "out_score"),
                                        _dev(out_index, i32, "out_index"), _pref(params), ctypes.c_void_p(_stream()))
    _check(st, "mdh_custom_reduce_static")
    return out_score, out_index


def mdh_static_scratch_bytes() -> int:
    return int(lib().mdh_static_scratch_bytes())


def mdh_matmul_ex(A, B, C, trans_a=False, trans_b=False, trans_c=False, params: Optional[TileParams] = None,
                  workspace=None):
    """A: (batch, M, K) or (batch, K, M) if trans_a; B: (batch, K, N) or (batch, N, K) if trans_b;
    C: (batch, M, N) or (batch, N, M) if trans_c."""
    import torch

    batch = A.shape[0]
    M, K = (A.shape[2], A.shape[1]) if trans_a else (A.shape[1], A.shape[2])
    N = B.shape[1] if trans_b else B.shape[2]
    assert B.shape[0] == batch and C.shape[0] == batch
    assert tuple(B.shape[1:]) == ((N, K) if trans_b else (K, N))
    assert tuple(C.shape[1:]) == ((N, M) if trans_c else (M, N))
    wp, wb = _ws(workspace)
    st = lib().mdh_matmul_ex(batch, M, N, K, _dev(A, torch.float32, "A"), int(trans_a), _dev(B, torch.float32, "B"),
                             int(trans_b), _dev(C, torch.float32, "C"), int(trans_c), _pref(params), wp, wb,
                             ctypes.c_void_p(_stream()))
    _check(st, "mdh_matmul_ex")
    return C


def mdh_dot(x, y, out, params: Optional[TileParams] = None, workspace=None):
    import torch

    K = x.numel()
    assert y.numel() == K and out.numel() == 1
    wp, wb = _ws(workspace)
    st = lib().mdh_dot(K, _dev(x, torch.float32, "x"), _dev(y, torch.float32, "y"), _dev(out, torch.float32, "out"),
                       _pref(params), wp, wb, ctypes.c_void_p(_stream()))
    _check(st, "mdh_dot")
    return out


def mdh_mcc_capsule(x, filt, out, stride=(1, 1), params: Optional[TileParams] = None):
    """x: (N,H,W,C,4,4), filt: (K,R,S,C,4,4), out: (N,P,Q,K,4,4)."""
    import torch

    N, H, W, C, MI, MK = x.shape
    K, R, S, C2, MK2, MJ = filt.shape
    assert (MI, MK, MJ, MK2) == (4, 4, 4, 4) and C == C2
    sh, sw = stride
    P, Q = (H - R) // sh + 1, (W - S) // sw + 1
    assert tuple(out.shape) == (N, P, Q, K, 4, 4)
    st = lib().mdh_mcc_capsule(N, H, W, C, K, R, S, sh, sw, _dev(x, torch.float32, "x"), _dev(filt, torch.float32, "filt"),
                               _dev(out, torch.float32, "out"), _pref(params), ctypes.c_void_p(_stream()))
    _check(st, "mdh_mcc_capsule")
    return out


def mdh_scan(x, out, params: Optional[TileParams] = None, workspace=None):
    """Row-wise inclusive prefix sums of the (R, n) matrix x (a vector counts as one row)."""
    import torch

    R, n = (1, x.numel()) if x.dim() == 1 else x.shape
    assert out.numel() == x.numel()
    wp, wb = _ws(workspace)
    st = lib().mdh_scan(R, n, _dev(x, torch.float32, "x"), _dev(out, torch.float32, "out"), _pref(params), wp, wb,
                        ctypes.c_void_p(_stream()))
    _check(st, "mdh_scan")
    return out


def mdh_scan_timed_out(x, params: Optional[TileParams] = None, workspace=None) -> bool:
    """After mdh_scan(x, ..., params, workspace): synchronises the stream and reports whether a bounded
    wait of the single-pass kernel expired (the output is then wrong and must be discarded)."""
    R, n = (1, x.numel()) if x.dim() == 1 else x.shape
    wp, _ = _ws(workspace)
    flag = ctypes.c_int32(0)
    _check(lib().mdh_scan_timed_out(R, n, _pref(params), wp, ctypes.c_void_p(_stream()), ctypes.byref(flag)),
           "mdh_scan_timed_out")
    return bool(flag.value)


def mdh_matvec(A, x, y, params: Optional[TileParams] = None, workspace=None):
    import torch

    M, K = A.shape
    assert x.numel() == K and y.numel() == M
    wp, wb = _ws(workspace)
    st = lib().mdh_matvec(M, K, _dev(A, torch.float32, "A"), _dev(x, torch.float32, "x"), _dev(y, torch.float32, "y"),
                          _pref(params), wp, wb, ctypes.c_void_p(_stream()))
    _check(st, "mdh_matvec")
    return y


class CustomDesc(ctypes.Structure):
    """Mirror of ``mdh_custom_desc`` (include/mdh.h)."""

    _fields_ = [
        ("D", ctypes.c_int32),
        ("sizes", ctypes.c_int64 * MDH_MAX_D),
        ("reduce", ctypes.c_uint8 * MDH_MAX_D),
        ("n_in", ctypes.c_int32),
        ("n_acc", ctypes.c_int32),
        ("acc_buf", ctypes.c_int32 * MDH_CUSTOM_MAX_ACC),
        ("out_elem_bytes", ctypes.c_int32),
        ("fast_dim", ctypes.c_int32),
        ("prelude", ctypes.c_char_p),
        ("in_type", ctypes.c_char_p * MDH_CUSTOM_MAX_IN),
        ("acc_index", ctypes.c_char_p * MDH_CUSTOM_MAX_ACC),
        ("out_type", ctypes.c_char_p),
        ("out_index", ctypes.c_char_p),
        ("f", ctypes.c_char_p),
        ("op", ctypes.c_char_p),
    ]


def custom_desc(sizes, reduce, in_types, accesses, out_type, out_elem_bytes, f, op=None, prelude=None,
                out_index=None, fast_dim=-1) -> CustomDesc:
    """Fill a ``mdh_custom_desc``: ``reduce[d]`` is 0 (++), 1 (pw(op)) or 2 (prefix-sum(op));
    ``accesses`` is a list of (input buffer number, index expression)."""
    d = CustomDesc()
    d.D = len(sizes)
    for i, (n, r) in enumerate(zip(sizes, reduce)):
        d.sizes[i] = int(n)
        d.reduce[i] = int(r)  # 0: ++, 1: pw(op), 2: prefix-sum(op)
    d.n_in, d.n_acc = len(in_types), len(accesses)
    for b, t in enumerate(in_types):
        d.in_type[b] = t.encode()
    for a, (buf, idx) in enumerate(accesses):
        d.acc_buf[a] = int(buf)
        d.acc_index[a] = idx.encode()
    d.out_type, d.out_elem_bytes, d.fast_dim = out_type.encode(), int(out_elem_bytes), int(fast_dim)
    d.f = f.encode()
    d.op = op.encode() if op is not None else None
    d.prelude = prelude.encode() if prelude is not None else None
    d.out_index = out_index.encode() if out_index is not None else None
    return d


def mdh_custom_default_params(desc: CustomDesc) -> TileParams:
    p = TileParams()
    _check(lib().mdh_custom_default_params(ctypes.byref(desc), ctypes.byref(p)), "mdh_custom_default_params")
    return p


def mdh_custom_validate_params(desc: CustomDesc, params: TileParams) -> int:
    return lib().mdh_custom_validate_params(ctypes.byref(desc), ctypes.byref(params))


def mdh_custom_num_candidates(desc: CustomDesc) -> int:
    return lib().mdh_custom_num_candidates(ctypes.byref(desc))


def mdh_custom_candidate(desc: CustomDesc, idx: int) -> TileParams:
    p = TileParams()
    _check(lib().mdh_custom_candidate(ctypes.byref(desc), idx, ctypes.byref(p)), "mdh_custom_candidate")
    return p


class CustomOp:
    """Handle of a compiled generic md_hom operation (``mdh_custom_op*``)."""

    def __init__(self, handle, log):
        self.handle, self.log = handle, log

    def __del__(self):
        if getattr(self, "handle", None):
            mdh_custom_destroy(self)


def mdh_custom_create(desc: CustomDesc, params: Optional[TileParams] = None) -> CustomOp:
    """Generate and compile (hipRTC, gfx950) the kernels of one description; needs no GPU."""
    h = ctypes.c_void_p()
    log = ctypes.create_string_buffer(16384)
    st = lib().mdh_custom_create(ctypes.byref(desc), _pref(params), ctypes.byref(h), log, len(log))
    if st != 0:
        raise MdhError(st, "mdh_custom_create: " + mdh_strerror(st) + "\n" + log.value.decode(errors="replace"))
    return CustomOp(h, log.value.decode(errors="replace"))


def mdh_custom_source(op: CustomOp) -> str:
    return lib().mdh_custom_source(op.handle).decode()


def mdh_custom_workspace_size(op: CustomOp) -> int:
    return lib().mdh_custom_workspace_size(op.handle)


def mdh_custom_run(op: CustomOp, inputs, output, workspace=None):
    n = len(inputs)
    ptrs = (ctypes.c_void_p * n)(*[ctypes.c_void_p(t.data_ptr()) for t in inputs])
    for t in list(inputs) + [output]:
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("device-resident contiguous tensors are required")
    wp, wb = _ws(workspace)
    st = lib().mdh_custom_run(op.handle, ptrs, ctypes.c_void_p(output.data_ptr()), wp, wb, ctypes.c_void_p(_stream()))
    _check(st, "mdh_custom_run")
    return output


def mdh_custom_tune(desc: CustomDesc, inputs, output, workspace=None, reps: int = 3, max_candidates: int = 0):
    """Compile and time the candidate configurations of desc; returns (best params, ms)."""
    n = len(inputs)
    ptrs = (ctypes.c_void_p * n)(*[ctypes.c_void_p(t.data_ptr()) for t in inputs])
    wp, wb = _ws(workspace)
    best, ms = TileParams(), ctypes.c_float()
    st = lib().mdh_custom_tune(ctypes.byref(desc), ptrs, ctypes.c_void_p(output.data_ptr()), wp, wb,
                               ctypes.c_void_p(_stream()), reps, max_candidates, ctypes.byref(best), ctypes.byref(ms))
    _check(st, "mdh_custom_tune")
    return best, ms.value


def mdh_custom_destroy(op: CustomOp):
    if op.handle:
        lib().mdh_custom_destroy(op.handle)
        op.handle = None


def mdh_calib_copy(src, dst):
    """Streaming device copy of src into dst (calibration of the HBM roofline)."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    _check(lib().mdh_calib_copy(ctypes.c_void_p(src.data_ptr()), ctypes.c_void_p(dst.data_ptr()), nbytes,
                                ctypes.c_void_p(_stream())), "mdh_calib_copy")


def mdh_calib_read(src, out):
    """Streaming read of src; out: MDH_CALIB_STREAM_LANES float32 partial sums."""
    import torch

    assert out.numel() >= MDH_CALIB_STREAM_LANES
    _check(lib().mdh_calib_read(ctypes.c_void_p(src.data_ptr()), src.numel() * src.element_size(),
                                _dev(out, torch.float32, "out"), ctypes.c_void_p(_stream())), "mdh_calib_read")


def mdh_calib_mfma(out, iters: int) -> int:
    """Register-resident FP32 MFMA loop; returns the floating-point operations of the launch."""
    import torch

    assert out.numel() >= MDH_CALIB_BLOCKS * 256
    n = ctypes.c_int64()
    _check(lib().mdh_calib_mfma(_dev(out, torch.float32, "out"), iters, ctypes.byref(n), ctypes.c_void_p(_stream())),
           "mdh_calib_mfma")
    return n.value


def mdh_calib_valu(out, iters: int) -> int:
    """Register-resident int32 VALU loop; returns lanes x operations of the launch."""
    import torch

    assert out.numel() >= MDH_CALIB_BLOCKS * 256
    n = ctypes.c_int64()
    _check(lib().mdh_calib_valu(_dev(out, torch.int32, "out"), iters, ctypes.byref(n), ctypes.c_void_p(_stream())),
           "mdh_calib_valu")
    return n.value


def mdh_calib_valu_kind(kind: int, out, iters: int, weights=None, clocks=None) -> int:
    """Register-resident loop of one VALU instruction kind (or the custom reduce's mix); returns lanes x
    VALU instructions of the launch.  `clocks` (2 x int64 on the GPU) receives shader-clock cycles and
    real-time ticks around the loop of workgroup 0."""
    import torch

    assert out.numel() >= MDH_CALIB_BLOCKS * 256
    assert weights is None or weights.numel() >= MDH_CALIB_MIX_WEIGHTS
    assert clocks is None or clocks.numel() >= 2
    n = ctypes.c_int64()
    st = lib().mdh_calib_valu_kind(int(kind), _dev(out, torch.int32, "out"),
                                   _dev(weights, torch.int32, "weights") if weights is not None else None, iters,
                                   ctypes.byref(n), _dev(clocks, torch.int64, "clocks") if clocks is not None else None,
                                   ctypes.c_void_p(_stream()))
    _check(st, "mdh_calib_valu_kind")
    return n.value


def mdh_calib_realtime_hz() -> int:
    return int(lib().mdh_calib_realtime_hz())


def mdh_tune(inst: int, sizes: Sequence[int], buffers, scalars=None, workspace=None, reps: int = 3):
    """Time every candidate configuration on the given device buffers; returns (best params, ms)."""
    n = len(buffers)
    bufs = (ctypes.c_void_p * n)(*[ctypes.c_void_p(b.data_ptr()) for b in buffers])
    sc = (ctypes.c_float * 2)(*scalars) if scalars is not None else None
    wp, wb = _ws(workspace)
    best, ms = TileParams(), ctypes.c_float()
    st = lib().mdh_tune(inst, _sizes(sizes), bufs, sc, wp, wb, ctypes.c_void_p(_stream()), reps, ctypes.byref(best),
                        ctypes.byref(ms))
    _check(st, "mdh_tune")
    return best, ms.value
