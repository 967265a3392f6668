"""Seeded synthetic inputs for the five benchmark configurations.

This module holds NONE of the method's arithmetic: it only draws numbers.  It is
the one piece shared by the GPU path's tests/bench and the CPU oracle's tests,
so that both sides see identical arrays.

Generator: counter based.  Element `n` of tensor `tid` under `seed` is derived
from  splitmix64(seed ^ (tid << 56) + n)  (the public-domain SplitMix64 output
function), so any slice can be generated independently and in any order.
    uniform[lo,hi):  lo + (hi-lo) * (x >> 11) * 2^-53, rounded to fp32
    normal(0,1):     Box-Muller on the two draws 2n and 2n+1, rounded to fp32
    integer[lo,hi]:  lo + x mod (hi-lo+1)
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Tuple

import numpy as np

_CHUNK = 1 << 22
_U = np.uint64


def _splitmix64(x: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        z = x + _U(0x9E3779B97F4A7C15)
        z = (z ^ (z >> _U(30))) * _U(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> _U(27))) * _U(0x94D049BB133111EB)
        return z ^ (z >> _U(31))


def _draw(seed: int, tid: int, start: int, count: int, stride: int = 1, phase: int = 0) -> np.ndarray:
    base = _U((seed ^ (tid << 56)) & 0xFFFFFFFFFFFFFFFF)
    n = np.arange(start, start + count, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _splitmix64(base + n * _U(stride) + _U(phase))


def _unit(x: np.ndarray) -> np.ndarray:
    return (x >> _U(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def uniform(seed: int, tid: int, shape, lo: float, hi: float) -> np.ndarray:
    total = int(np.prod(shape))
    out = np.empty(total, dtype=np.float32)
    for s in range(0, total, _CHUNK):
        c = min(_CHUNK, total - s)
        out[s : s + c] = (lo + (hi - lo) * _unit(_draw(seed, tid, s, c))).astype(np.float32)
    return out.reshape(shape)


def normal(seed: int, tid: int, shape) -> np.ndarray:
    total = int(np.prod(shape))
    out = np.empty(total, dtype=np.float32)
    for s in range(0, total, _CHUNK):
        c = min(_CHUNK, total - s)
        u1 = 1.0 - _unit(_draw(seed, tid, s, c, stride=2, phase=0))  # (0,1]
        u2 = _unit(_draw(seed, tid, s, c, stride=2, phase=1))
        out[s : s + c] = (np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)).astype(np.float32)
    return out.reshape(shape)


def integers(seed: int, tid: int, shape, lo: int, hi: int) -> np.ndarray:
    total = int(np.prod(shape))
    out = np.empty(total, dtype=np.int32)
    span = _U(hi - lo + 1)
    for s in range(0, total, _CHUNK):
        c = min(_CHUNK, total - s)
        out[s : s + c] = (_draw(seed, tid, s, c) % span).astype(np.int64) + lo
    return out.reshape(shape)


# ---------------------------------------------------------------------------
# The benchmark configurations (sizes, distributions, seeds)
# ---------------------------------------------------------------------------

SEED_BASE = 0x5EED0000

#: alphabet size of each of the 8 record fields of the custom-reduce workload
PRL_ALPHABETS = (4, 16, 64, 128, 256, 512, 1024, 1024)
PRL_WEIGHT_MAX = 1 << 16


@dataclass(frozen=True)
class MatmulCfg:
    M: int
    N: int
    K: int
    seed: int


@dataclass(frozen=True)
class BMatmulCfg:
    batch: int
    M: int
    N: int
    K: int
    trans: Tuple[int, int, int]  # views of A, B, C transposed
    seed: int


@dataclass(frozen=True)
class StencilCfg:
    nx: int
    ny: int
    nz: int
    c0: float
    c1: float
    seed: int


@dataclass(frozen=True)
class MccCfg:
    N: int
    H: int
    W: int
    C: int
    K: int
    R: int
    S: int
    stride: Tuple[int, int]
    seed: int


@dataclass(frozen=True)
class PrlCfg:
    nA: int
    nB: int
    nF: int
    seed: int


CONFIGS: Dict[str, object] = {
    "matmul_256": MatmulCfg(256, 256, 256, SEED_BASE + 1),
    "jacobi3d_512": StencilCfg(512, 512, 512, 0.5, float(np.float32(1.0 / 12.0)), SEED_BASE + 2),
    "matmul_4096": MatmulCfg(4096, 4096, 4096, SEED_BASE + 3),
    "matmul_ts": MatmulCfg(65536, 64, 4096, SEED_BASE + 4),
    "mcc_resnet": MccCfg(16, 230, 230, 64, 128, 7, 7, (1, 1), SEED_BASE + 5),
    "prl_2p16_2p18": PrlCfg(1 << 16, 1 << 18, 8, SEED_BASE + 6),
    # shapes of the paper's deep-learning study (Appendix "Data Characteristics used in Deep Neural
    # Networks"): first convolution of ResNet-50 (training, N = 16) and the small-M MatMuls
    "mcc_resnet50_first": MccCfg(16, 230, 230, 3, 64, 7, 7, (2, 2), SEED_BASE + 9),
    "matmul_resnet50_fc": MatmulCfg(16, 1000, 2048, SEED_BASE + 10),
    "matmul_vgg16_fc": MatmulCfg(16, 4096, 25088, SEED_BASE + 11),
    # bMatMul and MatMul^T of the paper's example table (Section "Examples"), at sizes that fill the chip
    "bmatmul_16x1024": BMatmulCfg(16, 1024, 1024, 1024, (0, 0, 0), SEED_BASE + 16),
    "matmul_t_4096": BMatmulCfg(1, 4096, 4096, 4096, (1, 1, 1), SEED_BASE + 17),
}


def matmul_inputs(cfg: MatmulCfg):
    """A (M x K), B (K x N): i.i.d. uniform[-1,1), fp32."""
    return (
        uniform(cfg.seed, 1, (cfg.M, cfg.K), -1.0, 1.0),
        uniform(cfg.seed, 2, (cfg.K, cfg.N), -1.0, 1.0),
    )


def bmatmul_inputs(cfg: BMatmulCfg):
    """A and B as the (possibly transposed) views store them: A[b,k,i] / B[b,j,k] when transposed."""
    ta, tb, _ = cfg.trans
    a = uniform(cfg.seed, 1, (cfg.batch, cfg.K, cfg.M) if ta else (cfg.batch, cfg.M, cfg.K), -1.0, 1.0)
    b = uniform(cfg.seed, 2, (cfg.batch, cfg.N, cfg.K) if tb else (cfg.batch, cfg.K, cfg.N), -1.0, 1.0)
    return a, b


def stencil_inputs(cfg: StencilCfg):
    """Haloed grid (nx+2, ny+2, nz+2): uniform[0,1), fp32."""
    return uniform(cfg.seed, 1, (cfg.nx + 2, cfg.ny + 2, cfg.nz + 2), 0.0, 1.0)


def mcc_inputs(cfg: MccCfg):
    """Input NHWC and filter KRSC: N(0,1), fp32."""
    return (
        normal(cfg.seed, 1, (cfg.N, cfg.H, cfg.W, cfg.C)),
        normal(cfg.seed, 2, (cfg.K, cfg.R, cfg.S, cfg.C)),
    )


def prl_alphabets(nF: int):
    return tuple(PRL_ALPHABETS[f % len(PRL_ALPHABETS)] for f in range(nF))


def prl_inputs(cfg: PrlCfg):
    """Record tables A (nA x nF), B (nB x nF): field f uniform in [0, alphabet_f);
    agree weights in [1, 2^16], disagree weights in [-2^16, 0]; all int32."""
    alph = prl_alphabets(cfg.nF)
    A = np.empty((cfg.nA, cfg.nF), dtype=np.int32)
    B = np.empty((cfg.nB, cfg.nF), dtype=np.int32)
    for f, a in enumerate(alph):
        A[:, f] = integers(cfg.seed, 1 + 2 * f, (cfg.nA,), 0, a - 1)
        B[:, f] = integers(cfg.seed, 2 + 2 * f, (cfg.nB,), 0, a - 1)
    w_agree = integers(cfg.seed, 40, (cfg.nF,), 1, PRL_WEIGHT_MAX)
    w_disagree = integers(cfg.seed, 41, (cfg.nF,), -PRL_WEIGHT_MAX, 0)
    return A, B, w_agree, w_disagree


# ---------------------------------------------------------------------------
# The same generator on the GPU (torch integer ops), for filling large benchmark
# buffers without a long host loop.  uniform and integers reproduce the numpy
# versions bit for bit (integer arithmetic mod 2^64, then exactly rounded fp64
# multiply/add); normal may differ in the last place (device log/cos/sqrt).
# ---------------------------------------------------------------------------


def _s64(c: int) -> int:
    c &= 0xFFFFFFFFFFFFFFFF
    return c - (1 << 64) if c >= (1 << 63) else c


def _lsr(x, k: int):
    return (x >> k) & ((1 << (64 - k)) - 1)


def _splitmix64_t(x):
    z = x + _s64(0x9E3779B97F4A7C15)
    z = (z ^ _lsr(z, 30)) * _s64(0xBF58476D1CE4E5B9)
    z = (z ^ _lsr(z, 27)) * _s64(0x94D049BB133111EB)
    return z ^ _lsr(z, 31)


def _draw_t(seed, tid, start, count, device, stride=1, phase=0):
    import torch

    base = _s64(seed ^ (tid << 56))
    n = torch.arange(start, start + count, dtype=torch.int64, device=device)
    return _splitmix64_t(n * stride + (base + phase))


def _unit_t(x):
    import torch

    return _lsr(x, 11).to(torch.float64) * (1.0 / 9007199254740992.0)


def device_uniform(seed: int, tid: int, shape, lo: float, hi: float, device="cuda"):
    import torch

    total = int(np.prod(shape))
    out = torch.empty(total, dtype=torch.float32, device=device)
    step = 1 << 24
    for s in range(0, total, step):
        c = min(step, total - s)
        out[s : s + c] = (lo + (hi - lo) * _unit_t(_draw_t(seed, tid, s, c, device))).to(torch.float32)
    return out.reshape(shape)


def device_normal(seed: int, tid: int, shape, device="cuda"):
    import math

    import torch

    total = int(np.prod(shape))
    out = torch.empty(total, dtype=torch.float32, device=device)
    step = 1 << 24
    for s in range(0, total, step):
        c = min(step, total - s)
        u1 = 1.0 - _unit_t(_draw_t(seed, tid, s, c, device, stride=2, phase=0))
        u2 = _unit_t(_draw_t(seed, tid, s, c, device, stride=2, phase=1))
        out[s : s + c] = (torch.sqrt(-2.0 * torch.log(u1)) * torch.cos(2.0 * math.pi * u2)).to(torch.float32)
    return out.reshape(shape)


def device_integers(seed: int, tid: int, shape, lo: int, hi: int, device="cuda"):
    import torch

    total = int(np.prod(shape))
    span = hi - lo + 1
    x = _draw_t(seed, tid, 0, total, device)
    # unsigned x mod span from the signed representation: split off the top bit
    r = (_lsr(x, 1) % span * 2 + (x & 1)) % span
    return (r + lo).to(torch.int32).reshape(shape)
