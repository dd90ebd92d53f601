"""Seeded synthetic inputs for the ternary x INT8 vector-LUT mpGeMM workloads.

This module only *generates* tensors (ternary weight matrices, fp32 activations,
the per-tensor weight scale).  It holds none of the method's arithmetic: no
quantiser, no packing, no table, no GEMM.  Both the CPU oracle's tests and the
GPU path's tests/bench feed from here so that they see the same bytes.

The generator is counter based: element i of stream s under seed z is a pure
function of (z, s, i), computed with the splitmix64 finaliser, so any slice of
any tensor can be regenerated independently and the result does not depend on
numpy's own random generators.

Shapes follow the real-model linear layers the paper benchmarks (its mpGeMM
kernel benchmark section uses BitNet-3B / Llama3-8B / Falcon3-1B GeMM shapes and
128..512-token prompts); the trained weights are replaced by iid ternary draws
with a stated zero probability because the kernel is exact and its run time does
not depend on the values.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

_U64 = np.uint64
_GOLDEN = _U64(0x9E3779B97F4A7C15)
_M1 = _U64(0xBF58476D1CE4E5B9)
_M2 = _U64(0x94D049BB133111EB)

# stream ids (one per tensor kind so tensors under one seed are independent)
STREAM_W = 1
STREAM_X = 2
STREAM_LATENT = 3
STREAM_OUTLIER = 4


def _mix(z: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser on a uint64 array (wrap-around arithmetic)."""
    z = (z ^ (z >> _U64(30))) * _M1
    z = (z ^ (z >> _U64(27))) * _M2
    return z ^ (z >> _U64(31))


def raw_u64(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """count 64-bit words for counters start .. start+count-1."""
    with np.errstate(over="ignore"):
        key = _mix(np.array([(seed * 0x10001 + stream * 0x9E3779B9 + 0x1234567) & (2**64 - 1)],
                            dtype=_U64))[0]
        ctr = np.arange(start, start + count, dtype=_U64)
        return _mix((ctr + _U64(1)) * _GOLDEN + key)


def uniform01(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """float64 uniforms in (0, 1): (top 53 bits + 0.5) / 2^53."""
    r = raw_u64(seed, stream, start, count) >> _U64(11)
    return (r.astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(seed: int, stream: int, count: int, sigma: float = 1.0,
           chunk: int = 1 << 22) -> np.ndarray:
    """count fp32 draws of N(0, sigma^2); Box-Muller in fp64 on counters (2i, 2i+1)."""
    out = np.empty(count, dtype=np.float32)
    for lo in range(0, count, chunk):
        n = min(chunk, count - lo)
        u = uniform01(seed, stream, 2 * lo, 2 * n)
        r = np.sqrt(-2.0 * np.log(u[0::2]))
        out[lo:lo + n] = (sigma * r * np.cos(2.0 * math.pi * u[1::2])).astype(np.float32)
    return out


def ternary(seed: int, M: int, K: int, p_zero: float, chunk: int = 1 << 22) -> np.ndarray:
    """int8 [M][K] with P(0) = p_zero and P(-1) = P(+1) = (1 - p_zero) / 2."""
    count = M * K
    out = np.empty(count, dtype=np.int8)
    p_neg = 0.5 * (1.0 - p_zero)
    for lo in range(0, count, chunk):
        n = min(chunk, count - lo)
        u = uniform01(seed, STREAM_W, lo, n)
        out[lo:lo + n] = (u >= p_neg).astype(np.int8) + (u >= p_neg + p_zero).astype(np.int8) - 1
    return out.reshape(M, K)


def latent_weight_scale(seed: int, M: int, K: int, sigma: float = 0.02,
                        chunk: int = 1 << 22) -> np.float32:
    """mean |W_fp| of an independent N(0, sigma^2) latent of the same shape, as fp32."""
    count = M * K
    total = 0.0
    for lo in range(0, count, chunk):
        n = min(chunk, count - lo)
        u = uniform01(seed, STREAM_LATENT, 2 * lo, 2 * n)
        r = np.sqrt(-2.0 * np.log(u[0::2]))
        v = (sigma * r * np.cos(2.0 * math.pi * u[1::2])).astype(np.float32)
        total += float(np.abs(v).astype(np.float64).sum())
    return np.float32(total / count)


def activations(seed: int, N: int, K: int, outlier_frac: float = 0.0,
                outlier_gain: float = 20.0) -> np.ndarray:
    """fp32 [N][K] (feature-contiguous, the framework-side layout) from N(0,1).

    With outlier_frac > 0 a fixed seeded set of ceil(outlier_frac*K) channels (the
    same for every token) is multiplied by outlier_gain before any quantisation.
    """
    x = normal(seed, STREAM_X, N * K).reshape(N, K)
    if outlier_frac > 0.0:
        n_out = int(math.ceil(outlier_frac * K))
        order = np.argsort(raw_u64(seed, STREAM_OUTLIER, 0, K), kind="stable")
        x[:, order[:n_out]] *= np.float32(outlier_gain)
    return x


@dataclass(frozen=True)
class Linear:
    name: str
    M: int
    K: int


@dataclass(frozen=True)
class Workload:
    name: str
    linears: Tuple[Linear, ...]
    N: Tuple[int, ...]
    p_zero: float
    unit_scale: bool = False          # w_scale = 1.0 instead of the latent mean
    outlier_frac: float = 0.0
    seeds: Tuple[int, ...] = (0,)
    note: str = ""


_LAYER_2B4 = (Linear("q", 2560, 2560), Linear("k", 640, 2560), Linear("v", 640, 2560),
              Linear("o", 2560, 2560), Linear("gate", 6912, 2560), Linear("up", 6912, 2560),
              Linear("down", 2560, 6912))

WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload("tiny", (Linear("tiny", 256, 256),), (8,), 1.0 / 3.0, unit_scale=True,
                     note="M=K=256, N=8, uniform ternary, scale 1"),
    "bitnet2b_ffn_up": Workload("bitnet2b_ffn_up", (Linear("up", 6912, 2560),), (128,), 0.4,
                                note="BitNet-2B-shaped FFN up projection, N=128"),
    "bitnet3b_prefill": Workload("bitnet3b_prefill",
                                 (Linear("up", 8640, 3200), Linear("down", 3200, 8640)), (256,), 0.4,
                                 note="3B-shaped up/down projections, N=256"),
    "llama8b_linears": Workload("llama8b_linears",
                                (Linear("qo", 4096, 4096), Linear("gateup", 14336, 4096),
                                 Linear("down", 4096, 14336)), (512,), 0.35, outlier_frac=0.01,
                                note="8B-shaped linears, N=512, 1% outlier channels x20"),
    "layer2b4_nsweep": Workload("layer2b4_nsweep", _LAYER_2B4, (1, 16, 64, 256, 1024), 0.4,
                                seeds=(0, 1, 2, 3, 4),
                                note="one 2.4B-style decoder layer, N sweep"),
}


def make_case(wl: Workload, lin: Linear, N: int, seed: int):
    """Returns (W int8 [M][K], w_scale fp32, x fp32 [N][K]) for one linear of a workload."""
    # decorrelate linears of one workload that share a seed
    sub = seed * 131 + (abs(hash_name(lin.name)) % 97)
    W = ternary(sub, lin.M, lin.K, wl.p_zero)
    w_scale = np.float32(1.0) if wl.unit_scale else latent_weight_scale(sub, lin.M, lin.K)
    x = activations(sub, N, lin.K, wl.outlier_frac)
    return W, w_scale, x


def hash_name(s: str) -> int:
    h = 0
    for ch in s.encode():
        h = (h * 131 + ch) & 0x7FFFFFFF
    return h


def small_case(seed: int, M: int, K: int, N: int, p_zero: float = 0.4, outlier_frac: float = 0.0):
    """Arbitrary small shape with the same distributions (ragged-tile parity cases)."""
    return (ternary(seed, M, K, p_zero), np.float32(1.0) if seed % 2 == 0 else
            latent_weight_scale(seed, M, K), activations(seed, N, K, outlier_frac))


def algorithmic_bytes(M: int, K: int, N: int) -> int:
    """HBM bytes one mpGeMM call must move: packed weights + INT8 activations + scales + fp32 out."""
    return M * K // 4 + K * N + 4 * N + 4 * M * N


def lookup_bytes(M: int, K: int, N: int) -> int:
    """Table bytes the lookups read: one INT16 per (row, k-group, token)."""
    return M * (K // 4) * N * 2
