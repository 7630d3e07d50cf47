"""Seeded synthetic inputs for the five benchmark workloads.

This module only draws random numbers, rounds them once to their storage type and
describes shapes.  It holds none of the operators' or the constructor's arithmetic, so
both the HIP path and the CPU oracle may be fed from it.  Everything is numpy; nothing
here touches a GPU.

Storage types are carried as numpy arrays of the raw bits:
  "f32"  -> np.float32
  "f16"  -> np.float16
  "bf16" -> np.uint16 holding the upper 16 bits of the fp32 value, rounded to nearest even
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, Tuple

import numpy as np

DTYPES = ("f32", "f16", "bf16")


def _rng(seed: int) -> np.random.Generator:
    # Philox is counter based: the stream depends on the seed alone.
    return np.random.Generator(np.random.Philox(int(seed)))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (nearest even) and return the 16 stored bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    nan = (u & 0x7FFFFFFF) > 0x7F800000
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16).astype(np.uint16)
    r[nan] = 0x7FC0
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round an fp32 array once to its storage type (the bits both sides then read)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "f16":
        return x.astype(np.float16)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(dtype)


def storage_to_f32(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return bf16_bits_to_f32(x)
    return x.astype(np.float32)


def uniform_pm1(seed: int, shape, dtype: str) -> np.ndarray:
    """i.i.d. uniform on [-1, 1)."""
    v = _rng(seed).random(size=shape, dtype=np.float32) * np.float32(2.0) - np.float32(1.0)
    return to_storage(v, dtype)


def normal(seed: int, shape, dtype: str, sigma: float = 1.0) -> np.ndarray:
    v = _rng(seed).standard_normal(size=shape, dtype=np.float32) * np.float32(sigma)
    return to_storage(v, dtype)


def small_ints(seed: int, shape, dtype: str, lo: int = -4, hi: int = 4) -> np.ndarray:
    """Integers in [lo, hi]: exactly representable in every storage type, so that sums
    of a few thousand products are exact in fp32 and any summation order agrees."""
    v = _rng(seed).integers(lo, hi + 1, size=shape).astype(np.float32)
    return to_storage(v, dtype)


# --------------------------------------------------------------------------------------
# workload descriptions
# --------------------------------------------------------------------------------------
@dataclass
class GemmWorkload:
    name: str
    dtype: str
    M: int
    N: int
    K: int
    transA: int = 0      # 0: A stored [M][K]; 1: A stored [K][M]
    transB: int = 0      # 0: B stored [K][N]; 1: B stored [N][K] (column-major B)
    batch: int = 1
    A: np.ndarray = field(default=None, repr=False)
    B: np.ndarray = field(default=None, repr=False)

    @property
    def flops(self) -> float:
        return 2.0 * self.batch * self.M * self.N * self.K


@dataclass
class ConvWorkload:
    name: str
    dtype: str
    n: int
    c: int
    h: int
    w: int
    k: int
    r: int
    s: int
    stride: int
    pad: int
    I: np.ndarray = field(default=None, repr=False)
    W: np.ndarray = field(default=None, repr=False)

    @property
    def p(self) -> int:
        return (self.h + 2 * self.pad - self.r) // self.stride + 1

    @property
    def q(self) -> int:
        return (self.w + 2 * self.pad - self.s) // self.stride + 1

    @property
    def flops(self) -> float:
        return 2.0 * self.n * self.k * self.p * self.q * self.c * self.r * self.s


def _seed(config: int, tensor: int) -> int:
    return 0x5EED0000 + 16 * config + tensor


def _a_shape(M, K, transA):
    return (K, M) if transA else (M, K)


def _b_shape(K, N, transB):
    return (N, K) if transB else (K, N)


def gemm_workload(name, dtype, M, N, K, transA, transB, gen_a, gen_b, batch=1) -> GemmWorkload:
    sa = _a_shape(M, K, transA)
    sb = _b_shape(K, N, transB)
    if batch > 1:
        sa = (batch,) + sa
        sb = (batch,) + sb
    return GemmWorkload(name, dtype, M, N, K, transA, transB, batch, gen_a(sa), gen_b(sb))


def config1_gemm_f32(scale: int = 1) -> GemmWorkload:
    """fp32 GEMM, M=N=K=512, both operands row-major, uniform[-1,1)."""
    n = 512 // scale
    return gemm_workload("cfg1_gemm_f32_512", "f32", n, n, n, 0, 0,
                         lambda s: uniform_pm1(_seed(1, 0), s, "f32"),
                         lambda s: uniform_pm1(_seed(1, 1), s, "f32"))


def config2_gemm_f16(size: int = 4096, dtype: str = "f16") -> GemmWorkload:
    """fp16 GEMM with fp32 accumulate/output, A row-major, B column-major, uniform[-1,1)."""
    return gemm_workload(f"cfg2_gemm_{dtype}_{size}", dtype, size, size, size, 0, 1,
                         lambda s: uniform_pm1(_seed(2, 0), s, dtype),
                         lambda s: uniform_pm1(_seed(2, 1), s, dtype))


def config3_gpt2(which: str, rows: int = 8192, dtype: str = "f16") -> GemmWorkload:
    """GPT-2-small MLP GEMMs: activations N(0,1) [rows x d_in] times weights N(0,0.02)
    [d_in x d_out], both row-major.  which = "up" (768->3072) or "down" (3072->768)."""
    d_in, d_out = (768, 3072) if which == "up" else (3072, 768)
    t = 0 if which == "up" else 2
    return gemm_workload(f"cfg3_gpt2_{which}_{dtype}", dtype, rows, d_out, d_in, 0, 0,
                         lambda s: normal(_seed(3, t), s, dtype, 1.0),
                         lambda s: normal(_seed(3, t + 1), s, dtype, 0.02))


def config4_bmm_scores(batch: int = 96, seq: int = 1024, head: int = 64, dtype: str = "f16",
                       materialised_kt: bool = False) -> GemmWorkload:
    """Attention scores Q.K^T per (batch, head): Q [b][seq][head], K [b][seq][head], N(0,1).
    The natural layout keeps K as stored and presents it with transB=1; with
    materialised_kt the same values are laid out as K^T [b][head][seq] (transB=0)."""
    w = gemm_workload(f"cfg4_bmm_scores_{dtype}", dtype, seq, seq, head, 0, 1,
                      lambda s: normal(_seed(4, 0), s, dtype, 1.0),
                      lambda s: normal(_seed(4, 1), s, dtype, 1.0), batch=batch)
    if materialised_kt:
        w.B = np.ascontiguousarray(np.swapaxes(w.B, -1, -2))
        w.transB = 0
        w.name += "_kt"
    return w


def config5_conv(which: str, n: int = 32, dtype: str = "f16", hw: int = 56) -> ConvWorkload:
    """ResNet-50 shaped convolutions, NCHW input N(0,1), KCRS weights He-normal
    (sigma = sqrt(2 / (C*R*S))).  which = "3x3" (C=64->K=64, stride 1, pad 1) or
    "1x1s2" (C=256->K=512, stride 2, pad 0)."""
    if which == "3x3":
        c, k, r, s, stride, pad, t = 64, 64, 3, 3, 1, 1, 0
    else:
        c, k, r, s, stride, pad, t = 256, 512, 1, 1, 2, 0, 2
    sigma = math.sqrt(2.0 / (c * r * s))
    cw = ConvWorkload(f"cfg5_conv_{which}_{dtype}", dtype, n, c, hw, hw, k, r, s, stride, pad)
    cw.I = normal(_seed(5, t), (n, c, hw, hw), dtype, 1.0)
    cw.W = normal(_seed(5, t + 1), (k, c, r, s), dtype, sigma)
    return cw


UNBALANCED_GEMMS = [(65536, 4, 1024), (32768, 64, 2048), (16384, 32, 1024), (65536, 1024, 4096), (8192, 8192, 8192)]


def unbalanced_gemm(index: int, dtype: str = "f16") -> GemmWorkload:
    """One of the paper's GEMM shapes with unbalanced dimensions, [M, K, N] as in its operator
    table (GEMM rows) and its unbalanced-shape experiments; A and B row-major, uniform [-1, 1)."""
    M, K, N = UNBALANCED_GEMMS[index]
    return gemm_workload(f"gemm_{M}x{K}x{N}_{dtype}", dtype, M, N, K, 0, 0,
                         lambda s: uniform_pm1(_seed(6 + index, 0), s, dtype),
                         lambda s: uniform_pm1(_seed(6 + index, 1), s, dtype))


# Few output tiles and a deep reduction, [M, K, N], transB: the shapes a split along k exists for (the other
# extreme of "unbalanced" from the paper's tall ones; not in its operator table).
DEEP_K_GEMMS = [("f16", 512, 32768, 512, 1), ("f16", 256, 65536, 256, 0), ("f16", 1024, 8192, 1024, 1), ("f32", 256, 16384, 256, 1)]


def deep_k_gemm(index: int) -> GemmWorkload:
    dtype, M, K, N, transB = DEEP_K_GEMMS[index]
    return gemm_workload(f"gemm_{M}x{K}x{N}_{dtype}_deepk", dtype, M, N, K, 0, transB,
                         lambda s: uniform_pm1(_seed(20 + index, 0), s, dtype),
                         lambda s: uniform_pm1(_seed(20 + index, 1), s, dtype))


GEMV_SHAPES = [(16384, 16384), (16384, 8192), (16384, 1000)]                      # V1-V3: [M, N]
POOL_SHAPES = [(16, 48, 48, 48, 2, 2), (128, 168, 83, 83, 2, 2), (128, 617, 21, 21, 3, 2)]   # P1-P3: n, c, h, w, F, S
PAPER_CONVS = [(128, 256, 30, 30, 256, 3, 2), (128, 128, 28, 28, 128, 3, 1), (128, 128, 58, 58, 128, 3, 2)]   # C1-C3: n, c, h, w, k, r, S


def gemv_workload(index: int, dtype: str = "f16"):
    """GEMV shape V1-V3 of the paper's operator table: (A [M][N], x [N]), uniform [-1, 1)."""
    M, N = GEMV_SHAPES[index]
    return uniform_pm1(_seed(11 + index, 0), (M, N), dtype), uniform_pm1(_seed(11 + index, 1), (N,), dtype)


def pool_workload(index: int, dtype: str = "f16"):
    """AvgPooling2d shape P1-P3 of the operator table: (input NCHW, F, S), N(0, 1) values."""
    n, c, h, w, f, s = POOL_SHAPES[index]
    return normal(_seed(14 + index, 0), (n, c, h, w), dtype, 1.0), f, s


def paper_conv(index: int, dtype: str = "f16") -> "ConvWorkload":
    """Conv2d shape C1-C3 of the operator table (inputs printed already padded: no padding here)."""
    n, c, h, w, k, r, stride = PAPER_CONVS[index]
    cw = ConvWorkload(f"conv_C{index + 1}_{dtype}", dtype, n, c, h, w, k, r, r, stride, 0)
    cw.I = normal(_seed(17 + index, 0), (n, c, h, w), dtype, 1.0)
    cw.W = normal(_seed(17 + index, 1), (k, c, r, r), dtype, math.sqrt(2.0 / (c * r * r)))
    return cw


def all_configs() -> Dict[str, object]:
    return {
        "cfg1": config1_gemm_f32(),
        "cfg2": config2_gemm_f16(),
        "cfg3_up": config3_gpt2("up"),
        "cfg3_down": config3_gpt2("down"),
        "cfg4": config4_bmm_scores(),
        "cfg5_3x3": config5_conv("3x3"),
        "cfg5_1x1s2": config5_conv("1x1s2"),
    }


def sample_indices(seed: int, shape: Tuple[int, ...], count: int) -> np.ndarray:
    """`count` distinct-ish output coordinates, always including the corners."""
    rng = _rng(seed)
    idx = np.stack([rng.integers(0, d, size=count) for d in shape], axis=1)
    corners = np.array([[0] * len(shape), [d - 1 for d in shape]])
    return np.concatenate([corners, idx], axis=0).astype(np.int64)
