"""Seeded synthetic inputs for the SQ-format linear layer.

This module only *draws inputs*: random activations with per-channel outliers,
random INT4 weights and their scales, plus the two container conversions every
consumer of those inputs needs (fp32 -> bf16 bit patterns, two INT4 codes per
byte).  It holds none of the method's arithmetic (no selection, no scales, no
quantisation of activations, no products), so both the CPU oracle and the HIP
path can be fed from it without sharing code with each other.

The activations stand in for real LLM activations, which have a few input
channels that are one to two orders of magnitude larger than the rest
(Section 3.2.2: per-channel outliers in activations); the shapes are the
Llama-7B / 70B projection shapes the benchmark configurations name.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional

import numpy as np

__all__ = [
    "Workload",
    "CONFIG_NAMES",
    "make",
    "f32_to_bf16_bits",
    "bf16_bits_to_f32",
    "pack_int4",
    "unpack_int4",
]


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-half-even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to the fp32 values they denote (exact)."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def pack_int4(w: np.ndarray) -> np.ndarray:
    """[R, K] integers in [-8, 7] -> [R, K/2] bytes; element 2i in bits 0-3, 2i+1 in bits 4-7."""
    w = np.asarray(w)
    assert w.shape[-1] % 2 == 0
    assert w.min() >= -8 and w.max() <= 7
    u = (w.astype(np.int16) & 0xF).astype(np.uint8)
    return (u[..., 0::2] | (u[..., 1::2] << 4)).astype(np.uint8)


def unpack_int4(p: np.ndarray) -> np.ndarray:
    """Inverse of pack_int4: [R, K/2] bytes -> [R, K] int8 in [-8, 7]."""
    p = np.asarray(p, dtype=np.uint8)
    lo = (p & 0xF).astype(np.int8)
    hi = (p >> 4).astype(np.int8)
    lo = np.where(lo >= 8, lo - 16, lo).astype(np.int8)
    hi = np.where(hi >= 8, hi - 16, hi).astype(np.int8)
    out = np.empty(p.shape[:-1] + (p.shape[-1] * 2,), dtype=np.int8)
    out[..., 0::2] = lo
    out[..., 1::2] = hi
    return out


@dataclasses.dataclass
class Workload:
    """One problem instance: everything the layer takes as input."""

    name: str
    M: int
    K: int
    N: int
    bank: int
    topk: int
    mode: str  # "dynamic" | "static"
    x_bits: np.ndarray  # [M, K] uint16 bf16 patterns
    wq_packed: np.ndarray  # [N, K/2] uint8
    w_scale: np.ndarray  # [N] float32
    outlier_channels: np.ndarray  # the channels that were scaled up
    calib_bits: Optional[np.ndarray] = None  # [T, K] uint16, static mode only
    seed: int = 0

    @property
    def ops(self) -> int:
        """Effective operations of the layer, 2*M*N*K."""
        return 2 * self.M * self.N * self.K


CONFIG_NAMES = ("c1_tiny", "c2_qkv7b", "c3_mlp7b", "c4_down7b_static", "c5_up70b")


def _weights(rng: np.random.Generator, N: int, K: int):
    # Drawn row block by row block so that the peak host footprint stays small.
    packed = np.empty((N, K // 2), dtype=np.uint8)
    step = 2048
    for r0 in range(0, N, step):
        r1 = min(N, r0 + step)
        w = rng.integers(-8, 8, size=(r1 - r0, K), dtype=np.int8)
        packed[r0:r1] = pack_int4(w)
    scale = rng.uniform(0.005, 0.02, size=N).astype(np.float32)
    return packed, scale


def _log_uniform(rng, lo, hi, n):
    return np.exp(rng.uniform(math.log(lo), math.log(hi), size=n))


def _normal_x(rng, M, K, chans, factors):
    x = rng.standard_normal(size=(M, K), dtype=np.float32)
    x[:, chans] *= factors.astype(np.float32)[None, :]
    return x


def _student_t3_x(rng, M, K, chans, factors):
    z = rng.standard_normal(size=(M, K), dtype=np.float32)
    chi = rng.chisquare(3.0, size=(M, K)).astype(np.float32)
    x = z / np.sqrt(chi / np.float32(3.0))
    x[:, chans] *= factors.astype(np.float32)[None, :]
    return x.astype(np.float32)


def make(
    name: str,
    *,
    M: Optional[int] = None,
    N: Optional[int] = None,
    bank: Optional[int] = None,
    topk: Optional[int] = None,
    with_weights: bool = True,
) -> Workload:
    """Build one of the five benchmark configurations (optionally with M, N, bank or topk overridden).

    Overriding N draws only the first N weight rows' worth of random numbers, so a
    reduced-N instance is *not* a slice of the full one; overriding M likewise.
    Every instance is a pure function of (name, M, N): the same call gives the same bytes.
    """
    if name == "c1_tiny":
        seed, m, k, n, b, tk, mode = 1001, 16, 512, 512, 64, 8, "dynamic"
    elif name == "c2_qkv7b":
        seed, m, k, n, b, tk, mode = 1002, 2048, 4096, 12288, 64, 8, "dynamic"
    elif name == "c3_mlp7b":
        seed, m, k, n, b, tk, mode = 1003, 4096, 4096, 22016, 64, 8, "dynamic"
    elif name == "c4_down7b_static":
        seed, m, k, n, b, tk, mode = 1004, 4096, 11008, 4096, 64, 8, "static"
    elif name == "c5_up70b":
        seed, m, k, n, b, tk, mode = 1005, 8192, 8192, 28672, 64, 8, "dynamic"
    else:
        raise KeyError(name)
    m = m if M is None else int(M)
    n = n if N is None else int(N)
    b = b if bank is None else int(bank)
    tk = tk if topk is None else int(topk)

    # Independent streams for activations, weights and calibration data, so that
    # changing M or N never changes the other operand.
    rx = np.random.Generator(np.random.PCG64([seed, 1]))
    rw = np.random.Generator(np.random.PCG64([seed, 2]))
    rc = np.random.Generator(np.random.PCG64([seed + 10000, 3]))

    calib = None
    if name == "c1_tiny":
        chans = np.sort(rx.choice(k, size=8, replace=False))
        factors = np.full(8, 30.0)
        x = _normal_x(rx, m, k, chans, factors)
    elif name in ("c2_qkv7b", "c3_mlp7b"):
        n_out = int(round(0.01 * k))
        chans = np.sort(rx.choice(k, size=n_out, replace=False))
        factors = _log_uniform(rx, 20.0, 50.0, n_out)
        x = _normal_x(rx, m, k, chans, factors)
    elif name == "c4_down7b_static":
        n_out = int(round(0.005 * k))
        chans = np.sort(rx.choice(k, size=n_out, replace=False))
        factors = _log_uniform(rx, 20.0, 50.0, n_out)
        x = _student_t3_x(rx, m, k, chans, factors)
        calib = f32_to_bf16_bits(_student_t3_x(rc, 512, k, chans, factors))
    else:  # c5_up70b
        n_out = int(round(0.01 * k))
        chans = np.sort(rx.choice(k, size=n_out, replace=False))
        factors = np.full(n_out, 30.0)
        x = _normal_x(rx, m, k, chans, factors)

    x_bits = f32_to_bf16_bits(x)
    if with_weights:
        wq, ws = _weights(rw, n, k)
    else:
        wq, ws = np.zeros((0, k // 2), np.uint8), np.zeros((0,), np.float32)
    return Workload(
        name=name, M=m, K=k, N=n, bank=b, topk=tk, mode=mode, x_bits=x_bits,
        wq_packed=wq, w_scale=ws, outlier_channels=chans, calib_bits=calib, seed=seed,
    )
