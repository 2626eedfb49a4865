"""Seeded synthetic inputs for the five benchmark workloads.

This module only draws random numbers and rounds them to the storage dtype.  It
holds none of the method's arithmetic (no masks, no patterns, no products), so
the CPU oracle and the HIP library can both be fed from it without sharing any
computation.  Everything is generated on the host with a seeded NumPy Generator
and rounded once; the same bytes go to both sides.

bf16 tensors are carried as ``uint16`` bit patterns (NumPy has no bf16); use
``bf16_to_f32`` / ``bf16_to_f64`` to view their exact values.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even), returned as uint16 bits."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    out = rounded.astype(np.uint16)
    nan = np.isnan(a)
    if nan.any():
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact float32 value of bf16 bit patterns."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    return bf16_to_f32(bits).astype(np.float64)


def xavier_uniform(rng: np.random.Generator, fan_out: int, fan_in: int) -> np.ndarray:
    lim = math.sqrt(6.0 / (fan_in + fan_out))
    return rng.uniform(-lim, lim, size=(fan_out, fan_in)).astype(np.float32)


@dataclass
class Workload:
    """A bag of named host arrays plus the scalar parameters of a config."""
    name: str
    dtype: str                      # "f32" or "bf16" (bf16 arrays are uint16 bits)
    arrays: dict = field(default_factory=dict)
    params: dict = field(default_factory=dict)

    def values(self, key: str) -> np.ndarray:
        """Exact values of an array as float64 (decodes bf16 bit patterns)."""
        a = self.arrays[key]
        return bf16_to_f64(a) if a.dtype == np.uint16 else a.astype(np.float64)


def _store(a: np.ndarray, dtype: str) -> np.ndarray:
    return f32_to_bf16_bits(a) if dtype == "bf16" else np.ascontiguousarray(a, dtype=np.float32)


def mlp_layer_f32(seed: int = 0, B: int = 64, I: int = 784, O: int = 1024) -> Workload:
    """Config 1: one fp32 MLP layer, X~N(0,1), W Xavier-uniform, dY~N(0,1)."""
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((B, I)).astype(np.float32)
    W = xavier_uniform(rng, O, I)
    dY = rng.standard_normal((B, O)).astype(np.float32)
    return Workload("mlp_layer_f32", "f32", dict(X=X, W=W, dY=dY),
                    dict(B=B, I=I, O=O, dp=2, b=1))


def mlp_chain(seed: int = 2, B: int = 1024, sizes=(784, 2048, 2048, 10), dtype: str = "bf16") -> Workload:
    """Config 2: MLP 784-2048-2048-10, inputs U(0,1), Xavier-uniform weights,
    output gradient N(0,1) standing in for a loss gradient."""
    rng = np.random.default_rng(seed)
    arrays = {"X0": _store(rng.uniform(0.0, 1.0, size=(B, sizes[0])).astype(np.float32), dtype)}
    for l in range(1, len(sizes)):
        arrays[f"W{l}"] = _store(xavier_uniform(rng, sizes[l], sizes[l - 1]), dtype)
    arrays["dY"] = _store(rng.standard_normal((B, sizes[-1])).astype(np.float32), dtype)
    return Workload("mlp_chain", dtype, arrays, dict(B=B, sizes=tuple(sizes)))


def tile_gemm(seed: int = 3, B: int = 4096, I: int = 4096, O: int = 4096, dtype: str = "bf16",
              tile: int = 64) -> Workload:
    """Config 3: W~N(0,0.02), X~N(0,1), dY~N(0,1)."""
    rng = np.random.default_rng(seed)
    W = (0.02 * rng.standard_normal((O, I))).astype(np.float32)
    X = rng.standard_normal((B, I)).astype(np.float32)
    dY = rng.standard_normal((B, O)).astype(np.float32)
    return Workload("tile_gemm", dtype, dict(X=_store(X, dtype), W=_store(W, dtype), dY=_store(dY, dtype)),
                    dict(B=B, I=I, O=O, tile_r=tile, tile_c=tile))


def lstm_layer(seed: int = 4, T: int = 64, B: int = 128, I: int = 1024, H: int = 1024,
               dtype: str = "bf16") -> Workload:
    """Config 4: x~N(0,1) [T,B,I], fused weight [4H, I+H] ~U(-1/sqrt(H), 1/sqrt(H))
    (1/32 for H=1024), gradient dh~N(0,1) on every h_t."""
    rng = np.random.default_rng(seed)
    lim = 1.0 / math.sqrt(H)
    x = rng.standard_normal((T, B, I)).astype(np.float32)
    W = rng.uniform(-lim, lim, size=(4 * H, I + H)).astype(np.float32)
    dh = rng.standard_normal((T, B, H)).astype(np.float32)
    return Workload("lstm_layer", dtype, dict(x=_store(x, dtype), W=_store(W, dtype), dh=_store(dh, dtype)),
                    dict(T=T, B=B, I=I, H=H))


def conv_layer(seed: int = 5, N: int = 128, C: int = 256, Cout: int = 256, H: int = 28, W: int = 28,
               dtype: str = "bf16", ksize: int = 3) -> Workload:
    """Config 5: A=ReLU(N(0,1)) NCHW, He-normal OIHW weights, dY~N(0,1)."""
    rng = np.random.default_rng(seed)
    A = np.maximum(rng.standard_normal((N, C, H, W)), 0.0).astype(np.float32)
    Wt = (math.sqrt(2.0 / (C * ksize * ksize)) * rng.standard_normal((Cout, C, ksize, ksize))).astype(np.float32)
    dY = rng.standard_normal((N, Cout, H, W)).astype(np.float32)
    return Workload("conv_layer", dtype, dict(A=_store(A, dtype), Wt=_store(Wt, dtype), dY=_store(dY, dtype)),
                    dict(N=N, C=C, Cout=Cout, H=H, W=W, ksize=ksize, rate=0.5))
