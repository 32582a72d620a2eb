"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU path's tests.

This module holds no arithmetic of the method: it only draws random tensors of the
workload shapes (layer shapes of GPT-3, LLaMA-65B and VGG-19 under 8-way tensor
parallelism, Section II-B and Table II of the paper) and rounds them to the 16-bit
storage type.  Weight matrices are returned in their mathematical shape [K x N];
callers lay them out as their side requires.

Recipe: a torch CPU generator seeded with `seed` (0 for every config); tensors drawn in
the order listed, as fp32 normal variates, scaled, then cast to the storage dtype.
X ~ N(0,1); GeMM weights ~ N(0, 1/K) with K the inner dimension; conv weights
He-normal N(0, 2/(9*C)).
"""
from __future__ import annotations

import math
from typing import Dict

import numpy as np
import torch


def _gen(seed: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return g


def _normal(g, shape, std, dtype):
    return (torch.randn(shape, generator=g, dtype=torch.float32) * std).to(dtype)


def to_f64(t: torch.Tensor) -> np.ndarray:
    """Exact widening of a (bf16/fp16/fp32) tensor to a float64 numpy array."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def mlp(M: int, K1: int, N1: int, N2: int, seed: int = 0, dtype=torch.bfloat16) -> Dict[str, torch.Tensor]:
    """X[M,K1], W1[K1,N1], W2[N1,N2]."""
    g = _gen(seed)
    return {
        "X": _normal(g, (M, K1), 1.0, dtype),
        "W1": _normal(g, (K1, N1), 1.0 / math.sqrt(K1), dtype),
        "W2": _normal(g, (N1, N2), 1.0 / math.sqrt(N1), dtype),
    }


def swiglu(M: int, K1: int, Nh: int, N2: int, seed: int = 0, dtype=torch.bfloat16) -> Dict[str, torch.Tensor]:
    """X[M,K1], Wgu[K1,2*Nh] = [Wgate | Wup], W2[Nh,N2]."""
    g = _gen(seed)
    return {
        "X": _normal(g, (M, K1), 1.0, dtype),
        "Wgu": _normal(g, (K1, 2 * Nh), 1.0 / math.sqrt(K1), dtype),
        "W2": _normal(g, (Nh, N2), 1.0 / math.sqrt(Nh), dtype),
    }


def attention(M: int, K1: int, heads: int, d: int, N2: int, seed: int = 0, dtype=torch.bfloat16) -> Dict[str, torch.Tensor]:
    """X[M,K1], Wqkv[K1,3*heads*d] (Q | K | V column blocks), Wo[heads*d,N2]."""
    g = _gen(seed)
    E = heads * d
    return {
        "X": _normal(g, (M, K1), 1.0, dtype),
        "Wqkv": _normal(g, (K1, 3 * E), 1.0 / math.sqrt(K1), dtype),
        "Wo": _normal(g, (E, N2), 1.0 / math.sqrt(E), dtype),
    }


def kv_cache(batch: int, cached: int, heads: int, d: int, seed: int = 0, dtype=torch.bfloat16) -> Dict[str, torch.Tensor]:
    """Keys and values of `cached` earlier tokens per sequence, [batch, cached, heads*d], N(0,1) like the
    K and V columns the QKV GeMM produces from N(0,1) activations and N(0,1/K) weights."""
    g = _gen(seed + 1000)
    E = heads * d
    return {"Kc": _normal(g, (batch, cached, E), 1.0, dtype), "Vc": _normal(g, (batch, cached, E), 1.0, dtype)}


def conv(B: int, H: int, W: int, C: int, K1: int, K2: int, seed: int = 0, dtype=torch.bfloat16) -> Dict[str, torch.Tensor]:
    """x[B,H,W,C] (NHWC), w1[K1,3,3,C], w2[K2,3,3,K1]."""
    g = _gen(seed)
    return {
        "x": _normal(g, (B, H, W, C), 1.0, dtype),
        "w1": _normal(g, (K1, 3, 3, C), math.sqrt(2.0 / (9 * C)), dtype),
        "w2": _normal(g, (K2, 3, 3, K1), math.sqrt(2.0 / (9 * K1)), dtype),
    }


# Workload shapes (one 8-way tensor-parallel shard on one GPU; Section II-B, Table II).
CFG1 = dict(M=256, K1=1024, N1=4096, N2=1024)
CFG2 = dict(K1=12288, N1=6144, N2=12288, Ms=(1, 64, 256, 512, 1024, 2048))
CFG3 = dict(K1=8192, Nh=2752, N2=8192, Ms=(1, 256, 1024, 2048))
CFG4 = dict(K1=12288, heads=12, d=128, N2=12288, Ms=(512, 2048))
CFG5 = dict(stages=((224, 64), (112, 128), (56, 256), (28, 512), (14, 512)), batches=(1, 4, 16, 32))
