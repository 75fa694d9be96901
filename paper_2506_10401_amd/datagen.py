"""Seeded synthetic tensors for the fused-operator workloads.

This module holds only the input generator.  It contains none of the
operators' arithmetic and is the single piece of code that both the GPU
library's callers and the CPU checker's callers draw their inputs from, so
both sides see identical fp32 bits.

Generator: a counter-based SplitMix64 stream per tensor (Steele, Lea, Flood,
"Fast splittable pseudorandom number generators", OOPSLA 2014; the 64-bit
finaliser with constants 0xBF58476D1CE4E5B9 / 0x94D049BB133111EB).  Draw i of
a stream with seed s is mix(s + (i+1)*0x9E3779B97F4A7C15), so any element can
be produced without the ones before it and the result does not depend on
chunking, thread count or library versions.

  uniform(a,b):  a + (b-a) * (u53 + 0.5) / 2**53   (open interval), -> fp32
  normal(mu,sd): Box-Muller in fp64 on draws 2i and 2i+1 of the stream,
                 mu + sd * sqrt(-2 ln u1) * cos(2 pi u2), -> fp32

The paper's operator benchmarks (basic operators, fused graphs, model blocks
of its Section 4.1) are not available; the five workloads below are synthetic
stand-ins with the operator classes of its Table 1 and the fused examples of
its Section 5.3, at the shapes and value distributions listed in `CONFIGS`.
"""
from __future__ import annotations

import math
import os
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, Tuple

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
BASE_SEED = 0x250610401
_CHUNK = 1 << 20


def splitmix64(seed: int, start: int, count: int) -> np.ndarray:
    """Draws start .. start+count-1 of the stream `seed` as uint64."""
    with np.errstate(over="ignore"):
        idx = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        z = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + idx * _GOLDEN
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def _unit_open(seed: int, start: int, count: int) -> np.ndarray:
    """count fp64 values strictly inside (0,1)."""
    u53 = (splitmix64(seed, start, count) >> np.uint64(11)).astype(np.float64)
    return (u53 + 0.5) * (1.0 / 9007199254740992.0)


def _fill(n: int, chunk_fn) -> np.ndarray:
    """out[s:s+c] = chunk_fn(s, c) for every chunk; chunks are independent
    (counter-based draws), so they are filled by a few threads."""
    out = np.empty(n, dtype=np.float32)

    def work(s):
        c = min(_CHUNK, n - s)
        out[s:s + c] = chunk_fn(s, c)

    starts = range(0, n, _CHUNK)
    if len(starts) <= 1:
        for s in starts:
            work(s)
    else:
        with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
            list(ex.map(work, starts))
    return out


def gen_uniform(seed: int, shape, lo: float, hi: float) -> np.ndarray:
    def chunk(s, c):
        return (lo + (hi - lo) * _unit_open(seed, s, c)).astype(np.float32)
    return _fill(int(np.prod(shape)), chunk).reshape(shape)


def gen_normal(seed: int, shape, mu: float, sd: float) -> np.ndarray:
    def chunk(s, c):
        u = _unit_open(seed, 2 * s, 2 * c)
        z = np.sqrt(-2.0 * np.log(u[0::2])) * np.cos((2.0 * math.pi) * u[1::2])
        return (mu + sd * z).astype(np.float32)
    return _fill(int(np.prod(shape)), chunk).reshape(shape)


def tensor_seed(config_index: int, tensor_index: int, variant: int = 0) -> int:
    """Seed of one tensor: base ^ (config<<8) ^ tensor, `variant` selects an
    independent replica (used for rotating buffer sets when timing)."""
    return BASE_SEED ^ (config_index << 8) ^ tensor_index ^ (variant << 20)


# name -> (tensor_index, shape, kind, p0, p1); kind 'u' = uniform(p0,p1), 'n' = normal(p0,p1)
Spec = Tuple[int, Tuple[int, ...], str, float, float]


def chain1_specs(M=64, K=256, N=256) -> Dict[str, Spec]:
    """GEMM + bias + ReLU + row softmax."""
    return {"X": (0, (M, K), "u", -1.0, 1.0),
            "W": (1, (K, N), "u", -1.0 / 16, 1.0 / 16),
            "bias": (2, (N,), "u", -0.1, 0.1)}


def chain2_specs(N=32, C=64, H=56, W=56) -> Dict[str, Spec]:
    """Per-channel affine + ReLU + residual, then global average pool."""
    return {"X": (0, (N, C, H, W), "n", 0.0, 1.0),
            "scale": (1, (C,), "n", 1.0, 0.1),
            "shift": (2, (C,), "n", 0.0, 0.1),
            "R": (3, (N, C, H, W), "n", 0.0, 1.0)}


def chain3_specs(M=8192, N=4096) -> Dict[str, Spec]:
    """Layernorm over the last dim + tanh-form GELU."""
    return {"X": (0, (M, N), "n", 0.0, 1.0),
            "gamma": (1, (N,), "n", 1.0, 0.1),
            "beta": (2, (N,), "n", 0.0, 0.1)}


def chain4_specs(N=32, C=64, H=56, W=56, K=128, R=3, S=3) -> Dict[str, Spec]:
    """NCHW conv2d + bias + ReLU; weights He-normal, std = sqrt(2 / (C*R*S))."""
    return {"in": (0, (N, C, H, W), "n", 0.0, 1.0),
            "wt": (1, (K, C, R, S), "n", 0.0, math.sqrt(2.0 / (C * R * S))),
            "bias": (2, (K,), "u", -0.1, 0.1)}


def chain5_specs(B=16, L=2048, D=64, Lk=None) -> Dict[str, Spec]:
    """Batched GEMM - softmax - GEMM."""
    Lk = L if Lk is None else Lk
    return {"Q": (0, (B, L, D), "n", 0.0, 1.0),
            "K": (1, (B, Lk, D), "n", 0.0, 1.0),
            "V": (2, (B, Lk, D), "n", 0.0, 1.0)}


def chain6_specs(M=4096, K=1024, N=4096) -> Dict[str, Spec]:
    """GEMM + bias + hash dropout + mean over features + softmax over the row means
    (the fused group of the paper's first case study, Section 5.3); W ~ N(0, 1/sqrt(K))
    keeps the pre-dropout activations at unit scale."""
    return {"X": (0, (M, K), "n", 0.0, 1.0),
            "W": (1, (K, N), "n", 0.0, 1.0 / math.sqrt(K)),
            "bias": (2, (N,), "u", -0.5, 0.5)}


# dropout probability and seed of workload 6 (scalars, not tensors)
CHAIN6_P = 0.25
CHAIN6_SEED = 0x2506_1040_1


def chain7_specs(N=32, C=64, H=56, W=56, K=128, R=3, S=3) -> Dict[str, Spec]:
    """VGG-style block: conv + bias, folded batch-norm scale/shift per output channel, ReLU, 2x2 max pool."""
    return {"in": (0, (N, C, H, W), "n", 0.0, 1.0),
            "wt": (1, (K, C, R, S), "n", 0.0, math.sqrt(2.0 / (C * R * S))),
            "bias": (2, (K,), "u", -0.1, 0.1),
            "scale": (3, (K,), "n", 1.0, 0.1),
            "shift": (4, (K,), "n", 0.0, 0.1)}


CONFIGS = {1: chain1_specs, 2: chain2_specs, 3: chain3_specs, 4: chain4_specs, 5: chain5_specs, 6: chain6_specs, 7: chain7_specs}


def make(config_index: int, variant: int = 0, **dims) -> Dict[str, np.ndarray]:
    """All input tensors of one workload, as contiguous fp32 numpy arrays.
    With no `dims` the shapes are the full-size ones of that workload."""
    specs = CONFIGS[config_index](**dims)
    out = {}
    for name, (ti, shape, kind, p0, p1) in specs.items():
        seed = tensor_seed(config_index, ti, variant)
        if 0 in shape:
            out[name] = np.zeros(shape, dtype=np.float32)
        elif kind == "u":
            out[name] = gen_uniform(seed, shape, p0, p1)
        else:
            out[name] = gen_normal(seed, shape, p0, p1)
    return out
