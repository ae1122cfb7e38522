"""Seeded synthetic inputs for the W4A16 skinny GEMM (paper Section 2, first paragraph:
an fp16 activation matrix, a packed int32 weight matrix, scale and zero parameters).

This module only draws random buffers of the right shape, dtype and distribution.
It contains none of the method's arithmetic: it never packs, unpacks, dequantises or
multiplies.  A packed word whose 32 bits are uniform is exactly a word whose eight
4-bit fields are independent and uniform on 0..15, so the packed tensors are drawn
directly as uniform 32-bit words and reinterpreted as int32.

Both the CPU oracle (through the tests) and the HIP path are fed from here.
The generator is numpy's counter-based Philox bit generator, so a (seed, shape)
pair names one set of buffers on every machine.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

#: value distributions of the paper-shaped workloads (llama-style square projections)
SCALE_LO = 0.001
SCALE_HI = 0.01

#: the five workload shapes: (name, m, n, k, group_size, split_k values to sweep)
CONFIGS = {
    "cfg1": dict(m=1, n=1024, k=1024, group_size=128, split_k=(4,)),
    "cfg2": dict(m=16, n=4096, k=4096, group_size=128, split_k=(1, 2, 4, 8, 16)),
    "cfg4": dict(m=16, n=8192, k=8192, group_size=128, split_k=(1, 2, 4, 8, 16, 32)),
    "cfg5": dict(m=8, n=16384, k=16384, group_size=128, split_k=(1, 4, 16, 32)),
}
#: the SplitK-vs-DP sweep: m x (n = k)
SWEEP_M = (1, 2, 4, 8, 16)
SWEEP_NK = (4096, 8192)


@dataclass
class W4A16Inputs:
    """Host buffers of one problem instance, all C-contiguous.

    A        float16 [m, k]
    qweight  int32   [k // 8, n]            eight 4-bit fields per word, along k
    scales   float16 [k // group_size, n]
    qzeros   int32   [k // group_size, n // 8]  eight 4-bit fields per word, along n
    """

    A: np.ndarray
    qweight: np.ndarray
    scales: np.ndarray
    qzeros: np.ndarray
    m: int
    n: int
    k: int
    group_size: int
    seed: int


def check_shape(m: int, n: int, k: int, group_size: int) -> None:
    if m < 1:
        raise ValueError("m must be >= 1")
    if n < 8 or n % 8:
        raise ValueError("n must be a positive multiple of 8")
    if group_size < 8 or group_size % 8:
        raise ValueError("group_size must be a positive multiple of 8")
    if k < group_size or k % group_size:
        raise ValueError("k must be a positive multiple of group_size")


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(seed))


def random_words(rng: np.random.Generator, shape) -> np.ndarray:
    """Uniform 32-bit words, returned as int32 (about half of them negative)."""
    w = rng.integers(0, 1 << 32, size=shape, dtype=np.uint32)
    return w.view(np.int32)


def make_weights(rng: np.random.Generator, n: int, k: int, group_size: int, bits: int = 4):
    """One (qweight, scales, qzeros) set drawn from `rng`, in that order.  `bits` is the field
    width (k * bits / 32 word rows, n * bits / 32 zero words per group; 3-bit fields come 32 to
    three words): uniform words are uniform independent fields at any width."""
    if (k * bits) % 32 or (n * bits) % 32:
        raise ValueError("k * bits and n * bits must be multiples of 32")
    qweight = random_words(rng, (k * bits // 32, n))
    scales = rng.uniform(SCALE_LO, SCALE_HI, size=(k // group_size, n)).astype(np.float16)
    qzeros = random_words(rng, (k // group_size, n * bits // 32))
    return qweight, scales, qzeros


def make_inputs(m: int, n: int, k: int, group_size: int = 128, seed: int = 0, bits: int = 4) -> W4A16Inputs:
    """The standard workload: A ~ N(0,1) rounded to fp16, fields uniform on 0..2^bits - 1 (the
    paper's are 4-bit), scales ~ U(0.001, 0.01) rounded to fp16.  Draw order: A, qweight,
    scales, qzeros."""
    check_shape(m, n, k, group_size)
    rng = _rng(seed)
    A = rng.standard_normal(size=(m, k), dtype=np.float32).astype(np.float16)
    qweight, scales, qzeros = make_weights(rng, n, k, group_size, bits)
    return W4A16Inputs(A, qweight, scales, qzeros, m, n, k, group_size, seed)


def make_weight_sets(count: int, n: int, k: int, group_size: int = 128, seed: int = 0, bits: int = 4):
    """`count` independent weight sets for the cold-cache timing rotation.
    They come from their own Philox key (seed, 1), so none of them repeats the weights
    that make_inputs draws for the same seed."""
    check_shape(1, n, k, group_size)
    rng = np.random.Generator(np.random.Philox(key=[seed, 1]))
    return [make_weights(rng, n, k, group_size, bits) for _ in range(count)]


def algorithmic_bytes(m: int, n: int, k: int, group_size: int = 128, bits: int = 4) -> int:
    """Bytes every call must move at least once: packed weights + scales + zeros + A + C."""
    g = k // group_size
    return (k * bits // 32) * n * 4 + g * n * 2 + g * (n * bits // 32) * 4 + m * k * 2 + m * n * 2
