"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds no arithmetic of the method: it only draws the weight and
activation matrices.  The shapes are those of the linear layers of the models
the paper evaluates (DeiT-small / DeiT-base, Section 5.1; Llama2-7B, Section
5.3); the values are generic stand-ins (the trained weights and datasets are
not used): W ~ N(0, 0.02^2), X ~ N(0, 1), drawn in fp32 and rounded to fp16
(round to nearest even).  For the Llama-shaped layers 1 % of the input columns
of W are multiplied by 10 to imitate outlier channels.

Draw order for one layer: W first, then the outlier column choice, then X, all
from numpy.random.default_rng(seed); W therefore does not depend on the token
count, and a shorter X is a prefix of a longer one.
"""

from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Layer:
    name: str
    out: int
    inn: int
    tokens: int
    V: int
    M: int
    seed: int
    outliers: bool = False


def make_weight_and_input(out: int, inn: int, tokens: int, seed: int,
                          outliers: bool = False, w_std: float = 0.02):
    """Return (W fp16 [out x in], X fp16 [tokens x in])."""
    rng = np.random.default_rng(seed)
    W = rng.standard_normal((out, inn), dtype=np.float32) * np.float32(w_std)
    if outliers:
        n_out = int(round(0.01 * inn))
        cols = rng.choice(inn, size=n_out, replace=False)
        W[:, cols] *= np.float32(10.0)
    X = rng.standard_normal((tokens, inn), dtype=np.float32)
    return W.astype(np.float16), X.astype(np.float16)


def layer_tensors(layer: Layer, tokens: int | None = None):
    """W and X of a Layer; `tokens` overrides the token count (W is unchanged
    and the shorter X is a prefix of the longer one)."""
    T = layer.tokens if tokens is None else tokens
    return make_weight_and_input(layer.out, layer.inn, T, layer.seed, layer.outliers)


def config_single_gemm():
    """Smallest case: one 128 x 128 layer, 16 tokens, 64:2:8, seed 0."""
    return [Layer("single", 128, 128, 16, 64, 8, 0)]


def config_deit_small(V: int = 64, M: int = 5):
    T = 64 * 197
    return [Layer("qkv", 1152, 384, T, V, M, 1000),
            Layer("proj", 384, 384, T, V, M, 1001),
            Layer("fc1", 1536, 384, T, V, M, 1002),
            Layer("fc2", 384, 1536, T, V, M, 1003)]


def config_deit_base(V: int = 64, M: int = 8):
    T = 64 * 197
    return [Layer("qkv", 2304, 768, T, V, M, 2000),
            Layer("proj", 768, 768, T, V, M, 2001),
            Layer("fc1", 3072, 768, T, V, M, 2002),
            Layer("fc2", 768, 3072, T, V, M, 2003)]


def config_llama2_7b(V: int = 64, M: int = 5, tokens: int = 4096):
    """The seven linear layers of one Llama-2-7B block at prefill."""
    names = [("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
             ("gate", 11008, 4096), ("up", 11008, 4096), ("down", 4096, 11008)]
    return [Layer(n, o, i, tokens, V, M, 3000 + k, outliers=True)
            for k, (n, o, i) in enumerate(names)]


def config_sweep():
    """V x M x tokens sweep on the two large Llama shapes."""
    layers = []
    for (n, o, i) in (("gate", 11008, 4096), ("down", 4096, 11008)):
        for V in (32, 64, 128):
            for M in (4, 5, 6, 7, 8, 16):
                for T in (16, 4096):
                    layers.append(Layer(f"{n}_V{V}_M{M}_T{T}", o, i, T, V, M, 4000, outliers=True))
    return layers


def small_integer_case(out: int, inn: int, tokens: int, seed: int, lo: int = -3, hi: int = 3):
    """Small-integer-valued fp16 W and X: every product and partial sum is
    exactly representable in fp32, so any correct product is exact."""
    rng = np.random.default_rng(seed)
    W = rng.integers(lo, hi + 1, size=(out, inn)).astype(np.float16)
    X = rng.integers(lo, hi + 1, size=(tokens, inn)).astype(np.float16)
    return W, X
