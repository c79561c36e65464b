"""Seeded synthetic inputs for the dual trit-plane linear layer.

This module only draws random tensors; it holds none of the method's
arithmetic (no packing, no trit-plane products, no scaling).  Both the CPU
oracle's tests and the HIP path's tests/benchmark take their inputs from here,
so the two sides are always fed identical data.

Recipe (stand-in for the quantised LLaMA weights the paper evaluates on, whose
checkpoints are not available): trits i.i.d. with P(-1)=P(+1)=0.3, P(0)=0.4,
the two planes independent; alpha1 = fp16(|z|), z ~ N(0, 0.02^2) per
(row, group); alpha2 = fp16(alpha1 * u), u ~ U(0.1, 0.5); x = fp16(N(0, 1)).
"""
from __future__ import annotations

import numpy as np

GROUP = 128  # paper, "Batch Processing": G = 128 columns per scale group

# (N = out features, K = in features), LLaMA-3-8B and LLaMA-3-70B decoder linears.
SHAPES_8B = {
    "q": (4096, 4096), "k": (1024, 4096), "v": (1024, 4096), "o": (4096, 4096),
    "gate": (14336, 4096), "up": (14336, 4096), "down": (4096, 14336),
}
SHAPES_70B = {
    "q": (8192, 8192), "k": (1024, 8192), "v": (1024, 8192), "o": (8192, 8192),
    "gate": (28672, 8192), "up": (28672, 8192), "down": (8192, 28672),
}
LINEAR_ORDER = ("q", "k", "v", "o", "gate", "up", "down")
N_LAYERS_8B = 32

_ROOT = 16989
_TRIT_LUT = np.array([-1, -1, -1, 1, 1, 1, 0, 0, 0, 0], dtype=np.int8)


def _rng(*key: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([_ROOT, *key])))


def make_trits(N: int, K: int, *key: int) -> np.ndarray:
    """int8 [N, K], values in {-1, 0, +1} with P = 0.3 / 0.4 / 0.3."""
    u = _rng(*key, 1).integers(0, 10, size=(N, K), dtype=np.uint8)
    return _TRIT_LUT[u]


def make_scales(N: int, K: int, *key: int, group: int = GROUP):
    """(alpha1, alpha2), each float16 [N, K // group]."""
    ng = K // group
    g = _rng(*key, 2)
    z = g.standard_normal((N, ng))
    a1 = np.abs(0.02 * z).astype(np.float16)
    u = g.uniform(0.1, 0.5, size=(N, ng))
    a2 = (a1.astype(np.float64) * u).astype(np.float16)
    return a1, a2


def make_x(M: int, K: int, *key: int) -> np.ndarray:
    """float16 [M, K] ~ N(0, 1)."""
    return _rng(*key, 3).standard_normal((M, K)).astype(np.float16)


def make_linear(N: int, K: int, *key: int, group: int = GROUP) -> dict:
    """One trit-plane linear layer: T1, T2 int8 [N, K]; a1, a2 float16 [N, K/group]."""
    a1, a2 = make_scales(N, K, *key, group=group)
    return {
        "T1": make_trits(N, K, *key, 11),
        "T2": make_trits(N, K, *key, 12),
        "a1": a1, "a2": a2, "N": N, "K": K, "group": group,
    }


def config0(M: int = 1):
    """BASELINE config 0: N = K = 1024, batch 1."""
    lin = make_linear(1024, 1024, 0)
    return lin, make_x(M, 1024, 0)


def layer_8b(layer: int = 0):
    """The seven linears of one 8B-shaped decoder layer (config 1 / one layer of config 3)."""
    return {name: make_linear(*SHAPES_8B[name], 1, layer, i)
            for i, name in enumerate(LINEAR_ORDER)}


def linear_8b(name: str, layer: int = 0):
    return make_linear(*SHAPES_8B[name], 1, layer, LINEAR_ORDER.index(name))


def linear_70b(name: str):
    return make_linear(*SHAPES_70B[name], 4, 0, LINEAR_ORDER.index(name))


def x_for(name: str, M: int, K: int, config: int = 1, layer: int = 0) -> np.ndarray:
    return make_x(M, K, config, layer, LINEAR_ORDER.index(name), M)


def integer_exact_case(N: int, K: int, M: int, *key: int, group: int = GROUP):
    """Inputs whose every partial sum is exactly representable in fp32, in any
    summation order: x integer in [-4, 4], alpha1 = 2^-5, alpha2 = 2^-7."""
    lin = {
        "T1": make_trits(N, K, *key, 21), "T2": make_trits(N, K, *key, 22),
        "a1": np.full((N, K // group), 2.0 ** -5, dtype=np.float16),
        "a2": np.full((N, K // group), 2.0 ** -7, dtype=np.float16),
        "N": N, "K": K, "group": group,
    }
    x = _rng(*key, 23).integers(-4, 5, size=(M, K)).astype(np.float16)
    return lin, x
