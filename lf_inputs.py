"""Seeded synthetic inputs for the sigmoid-MLP backpropagation path.

This module only draws random tensors (weights w^l, biases b^l, input x^1,
target y) with the shapes and distributions of the benchmark configurations.
It contains none of the method's arithmetic: no forward pass, no gradient.
Both the CPU oracle's tests and the GPU path's tests/benchmark take their
inputs from here so that the two sides see identical bits.

Notation follows the paper (section 2): layers are numbered 1..L, a^1 = x^1,
weights and biases exist for l = 2..L, every layer has N neurons, and
w^l is N x N with w^l[j][k] the weight from neuron k of layer l-1 into
neuron j of layer l.  A minibatch of B samples is stored sample-major:
x[b][n].  A spec may instead give every layer its own width n_l (the
paper's equations hold for any widths); w^l is then n_l x n_{l-1}.

Distributions: w^l ~ N(0, var=1/n_{l-1}), b^l ~ N(0, var=b_var), x, y ~ U[0,1).
The second argument of N(.,.) is read as a variance throughout.

Every tensor has its own random stream, keyed by
(seed, kind, layer), so a single layer of a large net can be drawn without
drawing the others.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Tuple

import numpy as np

_KIND_W, _KIND_B, _KIND_X, _KIND_Y = 1, 2, 3, 4


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bfloat16 (ties to even) and return
    them as fp32 (low 16 bits zero).  NaN/Inf do not occur in these inputs."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


@dataclass(frozen=True)
class NetSpec:
    """Shape, storage type and init of one configuration."""
    name: str
    L: int            # layers 1..L  (L-1 weight matrices)
    N: int            # neurons per layer
    B: int            # minibatch size (1 = the paper's single-sample case)
    dtype: str        # "f32" or "bf16": storage type of w, x, y and a^l
    ks: Tuple[int, ...]   # worker counts k the configuration is run with
    b_var: float      # variance of the bias init
    seed: int = 0
    widths: Tuple[int, ...] = ()   # neurons of layers 1..L when they differ; empty = N everywhere

    def width(self, l: int) -> int:
        """Neurons of layer l, l = 1..L."""
        return self.widths[l - 1] if self.widths else self.N


# The five benchmark configurations.
CONFIGS: Dict[str, NetSpec] = {
    "cfg1": NetSpec("cfg1", L=8, N=256, B=1, dtype="f32", ks=(2,), b_var=1.0),
    "cfg2": NetSpec("cfg2", L=32, N=1024, B=1, dtype="f32", ks=(1, 2, 4, 8), b_var=0.1),
    "cfg3": NetSpec("cfg3", L=64, N=4096, B=1, dtype="f32", ks=(1, 4, 8), b_var=0.1),
    "cfg4": NetSpec("cfg4", L=32, N=4096, B=256, dtype="f32", ks=(4,), b_var=0.1),
    "cfg5": NetSpec("cfg5", L=48, N=8192, B=512, dtype="bf16", ks=(8,), b_var=0.1),
}


class SyntheticNet:
    """Lazily drawn tensors of one net.  `w(l)`, `b(l)` take the paper's layer
    index l in 2..L.  All arrays are fp32; for dtype "bf16" the values of w, x
    and y are exactly representable in bfloat16 (b stays fp32)."""

    def __init__(self, spec: NetSpec, cache: bool = False):
        if spec.L < 2 or spec.N < 1 or spec.B < 1:
            raise ValueError("need L >= 2, N >= 1, B >= 1")
        if spec.dtype not in ("f32", "bf16"):
            raise ValueError("dtype must be 'f32' or 'bf16'")
        if spec.widths and (len(spec.widths) != spec.L or min(spec.widths) < 1):
            raise ValueError("widths needs one positive entry per layer")
        self.spec = spec
        self._cache = {} if cache else None

    def _rng(self, kind: int, layer: int) -> np.random.Generator:
        return np.random.default_rng([self.spec.seed, kind, layer])

    def _store(self, a: np.ndarray) -> np.ndarray:
        return round_to_bf16(a) if self.spec.dtype == "bf16" else a

    def _memo(self, key, make):
        if self._cache is None:
            return make()
        if key not in self._cache:
            self._cache[key] = make()
        return self._cache[key]

    def _check_layer(self, l: int) -> None:
        if not 2 <= l <= self.spec.L:
            raise IndexError(f"layer {l} has no weights (valid: 2..{self.spec.L})")

    def w(self, l: int) -> np.ndarray:
        self._check_layer(l)
        rows, cols = self.spec.width(l), self.spec.width(l - 1)

        def make():
            g = self._rng(_KIND_W, l).standard_normal((rows, cols), dtype=np.float32)
            g *= np.float32(1.0 / np.sqrt(cols))
            return self._store(g)
        return self._memo(("w", l), make)

    def b(self, l: int) -> np.ndarray:
        self._check_layer(l)

        def make():
            g = self._rng(_KIND_B, l).standard_normal(self.spec.width(l), dtype=np.float32)
            g *= np.float32(np.sqrt(self.spec.b_var))
            return g
        return self._memo(("b", l), make)

    def x(self) -> np.ndarray:
        s = self.spec
        return self._memo(("x", 0), lambda: self._store(
            self._rng(_KIND_X, 0).random((s.B, s.width(1)), dtype=np.float32)))

    def y(self) -> np.ndarray:
        s = self.spec
        return self._memo(("y", 0), lambda: self._store(
            self._rng(_KIND_Y, 0).random((s.B, s.width(s.L)), dtype=np.float32)))

    # Views indexable by the paper's layer index, for code that wants w[l], b[l].
    class _ByLayer:
        def __init__(self, fn, L):
            self._fn, self._L = fn, L

        def __getitem__(self, l):
            return self._fn(l)

        def keys(self):
            return range(2, self._L + 1)

    @property
    def w_by_layer(self):
        return SyntheticNet._ByLayer(self.w, self.spec.L)

    @property
    def b_by_layer(self):
        return SyntheticNet._ByLayer(self.b, self.spec.L)


def make_net(L: int, N, B: int = 1, dtype: str = "f32", b_var: float = 0.1,
             seed: int = 0, cache: bool = True, name: str = "custom") -> SyntheticNet:
    """A net of arbitrary shape with the configurations' init recipe.  N: the neurons of every layer, or a
    sequence of L widths (layer 1 first)."""
    if isinstance(N, int):
        return SyntheticNet(NetSpec(name, L, N, B, dtype, (1,), b_var, seed), cache=cache)
    widths = tuple(int(v) for v in N)
    return SyntheticNet(NetSpec(name, L, max(widths), B, dtype, (1,), b_var, seed, widths), cache=cache)


def config_net(name: str, cache: bool = False) -> SyntheticNet:
    return SyntheticNet(CONFIGS[name], cache=cache)
