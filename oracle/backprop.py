"""CPU oracle for one backpropagation pass of an L-layer sigmoid MLP.

TEST INFRASTRUCTURE ONLY.  This is the slow, plain reference that the GPU
library is checked against.  Only tests, the smoke check and the benchmark's
cpu-baseline leg may import it; no product code path may call it, and it
imports nothing from the GPU package.

Everything is fp64 numpy, one library call (a matrix product) per equation,
no blocking, no fusion.  Notation is the paper's (section 2): layers 1..L,
a^1 = x^1, weights w^l (N x N, w^l[j][k] = weight into neuron j of layer l
from neuron k of layer l-1) and biases b^l for l = 2..L.  A minibatch is
stored sample-major: a^l has shape (B, N), row b is sample b, so
"w^l a^{l-1}" for all samples at once is  a_prev @ w.T .
Nothing here assumes equal widths (the paper fixes N per layer for its cost
analysis only): every product takes its shape from w^l, which may be
n_l x n_{l-1}.

Arguments `w` and `b` are indexable by the paper's layer index (w[l] for
l = 2..L): a dict, or any object with __getitem__.  Entries of any float type
are widened exactly to fp64; nothing is rounded in between.

Readings of the paper taken here (where it is silent or inconsistent):
  * eq. (z) is printed without the bias, but b^l is defined and eq. (bp3)
    says dC/db^l = delta^l, which only holds if z^l = w^l a^{l-1} + b^l.
    That form is used.
  * sigma(z) = 1/(1+exp(-z)), sigma'(z) = sigma(z)(1 - sigma(z)).
  * the cost is quadratic, C = 1/2 sum_b ||a^L_b - y_b||^2 (summed over the
    minibatch, not averaged), so nabla_a^L C = a^L - y.
  * with a minibatch, eqs. (bp3) and (bp4) are summed over the samples.
  * Algorithm 1 as printed never applies (bp3),(bp4) at layer L (its first
    loop starts at L-1) while the proof of Theorem 1 says the parent covers
    every level above L-k; the parent therefore also does layer L here.

Pins (tests/test_oracle_pins.py): central finite differences of C for every
weight and bias of tiny nets; an fp64 autograd cross-check; the one-layer
closed form; the all-zero-weights closed form; the rank-one symmetric net
whose pass collapses to a scalar recurrence at any N; hand-computed values;
Algorithm 1 run literally equals the sequential pass bit for bit for every k;
finite differences and Algorithm 1 = sequential again for unequal widths;
the descent step by the first-order decrease of C it must produce.
"""
from __future__ import annotations

from typing import Dict, Iterator, List, Tuple

import numpy as np

F64 = np.float64


def _f64(a) -> np.ndarray:
    return np.asarray(a, dtype=F64)


def sigmoid(z: np.ndarray) -> np.ndarray:
    """sigma(z) = 1 / (1 + e^{-z})  (section 2; the paper names it only)."""
    with np.errstate(over="ignore"):
        return 1.0 / (1.0 + np.exp(-z))


def sigmoid_prime_from_a(a: np.ndarray) -> np.ndarray:
    """sigma'(z) written through a = sigma(z):  sigma' = a (1 - a)."""
    return a * (1.0 - a)


def forward(w, b, x, L: int) -> Dict[int, np.ndarray]:
    """Eqs. (x), (z), (a): a^1 = x^1;  z^l = w^l a^{l-1} + b^l;  a^l = sigma(z^l).

    x: (B, N).  Returns {l: a^l} for l = 1..L, each (B, N) fp64."""
    a = {1: np.atleast_2d(_f64(x))}
    for l in range(2, L + 1):
        z = a[l - 1] @ _f64(w[l]).T + _f64(b[l])[None, :]
        a[l] = sigmoid(z)
    return a


def cost(aL: np.ndarray, y) -> float:
    """Quadratic cost summed over the minibatch: C = 1/2 sum (a^L - y)^2."""
    d = aL - np.atleast_2d(_f64(y))
    return 0.5 * float(np.sum(d * d))


def output_error(aL: np.ndarray, y) -> np.ndarray:
    """Eq. (bp1): delta^L = nabla_a^L C (.) sigma'(z^L), with nabla_a^L C = a^L - y."""
    return (aL - np.atleast_2d(_f64(y))) * sigmoid_prime_from_a(aL)


def chain_step(w_next, delta_next: np.ndarray, a_l: np.ndarray) -> np.ndarray:
    """Eq. (bp2): delta^l = ((w^{l+1})^T delta^{l+1}) (.) sigma'(z^l).

    For sample b: ((w^{l+1})^T delta)[k] = sum_j w^{l+1}[j][k] delta[b][j]."""
    return (delta_next @ _f64(w_next)) * sigmoid_prime_from_a(a_l)


def bias_gradient(delta_l: np.ndarray) -> np.ndarray:
    """Eq. (bp3): dC/db^l_j = delta^l_j, summed over the samples."""
    return delta_l.sum(axis=0)


def weight_gradient(delta_l: np.ndarray, a_prev: np.ndarray) -> np.ndarray:
    """Eq. (bp4): dC/dw^l_jk = a^{l-1}_k delta^l_j, summed over the samples."""
    return delta_l.T @ a_prev


def backward_layers(w, a: Dict[int, np.ndarray], y, L: int,
                    want_nabla_w: bool = True
                    ) -> Iterator[Tuple[int, np.ndarray, np.ndarray, np.ndarray]]:
    """Sequential backward pass, yielding (l, delta^l, nabla_b^l, nabla_w^l)
    for l = L, L-1, ..., 2.  One layer's nabla_w is alive at a time so that
    large nets can be compared layer by layer."""
    delta = output_error(a[L], y)
    for l in range(L, 1, -1):
        if l < L:
            delta = chain_step(w[l + 1], delta, a[l])
        nw = weight_gradient(delta, a[l - 1]) if want_nabla_w else None
        yield l, delta, bias_gradient(delta), nw


def backward_sequential(w, a, y, L: int):
    """The plain pass (one worker).  Returns (delta, nabla_b, nabla_w), each a
    dict over l = 2..L."""
    delta, nb, nw = {}, {}, {}
    for l, d, gb, gw in backward_layers(w, a, y, L):
        delta[l], nb[l], nw[l] = d, gb, gw
    return delta, nb, nw


def backward_algorithm1(w, a, y, L: int, k: int):
    """Algorithm 1 ("Backpropagation with threads") carried out as written,
    the k threads run one after the other.

    The parent applies (bp1), then (bp2),(bp3),(bp4) at the k-1 layers below
    L, and hands thread j the error delta^{L-j}.  Every thread walks the
    whole remaining delta chain on its own (recomputing it) in blocks of k
    layers and applies (bp3),(bp4) only at the last layer of each block.

    Returns (nabla_b, nabla_w, owner, writes): owner[l] is "parent" or the
    thread number that saved layer l's gradients, writes[l] how many times
    they were saved (Theorem 1 claims exactly once for every layer)."""
    if not 1 <= k <= L - 1:
        raise ValueError("Algorithm 1 needs 1 <= k <= L-1")
    nb: Dict[int, np.ndarray] = {}
    nw: Dict[int, np.ndarray] = {}
    owner: Dict[int, object] = {}
    writes: Dict[int, int] = {l: 0 for l in range(2, L + 1)}

    def save(l, delta_l, who):
        nb[l] = bias_gradient(delta_l)
        nw[l] = weight_gradient(delta_l, a[l - 1])
        owner[l] = who
        writes[l] += 1

    # parent
    seeds = {L: output_error(a[L], y)}
    save(L, seeds[L], "parent")          # reading: the parent also does layer L
    for i in range(L - 1, L - k, -1):    # i = L-1, ..., L-k+1
        seeds[i] = chain_step(w[i + 1], seeds[i + 1], a[i])
        save(i, seeds[i], "parent")

    # Thread t is handed delta^{L-t}.  Its own layers are every k-th one below that: L-t-k, L-t-2k, ... down
    # to layer 2 at the lowest.  To reach the next of them it walks the k chain steps in between by itself
    # (so every thread recomputes the chain) and saves the gradients only where it arrives.
    for t in range(k):
        held = L - t                         # the layer whose delta the thread holds
        delta = seeds[held]
        for own in range(held - k, 1, -k):
            for l in range(held - 1, own - 1, -1):
                delta = chain_step(w[l + 1], delta, a[l])
            save(own, delta, t)
            held = own
    return nb, nw, owner, writes


def worker_of_layer(L: int, k: int) -> Dict[int, int]:
    """Which of the k interleaved workers saves layer l's gradients when
    Algorithm 1's thread rule is extended to the parent's layers as well:
    running the algorithm's index arithmetic (no numerics) shows thread t
    owns l = L-k-t-mk, i.e. (L-l) mod k == t; the same formula is used for
    the top k layers."""
    owner = {}
    for t in range(k):
        for own in range(L - t - k, 1, -k):      # the thread's layers: every k-th one below delta^{L-t}
            owner[own] = t
    for l in range(L, max(L - k, 1), -1):
        owner[l] = (L - l) % k
    return owner


def full_pass(w, b, x, y, L: int):
    """Forward then sequential backward.  Returns (a, delta, nabla_b, nabla_w, C)."""
    a = forward(w, b, x, L)
    delta, nb, nw = backward_sequential(w, a, y, L)
    return a, delta, nb, nw, cost(a[L], y)


def sgd_step(w, b, nabla_w, nabla_b, eta: float, L: int):
    """Plain gradient descent, the step that consumes (bp3),(bp4) (the paper itself stops at the gradients):
    w^l <- w^l - eta nabla_w^l,  b^l <- b^l - eta nabla_b^l  for l = 2..L.  Returns new dicts (w, b)."""
    w1 = {l: _f64(w[l]) - eta * nabla_w[l] for l in range(2, L + 1)}
    b1 = {l: _f64(b[l]) - eta * nabla_b[l] for l in range(2, L + 1)}
    return w1, b1


def normwise_error(got, want) -> float:
    """max|got - want| / max|want|  (0/0 := 0).  The error measure used for
    every tensor comparison against this oracle."""
    want = _f64(want)
    diff = float(np.max(np.abs(_f64(got) - want))) if want.size else 0.0
    scale = float(np.max(np.abs(want))) if want.size else 0.0
    if scale == 0.0:
        return 0.0 if diff == 0.0 else float("inf")
    return diff / scale
