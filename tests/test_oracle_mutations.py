"""The finite-difference pin must notice plausible mistakes: each test plants one
in the oracle (on the CPU, via monkeypatch) and expects the pin to fail."""
import numpy as np
import pytest

from lf_inputs import make_net
from oracle import backprop as O


def _fd_worst(L=4, N=4, B=2, seed=3):
    net = make_net(L, N, B, seed=seed, b_var=1.0)
    w = {l: net.w(l).astype(np.float64) * 3.0 for l in range(2, L + 1)}
    b = {l: net.b(l).astype(np.float64) for l in range(2, L + 1)}
    x, y = net.x().astype(np.float64), net.y().astype(np.float64)
    _, _, nb, nw, _ = O.full_pass(w, b, x, y, L)
    C = lambda: O.cost(O.forward(w, b, x, L)[L], y)
    h, worst = 1e-6, 0.0
    for l in range(2, L + 1):
        for idx in np.ndindex(N, N):
            w0 = w[l][idx]
            w[l][idx] = w0 + h; cp = C()
            w[l][idx] = w0 - h; cm = C()
            w[l][idx] = w0
            worst = max(worst, abs((cp - cm) / (2 * h) - nw[l][idx]))
        for j in range(N):
            b0 = b[l][j]
            b[l][j] = b0 + h; cp = C()
            b[l][j] = b0 - h; cm = C()
            b[l][j] = b0
            worst = max(worst, abs((cp - cm) / (2 * h) - nb[l][j]))
    return worst


def _forward_without_bias(w, b, x, L):
    a = {1: np.atleast_2d(np.asarray(x, float))}
    for l in range(2, L + 1):
        a[l] = O.sigmoid(a[l - 1] @ np.asarray(w[l], float).T)
    return a


def _forward_transposed(w, b, x, L):
    a = {1: np.atleast_2d(np.asarray(x, float))}
    for l in range(2, L + 1):
        a[l] = O.sigmoid(a[l - 1] @ np.asarray(w[l], float) + np.asarray(b[l], float))
    return a


def test_unmutated_oracle_passes():
    assert _fd_worst() < 2e-9


@pytest.mark.parametrize("name,mutant", [
    ("chain_step", lambda w_next, d, a_l: (d @ np.asarray(w_next, float).T) * a_l * (1 - a_l)),   # transposed w
    ("chain_step", lambda w_next, d, a_l: (d @ np.asarray(w_next, float)) * a_l),                  # sigma' truncated
    ("chain_step", lambda w_next, d, a_l: (d @ np.asarray(w_next, float)) * a_l * (1 + a_l)),      # sign
    ("weight_gradient", lambda d, a_prev: a_prev.T @ d),                                           # transposed nabla_w
    ("weight_gradient", lambda d, a_prev: d.T @ a_prev / d.shape[0]),                              # mean, not sum
    ("bias_gradient", lambda d: d.mean(axis=0)),
    ("output_error", lambda aL, y: (aL - np.atleast_2d(y))),                                       # sigma' dropped
    ("output_error", lambda aL, y: (np.atleast_2d(y) - aL) * aL * (1 - aL)),                       # sign
    ("sigmoid", lambda z: 1.0 / (1.0 + np.exp(z))),      # sigma(-z): its derivative is -a(1-a), the oracle's sigma' is then wrong
    ("forward", _forward_without_bias),                  # eq. (z) as printed: then dC/db = 0, not delta
    ("forward", _forward_transposed),                    # w^l used as its transpose
])
def test_planted_mistake_is_caught(monkeypatch, name, mutant):
    monkeypatch.setattr(O, name, mutant)
    assert _fd_worst() > 1e-4


def _first_order_defect(eta=1e-4, L=4, N=5, B=2, seed=8):
    """|(C(theta) - C(theta')) / eta - ||g||^2| / ||g||^2 for theta' = the oracle's descent step."""
    net = make_net(L, N, B, seed=seed, b_var=1.0)
    w = {l: net.w(l).astype(np.float64) * 3.0 for l in range(2, L + 1)}
    b = {l: net.b(l).astype(np.float64) for l in range(2, L + 1)}
    x, y = net.x().astype(np.float64), net.y().astype(np.float64)
    _, _, nb, nw, c0 = O.full_pass(w, b, x, y, L)
    g2 = sum(float(np.sum(nw[l] ** 2)) + float(np.sum(nb[l] ** 2)) for l in range(2, L + 1))
    w1, b1 = O.sgd_step(w, b, nw, nb, eta, L)
    c1 = O.cost(O.forward(w1, b1, x, L)[L], y)
    return abs((c0 - c1) / eta - g2) / g2


def test_unmutated_descent_step_passes():
    assert _first_order_defect() < 3e-3


@pytest.mark.parametrize("mutant", [
    lambda w, b, nw, nb, eta, L: ({l: w[l] + eta * nw[l] for l in w}, {l: b[l] - eta * nb[l] for l in b}),   # sign of the weight step
    lambda w, b, nw, nb, eta, L: ({l: w[l] - eta * nw[l] for l in w}, {l: b[l] for l in b}),                # biases left alone
    lambda w, b, nw, nb, eta, L: ({l: w[l] - 0.5 * eta * nw[l] for l in w}, {l: b[l] - eta * nb[l] for l in b}),  # a factor
    lambda w, b, nw, nb, eta, L: ({l: w[l] - eta * nw[l].T for l in w}, {l: b[l] - eta * nb[l] for l in b}),    # transposed gradient
])
def test_planted_mistake_in_the_descent_step_is_caught(monkeypatch, mutant):
    monkeypatch.setattr(O, "sgd_step", mutant)
    assert _first_order_defect() > 2e-2
