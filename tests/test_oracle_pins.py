"""Pins for the CPU oracle: what the paper and the mathematics fix, with no
implementation to compare against.  Each test is chosen so that a plausible
mistake in oracle/backprop.py (a dropped term, a wrong sign or index, a
transposed operand, a missing bias) fails at least one of them."""
import math

import numpy as np
import pytest

from lf_inputs import make_net
from oracle import backprop as O


def _net(L, N, B, seed=0, b_var=1.0):
    net = make_net(L, N, B, seed=seed, b_var=b_var)
    w = {l: net.w(l).astype(np.float64) * 3.0 for l in range(2, L + 1)}  # larger weights: less symmetric
    b = {l: net.b(l).astype(np.float64) for l in range(2, L + 1)}
    return w, b, net.x().astype(np.float64), net.y().astype(np.float64)


def _C(w, b, x, y, L):
    return O.cost(O.forward(w, b, x, L)[L], y)


# ---------------------------------------------------------------- finite differences
@pytest.mark.parametrize("L,N,B", [(2, 3, 1), (3, 2, 1), (4, 5, 1), (5, 3, 3), (3, 8, 2)])
def test_gradients_match_central_finite_differences(L, N, B):
    """(bp1)-(bp4) are the chain rule of C through (z),(a): every dC/dw^l_jk and
    dC/db^l_j must equal a central difference of C (section 2)."""
    w, b, x, y = _net(L, N, B, seed=L * 100 + N)
    _, _, nb, nw, _ = O.full_pass(w, b, x, y, L)
    h = 1e-6
    worst = 0.0
    for l in range(2, L + 1):
        for j in range(N):
            for k in range(N):
                w0 = w[l][j, k]
                w[l][j, k] = w0 + h
                cp = _C(w, b, x, y, L)
                w[l][j, k] = w0 - h
                cm = _C(w, b, x, y, L)
                w[l][j, k] = w0
                fd = (cp - cm) / (2 * h)
                worst = max(worst, abs(fd - nw[l][j, k]))
            b0 = b[l][j]
            b[l][j] = b0 + h
            cp = _C(w, b, x, y, L)
            b[l][j] = b0 - h
            cm = _C(w, b, x, y, L)
            b[l][j] = b0
            fd = (cp - cm) / (2 * h)
            worst = max(worst, abs(fd - nb[l][j]))
    assert worst < 2e-9, worst


@pytest.mark.parametrize("widths,B", [((3, 5, 2), 1), ((4, 2, 6, 3), 2), ((2, 7), 3), ((5, 1, 4, 1, 3), 1)])
def test_gradients_of_nets_with_unequal_widths_match_finite_differences(widths, B):
    """Section 2 fixes N neurons per layer for its cost analysis only; the equations hold for any widths.
    With w^l of shape n_l x n_{l-1} a transposed operand does not even have the right shape, and every
    dC/dw^l_jk, dC/db^l_j must still equal a central difference of C."""
    L = len(widths)
    net = make_net(L, widths, B, seed=sum(widths), b_var=1.0)
    w = {l: net.w(l).astype(np.float64) * 2.0 for l in range(2, L + 1)}
    b = {l: net.b(l).astype(np.float64) for l in range(2, L + 1)}
    x, y = net.x().astype(np.float64), net.y().astype(np.float64)
    assert x.shape == (B, widths[0]) and y.shape == (B, widths[-1])
    a, delta, nb, nw, _ = O.full_pass(w, b, x, y, L)
    h = 1e-6
    worst = 0.0
    for l in range(2, L + 1):
        assert w[l].shape == (widths[l - 1], widths[l - 2]) == nw[l].shape
        assert a[l].shape == delta[l].shape == (B, widths[l - 1]) and nb[l].shape == (widths[l - 1],)
        for j in range(widths[l - 1]):
            for k in range(widths[l - 2]):
                w0 = w[l][j, k]
                w[l][j, k] = w0 + h
                cp = _C(w, b, x, y, L)
                w[l][j, k] = w0 - h
                cm = _C(w, b, x, y, L)
                w[l][j, k] = w0
                worst = max(worst, abs((cp - cm) / (2 * h) - nw[l][j, k]))
            b0 = b[l][j]
            b[l][j] = b0 + h
            cp = _C(w, b, x, y, L)
            b[l][j] = b0 - h
            cm = _C(w, b, x, y, L)
            b[l][j] = b0
            worst = max(worst, abs((cp - cm) / (2 * h) - nb[l][j]))
    assert worst < 2e-9, worst


def test_unequal_widths_algorithm1_equals_sequential():
    """Theorem 1 does not depend on the widths: Algorithm 1 run literally gives the sequential pass's bits."""
    widths = (6, 3, 8, 2, 5, 4, 7)
    L = len(widths)
    net = make_net(L, widths, 2, seed=11)
    w, b = net.w_by_layer, net.b_by_layer
    a = O.forward(w, b, net.x(), L)
    _, nb, nw = O.backward_sequential(w, a, net.y(), L)
    for k in range(1, L):
        nb1, nw1, _, writes = O.backward_algorithm1(w, a, net.y(), L, k)
        assert all(writes[l] == 1 for l in range(2, L + 1))
        for l in range(2, L + 1):
            assert np.array_equal(nb[l], nb1[l]) and np.array_equal(nw[l], nw1[l])


def test_delta_is_dC_dz():
    """delta^l = dC/dz^l (the definition behind (bp1),(bp2)): perturb b^l, which
    enters z^l additively, one neuron and one layer at a time; B = 1."""
    L, N = 4, 4
    w, b, x, y = _net(L, N, 1, seed=7)
    _, delta, _, _, _ = O.full_pass(w, b, x, y, L)
    h = 1e-6
    for l in range(2, L + 1):
        for j in range(N):
            b[l][j] += h
            cp = _C(w, b, x, y, L)
            b[l][j] -= 2 * h
            cm = _C(w, b, x, y, L)
            b[l][j] += h
            assert abs((cp - cm) / (2 * h) - delta[l][0, j]) < 2e-9


# ---------------------------------------------------------------- identity (bp3),(bp4)
def test_outer_product_identity_single_sample():
    """(bp4): nabla_w^l[j][k] = a^{l-1}_k delta^l_j, (bp3): nabla_b^l = delta^l.
    Index order matters: a transposed nabla_w fails (a and delta differ)."""
    L, N = 5, 6
    w, b, x, y = _net(L, N, 1, seed=3)
    a, delta, nb, nw, _ = O.full_pass(w, b, x, y, L)
    for l in range(2, L + 1):
        for j in range(N):
            assert nb[l][j] == delta[l][0, j]
            for k in range(N):
                assert nw[l][j, k] == a[l - 1][0, k] * delta[l][0, j]


def test_minibatch_is_sum_of_single_samples():
    """Samples are independent; C is a sum over them, so are its gradients."""
    L, N, B = 4, 5, 4
    w, b, x, y = _net(L, N, B, seed=11)
    _, _, nb, nw, C = O.full_pass(w, b, x, y, L)
    nb_s = {l: 0.0 for l in nb}
    nw_s = {l: 0.0 for l in nw}
    C_s = 0.0
    for s in range(B):
        _, _, nb1, nw1, C1 = O.full_pass(w, b, x[s:s + 1], y[s:s + 1], L)
        C_s += C1
        for l in nb:
            nb_s[l] = nb_s[l] + nb1[l]
            nw_s[l] = nw_s[l] + nw1[l]
    assert abs(C - C_s) < 1e-14
    for l in nb:
        np.testing.assert_allclose(nb[l], nb_s[l], rtol=0, atol=1e-15)
        np.testing.assert_allclose(nw[l], nw_s[l], rtol=0, atol=1e-15)


# ---------------------------------------------------------------- closed forms
def test_hand_computed_one_neuron():
    """L=2, N=1, w=0, b=0: a^2 = 1/2, sigma' = 1/4, delta = (1/2 - y)/4,
    nabla_w = delta * x, C = (1/2 - y)^2 / 2.  With y = 0, x = 0.8:
    delta = 0.125, nabla_w = 0.1, C = 0.125."""
    a, delta, nb, nw, C = O.full_pass({2: [[0.0]]}, {2: [0.0]}, [[0.8]], [[0.0]], 2)
    assert a[2][0, 0] == 0.5
    assert delta[2][0, 0] == 0.125
    assert nb[2][0] == 0.125
    assert nw[2][0, 0] == pytest.approx(0.1, abs=1e-17)
    assert C == 0.125


def test_exact_small_cases_from_golden_file():
    """tests/golden/exact_small_cases.txt: values derived by hand from eqs. (z),(a),(bp1)-(bp4) for nets
    with all-zero parameters (every activation exactly 1/2, every sigma' exactly 1/4)."""
    import os
    want = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "exact_small_cases.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            case, name, *vals = line.split()
            want[(case, name)] = np.array([float(v) for v in vals])
    z1 = {2: np.zeros((1, 1))}
    a, delta, nb, nw, C = O.full_pass(z1, {2: np.zeros(1)}, [[0.8]], [[0.0]], 2)
    got = {("one_neuron", "a2"): a[2], ("one_neuron", "delta2"): delta[2], ("one_neuron", "nabla_b2"): nb[2],
           ("one_neuron", "nabla_w2"): nw[2], ("one_neuron", "C"): C}
    w = {2: np.zeros((2, 2)), 3: np.zeros((2, 2))}
    b = {2: np.zeros(2), 3: np.zeros(2)}
    a, delta, nb, nw, C = O.full_pass(w, b, [[1.0, 0.5]], [[0.0, 1.0]], 3)
    got.update({("two_by_two", "delta3"): delta[3], ("two_by_two", "delta2"): delta[2],
                ("two_by_two", "nabla_w3"): nw[3], ("two_by_two", "nabla_b3"): nb[3],
                ("two_by_two", "nabla_w2"): nw[2], ("two_by_two", "C"): C})
    a, delta, nb, nw, C = O.full_pass(z1, {2: np.zeros(1)}, [[0.8], [0.4]], [[0.0], [1.0]], 2)
    got.update({("two_samples", "nabla_b2"): nb[2], ("two_samples", "nabla_w2"): nw[2], ("two_samples", "C"): C})
    assert set(got) == set(want)
    for key, v in want.items():
        g = np.asarray(got[key], dtype=np.float64).reshape(-1)
        assert g.shape == v.shape, key
        assert np.allclose(g, v, rtol=0, atol=1e-16), (key, g, v)


def test_hand_computed_two_layers_scalar():
    """L=3, N=1, scalar chain written out with math.exp only."""
    w2, w3, b2, b3, x, y = 0.7, -1.3, 0.2, 0.4, 0.9, 0.25
    s = lambda t: 1.0 / (1.0 + math.exp(-t))
    a2 = s(w2 * x + b2)
    a3 = s(w3 * a2 + b3)
    d3 = (a3 - y) * a3 * (1 - a3)
    d2 = w3 * d3 * a2 * (1 - a2)
    a, delta, nb, nw, C = O.full_pass({2: [[w2]], 3: [[w3]]}, {2: [b2], 3: [b3]}, [[x]], [[y]], 3)
    assert a[3][0, 0] == pytest.approx(a3, rel=1e-15)
    assert delta[3][0, 0] == pytest.approx(d3, rel=1e-14)
    assert delta[2][0, 0] == pytest.approx(d2, rel=1e-14)
    assert nw[3][0, 0] == pytest.approx(d3 * a2, rel=1e-14)
    assert nw[2][0, 0] == pytest.approx(d2 * x, rel=1e-14)
    assert nb[2][0] == pytest.approx(d2, rel=1e-14)
    assert C == pytest.approx(0.5 * (a3 - y) ** 2, rel=1e-14)


def test_single_weight_layer_closed_form():
    """L=2: nabla_w^2 = ((sigma(w x + b) - y) (.) sigma') x^T, a one-line formula
    written here with explicit loops over j, k (no matrix product)."""
    N = 7
    w, b, x, y = _net(2, N, 1, seed=5)
    _, _, nb, nw, _ = O.full_pass(w, b, x, y, 2)
    for j in range(N):
        z = sum(w[2][j, k] * x[0, k] for k in range(N)) + b[2][j]
        aj = 1.0 / (1.0 + math.exp(-z))
        dj = (aj - y[0, j]) * aj * (1 - aj)
        assert nb[2][j] == pytest.approx(dj, rel=1e-12)
        for k in range(N):
            assert nw[2][j, k] == pytest.approx(dj * x[0, k], rel=1e-12)


def test_all_zero_weights():
    """w^l = 0 for all l: a^l = sigma(b^l); delta^l = 0 and nabla_w^l = 0 below L;
    nabla_w^L = ((sigma(b^L) - y) (.) sigma'(b^L)) sigma(b^{L-1})^T."""
    L, N = 4, 5
    _, b, x, y = _net(L, N, 1, seed=9)
    w = {l: np.zeros((N, N)) for l in range(2, L + 1)}
    a, delta, nb, nw, _ = O.full_pass(w, b, x, y, L)
    sig = lambda t: 1.0 / (1.0 + np.exp(-t))
    for l in range(2, L):
        assert np.all(delta[l] == 0) and np.all(nw[l] == 0) and np.all(nb[l] == 0)
        np.testing.assert_allclose(a[l][0], sig(b[l]), rtol=1e-15)
    aL = sig(b[L])
    dL = (aL - y[0]) * aL * (1 - aL)
    np.testing.assert_allclose(nw[L], np.outer(dL, sig(b[L - 1])), rtol=1e-13)
    np.testing.assert_allclose(nb[L], dL, rtol=1e-13)


@pytest.mark.parametrize("L,N", [(6, 4), (12, 64), (5, 1024)])
def test_rank_one_symmetric_net_scalar_recurrence(L, N):
    """w^l = (c/N) 1 1^T, b^l = beta 1, x = xi 1, y = eta 1  =>  a^l = alpha_l 1 with
    alpha_l = sigma(c alpha_{l-1} + beta); delta^l = d_l 1 with
    d_L = (alpha_L - eta) alpha_L (1 - alpha_L),  d_l = c d_{l+1} alpha_l (1 - alpha_l);
    nabla_w^l = d_l alpha_{l-1} 1 1^T.  Holds for any N, so it checks full-length
    reductions against a scalar recurrence."""
    c, beta, xi, eta = 1.7, -0.3, 0.6, 0.2
    w = {l: np.full((N, N), c / N) for l in range(2, L + 1)}
    b = {l: np.full(N, beta) for l in range(2, L + 1)}
    x = np.full((1, N), xi)
    y = np.full((1, N), eta)
    a, delta, nb, nw, _ = O.full_pass(w, b, x, y, L)
    alpha = {1: xi}
    for l in range(2, L + 1):
        alpha[l] = 1.0 / (1.0 + math.exp(-(c * alpha[l - 1] + beta)))
    d = {L: (alpha[L] - eta) * alpha[L] * (1 - alpha[L])}
    for l in range(L - 1, 1, -1):
        d[l] = c * d[l + 1] * alpha[l] * (1 - alpha[l])
    for l in range(2, L + 1):
        np.testing.assert_allclose(a[l], alpha[l], rtol=1e-12)
        np.testing.assert_allclose(delta[l], d[l], rtol=1e-10)
        np.testing.assert_allclose(nb[l], d[l], rtol=1e-10)
        np.testing.assert_allclose(nw[l], d[l] * alpha[l - 1], rtol=1e-10)


# ---------------------------------------------------------------- library cross-check
@pytest.mark.parametrize("L,N,B", [(4, 16, 1), (6, 33, 5)])
def test_matches_fp64_autograd(L, N, B):
    """A differently-built derivative (reverse-mode autodiff of the same cost in a
    tensor library) agrees to rounding."""
    import torch
    w, b, x, y = _net(L, N, B, seed=21)
    tw = {l: torch.tensor(w[l], dtype=torch.float64, requires_grad=True) for l in w}
    tb = {l: torch.tensor(b[l], dtype=torch.float64, requires_grad=True) for l in b}
    act = torch.tensor(x, dtype=torch.float64)
    for l in range(2, L + 1):
        act = torch.sigmoid(act @ tw[l].T + tb[l])
    C = 0.5 * ((act - torch.tensor(y)) ** 2).sum()
    C.backward()
    _, _, nb, nw, Co = O.full_pass(w, b, x, y, L)
    assert Co == pytest.approx(C.item(), rel=1e-13)
    for l in range(2, L + 1):
        assert O.normwise_error(nw[l], tw[l].grad.numpy()) < 1e-12
        assert O.normwise_error(nb[l], tb[l].grad.numpy()) < 1e-12


# ---------------------------------------------------------------- Algorithm 1 / Theorem 1
@pytest.mark.parametrize("L", [2, 3, 5, 8, 13])
def test_algorithm1_equals_sequential_for_every_k(L):
    """Theorem 1: the threaded algorithm computes the same (bp3),(bp4) at every
    layer; each layer is saved exactly once.  The comparison is bitwise: both
    modes apply the same operation to the same operands."""
    N, B = 6, 2
    w, b, x, y = _net(L, N, B, seed=L)
    a = O.forward(w, b, x, L)
    _, nb, nw = O.backward_sequential(w, a, y, L)
    for k in range(1, L):
        nb1, nw1, owner, writes = O.backward_algorithm1(w, a, y, L, k)
        assert sorted(nw1) == list(range(2, L + 1))
        assert all(c == 1 for c in writes.values()), (k, writes)
        for l in range(2, L + 1):
            assert np.array_equal(nb1[l], nb[l]) and np.array_equal(nw1[l], nw[l])
        # the parent owns the top k layers, thread t the layers with (L-l) mod k == t
        sched = O.worker_of_layer(L, k)
        for l in range(2, L + 1):
            if l > L - k:
                assert owner[l] == "parent"
            else:
                assert owner[l] == (L - l) % k == sched[l]


def test_algorithm1_rejects_bad_k():
    w, b, x, y = _net(4, 3, 1)
    a = O.forward(w, b, x, 4)
    for k in (0, 4, 9):
        with pytest.raises(ValueError):
            O.backward_algorithm1(w, a, y, 4, k)


@pytest.mark.parametrize("L", range(2, 40))
def test_schedule_is_a_partition(L):
    for k in range(1, L):
        sched = O.worker_of_layer(L, k)
        assert sorted(sched) == list(range(2, L + 1))
        assert all(0 <= t < k for t in sched.values())
        assert all(sched[l] == (L - l) % k for l in sched)


# ---------------------------------------------------------------- sanity of the workloads
def test_vanishing_gradient_rate_of_the_configs_init():
    """With the configurations' init, sigma' averages about 0.23 and |delta| shrinks
    by roughly that factor per layer (a property of the workload, used to size
    tolerances for deep fp32 nets)."""
    L, N = 16, 256
    net = make_net(L, N, 1, b_var=0.1, seed=0)
    a, delta, _, _, _ = O.full_pass(net.w_by_layer, net.b_by_layer, net.x(), net.y(), L)
    ratios = [np.abs(delta[l]).max() / np.abs(delta[l + 1]).max() for l in range(2, L)]
    assert 0.1 < np.exp(np.mean(np.log(ratios))) < 0.45


def test_descent_step_decreases_the_cost_to_first_order():
    """C(w - eta g, b - eta g_b) = C - eta ||g||^2 + O(eta^2): the sign, the pairing of each gradient with its
    own parameter and the absence of any extra factor are all fixed by this limit."""
    L, N, B = 4, 6, 3
    w, b, x, y = _net(L, N, B, seed=3)
    _, _, nb, nw, c0 = O.full_pass(w, b, x, y, L)
    g2 = sum(float(np.sum(nw[l] ** 2)) + float(np.sum(nb[l] ** 2)) for l in range(2, L + 1))
    prev = None
    for eta in (1e-2, 1e-3, 1e-4):
        w1, b1 = O.sgd_step(w, b, nw, nb, eta, L)
        c1 = _C(w1, b1, x, y, L)
        assert c1 < c0
        rel = abs((c0 - c1) / eta - g2) / g2
        assert rel < 30 * eta                      # the remainder is O(eta)
        assert prev is None or rel < prev
        prev = rel
    # a swapped pairing (the bias step taken with the wrong layer's gradient) does not pass
    nb_wrong = {l: nb[L + 2 - l] for l in range(2, L + 1)}
    w1, b1 = O.sgd_step(w, b, nw, nb_wrong, 1e-4, L)
    assert abs((c0 - _C(w1, b1, x, y, L)) / 1e-4 - g2) / g2 > 1e-2
    # eta = 0 changes nothing; inputs are not modified
    w0, b0 = O.sgd_step(w, b, nw, nb, 0.0, L)
    assert all(np.array_equal(w0[l], w[l]) and np.array_equal(b0[l], b[l]) for l in range(2, L + 1))


def test_normwise_error():
    assert O.normwise_error([1.0, 2.0], [1.0, 2.0]) == 0.0
    assert O.normwise_error([1.0, 2.5], [1.0, 2.0]) == 0.25
    assert O.normwise_error([0.0], [0.0]) == 0.0
    assert O.normwise_error([1.0], [0.0]) == float("inf")
