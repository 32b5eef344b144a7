"""Host-side checks of the C ABI (no GPU): the library loads, exports every symbol the header
declares, validates arguments and call order, and its schedule function agrees with Algorithm 1."""
import ctypes as C
import os
import re

import pytest

import paper_1801_04928_amd as P
from oracle import backprop as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "lf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lf_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    syms = _declared_symbols()
    assert {"lf_forward", "lf_backward_leapfrog", "lf_grads"} <= set(syms)
    lib = P.lib()
    for s in syms:
        assert hasattr(lib, s), f"{s} declared in lf.h but not exported"


def test_binding_has_same_names():
    for s in _declared_symbols():
        assert callable(getattr(P, s)), s


def test_workspace_bytes():
    assert P.lf_workspace_bytes(1, 256, 1, P.LF_F32) == 0          # L < 2
    assert P.lf_workspace_bytes(8, 255, 1, P.LF_F32) == 0          # N not a multiple of 4
    assert P.lf_workspace_bytes(8, 260, 1, P.LF_BF16) == 0         # N not a multiple of 8 for bf16
    assert P.lf_workspace_bytes(8, 256, 0, P.LF_F32) == 0
    assert P.lf_workspace_bytes(8, 256, 1, 7) == 0
    n = P.lf_workspace_bytes(8, 256, 1, P.LF_F32)
    assert n >= 7 * 256 * 4 * 2 and n % 256 == 0                   # a^2..a^L and delta^2..delta^L
    assert P.lf_workspace_bytes(8, 256, 8, P.LF_F32) > P.lf_workspace_bytes(8, 256, 2, P.LF_F32)


FAKE = 1 << 20   # a "device pointer" that is only checked for alignment, never dereferenced on the host


def _handle(L=8, N=256, B=1, dt=P.LF_F32):
    st, h = P.lf_create(L, N, B, dt, P.LF_COST_QUADRATIC, FAKE, P.lf_workspace_bytes(L, N, B, dt))
    assert st == P.LF_OK
    return h


def test_create_rejects_bad_arguments():
    ok = P.lf_workspace_bytes(8, 256, 1, P.LF_F32)
    for args in [(1, 256, 1, P.LF_F32, 0, FAKE, ok), (8, 254, 1, P.LF_F32, 0, FAKE, ok),
                 (8, 256, 0, P.LF_F32, 0, FAKE, ok), (8, 256, 1, 5, 0, FAKE, ok),
                 (8, 256, 1, P.LF_F32, 3, FAKE, ok), (8, 256, 1, P.LF_F32, 0, 0, ok),
                 (8, 256, 1, P.LF_F32, 0, FAKE + 16, ok), (8, 256, 1, P.LF_F32, 0, FAKE, ok - 1),
                 (5000, 256, 1, P.LF_F32, 0, FAKE, ok)]:
        st, h = P.lf_create(*args)
        assert st == P.LF_EINVAL and h is None, args
        assert "lf_create" in P.lf_last_error(None)


def test_unequal_widths_workspace_and_create():
    """lf_workspace_bytes_widths / lf_create_widths: one width per layer, the same limits as N; equal widths
    give lf_create's workspace; a net with hidden layers of different widths has no persistent path, one whose
    first and last layer alone are narrower has."""
    F = P.LF_F32
    assert P.lf_workspace_bytes_widths(3, [8, 16, 4], 1, F) > 0
    assert P.lf_workspace_bytes_widths(3, [8, 16, 4], 1, F) % 256 == 0
    assert P.lf_workspace_bytes_widths(3, [8, 15, 4], 1, F) == 0       # not a multiple of 4
    assert P.lf_workspace_bytes_widths(3, [8, 16, 4], 1, P.LF_BF16) == 0   # 4 is not a multiple of 8
    assert P.lf_workspace_bytes_widths(3, [8, 0, 4], 1, F) == 0
    assert P.lf_workspace_bytes_widths(1, [8], 1, F) == 0
    assert P.lf_workspace_bytes_widths(3, None, 1, F) == 0
    assert P.lf_workspace_bytes_widths(8, [256] * 8, 1, F) == P.lf_workspace_bytes(8, 256, 1, F)
    assert P.lf_workspace_bytes_widths(4, [64, 256, 256, 32], 16, F) <= P.lf_workspace_bytes(4, 256, 16, F)
    widths = [64, 256, 128, 32]
    nbytes = P.lf_workspace_bytes_widths(4, widths, 1, F)
    st, h = P.lf_create_widths(4, widths, 1, F, P.LF_COST_QUADRATIC, FAKE, nbytes)
    assert st == P.LF_OK
    assert P.lf_set_schedule(h, P.LF_SCHED_PERSISTENT) == P.LF_EUNSUPPORTED
    assert "one width" in P.lf_last_error(h)
    assert P.lf_set_schedule(h, P.LF_SCHED_STREAMS) == P.LF_OK
    assert P.lf_set_schedule(h, P.LF_SCHED_AUTO) == P.LF_OK
    P.lf_destroy(h)
    st, h = P.lf_create_widths(4, widths, 1, F, P.LF_COST_QUADRATIC, FAKE, nbytes - 1)
    assert st == P.LF_EINVAL and h is None
    st, h = P.lf_create_widths(4, [64, 256, 130, 32], 1, F, P.LF_COST_QUADRATIC, FAKE, nbytes)
    assert st == P.LF_EINVAL and "width" in P.lf_last_error(None)
    st, h = P.lf_create_widths(4, None, 1, F, P.LF_COST_QUADRATIC, FAKE, nbytes)
    assert st == P.LF_EINVAL
    # a narrower input and output around equal hidden layers: the persistent path is there; not with a wider input
    for w4, want in (([64, 256, 256, 32], P.LF_OK), ([512, 256, 256, 32], P.LF_EUNSUPPORTED)):
        st, h = P.lf_create_widths(4, w4, 1, F, P.LF_COST_QUADRATIC, FAKE, P.lf_workspace_bytes_widths(4, w4, 1, F))
        assert st == P.LF_OK and P.lf_set_schedule(h, P.LF_SCHED_PERSISTENT) == want
        P.lf_destroy(h)
    # equal widths through the general call: the persistent path is there
    st, h = P.lf_create_widths(8, [256] * 8, 1, F, P.LF_COST_QUADRATIC, FAKE, P.lf_workspace_bytes(8, 256, 1, F))
    assert st == P.LF_OK and P.lf_set_schedule(h, P.LF_SCHED_PERSISTENT) == P.LF_OK
    P.lf_destroy(h)


def test_sgd_argument_and_state_checks():
    """lf_set_sgd: eta finite and >= 0; fp32 storage only; available in both schedules."""
    h = _handle()
    assert P.lf_set_sgd(h, -1.0) == P.LF_EINVAL
    assert P.lf_set_sgd(h, float("nan")) == P.LF_EINVAL
    assert P.lf_set_sgd(h, float("inf")) == P.LF_EINVAL
    assert P.lf_set_sgd(h, 0.0) == P.LF_OK
    assert P.lf_set_sgd(h, 0.5) == P.LF_OK
    assert P.lf_set_schedule(h, P.LF_SCHED_PERSISTENT) == P.LF_OK
    assert P.lf_set_sgd(h, 0.25) == P.LF_OK
    assert P.lf_set_schedule(h, P.LF_SCHED_STREAMS) == P.LF_OK
    assert P.lf_set_sgd(None, 0.5) == P.LF_EINVAL
    # bf16 storage: the step is taken on fp32 master copies, which only such a net may register
    assert P.lf_set_master_weights(h, [FAKE] * 7) == P.LF_EINVAL and "bf16" in P.lf_last_error(h)
    P.lf_destroy(h)
    hb = _handle(4, 256, 8, P.LF_BF16)
    assert P.lf_set_sgd(hb, 0.5) == P.LF_OK
    assert P.lf_set_master_weights(hb, None) == P.LF_EINVAL
    assert P.lf_set_master_weights(hb, [FAKE, 0, FAKE]) == P.LF_EINVAL
    assert P.lf_set_master_weights(hb, [FAKE, FAKE + 4, FAKE]) == P.LF_EINVAL
    assert P.lf_set_master_weights(hb, [FAKE] * 3) == P.LF_OK
    assert P.lf_set_master_weights(None, [FAKE] * 3) == P.LF_EINVAL
    P.lf_destroy(hb)


def test_call_order_and_argument_checks():
    h = _handle()
    M = 7
    try:
        assert P.lf_forward(h, FAKE) == P.LF_ESTATE
        assert "lf_set_params" in P.lf_last_error(h)
        assert P.lf_set_params(h, None, None) == P.LF_EINVAL
        assert P.lf_set_params(h, [FAKE] * M, [FAKE] * (M - 1) + [0]) == P.LF_EINVAL
        assert P.lf_set_params(h, [FAKE] * (M - 1) + [FAKE + 4], [FAKE] * M) == P.LF_EINVAL
        assert P.lf_set_params(h, [FAKE] * M, [FAKE] * M) == P.LF_OK
        assert P.lf_backward_leapfrog(h, FAKE, 1) == P.LF_ESTATE          # no grad buffers
        assert P.lf_set_grad_buffers(h, [FAKE] * M, [FAKE + 8] * M) == P.LF_EINVAL
        assert P.lf_set_grad_buffers(h, [FAKE] * M, [FAKE] * M) == P.LF_OK
        assert P.lf_backward_leapfrog(h, FAKE, 1) == P.LF_ESTATE          # no forward yet
        assert "lf_forward" in P.lf_last_error(h)
        for k in (0, -1, 8, 100):
            assert P.lf_backward_leapfrog(h, FAKE, k) == P.LF_EINVAL      # 1 <= k <= L-1
        assert P.lf_backward_leapfrog(h, 0, 1) == P.LF_EINVAL
        assert P.lf_backward_leapfrog(h, FAKE + 2, 1) == P.LF_EINVAL
        assert P.lf_forward(h, 0) == P.LF_EINVAL
        assert P.lf_forward(h, FAKE + 4) == P.LF_EINVAL
        st, _, _ = P.lf_grads(h, 3)
        assert st == P.LF_ESTATE
        st, _, _ = P.lf_grads(h, 1)
        assert st == P.LF_EINVAL
        st, _, _ = P.lf_activations(h, 9)
        assert st == P.LF_EINVAL
        st, _, _ = P.lf_activations(h, 2)
        assert st == P.LF_ESTATE
        assert P.lf_set_cost_scale(h, 128) == P.LF_EINVAL
        assert P.lf_set_cost_scale(h, -127) == P.LF_EINVAL
        assert P.lf_set_cost_scale(h, 100) == P.LF_OK
        assert P.lf_set_schedule(h, 99) == P.LF_EINVAL
        assert P.lf_set_schedule(h, P.LF_SCHED_FUSED) == P.LF_OK           # B = 1, fp32, N <= 4096
        assert P.lf_set_schedule(h, P.LF_SCHED_STREAMS) == P.LF_OK
        assert P.lf_set_debug_flags(h, 2) == P.LF_EINVAL                    # unknown bit
        assert P.lf_set_debug_flags(h, P.LF_DEBUG_CHAIN_ONLY) == P.LF_OK
        assert P.lf_set_debug_flags(h, 0) == P.LF_OK
        assert P.lf_set_debug_flags(None, 0) == P.LF_EINVAL
    finally:
        P.lf_destroy(h)
    P.lf_destroy(None)


def test_null_handle_is_rejected():
    assert P.lf_forward(None, FAKE) == P.LF_EINVAL
    assert P.lf_backward_leapfrog(None, FAKE, 1) == P.LF_EINVAL
    assert P.lf_set_params(None, [FAKE], [FAKE]) == P.LF_EINVAL
    assert isinstance(P.lf_last_error(None), str)


@pytest.mark.parametrize("L", [2, 3, 8, 32, 64])
def test_schedule_matches_algorithm1(L):
    """The library's worker(l) equals what running Algorithm 1's index arithmetic gives."""
    for k in range(1, L):
        want = O.worker_of_layer(L, k)
        for l in range(2, L + 1):
            assert P.lf_schedule_worker(L, k, l) == want[l]
    assert P.lf_schedule_worker(L, 0, 2) == -1
    assert P.lf_schedule_worker(L, L, 2) == -1
    assert P.lf_schedule_worker(L, 1, 1) == -1
    assert P.lf_schedule_worker(L, 1, L + 1) == -1


@pytest.mark.parametrize("L", [2, 3, 5, 8, 13, 21])
def test_algorithm1_owner_matches_the_algorithm_run_literally(L):
    """lf_algorithm1_owner (who saves a layer's gradients under LF_SCHED_REDUNDANT) against the owners recorded
    by the oracle's literal run of Algorithm 1; LF_SCHED_REDUNDANT exists for single-sample fp32 nets only."""
    import numpy as np
    N = 2
    w = {l: np.zeros((N, N)) for l in range(2, L + 1)}
    a = {l: np.full((1, N), 0.5) for l in range(1, L + 1)}
    for k in range(1, L):
        _, _, owner, writes = O.backward_algorithm1(w, a, np.zeros((1, N)), L, k)
        assert all(v == 1 for v in writes.values())
        for l in range(2, L + 1):
            got = P.lf_algorithm1_owner(L, k, l)
            assert (got == k and owner[l] == "parent") or got == owner[l], (L, k, l, got, owner[l])
    assert P.lf_algorithm1_owner(L, 0, 2) == -1 and P.lf_algorithm1_owner(L, L, 2) == -1
    assert P.lf_algorithm1_owner(L, 1, 1) == -1 and P.lf_algorithm1_owner(L, 1, L + 1) == -1
    h = _handle()
    assert P.lf_set_schedule(h, P.LF_SCHED_REDUNDANT) == P.LF_OK
    P.lf_destroy(h)
    hb = _handle(4, 256, 8, P.LF_F32)
    assert P.lf_set_schedule(hb, P.LF_SCHED_REDUNDANT) == P.LF_EUNSUPPORTED
    assert P.lf_set_schedule(hb, P.LF_SCHED_FUSED) == P.LF_EUNSUPPORTED
    P.lf_destroy(hb)


def test_forward_without_a_gpu_fails_loudly():
    """No CPU fallback: on a machine without a GPU the pass reports LF_EHIP."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    h = _handle()
    try:
        assert P.lf_set_params(h, [FAKE] * 7, [FAKE] * 7) == P.LF_OK
        assert P.lf_forward(h, FAKE) == P.LF_EHIP
        assert P.lf_last_error(h)
    finally:
        P.lf_destroy(h)
