"""GPU tests of the schedules beside leapfrogging and of the persistent launch's guarantees: the on-chain
fusion (LF_SCHED_FUSED), the chain alone (LF_DEBUG_CHAIN_ONLY), two handles taking turns on one stream, and
an LF_SCHED_AUTO handle that loses a persistent pass and moves to the stream schedule."""
import numpy as np
import pytest

from lf_inputs import make_net
from tests.gpu_util import check_against_oracle, log, poison_buffers, run_gpu, to_np

pytestmark = pytest.mark.gpu


def _bits(g):
    return [to_np(t).copy().view(np.uint32) for t in g.nabla_w + g.nabla_b]


@pytest.mark.parametrize("L,N,split", [
    (2, 256, None),       # no chain step: the only layer is stored at the end
    (3, 4, None),         # smallest width
    (5, 260, None),       # ragged last strip
    (9, 512, None),       # 16-byte strips
    (6, 1000, None),      # not a multiple of any tile
    (32, 1024, None),     # configuration 2's shape: 32-byte strips, one chunk per step
    (4, 2052, None),      # just past a power of two
    (5, 3076, None),      # 256-byte strips in four row blocks, ragged
    (4, 4096, None),      # configuration 3's layer shape
    (6, 260, 2),          # ragged second row block
    (4, 4096, 1),         # the widest layer with whole-height strips: several chunks per step
])
def test_on_chain_fusion_matches_oracle_and_leapfrog(monkeypatch, L, N, split):
    """LF_SCHED_FUSED: the thread that multiplies an entry of w^{l+1} for (bp2) stores the same entry of
    nabla_w^{l+1} (bp4).  Against the oracle, and the same bits as the leapfrogged persistent pass."""
    import torch
    import paper_1801_04928_amd as P
    if split is not None:
        monkeypatch.setenv("LF_PERSISTENT_ROW_SPLIT", str(split))
    net = make_net(L, N, 1, seed=L * 100 + N)
    g = run_gpu(net, 1, sched=P.LF_SCHED_FUSED)
    rep = check_against_oracle(net, g)
    fused = _bits(g)
    g.set_schedule(P.LF_SCHED_PERSISTENT)
    poison_buffers(g, whole_workspace=False)
    g.forward()
    g.backward(min(2, L - 1))
    torch.cuda.synchronize()
    for a, b in zip(fused, _bits(g)):
        assert np.array_equal(a, b)
    log(f"on-chain fusion L={L} N={N} split={split}: worst {rep['worst']:.2e}")
    g.close()


def test_on_chain_fusion_limits():
    import paper_1801_04928_amd as P
    g = P.LeapfrogNet(4, 264, 20, "f32")            # a minibatch has no persistent kernels
    with pytest.raises(P.LfError) as e:
        g.set_schedule(P.LF_SCHED_FUSED)
    assert e.value.status == P.LF_EUNSUPPORTED
    g.close()
    net = make_net(4, 256, 1, seed=1)
    g = P.LeapfrogNet(4, 256, 1, "f32")
    g.load(net)
    g.set_schedule(P.LF_SCHED_FUSED)
    g.set_sgd(0.01)
    g.forward()
    with pytest.raises(P.LfError) as e:
        g.backward(1)
    assert e.value.status == P.LF_EUNSUPPORTED
    g.close()


@pytest.mark.parametrize("shape,B,dtype,sched", [
    ((9, 516), 1, "f32", "persistent"), ((5, 3076), 1, "f32", "persistent"), ((9, 516), 1, "f32", "streams"),
    ((5, 264), 70, "f32", "streams"), ((4, 264), 70, "bf16", "streams")])
def test_chain_only_flag(shape, B, dtype, sched):
    """LF_DEBUG_CHAIN_ONLY: the delta chain alone.  Every delta^l is the full pass's, bit for bit; no gradient
    buffer is touched; lf_grads refuses; clearing the flag gives the full pass back."""
    import torch
    import paper_1801_04928_amd as P
    L, N = shape
    k = 3
    s = {"streams": P.LF_SCHED_STREAMS, "persistent": P.LF_SCHED_PERSISTENT}[sched]
    net = make_net(L, N, B, dtype=dtype, seed=N + B)
    g = run_gpu(net, k, sched=s)
    check_against_oracle(net, g)
    want_delta = [to_np(g.delta(l)).copy().view(np.uint32) for l in range(2, L + 1)]
    want_grads = _bits(g)
    g.set_debug_flags(P.LF_DEBUG_CHAIN_ONLY)
    poison_buffers(g, whole_workspace=False)
    g.forward()
    g.backward(k)
    torch.cuda.synchronize()
    for l in range(2, L + 1):
        assert np.array_equal(to_np(g.delta(l)).view(np.uint32), want_delta[l - 2]), f"delta^{l}"
    for t in g.nabla_w + g.nabla_b:
        assert bool(torch.isnan(t).all()), "a gradient buffer was written"
    with pytest.raises(P.LfError) as e:
        g.grads(2)
    assert e.value.status == P.LF_ESTATE
    g.set_debug_flags(0)
    g.forward()
    g.backward(k)
    torch.cuda.synchronize()
    for a, b in zip(want_grads, _bits(g)):
        assert np.array_equal(a, b)
    g.close()


def test_two_persistent_handles_take_turns_on_one_stream():
    """Two nets on the persistent kernels, their passes enqueued alternately on the same stream (so they
    never overlap on the device): each keeps its own exchange state and tags; results as when run alone."""
    import torch
    import paper_1801_04928_amd as P
    nets = [make_net(9, 516, 1, seed=1), make_net(6, 1028, 1, seed=2)]
    alone = []
    for net in nets:
        g = run_gpu(net, 3, sched=P.LF_SCHED_PERSISTENT)
        check_against_oracle(net, g)
        alone.append(_bits(g))
        g.close()
    gs = []
    for net in nets:
        g = P.LeapfrogNet(net.spec.L, net.spec.N, 1, "f32")
        g.load(net)
        g.set_schedule(P.LF_SCHED_PERSISTENT)
        gs.append(g)
    for rep in range(6):
        for g in gs:
            g.forward()
        for g in reversed(gs):
            g.backward(1 + rep % 4)
    torch.cuda.synchronize()
    for g, want in zip(gs, alone):
        for a, b in zip(want, _bits(g)):
            assert np.array_equal(a, b)
        g.close()


def test_auto_handle_moves_to_streams_after_a_lost_persistent_pass(monkeypatch):
    """An LF_SCHED_AUTO handle whose persistent pass gives up a wait (forced from the host: a spin limit of one
    poll) reports LF_EHIP once and then runs on the stream schedule; its results match the oracle."""
    import torch
    import paper_1801_04928_amd as P
    monkeypatch.setenv("LF_PERSISTENT_SPIN_LIMIT", "1")
    net = make_net(12, 1024, 1, seed=1)
    g = P.LeapfrogNet(12, 1024, 1, "f32")
    g.load(net)
    stream = torch.cuda.current_stream().cuda_stream
    assert P.lf_forward(g.handle, g.x.data_ptr(), stream) == P.LF_OK
    torch.cuda.synchronize()
    st = P.lf_backward_leapfrog(g.handle, g.y.data_ptr(), 4, stream)
    if st == P.LF_OK:                       # the forward kernel's waits all found their data at once
        torch.cuda.synchronize()
        st, _, _ = P.lf_grads(g.handle, 2)
    assert st == P.LF_EHIP
    assert "stream schedule" in P.lf_last_error(g.handle)
    # the lost pass is gone (no forward pass on record), the handle works again
    assert P.lf_backward_leapfrog(g.handle, g.y.data_ptr(), 4, stream) == P.LF_ESTATE
    g.forward()
    g.backward(4)
    torch.cuda.synchronize()
    check_against_oracle(net, g)
    g.close()
