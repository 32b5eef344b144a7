"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs, element by element.  fp32: normwise error <= 1e-5 per tensor; bf16 storage with fp32
accumulation: <= 2e-2.  Gradients must be bit-identical for every k."""
import numpy as np
import pytest

from lf_inputs import config_net, make_net
from tests.gpu_util import check_against_oracle, log, poison_buffers, run_gpu, to_np

pytestmark = pytest.mark.gpu


def _free(g):
    g.close()


SCHEDS = {"streams": 1, "persistent": 2, "fused": 4}   # LF_SCHED_STREAMS, LF_SCHED_PERSISTENT, LF_SCHED_FUSED


# ---------------------------------------------------------------- single sample, fp32
@pytest.mark.parametrize("sched", ["streams", "persistent"])
@pytest.mark.parametrize("L,N,k", [
    (2, 256, 1),        # one weight layer
    (3, 4, 2),          # smallest width
    (5, 260, 2),        # ragged: one full strip of 256 columns + 4
    (8, 256, 2),        # configuration 1's shape
    (6, 1000, 3),       # not a multiple of any tile
    (4, 2052, 3),       # rows-per-wave 8 path, ragged
    (3, 4100, 2),       # rows-per-wave 16 path, ragged (wider than the persistent path: streams only)
    (4, 4096, 3),       # widest net of the persistent path
    (4, 3076, 2),       # persistent path, ragged, 4 column groups per thread
    (9, 512, 8),        # k = L-1, the largest allowed
])
def test_single_sample_fp32_matches_oracle(L, N, k, sched):
    if sched == "persistent" and N > 4096:
        import paper_1801_04928_amd as P
        g = P.LeapfrogNet(L, N, 1, "f32")
        with pytest.raises(P.LfError) as e:
            g.set_schedule(P.LF_SCHED_PERSISTENT)
        assert e.value.status == P.LF_EUNSUPPORTED
        _free(g)
        return
    net = make_net(L, N, 1, seed=L * 1000 + N)
    g = run_gpu(net, k, sched=SCHEDS[sched])
    rep = check_against_oracle(net, g)
    log(f"B=1 L={L} N={N} k={k} {sched}: worst normwise error {rep['worst']:.2e}")
    _free(g)


@pytest.mark.parametrize("sched", ["streams", "persistent"])
def test_single_sample_outer_product_is_exact(sched):
    """Eq. (bp4) at B = 1 is one multiplication per entry: nabla_w^l[j][k] must equal
    fl32(delta^l[j] * a^{l-1}[k]) of the GPU's own delta and a, bit for bit; nabla_b^l = delta^l."""
    net = make_net(6, 772, 1, seed=5)
    g = run_gpu(net, 2, sched=SCHEDS[sched])
    for l in range(2, 7):
        d = to_np(g.delta(l))[0].astype(np.float32)
        a = to_np(g.activation(l - 1))[0].astype(np.float32)
        gw, gb = g.grads(l)
        assert np.array_equal(to_np(gw), np.outer(d, a).astype(np.float32))
        assert np.array_equal(to_np(gb), d)
    _free(g)


@pytest.mark.parametrize("L,N,B,dtype,sched", [
    (12, 1024, 1, "f32", "streams"), (12, 1024, 1, "f32", "persistent"), (10, 2052, 1, "f32", "persistent"),
    (10, 392, 5, "f32", None), (10, 264, 9, "bf16", None), (9, 520, 260, "bf16", None)])
def test_gradients_bit_identical_for_every_k(L, N, B, dtype, sched):
    """Leapfrogging only reassigns who computes (bp3),(bp4) (Theorem 1): same bits for k = 1, 2, 4, 8 and
    the odd ones."""
    net = make_net(L, N, B, dtype=dtype, seed=77)
    ref = None
    for k in (1, 2, 4, 8, 5, L - 1):
        g = run_gpu(net, k, sched=SCHEDS.get(sched))
        cur = [(to_np(g.grads(l)[0]).copy(), to_np(g.grads(l)[1]).copy()) for l in range(2, L + 1)]
        if ref is None:
            ref = cur
        else:
            for (w0, b0), (w1, b1) in zip(ref, cur):
                assert np.array_equal(w0.view(np.uint32), w1.view(np.uint32))
                assert np.array_equal(b0.view(np.uint32), b1.view(np.uint32))
        _free(g)


def _grad_hash(g):
    """Order-sensitive 64-bit checksum of every gradient bit, computed on the device."""
    torch = g.torch
    h = torch.zeros((), dtype=torch.int64, device=g.device)
    for i, t in enumerate(g.nabla_w + g.nabla_b):
        v = t.view(torch.int32).to(torch.int64).flatten()
        h = h * 1000003 + (v * (torch.arange(v.numel(), device=g.device) % 8191 + 1)).sum() + i
    return int(h)


@pytest.mark.parametrize("sched", ["streams", "persistent", "fused"])
def test_repeated_passes_are_deterministic_and_overwrite(sched):
    """Gradients are overwritten (not accumulated) and identical on every one of 100 passes (a checksum of all
    gradient bits per pass); the activations, errors and gradients are poisoned with NaN before each pass so
    a worker that ran ahead of its delta would show."""
    import torch
    net = make_net(10, 640, 1, seed=3)
    g = run_gpu(net, 4, sched=SCHEDS[sched])
    first = [to_np(g.grads(l)[0]).copy() for l in range(2, 11)]
    want = _grad_hash(g)
    for i in range(100):
        poison_buffers(g, whole_workspace=False)
        g.forward()
        g.backward(4)
        torch.cuda.synchronize()
        assert _grad_hash(g) == want, f"pass {i} differs"
    for l in range(2, 11):
        assert np.array_equal(first[l - 2].view(np.uint32), to_np(g.grads(l)[0]).view(np.uint32))
    _free(g)


def test_rank_one_net_full_width():
    """The rank-one symmetric net collapses to a scalar recurrence (see the oracle pins); checks the
    full-length reductions of the GPU path at N = 4096 against that recurrence through the oracle."""
    import math
    import paper_1801_04928_amd as P
    import torch
    L, N = 5, 4096
    c, beta, xi, eta = 1.7, -0.3, 0.6, 0.2
    g = P.LeapfrogNet(L, N, 1, "f32")
    for t in g.w:
        t.fill_(c / N)
    for t in g.b:
        t.fill_(beta)
    g.x.fill_(xi)
    g.y.fill_(eta)
    g.forward()
    g.backward(2)
    torch.cuda.synchronize()
    alpha = {1: xi}
    for l in range(2, L + 1):
        alpha[l] = 1.0 / (1.0 + math.exp(-(c * alpha[l - 1] + beta)))
    d = {L: (alpha[L] - eta) * alpha[L] * (1 - alpha[L])}
    for l in range(L - 1, 1, -1):
        d[l] = c * d[l + 1] * alpha[l] * (1 - alpha[l])
    for l in range(2, L + 1):
        gw, gb = g.grads(l)
        np.testing.assert_allclose(to_np(gw), d[l] * alpha[l - 1], rtol=2e-5)
        np.testing.assert_allclose(to_np(gb), d[l], rtol=2e-5)
    _free(g)


@pytest.mark.parametrize("sched", ["streams", "persistent"])
def test_cost_scale_is_exact_and_lifts_deep_layers_out_of_the_subnormal_range(sched):
    """A power-of-two cost scale multiplies delta^L (eq. (bp1)) and, by linearity of (bp2)-(bp4), every
    gradient by the same power of two.  (i) Where nothing underflows the scaled result is the unscaled one
    times the scale, bit for bit.  (ii) In a net deep enough for delta to leave the fp32 normal range the
    scaled pass meets the relative tolerance at every layer, with no subnormal exception."""
    import paper_1801_04928_amd as P
    import torch
    # (i) exactness on a shallow net
    net = make_net(5, 516, 1, seed=9)
    g0 = run_gpu(net, 2, sched=SCHEDS[sched])
    g1 = P.LeapfrogNet(5, 516, 1, "f32")
    g1.load(net)
    g1.set_schedule(SCHEDS[sched])
    g1.set_cost_scale(20)
    g1.forward()
    g1.backward(2)
    torch.cuda.synchronize()
    for l in range(2, 6):
        assert np.array_equal(to_np(g1.grads(l)[0]), to_np(g0.grads(l)[0]) * np.float32(2.0 ** 20))
        assert np.array_equal(to_np(g1.grads(l)[1]), to_np(g0.grads(l)[1]) * np.float32(2.0 ** 20))
    _free(g0)
    _free(g1)
    # (ii) 72 layers: max|delta^2| is about 1e-45 unscaled
    from oracle import backprop as O
    from tests.gpu_util import compare
    L, N, e = 72, 512, 110
    net = make_net(L, N, 1, seed=10)
    g = P.LeapfrogNet(L, N, 1, "f32")
    g.load(net)
    g.set_schedule(SCHEDS[sched])
    g.set_cost_scale(e)
    g.forward()
    g.backward(8)
    torch.cuda.synchronize()
    a = O.forward(net.w_by_layer, net.b_by_layer, net.x(), L)
    report = {}
    for l, delta, nb, nw in O.backward_layers(net.w_by_layer, a, net.y(), L):
        gw, gb = g.grads(l)
        compare(f"nabla_w^{l}", to_np(gw), nw * 2.0 ** e, 1e-5, report)
        compare(f"nabla_b^{l}", to_np(gb), nb * 2.0 ** e, 1e-5, report)
    assert "subnormal" not in report
    assert float(np.max(np.abs(O.backward_sequential(net.w_by_layer, a, net.y(), L)[0][2]))) < 2.0 ** -126
    log(f"cost scale 2^{e}, L={L} {sched}: worst {report['worst']:.2e}")
    _free(g)


@pytest.mark.parametrize("L,N,k,split", [
    (5, 64, 2, 2),        # strips of 8 columns, two row blocks of 32 rows
    (6, 260, 3, 2),       # ragged last strip, ragged second row block
    (4, 1028, 1, 4),      # sequential pass, four row blocks, ragged
    (7, 2052, 4, 2),      # just past a power of two
    (5, 3076, 2, 4),      # 256-byte strips, ragged
    (3, 4096, 2, 4),
    (4, 4096, 3, 1),      # the widest layer with whole-height strips
])
def test_persistent_row_split_strips_match_oracle(monkeypatch, L, N, k, split):
    """The persistent backward kernel with every column strip shared by `split` row blocks (the layout
    wide layers take by default), forced at sizes that leave ragged strips and ragged row blocks."""
    import paper_1801_04928_amd as P
    monkeypatch.setenv("LF_PERSISTENT_ROW_SPLIT", str(split))
    net = make_net(L, N, 1, seed=N + 31 * split)
    g = run_gpu(net, k, sched=P.LF_SCHED_PERSISTENT)
    rep = check_against_oracle(net, g)
    # same bits for another k (the partial sums are added in row-block order whatever the timing)
    ref = [to_np(t).copy() for t in g.nabla_w] + [to_np(t).copy() for t in g.nabla_b]
    g.forward()
    g.backward(1 if k > 1 else min(2, L - 1))
    import torch
    torch.cuda.synchronize()
    got = [to_np(t) for t in g.nabla_w] + [to_np(t) for t in g.nabla_b]
    for a, b in zip(ref, got):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    log(f"row split {split}: L={L} N={N} k={k}: worst {rep['worst']:.2e}")
    _free(g)


@pytest.mark.parametrize("L,N,k,split", [
    (5, 3076, 2, 4),      # ragged strips and row blocks, with workers
    (4, 4096, 1, 4),      # the sequential pass
    (4, 2052, 3, 2),      # a forced row split below the width that takes it by default
])
def test_persistent_wide_layer_instances_with_streamed_weights(monkeypatch, L, N, k, split):
    """The wide-layer instances that read the weights with non-temporal loads (taken by default only by nets whose
    weights are far larger than the cache), forced on small nets: the oracle's numbers, and the same bits as the
    instances with ordinary loads -- how a load is cached changes no value."""
    import torch
    import paper_1801_04928_amd as P
    monkeypatch.setenv("LF_PERSISTENT_ROW_SPLIT", str(split))
    net = make_net(L, N, 1, seed=N + 7 * split)
    bits = []
    for stream in ("1", "0"):
        monkeypatch.setenv("LF_PERSISTENT_STREAM_WEIGHTS", stream)
        g = run_gpu(net, k, sched=P.LF_SCHED_PERSISTENT)
        if stream == "1":
            rep = check_against_oracle(net, g)
            log(f"streamed weights: L={L} N={N} k={k} split {split}: worst {rep['worst']:.2e}")
        bits.append([to_np(t).copy().view(np.uint32) for t in g.nabla_w + g.nabla_b] +
                    [to_np(g.activation(l)).copy().view(np.uint32) for l in range(2, L + 1)])
        _free(g)
    for a, b in zip(*bits):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("L,N,k,groups", [(5, 1024, 2, 16), (4, 2048, 3, 32), (6, 520, 1, 8), (4, 1000, 2, 4)])
def test_persistent_with_few_workgroups(monkeypatch, L, N, k, groups):
    """The launch shapes a device with few compute units would get (many rows per forward workgroup, several
    chunks per wave and layer; wide backward strips), forced through the workgroup-count override."""
    import paper_1801_04928_amd as P
    monkeypatch.setenv("LF_PERSISTENT_GROUPS", str(groups))
    net = make_net(L, N, 1, seed=N + groups)
    g = run_gpu(net, k, sched=P.LF_SCHED_PERSISTENT)
    rep = check_against_oracle(net, g)
    log(f"{groups} workgroups: L={L} N={N} k={k}: worst {rep['worst']:.2e}")
    _free(g)


@pytest.mark.parametrize("stride,nap", [("1024", "0"), ("256", "3")])
def test_persistent_exchange_layout_and_pause_knobs(monkeypatch, stride, nap):
    """The tuning knobs that change where the exchanged words lie and when they are first polled change
    no result: spread words (groups of eight, `stride` bytes apart) and another pause give the same bits."""
    import paper_1801_04928_amd as P
    import torch
    net = make_net(6, 1000, 1, seed=77)
    ref = run_gpu(net, 3, sched=P.LF_SCHED_PERSISTENT)
    want = [to_np(t).copy() for t in ref.nabla_w] + [to_np(t).copy() for t in ref.nabla_b]
    _free(ref)
    monkeypatch.setenv("LF_PERSISTENT_LL_STRIDE", stride)
    monkeypatch.setenv("LF_PERSISTENT_NAP_FWD", nap)
    monkeypatch.setenv("LF_PERSISTENT_NAP_BWD", nap)
    g = run_gpu(net, 3, sched=P.LF_SCHED_PERSISTENT)
    check_against_oracle(net, g)
    got = [to_np(t) for t in g.nabla_w] + [to_np(t) for t in g.nabla_b]
    for a, b in zip(want, got):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    _free(g)


@pytest.mark.parametrize("L,N,k", [(11, 1000, 8), (7, 2052, 4), (19, 516, 16)])
def test_persistent_worker_partition_layout_and_pacing_change_no_bits(monkeypatch, L, N, k):
    """Which workgroups make up a worker partition (all XCDs for k a multiple of 4, or workgroup index mod k)
    decides only who stores which rows of nabla_w^l, and pacing only when: the oracle's numbers and the same bits
    every way."""
    import paper_1801_04928_amd as P
    net = make_net(L, N, 1, seed=N + k)
    g = run_gpu(net, k, sched=P.LF_SCHED_PERSISTENT)
    rep = check_against_oracle(net, g)
    want = [to_np(t).copy() for t in g.nabla_w] + [to_np(t).copy() for t in g.nabla_b]
    want += [to_np(g.activation(l)).copy() for l in range(2, L + 1)]
    _free(g)
    # the other layout; then the default layout with the stores paced by the chain's steps (the default only for
    # nets too large for the cache): k bursts per layer, and three
    # ... the forward kernel's other dealing of row blocks to XCDs (the default only for nets read from memory), and
    # other dealings of the chain's strips (wide layers only)
    for env in ({"LF_PERSISTENT_SPREAD": "0"}, {"LF_PERSISTENT_PACE": str(k)}, {"LF_PERSISTENT_PACE": "3"},
                {"LF_PERSISTENT_FWD_BAND": "1"}, {"LF_PERSISTENT_STRIP_RUN": "8"}, {"LF_PERSISTENT_STRIP_RUN": "1"}):
        for name, value in env.items():
            monkeypatch.setenv(name, value)
        g = run_gpu(net, k, sched=P.LF_SCHED_PERSISTENT)
        check_against_oracle(net, g)
        got = [to_np(t) for t in g.nabla_w] + [to_np(t) for t in g.nabla_b]
        got += [to_np(g.activation(l)) for l in range(2, L + 1)]
        for a, b in zip(want, got):
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
        _free(g)
        for name in env:
            monkeypatch.delenv(name)
    log(f"partition layouts and pacing: L={L} N={N} k={k}: worst {rep['worst']:.2e}")


def test_persistent_pass_replays_from_a_hip_graph():
    """A forward + backward pass recorded in a HIP graph and replayed: every replay (with eager passes of the
    same handle and synchronisations in between) must give the bits of the eager pass.  The launches carry
    no per-launch argument -- the tag of the exchanged words is kept in device memory -- so a replay cannot
    mistake the words of the launch before it for its own."""
    import paper_1801_04928_amd as P
    import torch
    net = make_net(9, 516, 1, seed=21)
    g = P.LeapfrogNet(9, 516, 1, "f32")
    g.load(net)
    g.set_schedule(P.LF_SCHED_PERSISTENT)
    g.forward()
    g.backward(3)
    torch.cuda.synchronize()
    check_against_oracle(net, g)
    want = [to_np(t).copy() for t in g.nabla_w] + [to_np(t).copy() for t in g.nabla_b]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        g.forward()
        g.backward(3)
    for replay in range(4):
        for t in g.nabla_w + g.nabla_b:
            t.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = [to_np(t) for t in g.nabla_w] + [to_np(t) for t in g.nabla_b]
        for a, b in zip(want, got):
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), f"replay {replay} differs"
        # eager work of the same handle between the replays
        g.forward()
        g.backward(1 + replay % 2)
        torch.cuda.synchronize()
    _free(g)


@pytest.mark.parametrize("L,N,B,dtype,k", [(5, 520, 130, "f32", 3), (4, 516, 1, "f32", 2), (4, 520, 260, "bf16", 2)])
def test_stream_schedule_pass_replays_from_a_hip_graph(L, N, B, dtype, k):
    """The stream schedule recorded in a HIP graph: the worker streams fork from and join the capturing stream
    through events, so the whole leapfrogged pass becomes one graph; every replay, with eager passes of the
    same handle in between, must give the bits of the eager pass."""
    import paper_1801_04928_amd as P
    import torch
    net = make_net(L, N, B, dtype=dtype, seed=5)
    g = P.LeapfrogNet(L, N, B, dtype)
    g.load(net)
    g.set_schedule(P.LF_SCHED_STREAMS)
    g.forward()
    g.backward(k)
    torch.cuda.synchronize()
    check_against_oracle(net, g)
    want = [to_np(t).copy() for t in g.nabla_w] + [to_np(t).copy() for t in g.nabla_b]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        g.forward()
        g.backward(k)
    for replay in range(3):
        for t in g.nabla_w + g.nabla_b:
            t.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = [to_np(t) for t in g.nabla_w] + [to_np(t) for t in g.nabla_b]
        for a, b in zip(want, got):
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), f"replay {replay} differs"
        g.forward()
        g.backward(1 + replay % 2)
        torch.cuda.synchronize()
    _free(g)


def test_persistent_wait_that_gives_up_is_reported(monkeypatch):
    """Failure handling of the persistent path, forced from the host: with a spin limit of one poll the
    first wait that does not find its data at once gives up.  Every kernel still exits normally; the next
    call on the handle reports LF_EHIP and says where the wait was."""
    import paper_1801_04928_amd as P
    import torch
    monkeypatch.setenv("LF_PERSISTENT_SPIN_LIMIT", "1")
    net = make_net(12, 1024, 1, seed=1)
    g = P.LeapfrogNet(12, 1024, 1, "f32")
    g.load(net)
    g.set_schedule(P.LF_SCHED_PERSISTENT)
    g.forward()
    torch.cuda.synchronize()
    # the forward kernel's first gather very likely gave up; if not, the backward kernel's will
    failed = P.lf_backward_leapfrog(g.handle, g.y.data_ptr(), 4, torch.cuda.current_stream().cuda_stream)
    message = P.lf_last_error(g.handle)
    if failed == P.LF_OK:
        torch.cuda.synchronize()
        failed, _, _ = P.lf_grads(g.handle, 2)
        message = P.lf_last_error(g.handle)
    assert failed == P.LF_EHIP
    assert "gave up waiting" in message
    # the handle stays failed (its exchange state is undefined); a new handle works
    assert P.lf_forward(g.handle, g.x.data_ptr(), 0) == P.LF_EHIP
    _free(g)
    monkeypatch.delenv("LF_PERSISTENT_SPIN_LIMIT")
    g = run_gpu(net, 4, sched=P.LF_SCHED_PERSISTENT)
    check_against_oracle(net, g)
    _free(g)


# ---------------------------------------------------------------- minibatch
@pytest.mark.parametrize("L,N,B,dtype,k", [
    (4, 132, 3, "f32", 2),       # one ragged tile in every dimension
    (3, 260, 37, "f32", 1),
    (5, 512, 256, "f32", 4),     # several full tiles; split-K on the chain
    (3, 1024, 130, "f32", 2),
    (4, 136, 5, "bf16", 2),
    (3, 264, 70, "bf16", 1),
    (5, 512, 192, "bf16", 4),
    (3, 392, 1, "bf16", 2),      # B = 1 through the minibatch kernels
])
def test_minibatch_matches_oracle(L, N, B, dtype, k):
    net = make_net(L, N, B, dtype=dtype, seed=L * 1000 + N + B)
    g = run_gpu(net, k)
    rep = check_against_oracle(net, g)
    log(f"B={B} L={L} N={N} {dtype} k={k}: worst normwise error {rep['worst']:.2e}")
    _free(g)


@pytest.mark.parametrize("tile", ["stream", "half", "big"])
@pytest.mark.parametrize("L,N,B,k", [
    (3, 264, 70, 1),        # one ragged tile per product; a ragged last k-tile
    (4, 520, 260, 2),       # 3 x 3 tiles with ragged edges, split K on the chain side
    (3, 1024, 512, 2),      # full tiles only
    (4, 2056, 136, 3),      # ragged last column tile, two row tiles of the 128 x 256 kernel, long K split
])
def test_minibatch_bf16_large_tile_kernel_matches_oracle(monkeypatch, L, N, B, k, tile):
    """The bf16 contraction kernels of wide nets (256 x 256 tiles, the gradient product streamed through resident
    workgroups: the default; 256 x 256 tiles with a workgroup per tile; 128 x 256 tiles, two workgroups per
    compute unit), forced at sizes the oracle finishes quickly and that leave ragged tiles in
    every dimension.  Both kernels give the same bits for every k."""
    import torch
    monkeypatch.setenv("LF_GEMM_BIG", "1")
    monkeypatch.setenv("LF_GEMM_CHAIN_TILE", "big" if tile == "stream" else tile)
    monkeypatch.setenv("LF_GEMM_GRAD_TILE", tile)
    if tile == "stream" and N > 2000:
        monkeypatch.setenv("LF_GEMM_STREAM_GROUPS", "24")      # several tiles per resident workgroup
    net = make_net(L, N, B, dtype="bf16", seed=7 * N + B)
    g = run_gpu(net, k)
    rep = check_against_oracle(net, g)
    ref = [to_np(t).copy() for t in g.nabla_w] + [to_np(t).copy() for t in g.nabla_b]
    poison_buffers(g, whole_workspace=False)
    g.forward()
    g.backward(1 if k > 1 else 2)
    torch.cuda.synchronize()
    for a, b in zip(ref, [to_np(t) for t in g.nabla_w] + [to_np(t) for t in g.nabla_b]):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    log(f"wide-net bf16 kernel {tile}: B={B} L={L} N={N} k={k}: worst normwise error {rep['worst']:.2e}")
    _free(g)


def test_minibatch_sharing_knobs_change_no_bits(monkeypatch):
    """How a minibatch net shares the chip between chain and workers -- resident workgroups of the streamed
    gradient product, streams the workers share -- is a matter of time only: the gradients are the same bits.
    (The number of K splits of the chain product is part of the arithmetic and is not varied here.)"""
    import torch
    monkeypatch.setenv("LF_GEMM_BIG", "1")
    net = make_net(6, 1032, 136, dtype="bf16", seed=99)
    want = None
    for groups, streams in (("96", "2"), ("8", "1"), ("256", "3"), ("40", "8")):
        monkeypatch.setenv("LF_GEMM_STREAM_GROUPS", groups)
        monkeypatch.setenv("LF_WORKER_STREAMS", streams)
        g = run_gpu(net, 4)
        got = [to_np(t).copy().view(np.uint32) for t in g.nabla_w + g.nabla_b]
        if want is None:
            check_against_oracle(net, g)
            want = got
        else:
            for a, b in zip(want, got):
                assert np.array_equal(a, b), f"groups {groups}, streams {streams}"
        _free(g)


@pytest.mark.parametrize("target", ["512", "1024"])
def test_minibatch_bf16_half_tile_kernel_deeper_split(monkeypatch, target):
    """The 128 x 256-tile kernel with the chain-side products split further along K (more, shorter workgroups)."""
    monkeypatch.setenv("LF_GEMM_BIG", "1")
    monkeypatch.setenv("LF_GEMM_CHAIN_TILE", "half")
    monkeypatch.setenv("LF_GEMM_GRAD_TILE", "half")
    monkeypatch.setenv("LF_GEMM_SPLIT_TARGET", target)
    net = make_net(3, 2048, 136, dtype="bf16", seed=int(target))
    g = run_gpu(net, 2)
    rep = check_against_oracle(net, g)
    log(f"wide-net bf16 kernel, split target {target}: worst normwise error {rep['worst']:.2e}")
    _free(g)


# ---------------------------------------------------------------- the five configurations, full size
# ---------------------------------------------------------------- layers of unequal widths
@pytest.mark.parametrize("widths,B,dtype,k,big", [
    ((260, 1028, 516, 2052, 64), 1, "f32", 2, None),     # single sample: every matrix ragged, rows-per-wave 4 and 8
    ((1000, 4100, 300, 4100), 1, "f32", 3, None),        # rows-per-wave 16 on a 4100 x 300 and a 300 x 4100 matrix
    ((4100, 4100, 8), 1, "f32", 1, None),                # four rows per wave forward; an 8 x 4100 last layer
    ((8, 4), 1, "f32", 1, None),                         # one tiny weight layer
    ((264, 520, 136, 392), 70, "f32", 2, None),          # minibatch fp32 MFMA, ragged in every dimension
    ((136, 1032, 264), 300, "f32", 1, None),             # several row tiles
    ((264, 520, 136, 392), 70, "bf16", 3, "0"),          # bf16, 128 x 128 tiles
    ((520, 264, 1032, 264), 260, "bf16", 2, "1"),        # bf16, 256 x 256 tiles, split K of unequal lengths
])
def test_unequal_layer_widths_match_oracle(monkeypatch, widths, B, dtype, k, big):
    """Nets whose layers differ in width (w^l is n_l x n_{l-1}; x has n_1 and y has n_L entries): the stream
    schedule's kernels against the oracle, and the same bits for another k."""
    import torch
    if big is not None:
        monkeypatch.setenv("LF_GEMM_BIG", big)
    L = len(widths)
    net = make_net(L, widths, B, dtype=dtype, seed=sum(widths) + B)
    g = run_gpu(net, k)
    rep = check_against_oracle(net, g)
    for l in range(2, L + 1):
        gw, gb = g.grads(l)
        assert tuple(gw.shape) == (widths[l - 1], widths[l - 2]) and tuple(gb.shape) == (widths[l - 1],)
    if L > 2:
        ref = [to_np(t).copy() for t in g.nabla_w] + [to_np(t).copy() for t in g.nabla_b]
        g.forward()
        g.backward(1 if k > 1 else 2)
        torch.cuda.synchronize()
        got = [to_np(t) for t in g.nabla_w] + [to_np(t) for t in g.nabla_b]
        for a, b in zip(ref, got):
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    log(f"widths {widths} B={B} {dtype} k={k}: worst normwise error {rep['worst']:.2e}")
    _free(g)


def test_unequal_layer_widths_outer_product_is_exact():
    """Eq. (bp4) at B = 1 with a non-square w^l: nabla_w^l[j][k] = fl32(delta^l[j] * a^{l-1}[k]) bit for bit."""
    widths = (772, 260, 1284, 516)
    net = make_net(4, widths, 1, seed=9)
    g = run_gpu(net, 2)
    for l in range(2, 5):
        d = to_np(g.delta(l))[0].astype(np.float32)
        a = to_np(g.activation(l - 1))[0].astype(np.float32)
        gw, gb = g.grads(l)
        assert np.array_equal(to_np(gw), np.outer(d, a).astype(np.float32))
        assert np.array_equal(to_np(gb), d)
    _free(g)


# ---------------------------------------------------------------- descent step fused into the workers
@pytest.mark.parametrize("shape,B,k,sched", [
    ((5, 516), 1, 2, "streams"),                   # single sample, ragged strips
    ((3, 4100), 1, 1, "streams"),                  # sequential pass; rows read ahead past a ragged end
    ((260, 1028, 516, 64), 1, 3, "streams"),       # unequal widths
    ((4, 520), 130, 2, "streams"),                 # minibatch fp32 MFMA epilogue
    ((264, 520, 136, 392), 70, 1, "streams"),      # minibatch, unequal widths, sequential
    ((5, 516), 1, 2, "persistent"),                # worker workgroups step the weights behind the chain
    ((9, 1000), 1, 1, "persistent"),               # k = 1: one partition of workers does every layer
    ((6, 1028), 1, 5, "persistent"),               # k = L-1
    ((4, 3076), 1, 3, "persistent"),               # strips in row blocks, several float4 groups per thread
    ((2, 256), 1, 1, "persistent"),                # no chain step: nothing to wait for
    ((32, 1024), 1, 8, "persistent"),              # configuration 2's shape: 31 layers stepped behind the chain
    ((64, 256, 256, 32), 1, 2, "persistent"),      # a narrower first and last layer
    ((1024, 3076, 3076, 260), 1, 3, "persistent"), # the same with strips in row blocks
])
def test_fused_descent_step(shape, B, k, sched):
    """lf_set_sgd: the pass applies w <- w - eta nabla_w, b <- b - eta nabla_b in place.  Checked (i) against
    the gradients the same library stores without it -- each entry must be the fp32 value nearest to
    w - eta g, give or take the double rounding of the host's reference -- which isolates the step from the
    chain; (ii) against the oracle's step; (iii) for the same bits with another k; (iv) for the call order."""
    import torch
    import paper_1801_04928_amd as P
    from oracle import backprop as O
    if len(shape) == 2:                            # (L, N); longer tuples are widths
        L, N = shape
        widths = [N] * L
        net = make_net(L, N, B, seed=N + B)
    else:
        widths = list(shape)
        L = len(widths)
        net = make_net(L, widths, B, seed=sum(widths) + B)
    g = run_gpu(net, k, sched=SCHEDS[sched])
    check_against_oracle(net, g)
    grads_w = [to_np(t).astype(np.float64) for t in g.nabla_w]
    grads_b = [to_np(t).astype(np.float64) for t in g.nabla_b]
    eta = float(np.float32(0.1 * np.max(np.abs(net.w(L))) / np.max(np.abs(grads_w[-1]))))
    g.set_sgd(eta)
    g.forward()
    g.backward(k)
    torch.cuda.synchronize()
    new_w = [to_np(t).copy() for t in g.w]
    new_b = [to_np(t).copy() for t in g.b]
    # (i) the step itself
    for i in range(L - 1):
        for new, old, grad in ((new_w[i], net.w(i + 2), grads_w[i]), (new_b[i], net.b(i + 2), grads_b[i])):
            want = old.astype(np.float64) - eta * grad
            ulp = np.spacing(np.abs(want).astype(np.float32)).astype(np.float64)
            assert np.all(np.abs(new.astype(np.float64) - want) <= 0.5000001 * ulp + 1e-300), f"layer {i + 2}"
    # (ii) against the oracle: the applied step, in units of the gradient
    w, b = net.w_by_layer, net.b_by_layer
    a = O.forward(w, b, net.x(), L)
    _, nb, nw = O.backward_sequential(w, a, net.y(), L)
    w1, b1 = O.sgd_step(w, b, nw, nb, eta, L)
    for l in range(2, L + 1):
        for new, old, want, grad in ((new_w[l - 2], net.w(l), w1[l], nw[l]), (new_b[l - 2], net.b(l), b1[l], nb[l])):
            applied = (old.astype(np.float64) - new.astype(np.float64)) / eta
            floor = 2.0 ** -23 * float(np.max(np.abs(old))) / eta      # rounding of the stored result
            assert np.max(np.abs(applied - grad)) <= 1e-5 * np.max(np.abs(grad)) + floor, f"layer {l}"
            assert np.max(np.abs(new - want)) <= 1e-6 * np.max(np.abs(want))
    # (iv) stale activations, gradients not stored
    with pytest.raises(P.LfError) as e:
        g.backward(k)
    assert e.value.status == P.LF_ESTATE
    with pytest.raises(P.LfError) as e:
        g.grads(2)
    assert e.value.status == P.LF_ESTATE
    # the next forward pass runs on the stepped weights
    c0 = O.cost(a[L], net.y())
    g.forward()
    torch.cuda.synchronize()
    a1 = O.forward(w1, b1, net.x(), L)
    assert O.normwise_error(to_np(g.activation(L)), a1[L]) <= 1e-5
    c1 = O.cost(a1[L], net.y())
    # (iii) another k from the same start gives the same bits
    if L > 2:
        g.load(net)
        g.forward()
        g.backward(1 if k > 1 else 2)
        torch.cuda.synchronize()
        for i in range(L - 1):
            assert np.array_equal(to_np(g.w[i]).view(np.uint32), new_w[i].view(np.uint32))
            assert np.array_equal(to_np(g.b[i]).view(np.uint32), new_b[i].view(np.uint32))
    log(f"fused descent step {shape} B={B} k={k} {sched}: eta {eta:.3g}, cost {c0:.6g} -> {c1:.6g}")
    _free(g)


@pytest.mark.parametrize("L,N,B,k,big,tile", [(4, 264, 70, 2, "0", "half"), (3, 520, 260, 1, "1", "half"),
                                              (3, 520, 260, 1, "1", "big")])
def test_fused_descent_step_bf16_master_weights(monkeypatch, L, N, B, k, big, tile):
    """bfloat16 storage: the step is taken on fp32 master copies and the bf16 weights are rewritten as their
    rounding.  Checked against the gradients the library stores without the step (master' is the fp32 value
    nearest to master - eta g), against the oracle's step within the bf16 tolerance, for w = rne(master')
    bit for bit, and for the order of calls."""
    import torch
    import paper_1801_04928_amd as P
    from lf_inputs import round_to_bf16
    from oracle import backprop as O
    monkeypatch.setenv("LF_GEMM_BIG", big)
    monkeypatch.setenv("LF_GEMM_GRAD_TILE", tile)
    net = make_net(L, N, B, dtype="bf16", seed=N + B)
    g = run_gpu(net, k)
    check_against_oracle(net, g)
    grads_w = [to_np(t).astype(np.float64) for t in g.nabla_w]
    grads_b = [to_np(t).astype(np.float64) for t in g.nabla_b]
    eta = float(np.float32(0.05 * np.max(np.abs(net.w(L))) / np.max(np.abs(grads_w[-1]))))
    # without master weights the pass refuses
    st = P.lf_set_sgd(g.handle, eta)
    assert st == P.LF_OK
    g.forward()
    with pytest.raises(P.LfError) as e:
        g.backward(k)
    assert e.value.status == P.LF_ESTATE and "master" in str(e.value)
    g.set_sgd(eta)                       # the binding creates the masters from the bf16 weights
    g.forward()
    g.backward(k)
    torch.cuda.synchronize()
    w, b = net.w_by_layer, net.b_by_layer
    a = O.forward(w, b, net.x(), L)
    _, nb, nw = O.backward_sequential(w, a, net.y(), L)
    for l in range(2, L + 1):
        master = to_np(g.master_w[l - 2])
        want = net.w(l).astype(np.float64) - eta * grads_w[l - 2]
        ulp = np.spacing(np.abs(want).astype(np.float32)).astype(np.float64)
        assert np.all(np.abs(master.astype(np.float64) - want) <= 0.5000001 * ulp + 1e-300), f"layer {l}"
        assert np.array_equal(to_np(g.w[l - 2]).view(np.uint32), round_to_bf16(master).view(np.uint32)), f"layer {l}"
        applied = (net.w(l).astype(np.float64) - master.astype(np.float64)) / eta
        floor = 2.0 ** -23 * float(np.max(np.abs(net.w(l)))) / eta
        assert np.max(np.abs(applied - nw[l])) <= 2e-2 * np.max(np.abs(nw[l])) + floor, f"layer {l}"
        bias = to_np(g.b[l - 2]).astype(np.float64)
        want_b = net.b(l).astype(np.float64) - eta * grads_b[l - 2]
        assert np.all(np.abs(bias - want_b) <= 0.5000001 * np.spacing(np.abs(want_b).astype(np.float32)) + 1e-300)
    with pytest.raises(P.LfError) as e:
        g.backward(k)
    assert e.value.status == P.LF_ESTATE
    _free(g)


# ---------------------------------------------------------------- the limits of the shape
def test_widest_single_sample_net():
    """N = 16384, the widest net of the single-sample kernels (a 1 GiB matrix per layer; the forward kernel keeps
    all of a^{l-1} in 64 KiB of LDS)."""
    net = make_net(3, 16384, 1, seed=16384, cache=False)
    g = run_gpu(net, 2)
    rep = check_against_oracle(net, g, sample_tiles=(24, 96), rng=np.random.default_rng(1))
    log(f"B=1 L=3 N=16384: worst normwise error {rep['worst']:.2e}")
    _free(g)


def test_single_sample_wider_than_the_gemv_kernels_takes_the_matrix_kernels():
    """Past N = 16384 a single sample runs as a minibatch of one through the MFMA kernels."""
    net = make_net(2, 16392, 1, seed=3, cache=False)
    g = run_gpu(net, 1)
    rep = check_against_oracle(net, g, sample_tiles=(24, 96), rng=np.random.default_rng(2))
    log(f"B=1 L=2 N=16392: worst normwise error {rep['worst']:.2e}")
    _free(g)


@pytest.mark.parametrize("L,sched", [(1025, "persistent"), (1030, "auto")])
def test_deepest_nets(L, sched):
    """L = 1025 is the deepest net of the persistent kernels (their per-layer pointer tables live in LDS); deeper
    nets take the stream schedule.  delta vanishes by about 4x per layer, so below the top 60 layers the
    gradients are subnormal or zero and are compared absolutely; the activations are compared at every layer."""
    import paper_1801_04928_amd as P
    N = 16
    net = make_net(L, N, 1, seed=L)
    g = P.LeapfrogNet(L, N, 1, "f32")
    g.load(net)
    if sched == "persistent":
        g.set_schedule(P.LF_SCHED_PERSISTENT)
    else:
        with pytest.raises(P.LfError) as e:
            g.set_schedule(P.LF_SCHED_PERSISTENT)
        assert e.value.status == P.LF_EUNSUPPORTED
    poison_buffers(g)
    g.forward()
    g.backward(8)
    import torch
    torch.cuda.synchronize()
    rep = check_against_oracle(net, g)
    assert len(rep.get("subnormal", [])) < 3 * (L - 1)      # the top layers met the relative bound
    log(f"L={L} N={N} {sched}: worst {rep['worst']:.2e}, {len(rep.get('subnormal', []))} tensors compared absolutely")
    _free(g)


# ---------------------------------------------------------------- Algorithm 1 as printed
@pytest.mark.parametrize("shape,k", [
    ((9, 516), 1),                  # one thread walks everything
    ((9, 516), 3),
    ((9, 516), 8),                  # k = L-1: the parent does every layer
    ((12, 1028), 5),                # some threads stop above layer 2
    ((260, 1028, 516, 64, 132, 8), 2),   # unequal widths
    ((4, 4100), 2),
])
def test_algorithm1_as_printed(shape, k):
    """LF_SCHED_REDUNDANT: every worker stream recomputes the delta chain it needs (Algorithm 1).  Theorem 1:
    the same gradients as the sequential pass -- here the same bits as the stream schedule, whose kernels
    it uses -- and the oracle's within the fp32 tolerance."""
    import torch
    import paper_1801_04928_amd as P
    if len(shape) == 2:
        L, N = shape
        net = make_net(L, N, 1, seed=N + k)
    else:
        L = len(shape)
        net = make_net(L, list(shape), 1, seed=sum(shape) + k)
    ref = run_gpu(net, min(2, L - 1), sched=P.LF_SCHED_STREAMS)
    want = [to_np(t).copy() for t in ref.nabla_w] + [to_np(t).copy() for t in ref.nabla_b]
    _free(ref)
    g = run_gpu(net, k, sched=P.LF_SCHED_REDUNDANT)
    rep = check_against_oracle(net, g)
    got = [to_np(t) for t in g.nabla_w] + [to_np(t) for t in g.nabla_b]
    for a, b in zip(want, got):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    # a second pass (the threads' private vectors are reused), then the limits
    poison_buffers(g, whole_workspace=False)
    g.forward()
    g.backward(k)
    torch.cuda.synchronize()
    for a, b in zip(want, [to_np(t) for t in g.nabla_w] + [to_np(t) for t in g.nabla_b]):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    if L - 1 > 8:
        with pytest.raises(P.LfError) as e:
            g.backward(9)
        assert e.value.status == P.LF_EUNSUPPORTED
    log(f"Algorithm 1 as printed {shape} k={k}: worst {rep['worst']:.2e}")
    _free(g)


def test_config1_full():
    net = config_net("cfg1", cache=True)
    g = run_gpu(net, 2)
    rep = check_against_oracle(net, g)
    log(f"cfg1: worst {rep['worst']:.2e}")
    _free(g)


def _clone_grads(g):
    return [t.clone() for t in g.nabla_w + g.nabla_b]


def _assert_same_bits(g, ref, what):
    torch = g.torch
    for i, (t, r) in enumerate(zip(g.nabla_w + g.nabla_b, ref)):
        assert bool(torch.equal(t.view(torch.int32), r.view(torch.int32))), f"{what}: tensor {i} differs"


@pytest.mark.parametrize("sched", ["streams", "persistent", "fused"])
@pytest.mark.parametrize("k", [1, 2, 4, 8])
def test_config2_full(k, sched):
    net = config_net("cfg2", cache=True)
    g = run_gpu(net, k, sched=SCHEDS[sched])
    rep = check_against_oracle(net, g)
    log(f"cfg2 k={k} {sched}: worst {rep['worst']:.2e}")
    _free(g)


@pytest.mark.parametrize("sched", ["streams", "persistent"])
def test_config2_same_bits_for_k_1_2_4_8(sched):
    """Configuration 2 at full size: the gradients of k = 1, 2, 4, 8 are the same bits (Theorem 1: leapfrogging
    changes who computes (bp3),(bp4), never what), and so are the on-chain fusion's."""
    import torch
    import paper_1801_04928_amd as P
    net = config_net("cfg2", cache=True)
    g = run_gpu(net, 1, sched=SCHEDS[sched])
    ref = _clone_grads(g)
    for k in (2, 4, 8):
        poison_buffers(g, whole_workspace=False)
        g.forward()
        g.backward(k)
        torch.cuda.synchronize()
        _assert_same_bits(g, ref, f"cfg2 {sched} k={k}")
    if sched == "persistent":
        g.set_schedule(P.LF_SCHED_FUSED)
        poison_buffers(g, whole_workspace=False)
        g.forward()
        g.backward(1)
        torch.cuda.synchronize()
        _assert_same_bits(g, ref, "cfg2 fused")
    _free(g)


def test_config3_full():
    """L=64: delta underflows into the fp32 subnormal range near the input; those layers are
    compared in denormal ulps and listed.  Persistent kernels, k = 8: against the oracle; k = 1 (the chain
    workgroups' in-line gradient bursts, rows taken from the row block), k = 4 and the on-chain fusion: the same
    bits as k = 8.  Stream schedule, k = 4 (another summation order): against the oracle."""
    import torch
    import paper_1801_04928_amd as P
    net = config_net("cfg3", cache=True)
    g = run_gpu(net, 8, sched=SCHEDS["persistent"])
    rep = check_against_oracle(net, g)
    log(f"cfg3 k=8 persistent: worst {rep['worst']:.2e}; subnormal tensors: {rep.get('subnormal', [])}")
    ref = _clone_grads(g)
    for k, sched in ((1, "persistent"), (4, "persistent"), (8, "fused")):
        g.set_schedule(SCHEDS[sched])
        poison_buffers(g, whole_workspace=False)
        g.forward()
        g.backward(k)
        torch.cuda.synchronize()
        _assert_same_bits(g, ref, f"cfg3 {sched} k={k}")
        log(f"cfg3 k={k} {sched}: same bits as k=8")
    del ref
    _free(g)
    g = run_gpu(net, 4, sched=SCHEDS["streams"])
    rep = check_against_oracle(net, g)
    log(f"cfg3 k=4 streams: worst {rep['worst']:.2e}; subnormal tensors: {rep.get('subnormal', [])}")
    _free(g)


def test_config3_fused_descent_step():
    """Configuration 3's shape with the descent step on, in the launch configuration the benchmark times
    (256 chain workgroups in row blocks, 256 worker workgroups, k = 8): the workers rewrite 63 matrices of
    64 MiB behind the chain.  Layer by layer, every stepped entry must be the fp32 value nearest to
    w - eta g for the g the library stores without the step (a worker that overwrote w^l before the chain had
    read it would change delta^{l-1} and with it every layer below)."""
    import torch
    import paper_1801_04928_amd as P
    net = config_net("cfg3", cache=False)
    s = net.spec
    g = P.LeapfrogNet(s.L, s.N, 1, "f32")
    g.load(net)
    g.set_cost_scale(60)                 # keeps the bottom layers' gradients in the normal range
    g.forward()
    g.backward(8)
    torch.cuda.synchronize()
    top = float(torch.max(torch.abs(g.nabla_w[-1])))
    eta = float(np.float32(0.05 * float(torch.max(torch.abs(g.w[-1]))) / top))
    grads = [t.clone() for t in g.nabla_w]
    old = [t.clone() for t in g.w]
    old_b = [to_np(t).copy() for t in g.b]
    grads_b = [to_np(t).astype(np.float64) for t in g.nabla_b]
    g.set_sgd(eta)
    g.forward()
    g.backward(8)
    torch.cuda.synchronize()
    for i in range(s.L - 1):
        want = to_np(old[i]).astype(np.float64) - eta * to_np(grads[i]).astype(np.float64)
        ulp = np.spacing(np.abs(want).astype(np.float32)).astype(np.float64)
        bad = np.abs(to_np(g.w[i]).astype(np.float64) - want) > 0.5000001 * ulp + 1e-300
        assert not bad.any(), f"layer {i + 2}: {int(bad.sum())} entries off"
        want_b = old_b[i].astype(np.float64) - eta * grads_b[i]
        assert np.all(np.abs(to_np(g.b[i]).astype(np.float64) - want_b)
                      <= 0.5000001 * np.spacing(np.abs(want_b).astype(np.float32)) + 1e-300)
        if (i + 2) % 16 == 0:
            log(f"  cfg3 fused step: layer {i + 2} checked")
    _free(g)


def _check_whole_gradient_against_library_product(g, layers, tol):
    """nabla_w^l as a whole against a plain fp32 matrix product (the vendor library's) of the GPU's own delta^l
    and a^{l-1}: every tile of the hand-written contraction, not only the sampled ones, must agree with an
    independent contraction of the same operands.  (For bf16 nets the operand is the bf16 copy of delta.)"""
    torch = g.torch
    for l in layers:
        d = g.delta(l)
        if g.dtype == "bf16":
            d = d.to(torch.bfloat16)
        want = d.float().t() @ g.activation(l - 1).float()
        got = g.grads(l)[0]
        err = float((got - want).abs().max() / want.abs().max())
        assert err <= tol, f"nabla_w^{l}: whole-matrix normwise difference {err:.2e}"
        del want


def test_config4_full_sampled():
    net = config_net("cfg4", cache=True)
    g = run_gpu(net, 4)
    rep = check_against_oracle(net, g, sample_tiles=(64, 128), rng=np.random.default_rng(4))
    assert rep["tiles_per_layer"] >= 64
    _check_whole_gradient_against_library_product(g, (2, 17, 32), 1e-5)
    log(f"cfg4 k=4: worst {rep['worst']:.2e} ({rep['tiles_per_layer']} tiles of 128 x 128 per layer)")
    _free(g)


def test_config5_full_sampled():
    net = config_net("cfg5", cache=False)
    g = run_gpu(net, 8)
    rep = check_against_oracle(net, g, sample_tiles=(64, 128), rng=np.random.default_rng(5))
    assert rep["tiles_per_layer"] >= 64
    _check_whole_gradient_against_library_product(g, (2, 25, 48), 1e-5)
    log(f"cfg5 k=8: worst {rep['worst']:.2e} ({rep['tiles_per_layer']} tiles of 128 x 128 per layer)")
    _free(g)
