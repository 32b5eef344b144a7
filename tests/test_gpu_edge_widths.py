"""GPU tests of the persistent kernels on nets whose first and last layer are narrower than the rest (section 2:
the equations hold for any widths): an input of n_1 and an output of n_L neurons around hidden layers of one
width N.  w^2 is N x n_1, w^L is n_L x N; every step in between is the square one of the five configurations."""
import numpy as np
import pytest

from lf_inputs import make_net
from tests.gpu_util import check_against_oracle, log, run_gpu, to_np

pytestmark = pytest.mark.gpu


def _bits(g):
    return [to_np(t).copy().view(np.uint32) for t in g.nabla_w + g.nabla_b]


SHAPES = [
    ((8, 4), (1,)),                                  # one weight layer, 4 x 8
    ((4, 8), (1,)),                                  # one weight layer, 8 x 4
    ((64, 256, 32), (1, 2)),                         # one hidden layer: both matrices are edge matrices
    ((64, 256, 256, 256, 32), (1, 2, 4)),            # one chunk per step
    ((4, 260, 260, 260, 260), (1, 3)),               # the narrowest input, ragged strips, a full-width output
    ((516, 1028, 1028, 1028, 1028, 260), (1, 2, 5)), # ragged everywhere
    ((1000, 1000, 1000, 8), (1, 2)),                 # a full-width input, a two-vector output
    ((512, 2048, 2048, 2048, 128), (1, 3)),          # whole-height strips, several chunks per step
    ((1024, 3076, 3076, 3076, 12), (1, 3)),          # four row blocks per strip, ragged; most row blocks of w^L empty
    ((1024, 4096, 4096, 4096, 4096, 4096, 256), (1, 4)),   # 1024 in, five hidden layers of 4096, 256 out
]


@pytest.mark.parametrize("widths,ks", SHAPES)
def test_narrow_first_and_last_layer_on_the_persistent_path(widths, ks):
    """Forward and backward through the persistent kernels (the schedule is set explicitly: a shape they do not
    take would be refused) against the oracle; the same bits for every k; the same bits from the on-chain
    fusion."""
    import torch
    import paper_1801_04928_amd as P
    L = len(widths)
    net = make_net(L, list(widths), 1, seed=sum(widths) + L)
    ref = None
    for k in ks:
        if k > L - 1:
            continue
        g = run_gpu(net, k, sched=P.LF_SCHED_PERSISTENT)
        rep = check_against_oracle(net, g)
        for l in range(2, L + 1):
            gw, gb = g.grads(l)
            assert tuple(gw.shape) == (widths[l - 1], widths[l - 2]) and tuple(gb.shape) == (widths[l - 1],)
        bits = _bits(g)
        if ref is None:
            ref = bits
            log(f"widths {widths} k={k}: worst normwise error {rep['worst']:.2e}")
        else:
            for i, (a, b) in enumerate(zip(ref, bits)):
                assert np.array_equal(a, b), f"k={k}: tensor {i} differs from k={ks[0]}"
        # a second pass on the same handle (the tags of the first are still in the exchange buffers)
        g.forward()
        g.backward(k)
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(zip(ref, _bits(g))):
            assert np.array_equal(a, b), f"k={k}, second pass: tensor {i}"
        g.close()
    g = run_gpu(net, 1, sched=P.LF_SCHED_FUSED)
    check_against_oracle(net, g)
    for i, (a, b) in enumerate(zip(ref, _bits(g))):
        assert np.array_equal(a, b), f"on-chain fusion: tensor {i}"
    g.close()


def test_auto_takes_the_persistent_kernels_for_such_a_net():
    """LF_SCHED_AUTO gives the bits of LF_SCHED_PERSISTENT (the stream schedule sums in another order), and the
    stream schedule still agrees with the oracle."""
    import paper_1801_04928_amd as P
    widths = [132, 520, 520, 520, 68]
    net = make_net(len(widths), widths, 1, seed=77)
    g = run_gpu(net, 2, sched=P.LF_SCHED_PERSISTENT)
    want = _bits(g)
    g.close()
    g = run_gpu(net, 2)
    for a, b in zip(want, _bits(g)):
        assert np.array_equal(a, b)
    g.close()
    g = run_gpu(net, 2, sched=P.LF_SCHED_STREAMS)
    check_against_oracle(net, g)
    g.close()


def test_shapes_the_persistent_kernels_refuse():
    """A hidden layer of another width, or an input or output wider than the hidden layers: stream schedule."""
    import paper_1801_04928_amd as P
    for widths in ([64, 256, 128, 256, 32], [512, 256, 256, 32], [64, 256, 256, 512]):
        g = P.LeapfrogNet(len(widths), widths, 1, "f32")
        with pytest.raises(P.LfError) as e:
            g.set_schedule(P.LF_SCHED_PERSISTENT)
        assert e.value.status == P.LF_EUNSUPPORTED
        g.close()


def test_cost_scale_on_a_narrow_output():
    """The power-of-two cost scale enters at delta^L, here a vector shorter than N: gradients scale exactly."""
    import torch
    import paper_1801_04928_amd as P
    widths = [64, 256, 256, 32]
    net = make_net(4, widths, 1, seed=5)
    g = run_gpu(net, 2, sched=P.LF_SCHED_PERSISTENT)
    plain = [to_np(t).copy() for t in g.nabla_w + g.nabla_b]
    g.set_cost_scale(10)
    g.forward()
    g.backward(2)
    torch.cuda.synchronize()
    for a, b in zip(plain, [to_np(t) for t in g.nabla_w + g.nabla_b]):
        assert np.array_equal(a * np.float32(1024.0), b)
    g.close()
