"""sdnn_forward_noalloc (the entry point for callers that cannot allocate) against sdnn_forward,
through the C ABI: same bits, on two calls in a row, the second with a smaller input; the limits
are refused with a clear error."""
import numpy as np
import pytest
import torch

from paper_2104_11805_amd import sdnn, workloads as wl
from tests import parity as P

pytestmark = pytest.mark.gpu


def _net(seed, sizes, density, max_batch):
    layers = [wl.random_layer(seed * 100 + l, sizes[l + 1], sizes[l], density) for l in range(len(sizes) - 1)]
    return layers, sdnn.Net(layers, 1.5, max_batch, training=False)


def test_noalloc_forward_equals_forward_twice_in_a_row_and_the_oracle():
    sizes = (300, 1000, 517, 1000, 64)
    layers, net = _net(31, sizes, 0.03, 260)
    for b in (260, 37):            # the second call is smaller: stale contents of the array stay out of the result
        x = wl.normal_inputs(7700 + b, sizes[0], b)
        xd = P.dev(x)
        ref = torch.empty(sizes[-1], b, device=P.DEV)
        got = torch.full((sizes[-1], b), -7.0, device=P.DEV)
        net.sdnn_forward(xd, ref)
        net.sdnn_forward_noalloc(xd, got)
        assert torch.equal(ref, got), f"B = {b}"
        orc = P.O32.forward(layers, x, 1.5)[-1]
        P.assert_forward_close(P.host(got), orc, f"noalloc B = {b}")
        assert np.array_equal(P.host(got), orc)
    net.close()


def test_noalloc_uniform_net_and_one_layer_net():
    work = wl.make_config(1, n_layers=9, density=0.35)
    net = sdnn.Net(work.layers, work.act_cap, 64, training=False)
    xd = P.dev(work.x_infer)
    ref = torch.empty(1024, 64, device=P.DEV)
    got = torch.empty(1024, 64, device=P.DEV)
    net.sdnn_forward(xd, ref)
    net.sdnn_forward_noalloc(xd, got)
    assert torch.equal(ref, got) and float(got.max()) > 0
    net.close()
    one = sdnn.Net(work.layers[:1], work.act_cap, 64, training=False)   # no staging needed at all
    one.sdnn_forward(xd, ref)
    one.sdnn_forward_noalloc(xd, got)
    assert torch.equal(ref, got)
    one.close()


def test_noalloc_refuses_what_does_not_fit_and_training_nets():
    n = 4096
    layers = [wl.regular_layer(88 + l, n, 4, 0.25, -0.1) for l in range(2)]
    net = sdnn.Net(layers, 32.0, 1024, training=False)
    limit = sdnn.SDNN_NOALLOC_SCRATCH_BYTES // 2 // (4 * n)            # 512 samples
    x = torch.zeros(n, limit + 1, device=P.DEV)
    out = torch.empty(n, limit + 1, device=P.DEV)
    with pytest.raises(sdnn.SdnnError) as e:
        net.sdnn_forward_noalloc(x, out)
    assert e.value.code == sdnn.SDNN_EINVAL and "smaller B" in str(e.value)
    xs = P.dev(wl.binary_inputs(5, n, limit, 0.5))
    ref = torch.empty(n, limit, device=P.DEV)
    got = torch.empty(n, limit, device=P.DEV)
    net.sdnn_forward(xs, ref)
    net.sdnn_forward_noalloc(xs, got)                                   # exactly at the limit
    assert torch.equal(ref, got) and float(got.max()) > 0
    net.close()
    tr = sdnn.Net(layers, 32.0, 8, training=True)
    with pytest.raises(sdnn.SdnnError) as e:
        tr.sdnn_forward_noalloc(torch.zeros(n, 8, device=P.DEV), torch.empty(n, 8, device=P.DEV))
    assert e.value.code == sdnn.SDNN_ESTATE
    tr.close()
