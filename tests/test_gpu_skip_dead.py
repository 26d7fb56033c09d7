"""Inference with dead samples dropped (sdnn_forward_skip_dead) against the oracle's plain forward
pass and against sdnn_forward: the results must be identical, whatever the packing interval."""
import numpy as np
import pytest
import torch

from paper_2104_11805_amd import sdnn, workloads as wl
from tests import parity as P

pytestmark = pytest.mark.gpu

MIX = (0.02, 0.10, 0.25, 0.30, 0.33, 0.40)      # input densities: die at once ... never die


def _mixed_config1(b, n_layers=24):
    work = wl.make_config(1, n_layers=n_layers, b_infer=b, b_train=min(b, 64))
    work.x_infer = wl.mixed_density_inputs(8800 + b, work.layers[0].n_in, b, MIX)
    return work


@pytest.mark.parametrize("check_every", [1, 3, 8, 100])
@pytest.mark.parametrize("b", [200, 256, 1])
def test_skip_dead_equals_plain_forward(check_every, b):
    work = _mixed_config1(b)
    xs = P.O32.forward(work.layers, work.x_infer, work.act_cap)
    ref = xs[-1]
    if b > 1:
        dead_at_end = int((~(ref != 0).any(axis=0)).sum())
        alive_l1 = int((xs[1] != 0).any(axis=0).sum())
        assert 0 < dead_at_end < b and alive_l1 > b - dead_at_end, "the mix must hold samples that die at different depths"
    net = sdnn.Net(work.layers, work.act_cap, b, training=False)
    out = torch.full((work.layers[-1].n_out, b), 7.0, device=P.DEV)
    n_live = torch.full((1,), -1, dtype=torch.int32, device=P.DEV)
    for _ in range(2):                         # second call: the scratch state of the first must not leak
        net.sdnn_forward_skip_dead(P.dev(work.x_infer), out, check_every=check_every, n_live=n_live)
        assert np.array_equal(P.host(out), ref)
    # live count = non-zero columns at the last packing layer (none: the whole block)
    L = len(work.layers)
    last_check = ((L - 1) // check_every) * check_every
    expect = b if last_check == 0 or b == 1 else int((xs[last_check] != 0).any(axis=0).sum())   # one sample: never packed
    assert int(n_live.item()) == expect
    plain = torch.empty_like(out)
    net.sdnn_forward(P.dev(work.x_infer), plain)
    assert torch.equal(plain, out)
    net.close()


def test_skip_dead_all_dead_and_all_live():
    work = wl.make_config(1, n_layers=10, b_infer=128, b_train=64, density=0.40)
    net = sdnn.Net(work.layers, work.act_cap, 128, training=False)
    n_live = torch.zeros(1, dtype=torch.int32, device=P.DEV)
    out = torch.empty(1024, 128, device=P.DEV)
    ref = P.O32.forward(work.layers, work.x_infer, work.act_cap)[-1]
    net.sdnn_forward_skip_dead(P.dev(work.x_infer), out, check_every=2, n_live=n_live)
    assert np.array_equal(P.host(out), ref) and int(n_live.item()) == 128 and (ref != 0).all()
    zeros = torch.zeros(1024, 128, device=P.DEV)
    out.fill_(3.0)
    net.sdnn_forward_skip_dead(zeros, out, check_every=2, n_live=n_live)
    assert int(n_live.item()) == 0 and not out.any()
    net.close()


def test_skip_dead_rectangular_irregular_net():
    """Uneven rows, rectangular layers, mixed-sign weights, biases forced <= 0; a third of the input
    columns are zero and die in layer 1, others die by chance later or never."""
    work = wl.tiny_net(71, sizes=(90, 300, 150, 260, 40, 120), density=0.08, b=131)
    for l in work.layers:
        l.bias = -np.abs(l.bias)
    work.x_infer[:, ::3] = 0.0
    ref = P.O32.forward(work.layers, work.x_infer, work.act_cap)
    assert (ref[-1] != 0).any() and not ref[1][:, ::3].any()
    net = sdnn.Net(work.layers, work.act_cap, 131, training=False)
    out = torch.empty(120, 131, device=P.DEV)
    for k in (1, 2):
        net.sdnn_forward_skip_dead(P.dev(work.x_infer), out, check_every=k)
        assert np.array_equal(P.host(out), ref[-1])
    net.close()


def test_skip_dead_refuses_nets_where_dead_samples_can_revive():
    work = wl.tiny_net(72, sizes=(20, 30, 25, 10), density=0.3, b=8)
    x, out = P.dev(work.x_infer), torch.empty(10, 8, device=P.DEV)

    def refused(net, why):
        with pytest.raises(sdnn.SdnnError) as e:
            net.sdnn_forward_skip_dead(x, out)
        assert e.value.code == sdnn.SDNN_ESTATE and why in str(e.value)
        net.close()

    assert any((l.bias > 0).any() for l in work.layers[1:])
    refused(sdnn.Net(work.layers, work.act_cap, 8, training=False), "bias")
    for l in work.layers:
        l.bias = -np.abs(l.bias)
    refused(sdnn.Net(work.layers, work.act_cap, 8, training=True), "inference")
    refused(sdnn.Net(work.layers, work.act_cap, 8, training=False, activation="sigmoid"), "ReLU")
    # a positive bias in layer 1 alone is harmless; replacing a later bias is not inspected, hence refused
    work.layers[0].bias = np.abs(work.layers[0].bias)
    net = sdnn.Net(work.layers, work.act_cap, 8, training=False)
    net.sdnn_forward_skip_dead(x, out, check_every=1)
    assert np.array_equal(P.host(out), P.O32.forward(work.layers, work.x_infer, work.act_cap)[-1])
    with pytest.raises(sdnn.SdnnError) as e:
        net.sdnn_forward_skip_dead(x, out, check_every=0)
    assert e.value.code == sdnn.SDNN_EINVAL
    net.sdnn_set_weights(2, None, P.dev(work.layers[1].bias))
    refused(net, "bias")


def test_skip_dead_block_size_limits():
    """The packing kernel holds one position per sample in LDS: 8192 samples work, more are refused."""
    work = wl.tiny_net(73, sizes=(24, 40, 16), density=0.3, b=8192)
    for l in work.layers:
        l.bias = -np.abs(l.bias)
    work.x_infer[:, 5::7] = 0.0
    ref = P.O32.forward(work.layers, work.x_infer, work.act_cap)[-1]
    net = sdnn.Net(work.layers, work.act_cap, 9000, training=False)
    out = torch.empty(16, 8192, device=P.DEV)
    n_live = torch.zeros(1, dtype=torch.int32, device=P.DEV)
    net.sdnn_forward_skip_dead(P.dev(work.x_infer), out, check_every=1, n_live=n_live)
    assert np.array_equal(P.host(out), ref)
    assert 0 < int(n_live.item()) <= 8192 - len(range(5, 8192, 7))
    big = torch.zeros(24, 9000, device=P.DEV)
    with pytest.raises(sdnn.SdnnError) as e:
        net.sdnn_forward_skip_dead(big, torch.empty(16, 9000, device=P.DEV))
    assert e.value.code == sdnn.SDNN_EINVAL and "8192" in str(e.value)
    net.close()


@pytest.mark.parametrize("seed", range(8))
def test_skip_dead_seeded_random_nets(seed):
    rng = np.random.default_rng(9500 + seed)
    depth = int(rng.integers(2, 7))
    sizes = tuple(int(x) for x in rng.integers(1, 200, size=depth + 1))
    b = int(rng.choice([2, 31, 64, 65, 255, 256, 300, 1024]))
    k = int(rng.choice([1, 2, 3, 5]))
    work = wl.tiny_net(400 + seed, sizes=sizes, density=float(rng.choice([0.05, 0.2, 0.6])), b=b,
                       cap=float(rng.choice([np.inf, 2.0])))
    for l in work.layers:
        l.bias = -np.abs(l.bias) * float(rng.choice([0.0, 1.0, 4.0]))     # larger negative biases kill more samples
    work.x_infer[:, rng.random(b) < 0.3] = 0.0
    ref = P.O32.forward(work.layers, work.x_infer, work.act_cap)[-1]
    net = sdnn.Net(work.layers, work.act_cap, b, training=False)
    out = torch.full((sizes[-1], b), -1.0, device=P.DEV)
    net.sdnn_forward_skip_dead(P.dev(work.x_infer), out, check_every=k)
    assert np.array_equal(P.host(out), ref), f"seed {seed}: sizes {sizes} b {b} every {k}"
    net.close()
