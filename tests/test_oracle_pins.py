"""Pins for the CPU oracle: checks against things other than itself.

The paper prints no numeric worked example (its example figures are images), so
the oracle is pinned by: dense matrix algebra on tiny nets (numpy), an
independent sparse library (scipy) in the linear special case, closed forms on
the benchmark topology, central finite differences of the loss for every
stored weight and bias, and structural invariants.  CPU only.
"""
import numpy as np
import pytest
import scipy.sparse as sp

from oracle.sdnn_oracle import (Oracle, mse_dloss, mse_loss, softmax_ce_dloss, softmax_ce_loss)
from paper_2104_11805_amd import workloads as wl

O32 = Oracle(np.float32)
O64 = Oracle(np.float64)


def dense(layer, dtype=np.float64):
    w = np.zeros((layer.n_out, layer.n_in), dtype=dtype)
    for j in range(layer.n_out):
        for p in range(layer.row_ptr[j], layer.row_ptr[j + 1]):
            w[j, layer.col_idx[p]] = layer.values[p]
    return w


def dense_forward(layers, x0, cap):
    """Eq. 3 with dense fp64 matrices; returns (xs, zs)."""
    xs, zs = [x0.astype(np.float64)], [None]
    for l in layers:
        z = dense(l) @ xs[-1] + l.bias.astype(np.float64)[:, None]
        zs.append(z)
        xs.append(np.minimum(np.maximum(z, 0.0), cap))
    return xs, zs


# --------------------------------------------------------------------------
# forward: dense algebra, library routine, closed forms
# --------------------------------------------------------------------------

@pytest.mark.parametrize("seed", [1, 2, 3])
@pytest.mark.parametrize("cap", [np.inf, 0.9])
def test_forward_matches_dense_algebra(seed, cap):
    net = wl.tiny_net(seed, sizes=(11, 17, 13, 9), b=6, cap=cap)
    ref, _ = dense_forward(net.layers, net.x_infer, cap)
    got64 = O64.forward(net.layers, net.x_infer, cap)
    got32 = O32.forward(net.layers, net.x_infer, cap)
    for k in range(1, len(ref)):
        np.testing.assert_allclose(got64[k], ref[k], rtol=1e-13, atol=1e-14)
        np.testing.assert_allclose(got32[k], ref[k], rtol=2e-6, atol=1e-6)
    if np.isfinite(cap):
        assert any((x == cap).any() for x in got64[1:]), "cap never reached: test does not bite"
    assert any((x == 0).any() for x in got64[1:])


def test_forward_linear_case_is_a_chain_of_scipy_products():
    """cap = inf, weights, inputs and biases >= 0: ReLU is the identity."""
    rng = np.random.default_rng(7)
    layers = []
    for l in range(4):
        lay = wl.random_layer(70 + l, 40, 40, 0.2)
        lay.values = np.abs(lay.values)
        lay.bias = np.abs(lay.bias)
        layers.append(lay)
    x0 = rng.random((40, 9)).astype(np.float32)
    got = O64.forward(layers, x0, np.inf)[-1]
    x = x0.astype(np.float64)
    for lay in layers:
        m = sp.csr_matrix((lay.values.astype(np.float64), lay.col_idx, lay.row_ptr),
                          shape=(lay.n_out, lay.n_in))
        x = m @ x + lay.bias.astype(np.float64)[:, None]
    np.testing.assert_allclose(got, x, rtol=1e-13)


@pytest.mark.parametrize("bias", [-0.3, -0.45, 0.25])
def test_forward_closed_form_on_benchmark_topology(bias):
    """32 links of weight 1/16 per neuron: every row sums to 2, whatever the
    pattern.  With an all-ones input every neuron of layer k therefore equals
    u_k = min(32, max(0, 2 u_{k-1} + b)), u_0 = 1 (a scalar recurrence)."""
    layers = [wl.regular_layer(300 + l, 512, 32, 0.0625, bias) for l in range(9)]
    xs = O32.forward(layers, np.ones((512, 3), np.float32), 32.0)
    u = 1.0
    for k in range(1, 10):
        u = min(32.0, max(0.0, 2.0 * u + float(np.float32(bias))))
        np.testing.assert_allclose(xs[k], u, rtol=1e-6)
    assert (xs[9] == 32.0).all()
    # all-zero input: b <= 0 stays dead, b > 0 grows as b (2^k - 1)
    xs0 = O32.forward(layers, np.zeros((512, 2), np.float32), 32.0)
    for k in range(1, 6):
        expect = 0.0 if bias <= 0 else min(32.0, float(np.float32(bias)) * (2 ** k - 1))
        np.testing.assert_allclose(xs0[k], expect, rtol=1e-6, atol=0)


def test_forward_samples_are_independent_bitwise():
    net = wl.make_config(1, n=256, n_layers=5, b_infer=16, density=0.4)
    full = O32.forward(net.layers, net.x_infer, net.act_cap)
    for s in (0, 7, 15):
        one = O32.forward(net.layers, net.x_infer[:, s:s + 1], net.act_cap)
        for k in range(len(full)):
            assert np.array_equal(full[k][:, s], one[k][:, 0])


def test_range_and_degeneracy_of_nominal_config1():
    """0 <= x <= cap everywhere; at the nominal 10% input density the net is
    dead from layer 2 on (every activation exactly zero)."""
    net = wl.make_config(1, n_layers=6)
    xs = O32.forward(net.layers, net.x_infer, net.act_cap)
    for x in xs:
        assert (x >= 0).all() and (x <= net.act_cap).all()
    assert (xs[1] > 0).mean() > 0.1
    assert all((x == 0).all() for x in xs[2:])
    live = wl.make_config(1, n_layers=6, density=0.4)
    xl = O32.forward(live.layers, live.x_infer, live.act_cap)
    assert all((x > 0).mean() > 0.99 and (x < 32).all() for x in xl[1:])


# --------------------------------------------------------------------------
# backward / gradient: dense algebra
# --------------------------------------------------------------------------

@pytest.mark.parametrize("cap", [np.inf, 0.9])
def test_backward_and_gradient_match_dense_algebra(cap):
    net = wl.tiny_net(5, sizes=(10, 14, 12, 8), b=7, cap=cap)
    xs, zs = dense_forward(net.layers, net.x_infer, cap)
    dloss = np.random.default_rng(3).standard_normal(xs[-1].shape)
    oxs = O64.forward(net.layers, net.x_infer, cap)
    od = O64.backward(net.layers, oxs, dloss, cap)
    og = O64.gradients(net.layers, oxs, od)
    L = len(net.layers)
    fp = lambda z: ((z > 0) & (z < cap)).astype(np.float64)
    d = [None] * (L + 1)
    d[L] = dloss * fp(zs[L])
    for k in range(L, 1, -1):
        d[k - 1] = (dense(net.layers[k - 1]).T @ d[k]) * fp(zs[k - 1])
    assert od[0] is None
    for k in range(1, L + 1):
        np.testing.assert_allclose(od[k], d[k], rtol=1e-12, atol=1e-14)
        lay = net.layers[k - 1]
        full = d[k] @ xs[k - 1].T                       # the dense outer-product sum
        rows = np.repeat(np.arange(lay.n_out), np.diff(lay.row_ptr))
        np.testing.assert_allclose(og[k - 1][0], full[rows, lay.col_idx], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(og[k - 1][1], d[k].sum(axis=1), rtol=1e-12, atol=1e-14)
    assert any((np.asarray(x) == 0).any() for x in od[1:]), "mask never bites"


def test_backward_closed_form_counts_column_links():
    """All masks open and a uniform delta gamma: (W^T delta)(i) = gamma * colnnz(i)/16,
    and g(p) = B * gamma * x_prev for every stored entry."""
    lay = wl.regular_layer(41, 512, 32, 0.0625, -0.3)
    b = 4
    xprev = np.full((512, b), 0.5, np.float32)
    delta = np.full((512, b), 0.25, np.float32)
    got = O32.backward_layer(lay, delta, xprev, 32.0)
    colnnz = np.bincount(lay.col_idx, minlength=512)
    assert colnnz.sum() == lay.nnz and colnnz.min() != colnnz.max()
    np.testing.assert_array_equal(got, (0.25 * colnnz / 16.0).astype(np.float32)[:, None].repeat(b, 1))
    g, gb = O32.weight_grad(lay, delta, xprev)
    np.testing.assert_array_equal(g, np.float32(b * 0.25 * 0.5))
    np.testing.assert_array_equal(gb, np.float32(b * 0.25))
    # closed mask (x_prev at 0 or at the cap) kills the delta
    assert (O32.backward_layer(lay, delta, np.zeros_like(xprev), 32.0) == 0).all()
    assert (O32.backward_layer(lay, delta, np.full_like(xprev, 32.0), 32.0) == 0).all()


def test_output_delta_mask():
    x = np.array([[0.0, 0.5, 32.0, 31.999]], np.float32)
    dl = np.array([[2.0, 3.0, 4.0, 5.0]], np.float32)
    np.testing.assert_array_equal(O32.output_delta(dl, x, 32.0), [[0.0, 3.0, 0.0, 5.0]])
    np.testing.assert_array_equal(O32.output_delta(dl, x, np.inf), [[0.0, 3.0, 4.0, 5.0]])


# --------------------------------------------------------------------------
# gradients: central finite differences of the loss (delta is dJ/dz, Section 3.2)
# --------------------------------------------------------------------------

def _kink_free(layers, x0, cap, margin):
    _, zs = dense_forward(layers, x0, cap)
    for z in zs[1:]:
        if (np.abs(z) < margin).any():
            return False
        if np.isfinite(cap) and (np.abs(z - cap) < margin).any():
            return False
    return True


def _fd_check(net, loss_fn, dloss_fn, cap, h=1e-6, tol=2e-7):
    x0 = net.x_infer
    assert _kink_free(net.layers, x0, cap, 1e-3), "reseed: a pre-activation sits on a kink"
    xs = O64.forward(net.layers, x0, cap)
    deltas = O64.backward(net.layers, xs, dloss_fn(xs[-1]), cap)
    grads = O64.gradients(net.layers, xs, deltas)

    def J():
        return loss_fn(O64.forward(net.layers, x0, cap)[-1])

    checked = nonzero = 0
    for k, lay in enumerate(net.layers):
        lay.values = lay.values.astype(np.float64)
        lay.bias = lay.bias.astype(np.float64)
    scale = max(max(np.abs(g).max(), np.abs(gb).max()) for g, gb in grads)
    for k, lay in enumerate(net.layers):
        for arr, g in ((lay.values, grads[k][0]), (lay.bias, grads[k][1])):
            for p in range(arr.size):
                keep = arr[p]
                arr[p] = keep + h
                jp = J()
                arr[p] = keep - h
                jm = J()
                arr[p] = keep
                fd = (jp - jm) / (2 * h)
                assert abs(fd - g[p]) <= tol * scale + 1e-9 * abs(g[p]), (k, p, fd, g[p])
                checked += 1
                nonzero += g[p] != 0
    assert nonzero > checked // 4, "most gradients are zero: test does not bite"
    return xs


@pytest.mark.parametrize("seed", [11, 12])
def test_gradients_by_finite_differences_mse(seed):
    net = wl.tiny_net(seed, sizes=(6, 8, 7, 5), b=4, density=0.5)
    _fd_check(net, lambda xl: mse_loss(xl, net.targets), lambda xl: mse_dloss(xl, net.targets), np.inf)


def test_gradients_by_finite_differences_with_active_cap():
    net = wl.tiny_net(19, sizes=(6, 8, 7, 5), b=4, density=0.6, scale=1.5)
    cap = 2.0
    xs = _fd_check(net, lambda xl: mse_loss(xl, net.targets), lambda xl: mse_dloss(xl, net.targets), cap)
    assert sum(int((x == cap).sum()) for x in xs[1:]) >= 3, "no neuron sits at the cap"


def test_gradients_by_finite_differences_softmax_ce():
    net = wl.tiny_net(14, sizes=(6, 9, 8), b=5, density=0.5)
    labels = np.array([0, 2, 1, 2, 0])
    _fd_check(net, lambda xl: softmax_ce_loss(xl, labels, 3), lambda xl: softmax_ce_dloss(xl, labels, 3), np.inf)


# --------------------------------------------------------------------------
# update: invariants
# --------------------------------------------------------------------------

def test_sgd_step_invariants():
    net = wl.tiny_net(21, sizes=(9, 12, 10), b=6)
    patt = [(l.row_ptr.copy(), l.col_idx.copy()) for l in net.layers]
    dfn = lambda xl: mse_dloss(xl, net.targets)
    xs, deltas, grads, new = O32.train_step(net.layers, net.x_infer, np.inf, dfn, 0.01)
    for lay, (rp, ci), (g, gb), (v, b) in zip(net.layers, patt, grads, new):
        assert np.array_equal(lay.row_ptr, rp) and np.array_equal(lay.col_idx, ci)
        assert v.shape == lay.values.shape and v.dtype == np.float32
        lr = np.float64(np.float32(0.01))
        np.testing.assert_array_equal(v, (lay.values.astype(np.float64) - lr * g.astype(np.float64)).astype(np.float32))
        np.testing.assert_array_equal(b, (lay.bias.astype(np.float64) - lr * gb.astype(np.float64)).astype(np.float32))
        assert (v != lay.values).any()
    _, _, _, same = O32.train_step(net.layers, net.x_infer, np.inf, dfn, 0.0)
    for lay, (v, b) in zip(net.layers, same):
        assert np.array_equal(v, lay.values) and np.array_equal(b, lay.bias)
    _, _, _, frozen = O32.train_step(net.layers, net.x_infer, np.inf, dfn, 0.01, update_bias=False)
    assert all(np.array_equal(b, lay.bias) for lay, (v, b) in zip(net.layers, frozen))


def test_sgd_step_decreases_the_loss():
    net = wl.tiny_net(22, sizes=(9, 12, 10), b=6)
    dfn = lambda xl: mse_dloss(xl, net.targets)
    j0 = mse_loss(O64.forward(net.layers, net.x_infer, np.inf)[-1], net.targets)
    for _ in range(20):
        _, _, _, new = O64.train_step(net.layers, net.x_infer, np.inf, dfn, 0.05)
        for lay, (v, b) in zip(net.layers, new):
            lay.values, lay.bias = v, b
    j1 = mse_loss(O64.forward(net.layers, net.x_infer, np.inf)[-1], net.targets)
    assert j1 < 0.9 * j0


def test_backward_samples_are_independent_bitwise():
    net = wl.make_config(1, n=256, n_layers=5, b_infer=8, density=0.4)
    xs = O32.forward(net.layers, net.x_infer, net.act_cap)
    dl = mse_dloss(xs[-1], net.targets)
    full = O32.backward(net.layers, xs, dl, net.act_cap)
    s = 3
    one = O32.backward(net.layers, [x[:, s:s + 1] for x in xs], dl[:, s:s + 1], net.act_cap)
    for k in range(1, len(full)):
        assert np.array_equal(full[k][:, s], one[k][:, 0])
        assert (full[k] != 0).any()


def test_cap_is_a_number_of_the_storage_precision():
    """A neuron clamped at a cap that fp32 cannot represent exactly (0.9) must
    still read as saturated (derivative 0) from its stored fp32 output."""
    lay = wl.random_layer(1, 4, 4, 1.0)
    lay.values = np.full(lay.nnz, 1.0, np.float32)
    lay.bias = np.zeros(4, np.float32)
    x1 = O32.forward_layer(lay, np.ones((4, 1), np.float32), 0.9)
    assert (x1 == np.float32(0.9)).all()
    d = O32.output_delta(np.ones((4, 1), np.float32), x1, 0.9)
    assert (d == 0).all()


# --------------------------------------------------------------------------
# sigmoid activation (the paper's own training setup, Section 6.1)
# --------------------------------------------------------------------------

S64 = Oracle(np.float64, "sigmoid")
S32 = Oracle(np.float32, "sigmoid")


def test_sigmoid_forward_backward_match_dense_algebra():
    net = wl.tiny_net(41, sizes=(9, 13, 11, 7), b=5)
    sig = lambda z: 1.0 / (1.0 + np.exp(-z))
    xs = [net.x_infer.astype(np.float64)]
    for l in net.layers:
        xs.append(sig(dense(l) @ xs[-1] + l.bias.astype(np.float64)[:, None]))
    got = S64.forward(net.layers, net.x_infer, np.inf)
    for k in range(1, 4):
        np.testing.assert_allclose(got[k], xs[k], rtol=1e-13)
        np.testing.assert_allclose(S32.forward(net.layers, net.x_infer, np.inf)[k], xs[k], rtol=3e-7)
        assert (got[k] > 0).all() and (got[k] < 1).all()
    dloss = np.random.default_rng(4).standard_normal(xs[-1].shape)
    od = S64.backward(net.layers, got, dloss, np.inf)
    d = [None] * 4
    d[3] = dloss * xs[3] * (1 - xs[3])
    for k in (3, 2):
        d[k - 1] = (dense(net.layers[k - 1]).T @ d[k]) * xs[k - 1] * (1 - xs[k - 1])
    for k in (1, 2, 3):
        np.testing.assert_allclose(od[k], d[k], rtol=1e-12, atol=1e-15)
    # closed form: zero weights and bias give 0.5 everywhere, f' = 0.25
    lay = wl.regular_layer(5, 64, 32, 0.0, 0.0)
    assert (S32.forward_layer(lay, np.ones((64, 2), np.float32), np.inf) == 0.5).all()
    assert (S32.output_delta(np.ones((64, 2), np.float32), np.full((64, 2), 0.5, np.float32), np.inf) == 0.25).all()


def test_sigmoid_gradients_by_finite_differences():
    net = wl.tiny_net(42, sizes=(6, 8, 7, 5), b=3, density=0.5)
    x0 = net.x_infer
    xs = S64.forward(net.layers, x0, np.inf)
    deltas = S64.backward(net.layers, xs, mse_dloss(xs[-1], net.targets), np.inf)
    grads = S64.gradients(net.layers, xs, deltas)
    for lay in net.layers:
        lay.values = lay.values.astype(np.float64)
        lay.bias = lay.bias.astype(np.float64)
    J = lambda: mse_loss(S64.forward(net.layers, x0, np.inf)[-1], net.targets)
    h, worst, scale = 1e-5, 0.0, max(np.abs(g).max() for g, _ in grads)
    for k, lay in enumerate(net.layers):
        for arr, g in ((lay.values, grads[k][0]), (lay.bias, grads[k][1])):
            for p in range(arr.size):
                keep = arr[p]
                arr[p] = keep + h; jp = J()
                arr[p] = keep - h; jm = J()
                arr[p] = keep
                worst = max(worst, abs((jp - jm) / (2 * h) - g[p]))
                assert g[p] != 0
    assert worst <= 1e-8 * max(scale, 1e-3), worst      # smooth activation: O(h^2) error only


def test_oracle_results_do_not_depend_on_the_thread_count():
    """The OpenMP loops split independent outputs only: one thread and all threads give the same bits
    in every pass (this is what lets the timing leg change the thread count)."""
    from oracle.sdnn_oracle import Oracle, mse_dloss
    work = wl.tiny_net(97, sizes=(60, 90, 70, 40), density=0.2, b=37)
    orc = Oracle(np.float32)
    n_all = orc.threads()
    dfn = lambda x: mse_dloss(x, work.targets)
    try:
        orc.set_threads(1)
        one = orc.train_step(work.layers, work.x_infer, work.act_cap, dfn, 0.05)
        orc.set_threads(max(2, n_all))
        many = orc.train_step(work.layers, work.x_infer, work.act_cap, dfn, 0.05)
    finally:
        orc.set_threads(n_all)
    for a, c in zip(one[0], many[0]):
        assert np.array_equal(a, c)
    for a, c in zip(one[1][1:], many[1][1:]):
        assert np.array_equal(a, c)
    for (ga, gba), (gc, gbc) in zip(one[2], many[2]):
        assert np.array_equal(ga, gc) and np.array_equal(gba, gbc)
    for (va, ba), (vc, bc) in zip(one[3], many[3]):
        assert np.array_equal(va, vc) and np.array_equal(ba, bc)
