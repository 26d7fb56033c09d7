"""GPU-vs-oracle parity through the C ABI, on seeded synthetic workloads.

Bar: forward max relative error 1e-5 and identical active sets; deltas,
gradients and updated weights within 1e-4 relative or 1e-6 absolute.  Since
both sides accumulate exact fp32 x fp32 products in fp64 in the same order,
the forward and backward results are in fact expected to be bit-identical and
the tests say so where the kernel's summation order equals the oracle's.
"""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2104_11805_amd import sdnn, workloads as wl
from tests import parity as P

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("b", [1, 5, 64, 67, 130, 260])
@pytest.mark.parametrize("cap", [float("inf"), 0.9])
def test_tiny_rectangular_net_all_passes(b, cap):
    work = wl.tiny_net(31, sizes=(37, 70, 33, 129, 20), density=0.3, b=b, cap=cap)
    x0 = work.x_infer
    g = P.gpu_train_step(work, x0, lr=0.05)
    o = P.oracle_train_step(work, x0, lr=0.05)
    st = P.compare_step(g, o, f"tiny b={b} cap={cap}")
    assert st["live_d"] == st["layers"] and st["live_g"] == st["layers"]
    assert st["bitexact_d"] == st["layers"]
    for lay, (v, bias) in zip(work.layers, g["new"]):
        assert (v != lay.values).any() and (bias != lay.bias).any()


def test_empty_rows_empty_columns_and_zero_nnz_layer():
    work = wl.tiny_net(32, sizes=(12, 40, 16, 9), density=0.08, b=7)
    lens = [np.diff(l.row_ptr) for l in work.layers]
    assert any((x == 0).any() for x in lens), "no empty row drawn"
    # make the middle layer completely empty: its outputs are f(bias)
    mid = work.layers[1]
    mid.row_ptr = np.zeros_like(mid.row_ptr); mid.col_idx = mid.col_idx[:0]; mid.values = mid.values[:0]
    g = P.gpu_train_step(work, work.x_infer, lr=0.05)
    o = P.oracle_train_step(work, work.x_infer, lr=0.05)
    P.compare_step(g, o, "empty")
    assert g["new"][1][0].size == 0
    assert (g["new"][1][1] != mid.bias).any(), "bias of a link-less neuron must still train"


def test_live_config1_prefix_training_step():
    """Depth-6 prefix of config 1 at input density 0.40: every mask open, dense
    non-zero deltas and gradients in every layer."""
    work = wl.make_config(1, n_layers=6, density=0.40)
    g = P.gpu_train_step(work, work.x_train)
    o = P.oracle_train_step(work, work.x_train)
    st = P.compare_step(g, o, "cfg1-live")
    assert st["live_d"] == 6 and st["live_g"] == 6 and st["bitexact_d"] == 6
    for k in range(1, 7):
        assert (o["deltas"][k] != 0).mean() > 0.9


@pytest.mark.parametrize("density", [0.10, 0.30])
def test_config1_full_depth(density):
    """Config 1 verbatim (dead after layer 1 at density 0.10) and its live
    forward companion at 0.30 (mixed transient, then saturated or dead)."""
    work = wl.make_config(1, density=density)
    g = P.gpu_train_step(work, work.x_train)
    o = P.oracle_train_step(work, work.x_train)
    st = P.compare_step(g, o, f"cfg1 d={density}")
    frac = [float((x > 0).mean()) for x in o["xs"]]
    if density == 0.10:
        assert frac[1] > 0.1 and max(frac[2:]) == 0.0          # the degeneracy is visible
        assert all((d == 0).all() for d in g["deltas"][1:])
    else:
        assert min(frac[1:8]) > 0.05 and any(0.0 < f < 1.0 for f in frac[3:12])
    for lay, x in zip(work.layers, g["xs"][1:]):
        assert (x >= 0).all() and (x <= 32).all()


def test_irregular_net_scaled_config5():
    """Heavy-tailed row degrees, mixed-sign weights, no cap, softmax-CE on the
    last 10 neurons; gradients scaled by 2^12 so they clear the absolute floor."""
    work = wl.make_config(5, n=1024, n_layers=5, b_infer=96, b_train=96)
    lens = np.diff(work.layers[0].row_ptr)
    assert lens.max() >= 20 * lens.min()
    for scale in (1.0, 4096.0):
        g = P.gpu_train_step(work, work.x_train, scale=scale)
        o = P.oracle_train_step(work, work.x_train, scale=scale)
        st = P.compare_step(g, o, f"cfg5-scaled x{scale}")
        assert st["live_g"] == 5
    assert max(np.abs(gr[0]).max() for gr in o["grads"]) > 1e-4


def test_inference_mode_matches_training_forward_and_oracle():
    work = wl.make_config(1, n=512, n_layers=7, b_infer=200, density=0.4)
    x0 = P.dev(work.x_infer)
    ref = P.O32.forward(work.layers, work.x_infer, work.act_cap)[-1]
    for training in (False, True):
        net = sdnn.Net(work.layers, work.act_cap, 256, training=training)
        xl = torch.empty(512, 200, device=P.DEV)
        net.sdnn_forward(x0, xl)
        assert np.array_equal(P.host(xl), ref)
        net.close()
    # a block of the batch gives the same columns (samples are independent)
    net = sdnn.Net(work.layers, work.act_cap, 256, training=False)
    blk = torch.empty(512, 72, device=P.DEV)
    net.sdnn_forward(P.dev(work.x_infer[:, 64:136]), blk)
    assert np.array_equal(P.host(blk), ref[:, 64:136])
    net.close()


def test_two_runs_are_bit_identical():
    work = wl.make_config(5, n=512, n_layers=4, b_infer=64, b_train=64)
    a = P.gpu_train_step(work, work.x_train, scale=4096.0)
    b = P.gpu_train_step(work, work.x_train, scale=4096.0)
    for k in range(4):
        assert np.array_equal(a["deltas"][k + 1], b["deltas"][k + 1])
        assert np.array_equal(a["grads"][k][0], b["grads"][k][0])
        assert np.array_equal(a["new"][k][0], b["new"][k][0])
        assert np.array_equal(a["new"][k][1], b["new"][k][1])


def test_update_options_and_pattern_confinement():
    work = wl.tiny_net(33, sizes=(20, 30, 25), density=0.3, b=16)
    base = P.gpu_train_step(work, work.x_infer, lr=0.0)
    for lay, (v, b) in zip(work.layers, base["new"]):
        assert np.array_equal(v, lay.values) and np.array_equal(b, lay.bias)   # lr = 0: untouched
        assert v.size == lay.nnz                                               # pattern size fixed
    frozen = P.gpu_train_step(work, work.x_infer, lr=0.05, update_bias=False)
    o = P.oracle_train_step(work, work.x_infer, lr=0.05, update_bias=False)
    for lay, (v, b), (ov, ob) in zip(work.layers, frozen["new"], o["new"]):
        assert np.array_equal(b, lay.bias)
        P.assert_grad_close(v, ov)


def test_call_order_and_size_errors():
    work = wl.tiny_net(34, sizes=(8, 10, 6), b=4)
    net = sdnn.Net(work.layers, work.act_cap, 4, training=True)
    x0 = P.dev(work.x_infer)
    dl = torch.zeros(6, 4, device=P.DEV)
    with pytest.raises(sdnn.SdnnError) as e:
        net.sdnn_backward(dl)
    assert e.value.code == sdnn.SDNN_ESTATE
    with pytest.raises(sdnn.SdnnError) as e:
        net.sdnn_sgd_step(0.1)
    assert e.value.code == sdnn.SDNN_ESTATE
    with pytest.raises(sdnn.SdnnError) as e:
        net.sdnn_forward(torch.zeros(8, 5, device=P.DEV))
    assert e.value.code == sdnn.SDNN_EINVAL
    net.sdnn_forward(x0)
    net.sdnn_backward(dl)
    net.sdnn_sgd_step(0.1)
    with pytest.raises(sdnn.SdnnError) as e:
        net.sdnn_sgd_step(0.1)           # the backward pass was consumed
    assert e.value.code == sdnn.SDNN_ESTATE
    net.close()
    inf = sdnn.Net(work.layers, work.act_cap, 4, training=False)
    with pytest.raises(sdnn.SdnnError) as e:
        inf.sdnn_forward(x0)             # inference needs an output buffer
    assert e.value.code == sdnn.SDNN_EINVAL
    out = torch.empty(6, 4, device=P.DEV)
    inf.sdnn_forward(x0, out)
    with pytest.raises(sdnn.SdnnError) as e:
        inf.sdnn_backward(dl)
    assert e.value.code == sdnn.SDNN_ESTATE
    inf.close()


def test_loss_gradient_kernels():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((40, 33)).astype(np.float32)
    y = rng.random((40, 33)).astype(np.float32)
    got = P.host(sdnn.sdnn_mse_dloss(P.dev(x), P.dev(y)))
    assert np.array_equal(got, P.mse_dloss(x, y))
    lab = rng.integers(0, 10, 33)
    got = P.host(sdnn.sdnn_softmax_ce_dloss(P.dev(x), P.dev(lab, torch.int32), 10))
    ref = P.softmax_ce_dloss(x, lab, 10)
    assert (got[:30] == 0).all()
    np.testing.assert_allclose(got, ref, rtol=1e-6, atol=1e-9)
    assert abs(got[30:].sum()) < 1e-6


@pytest.mark.parametrize("b", [1, 3, 64, 128])
def test_sigmoid_training_step(b):
    """The paper's own activation (Section 6.1), small rectangular net, several batch sizes
    including one vector per step (B = 1 takes the lane-per-row kernels)."""
    work = wl.tiny_net(51, sizes=(40, 70, 33, 50), density=0.3, b=b)
    work.activation = "sigmoid"
    g = P.gpu_train_step(work, work.x_infer, lr=0.05)
    o = P.oracle_train_step(work, work.x_infer, lr=0.05)
    st = P.compare_step(g, o, f"sigmoid b={b}", exact_fwd=False)
    assert st["live_g"] == 3 and st["live_d"] == 3
    assert st["bitexact_x"] >= 3          # exp() may differ in the last bit of a double, rarely visible in fp32


def test_paper_training_setup_one_vector_per_step():
    """Sigmoid, weights U[-1,1], lr 0.01, B = 1 on a 1024-wide, 12-layer stand-in net: three
    consecutive SGD steps on three input vectors, weights carried over, against the oracle."""
    work = wl.paper_training_setup(1024, n_layers=12, n_inputs=4)
    orc = P.ORACLES["sigmoid"]
    net = sdnn.Net(work.layers, work.act_cap, 1, training=True, activation="sigmoid")
    layers = work.layers
    for s in range(3):
        x0 = np.ascontiguousarray(work.x_infer[:, s:s + 1])
        y = np.ascontiguousarray(work.targets[:, s:s + 1])
        xl = torch.empty(1024, 1, device=P.DEV)
        net.sdnn_forward(P.dev(x0), xl)
        net.sdnn_backward(sdnn.sdnn_mse_dloss(xl, P.dev(y)))
        net.sdnn_sgd_step(work.lr)
        xs, deltas, grads, new = orc.train_step(layers, x0, work.act_cap, lambda x: P.mse_dloss(x, y), work.lr)
        P.assert_forward_close(P.host(xl), xs[-1], f"step {s} X_L")
        for k, (lay, (v, b)) in enumerate(zip(layers, new)):
            gv, gb = (P.host(t) for t in net.sdnn_get_weights(k + 1))
            P.assert_grad_close(gv, v, f"step {s} layer {k + 1} weights")
            P.assert_grad_close(gb, b, f"step {s} layer {k + 1} bias")
            assert (v != lay.values).any()
            # carry the ORACLE's weights forward on the oracle side, the GPU keeps its own
            lay.values, lay.bias = v, b
    net.close()


@pytest.mark.parametrize("training", [False, True])
def test_two_stream_half_batches_match_oracle(training):
    """B a multiple of 128 on small layers: forward (and backward) run as two half-batch chains on
    two streams; inference mode shares the ping-pong buffers between them."""
    work = wl.make_config(1, n=512, n_layers=9, b_infer=256, b_train=256, density=0.4)
    ref = P.O32.forward(work.layers, work.x_infer, work.act_cap)
    net = sdnn.Net(work.layers, work.act_cap, 256, training=training)
    out = torch.empty(512, 256, device=P.DEV)
    for _ in range(3):                       # repeated passes: the fork/join events are reused
        out.zero_()
        net.sdnn_forward(P.dev(work.x_infer), out)
        assert np.array_equal(P.host(out), ref[-1])
    if training:
        g = P.gpu_train_step(work, work.x_train)
        o = P.oracle_train_step(work, work.x_train)
        st = P.compare_step(g, o, "split")
        assert st["bitexact_d"] == 9 and st["live_g"] >= 6
    net.close()


@pytest.mark.parametrize("activation", ["relu", "sigmoid"])
def test_one_vector_wide_layers_take_the_staged_kernels(activation):
    """B = 1 on layers of 2000+ rows with short uneven rows (Bernoulli pattern, some rows empty): the
    products are formed by all lanes over a contiguous stretch of entries and summed per row in
    storage order; row counts that are no multiple of the rows per workgroup."""
    work = wl.tiny_net(61, sizes=(3000, 2500, 4100, 2049), density=0.01, b=1)
    work.activation = activation
    lens = np.concatenate([np.diff(l.row_ptr) for l in work.layers])
    assert lens.min() <= 12 and lens.max() >= 50
    g = P.gpu_train_step(work, work.x_infer, lr=0.05)
    o = P.oracle_train_step(work, work.x_infer, lr=0.05)
    st = P.compare_step(g, o, f"staged b=1 {activation}", exact_fwd=(activation == "relu"))
    assert st["live_g"] == 3 and st["live_d"] == 3
    if activation == "relu":
        assert st["bitexact_d"] == 3
    # the same step with the gradient formed in the backward sweep (one product per entry at B = 1)
    gf = P.gpu_train_step(work, work.x_infer, lr=0.05, fuse_gradient=1)
    stf = P.compare_step(gf, o, f"staged b=1 {activation}, fused", exact_fwd=(activation == "relu"))
    assert stf["live_g"] == 3 and stf["live_d"] == 3
    for k in range(1, 4):
        assert np.array_equal(gf["deltas"][k], g["deltas"][k])


def test_one_vector_rows_longer_than_a_stage():
    """B = 1, rows and columns of 2500-3000 entries (several staging segments each) among rows of
    about three entries, in both orientations."""
    layers = [wl.ragged_layer(7101, 2300, 5000, 0.0006, 3, 2700, 4, 2000),
              wl.ragged_layer(7102, 4200, 2300, 0.0012, 2, 2200, 3, 3000)]
    for l in layers:
        assert l.nnz < 128 * l.n_out and np.diff(l.row_ptr).max() > 2048 and np.diff(l.row_ptr).min() <= 1
    x = wl.normal_inputs(7190, 5000, 1)
    tg = wl.uniform_targets(7191, 4200, 1)
    work = wl.Workload("ragged-b1", layers, float("inf"), x, 1, "mse", 0.01, targets=tg)
    g = P.gpu_train_step(work, work.x_infer, lr=0.05)
    o = P.oracle_train_step(work, work.x_infer, lr=0.05)
    st = P.compare_step(g, o, "ragged b=1")
    assert st["bitexact_d"] == 2 and st["live_g"] == 2
    gf = P.gpu_train_step(work, work.x_infer, lr=0.05, fuse_gradient=1)
    stf = P.compare_step(gf, o, "ragged b=1, fused")
    assert stf["bitexact_d"] == 2 and stf["live_g"] == 2


def test_paper_training_setup_wide_net_two_steps():
    """The paper's setup (sigmoid, U[-1,1] weights, one vector per step) at N = 4096, where B = 1
    takes the staged product kernels and the two-rows-per-wavefront update."""
    work = wl.paper_training_setup(4096, n_layers=5, n_inputs=2)
    orc = P.ORACLES["sigmoid"]
    net = sdnn.Net(work.layers, work.act_cap, 1, training=True, activation="sigmoid")
    layers = work.layers
    for s in range(2):
        x0 = np.ascontiguousarray(work.x_infer[:, s:s + 1])
        y = np.ascontiguousarray(work.targets[:, s:s + 1])
        xl = torch.empty(4096, 1, device=P.DEV)
        net.sdnn_forward(P.dev(x0), xl)
        net.sdnn_backward(sdnn.sdnn_mse_dloss(xl, P.dev(y)))
        net.sdnn_sgd_step(work.lr)
        xs, deltas, grads, new = orc.train_step(layers, x0, work.act_cap, lambda x: P.mse_dloss(x, y), work.lr)
        P.assert_forward_close(P.host(xl), xs[-1], f"step {s} X_L")
        for k, (lay, (v, b)) in enumerate(zip(layers, new)):
            gv, gb = (P.host(t) for t in net.sdnn_get_weights(k + 1))
            P.assert_grad_close(gv, v, f"step {s} layer {k + 1} weights")
            P.assert_grad_close(gb, b, f"step {s} layer {k + 1} bias")
            lay.values, lay.bias = v, b
    net.close()


@pytest.mark.parametrize("b", [256, 64, 1])
def test_training_step_captured_in_a_graph_replays_like_eager(b):
    """The library allocates nothing and orders all work on the caller's stream (the helper stream
    of the two-half-batch path is forked and joined with events), so a whole step can be captured
    in a HIP graph.  Every replay is checked against an eager twin net, with eager work and
    synchronisations between the replays; the oracle checks the first step."""
    work = wl.make_config(1, n=512, n_layers=7, b_infer=b, b_train=b, density=0.4)
    x0, y = P.dev(work.x_train), P.dev(work.targets)

    def step(net, xl, dl):
        net.sdnn_forward(x0, xl)
        sdnn.sdnn_mse_dloss(xl, y, out=dl)
        net.sdnn_backward(dl)
        net.sdnn_sgd_step(work.lr)

    eager = sdnn.Net(work.layers, work.act_cap, b, training=True)
    graphed = sdnn.Net(work.layers, work.act_cap, b, training=True)
    xe, de = torch.empty(512, b, device=P.DEV), torch.empty(512, b, device=P.DEV)
    xg, dg = torch.empty_like(xe), torch.empty_like(xe)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):       # capture records, it does not run
        step(graphed, xg, dg)
    torch.cuda.synchronize()
    for it in range(4):
        graph.replay()
        step(eager, xe, de)                           # eager work of the program between replays
        torch.cuda.synchronize()
        assert torch.equal(xg, xe), f"replay {it}: X_L differs from the eager step"
        for k in (1, 4, 7):
            for a, c in zip(graphed.sdnn_get_weights(k), eager.sdnn_get_weights(k)):
                assert torch.equal(a, c), f"replay {it}: layer {k} differs from the eager step"
        if it == 0:
            o = P.oracle_train_step(work, work.x_train)
            assert np.array_equal(P.host(xg), o["xs"][-1])
            P.assert_grad_close(P.host(graphed.sdnn_get_weights(7)[0]), o["new"][6][0], "graph step weights")
    eager.close(); graphed.close()


@pytest.mark.parametrize("b", [5, 64, 128, 130])
@pytest.mark.parametrize("activation", ["relu", "sigmoid"])
def test_fused_backward_and_gradient(b, activation):
    """SDNN_FUSE_ON: back-propagation and the gradient of the stored entries in one sweep (whole batch
    for B <= 64, two half-batch launches for B = 128; B = 130 cannot be fused and takes the separate
    update), then the streaming descent step.  Uneven rows, several 16-entry groups per row, empty rows."""
    work = wl.tiny_net(81, sizes=(150, 90, 200, 60, 110), density=0.25, b=b)
    work.activation = activation
    lens = np.concatenate([np.diff(l.row_ptr) for l in work.layers])
    assert lens.max() > 40 and lens.min() < 16
    g = P.gpu_train_step(work, work.x_infer, lr=0.05, fuse_gradient=sdnn.SDNN_FUSE_ON)
    o = P.oracle_train_step(work, work.x_infer, lr=0.05)
    st = P.compare_step(g, o, f"fused b={b} {activation}", exact_fwd=(activation == "relu"))
    assert st["live_g"] == 4 and st["live_d"] == 4
    plain = P.gpu_train_step(work, work.x_infer, lr=0.05, fuse_gradient=sdnn.SDNN_FUSE_OFF)
    for k in range(1, 5):
        assert np.array_equal(g["deltas"][k], plain["deltas"][k]), "the fused sweep must back-propagate the same bits"
    for (v, bias), (pv, pb) in zip(g["new"], plain["new"]):
        P.assert_grad_close(v, pv, "fused vs separate update")     # two fp32 partial sums instead of one
        P.assert_grad_close(bias, pb, "fused vs separate bias update")


def test_fused_gradient_options_and_empty_layer():
    """Fused path with update_bias off, a layer without entries, and lr = 0 (weights bit-identical)."""
    work = wl.tiny_net(82, sizes=(30, 50, 40, 20), density=0.2, b=33)
    mid = work.layers[1]
    mid.row_ptr = np.zeros_like(mid.row_ptr); mid.col_idx = mid.col_idx[:0]; mid.values = mid.values[:0]
    g = P.gpu_train_step(work, work.x_infer, lr=0.05, update_bias=False, fuse_gradient=sdnn.SDNN_FUSE_ON)
    o = P.oracle_train_step(work, work.x_infer, lr=0.05, update_bias=False)
    P.compare_step(g, o, "fused no-bias")
    for lay, (v, bias) in zip(work.layers, g["new"]):
        assert np.array_equal(bias, lay.bias)
    z = P.gpu_train_step(work, work.x_infer, lr=0.0, fuse_gradient=sdnn.SDNN_FUSE_ON)
    for lay, (v, bias) in zip(work.layers, z["new"]):
        assert np.array_equal(v, lay.values) and np.array_equal(bias, lay.bias)


@pytest.mark.parametrize("seed", range(24))
def test_seeded_random_small_nets(seed):
    """A seeded sweep over shapes, densities, batch sizes, activations, caps and the gradient-fusion
    switch: every pass of every case against the oracle."""
    rng = np.random.default_rng(9000 + seed)
    depth = int(rng.integers(1, 5))
    sizes = tuple(int(x) for x in rng.integers(1, 260, size=depth + 1))
    density = float(rng.choice([0.02, 0.1, 0.3, 0.7, 1.0]))
    b = int(rng.choice([1, 2, 3, 17, 63, 64, 65, 100, 128, 129, 192, 256]))
    activation = str(rng.choice(["relu", "sigmoid"]))
    cap = float(rng.choice([np.inf, 1.5])) if activation == "relu" else float("inf")
    fuse = int(rng.choice([sdnn.SDNN_FUSE_AUTO, sdnn.SDNN_FUSE_ON, sdnn.SDNN_FUSE_OFF]))
    update_bias = bool(rng.integers(0, 2))
    work = wl.tiny_net(300 + seed, sizes=sizes, density=density, b=b, cap=cap, scale=float(rng.choice([0.3, 1.0])))
    work.activation = activation
    what = f"seed {seed}: sizes {sizes} density {density} b {b} {activation} cap {cap} fuse {fuse} bias {update_bias}"
    g = P.gpu_train_step(work, work.x_infer, lr=0.05, update_bias=update_bias, fuse_gradient=fuse)
    o = P.oracle_train_step(work, work.x_infer, lr=0.05, update_bias=update_bias)
    P.compare_step(g, o, what, exact_fwd=(activation == "relu"))


@pytest.mark.parametrize("n,d,b,training", [(1000, 24, 2900, False), (1500, 8, 701, False), (2048, 40, 1026, True),
                                             (777, 16, 4096, False), (1000, 24, 1024, False), (515, 16, 300, True),
                                             (1030, 32, 390, False)])
def test_uniform_rows_wide_batches(n, d, b, training):
    """Layers whose rows all hold d entries, batches of several tiles: 2 to 7 tiles (a wavefront keeps
    its row and walks the tiles) and 8 and more (tiles dealt to the XCDs); row counts that are no
    multiple of the rows per workgroup, ragged last tile, 1, 2 and 4 samples per lane; mixed-sign
    weights and biases."""
    rng = np.random.default_rng(n + d)
    layers = []
    for l in range(3):
        lay = wl.regular_layer(6000 + 10 * n + l, n, d, 1.0, 0.0)
        lay.values = (rng.standard_normal(lay.values.size) / np.sqrt(d)).astype(np.float32)
        lay.bias = (0.2 * rng.standard_normal(n)).astype(np.float32)
        layers.append(lay)
    x = wl.normal_inputs(6900 + n, n, b)
    ref = P.O32.forward(layers, x, 1.0)
    assert (ref[-1] > 0).any() and (ref[-1] == 0).any() and (ref[1] == 1.0).any()
    net = sdnn.Net(layers, 1.0, b, training=training)
    out = torch.empty(n, b, device=P.DEV)
    net.sdnn_forward(P.dev(x), out)
    assert np.array_equal(P.host(out), ref[-1])
    if training:
        for k in (1, 2):
            assert np.array_equal(P.host(net.sdnn_get_activation(k, b)), ref[k])
    net.close()


@pytest.mark.parametrize("b", [64, 128, 17])
def test_fused_gradient_layout_over_several_steps(b):
    """The fused sweep keeps the values a second time, in the order of the transposed index, and the step writes
    both copies: layers of 31521, 69286 and 39647 entries (several spans and chunks of the way back to the CSR order,
    none a multiple of four), four steps with the weights carried over: fused, then a batch of 100 (not fusable: the
    separate update steps the CSR copy only and the next sweep must bring the other copy up to date), fused again,
    and fused after one layer's weights were replaced.  After every step the forward pass (CSR copy), the deltas
    (transposed copy) and the gradient handed out in CSR order must all be the oracle's."""
    sizes = (900, 700, 1100, 600)
    layers = [wl.random_layer(8130 + l, sizes[l + 1], sizes[l], (0.05, 0.09, 0.06)[l], scale=0.3) for l in range(3)]
    assert all(l.nnz > 3 * 8192 and l.nnz % 4 for l in layers) and max(l.nnz for l in layers) > 4 * 16384
    batches = [b, 100, b, b]
    x = wl.normal_inputs(8190, sizes[0], sum(batches))
    tg = wl.uniform_targets(8191, sizes[-1], sum(batches))
    work = wl.Workload("fused-layout", layers, 4.0, x, b, "mse", 0.05, targets=tg)
    net = sdnn.Net(layers, work.act_cap, 128, training=True, fuse_gradient=1)
    at = 0
    for s, bs in enumerate(batches):
        x0 = np.ascontiguousarray(x[:, at:at + bs])
        y = np.ascontiguousarray(tg[:, at:at + bs])
        at += bs
        if s == 3:      # new values for layer 2: both copies must follow
            rng = np.random.default_rng(8199)
            layers[1].values = (layers[1].values * rng.uniform(0.5, 1.5, layers[1].nnz)).astype(np.float32)
            net.sdnn_set_weights(2, P.dev(layers[1].values), P.dev(layers[1].bias))
        xl = torch.empty(sizes[-1], bs, device=P.DEV)
        net.sdnn_forward(P.dev(x0), xl)
        net.sdnn_backward(sdnn.sdnn_mse_dloss(xl, P.dev(y)))
        got_d = [P.host(net.sdnn_get_delta(k, bs)) for k in range(1, 4)]
        got_g = [tuple(P.host(t) for t in net.sdnn_weight_grad(k)) for k in range(1, 4)]
        net.sdnn_sgd_step(work.lr)
        xs, deltas, grads, new = P.O32.train_step(layers, x0, work.act_cap, lambda v: P.mse_dloss(v, y), work.lr)
        assert np.array_equal(P.host(xl), xs[-1]), f"step {s}: X_L"
        for k in range(3):
            assert np.array_equal(got_d[k], deltas[k + 1]), f"step {s}: delta {k + 1}"
            P.assert_grad_close(got_g[k][0], grads[k][0], f"step {s} layer {k + 1} gradient")
            P.assert_grad_close(got_g[k][1], grads[k][1], f"step {s} layer {k + 1} bias gradient")
            gv, gb = (P.host(t) for t in net.sdnn_get_weights(k + 1))
            P.assert_grad_close(gv, new[k][0], f"step {s} layer {k + 1} weights")
            P.assert_grad_close(gb, new[k][1], f"step {s} layer {k + 1} bias")
            assert (new[k][0] != layers[k].values).any()
            layers[k].values, layers[k].bias = gv, gb      # both sides go on from the GPU's weights: bits stay comparable
    net.close()


def test_fused_gradient_layout_at_the_sizes_of_its_spans_and_chunks():
    """Entry counts at the edges of the way back to the CSR order: exactly one span (8192), exactly one chunk
    (16384), five entries, none (a layer without entries sends only f(bias) on and no delta back), and just over a chunk.
    Two steps, so that the second one reads the values the first one wrote."""
    rng = np.random.default_rng(8300)

    def with_random_weights(lay, scale):
        lay.values = (rng.standard_normal(lay.nnz) * scale).astype(np.float32)
        lay.bias = (rng.standard_normal(lay.n_out) * 0.3).astype(np.float32)
        return lay

    few = wl.random_layer(8303, 64, 512, 0.0001, scale=0.5)
    few.bias = np.abs(few.bias) + 0.1          # its outputs stay alive without inputs
    none = wl.random_layer(8304, 96, 64, 0.0, scale=0.5)
    none.bias = np.abs(none.bias) + 0.1
    last = wl.random_layer(8305, 173, 96, 0.99, scale=0.2)
    layers = [with_random_weights(wl.regular_layer(8301, 256, 32, 0.0, 0.0), 0.3),
              with_random_weights(wl.regular_layer(8302, 512, 32, 0.0, 0.0, n_in=256), 0.3), few, none, last]
    wide = wl.random_layer(8306, 300, 173, 0.3158, scale=0.2)
    layers.append(wide)
    assert [l.nnz for l in layers[:4]] == [8192, 16384, 5, 0] and layers[5].nnz in range(16385, 16500)
    b = 64
    x = wl.normal_inputs(8390, 256, 2 * b)
    tg = wl.uniform_targets(8391, 300, 2 * b)
    net = sdnn.Net(layers, 4.0, b, training=True, fuse_gradient=1)
    for s in range(2):
        x0 = np.ascontiguousarray(x[:, s * b:(s + 1) * b])
        y = np.ascontiguousarray(tg[:, s * b:(s + 1) * b])
        xl = torch.empty(300, b, device=P.DEV)
        net.sdnn_forward(P.dev(x0), xl)
        net.sdnn_backward(sdnn.sdnn_mse_dloss(xl, P.dev(y)))
        got_d = [P.host(net.sdnn_get_delta(k, b)) for k in range(1, 7)]
        net.sdnn_sgd_step(0.05)
        xs, deltas, grads, new = P.O32.train_step(layers, x0, 4.0, lambda v: P.mse_dloss(v, y), 0.05)
        assert np.array_equal(P.host(xl), xs[-1]), f"step {s}: X_L"
        for k in range(6):
            assert np.array_equal(got_d[k], deltas[k + 1]), f"step {s}: delta {k + 1}"
            gv, gb = (P.host(t) for t in net.sdnn_get_weights(k + 1))
            P.assert_grad_close(gv, new[k][0], f"step {s} layer {k + 1} weights")
            P.assert_grad_close(gb, new[k][1], f"step {s} layer {k + 1} bias")
            layers[k].values, layers[k].bias = gv, gb
        assert (deltas[5] != 0).any() and (deltas[6] != 0).any()
    net.close()


@pytest.mark.parametrize("b", [256, 96, 36, 4, 130])
def test_fused_gradient_on_long_rows_four_samples_per_lane(b):
    """Rows of hundreds of entries (heavy-tailed degrees, and a layer with rows of 270 to 939 entries): the
    backward sweep forms the gradient with four samples per lane for batches of up to 256 samples that are a multiple
    of four; b = 130 takes the separate kernels on the same net.  Two steps, weights carried over."""
    work = wl.make_config(5, n=1024, n_layers=3, b_infer=2 * b, b_train=b)
    layers = work.layers + [wl.ragged_layer(8500, 700, 1024, 0.3, 3, 900, 5, 400)]
    assert sum(l.nnz for l in layers) >= 128 * sum(l.n_out for l in layers)
    x = wl.normal_inputs(8501, 1024, 2 * b)
    tg = wl.uniform_targets(8502, 700, 2 * b)
    net = sdnn.Net(layers, float("inf"), b, training=True, fuse_gradient=1)
    for s in range(2):
        x0 = np.ascontiguousarray(x[:, s * b:(s + 1) * b])
        y = np.ascontiguousarray(tg[:, s * b:(s + 1) * b])
        xl = torch.empty(700, b, device=P.DEV)
        net.sdnn_forward(P.dev(x0), xl)
        net.sdnn_backward(sdnn.sdnn_mse_dloss(xl, P.dev(y)))
        got_d = [P.host(net.sdnn_get_delta(k, b)) for k in range(1, 5)]
        got_g = [tuple(P.host(t) for t in net.sdnn_weight_grad(k)) for k in range(1, 5)]
        net.sdnn_sgd_step(0.01)
        xs, deltas, grads, new = P.O32.train_step(layers, x0, float("inf"), lambda v: P.mse_dloss(v, y), 0.01)
        assert np.array_equal(P.host(xl), xs[-1]), f"step {s}: X_L"
        for k in range(4):
            assert np.array_equal(got_d[k], deltas[k + 1]), f"step {s}: delta {k + 1}"
            P.assert_grad_close(got_g[k][0], grads[k][0], f"step {s} layer {k + 1} gradient")
            P.assert_grad_close(got_g[k][1], grads[k][1], f"step {s} layer {k + 1} bias gradient")
            gv, gb = (P.host(t) for t in net.sdnn_get_weights(k + 1))
            P.assert_grad_close(gv, new[k][0], f"step {s} layer {k + 1} weights")
            layers[k].values, layers[k].bias = gv, gb
        assert all((g[0] != 0).any() for g in grads)
    net.close()


def test_fused_gradient_long_row_kernels_on_empty_and_short_rows():
    """A net that is dense enough overall to take the long-row kernels (scalar entry loads, four samples per lane)
    also has a layer with empty rows, empty columns and rows of one to seven entries: every group size of the
    scalar loads and of the parked rows, and rows with nothing to do."""
    dense = wl.random_layer(8601, 600, 600, 0.6, scale=0.05)
    sparse = wl.ragged_layer(8602, 300, 600, 0.003, 2, 333, 2, 150)
    tail = wl.random_layer(8603, 64, 300, 0.5, scale=0.2)
    layers = [dense, sparse, tail]
    lens = np.diff(sparse.row_ptr)
    cols = np.bincount(sparse.col_idx, minlength=600)
    assert (lens == 0).any() and (cols == 0).any() and ((lens > 0) & (lens < 8)).any() and lens.max() > 300
    assert sum(l.nnz for l in layers) >= 128 * sum(l.n_out for l in layers)
    b = 100
    x = wl.normal_inputs(8690, 600, b)
    tg = wl.uniform_targets(8691, 64, b)
    work = wl.Workload("long-row-edges", layers, float("inf"), x, b, "mse", 0.02, targets=tg)
    o = P.oracle_train_step(work, x)
    for fuse in (1, -1):
        g = P.gpu_train_step(work, x, fuse_gradient=fuse)
        st = P.compare_step(g, o, f"long-row edges fuse={fuse}")
        assert st["bitexact_x"] == 4 and st["bitexact_d"] == 3 and st["live_g"] == 3
