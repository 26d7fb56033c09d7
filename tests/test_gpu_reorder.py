"""Options that change how the work is laid out on the chip, never what is computed: the row order
chosen for gather locality (reorder_rows) and the column-panel sweep of wide layers (panel_cols).
Every result must be the bits of the oracle (forward, deltas) or within the usual bar (gradients)."""
import numpy as np
import pytest
import torch

from paper_2104_11805_amd import sdnn, workloads as wl
from tests import parity as P

pytestmark = pytest.mark.gpu


def _work(layers, b, seed, cap=1.5, inputs="normal"):
    n_in, n_out = layers[0].n_in, layers[-1].n_out
    x = wl.normal_inputs(seed, n_in, b) if inputs == "normal" else wl.binary_inputs(seed, n_in, b, 0.4)
    return wl.Workload("layout", layers, cap, x, b, "mse", 0.05, targets=wl.uniform_targets(seed + 1, n_out, b))


@pytest.mark.parametrize("b,fuse", [(64, 0), (64, 1), (128, 1), (300, 0), (1, 0)])
def test_reordered_rows_structured_net(b, fuse):
    """Butterfly-like pattern (32 rows share each column set): the clustered schedule gives the oracle's result."""
    layers = [wl.strided_layer(600 + l, 2048) for l in range(4)]
    work = _work(layers, b, 610)
    g = P.gpu_train_step(work, work.x_train, fuse_gradient=fuse, reorder_rows=True)
    o = P.oracle_train_step(work, work.x_train)
    st = P.compare_step(g, o, f"reordered strided b={b} fuse={fuse}")
    assert st["live_g"] == 4
    plain = P.gpu_train_step(work, work.x_train, fuse_gradient=fuse, reorder_rows=False)
    for k in range(5):
        assert np.array_equal(g["xs"][k], plain["xs"][k])
    for k in range(1, 5):
        assert np.array_equal(g["deltas"][k], plain["deltas"][k])
        assert np.array_equal(g["new"][k - 1][0], plain["new"][k - 1][0])


def test_reordered_rows_irregular_and_random_nets():
    work = wl.make_config(5, n=1024, n_layers=3, b_infer=96, b_train=96)
    g = P.gpu_train_step(work, work.x_train, scale=4096.0, reorder_rows=True)
    o = P.oracle_train_step(work, work.x_train, scale=4096.0)
    P.compare_step(g, o, "reordered irregular")
    work = wl.make_config(1, n_layers=6, density=0.40)
    g = P.gpu_train_step(work, work.x_train, reorder_rows=True)
    o = P.oracle_train_step(work, work.x_train)
    assert P.compare_step(g, o, "reordered cfg1")["live_g"] == 6
    layers = [wl.ragged_layer(40 + l, 500, 500, 0.01, 3, 300, 3, 200) for l in range(2)]   # long rows, empty rows
    work = _work(layers, 70, 45, cap=float("inf"))
    g = P.gpu_train_step(work, work.x_train, reorder_rows=True)
    o = P.oracle_train_step(work, work.x_train)
    P.compare_step(g, o, "reordered ragged")


def test_reordered_rows_inference_and_skip_dead():
    layers = [wl.strided_layer(700 + l, 1024, value=0.0625, bias=-0.3) for l in range(8)]
    x = wl.mixed_density_inputs(705, 1024, 200, (0.05, 0.30, 0.45))
    ref = P.O32.forward(layers, x, 32.0)[-1]
    net = sdnn.Net(layers, 32.0, 200, training=False, reorder_rows=True)
    out = torch.empty(1024, 200, device=P.DEV)
    net.sdnn_forward(P.dev(x), out)
    assert np.array_equal(P.host(out), ref)
    out2 = torch.full((1024, 200), -1.0, device=P.DEV)
    net.sdnn_forward_skip_dead(P.dev(x), out2, check_every=2)
    assert np.array_equal(P.host(out2), ref)
    net.close()


@pytest.mark.parametrize("b,cols,n", [(37, 7, 333), (64, 50, 333), (100, 1000, 333), (130, 16, 333), (128, 9, 333),
                                      (64, 300, 5000), (520, 100, 5000)])
def test_panel_sweep_forced_on_small_nets(b, cols, n):
    """panel_cols forced: many narrow panels, ragged rows (some empty), partial last tile; the last case has
    eight or more tiles, so every XCD sweeps its own tiles with several rows per wavefront."""
    sizes = (150, n, 97, 210)
    dens = (0.12, 0.12 if n < 1000 else 0.006, 0.12)
    layers = [wl.random_layer(900 + l, sizes[l + 1], sizes[l], dens[l], scale=0.5) for l in range(3)]
    assert max(int(np.diff(l.row_ptr).max()) for l in layers) <= 64
    work = _work(layers, b, 77, cap=1.2)
    g = P.gpu_train_step(work, work.x_train, fuse_gradient=-1, panel_cols=cols)
    o = P.oracle_train_step(work, work.x_train)
    assert P.compare_step(g, o, f"panel b={b} cols={cols}")["live_g"] == 3
    if b <= 64 or b == 128:      # the fused backward sweep next to a panel-swept forward
        g = P.gpu_train_step(work, work.x_train, fuse_gradient=1, panel_cols=cols)
        assert P.compare_step(g, o, f"fused panel b={b} cols={cols}")["live_g"] == 3
    net = sdnn.Net(layers, 1.2, b, training=False, panel_cols=cols)
    out = torch.empty(sizes[-1], b, device=P.DEV)
    net.sdnn_forward(P.dev(work.x_train), out)
    assert np.array_equal(P.host(out), o["xs"][-1])
    net.close()


def test_panel_sweep_by_policy_on_a_wide_layer_and_long_rows_fall_back():
    """65536 columns: the policy sweeps in panels (forward and the separate backward product; rows per
    wavefront chosen from the row count); a layer with a row of more than 64 entries does not."""
    work = wl.make_config(4, n_layers=3, density=0.60, b_infer=64, b_train=64)
    for opts in (dict(fuse_gradient=-1), dict(fuse_gradient=-1, panel_cols=-1), dict(fuse_gradient=-1, reorder_rows=True),
                 dict(fuse_gradient=1), dict(fuse_gradient=1, panel_cols=-1)):
        g = P.gpu_train_step(work, work.x_train, **opts)
        if "o" not in locals():
            o = P.oracle_train_step(work, work.x_train)
        assert P.compare_step(g, o, f"cfg4 {opts}")["live_g"] == 3
    layers = [wl.ragged_layer(50 + l, 400, 400, 0.02, 2, 100, 2, 90) for l in range(2)]
    assert max(int(np.diff(l.row_ptr).max()) for l in layers) > 64
    work = _work(layers, 64, 55, cap=float("inf"))
    g = P.gpu_train_step(work, work.x_train, fuse_gradient=-1, panel_cols=32)
    o = P.oracle_train_step(work, work.x_train)
    P.compare_step(g, o, "panel refused for long rows")


@pytest.mark.parametrize("activation", ["relu", "sigmoid"])
@pytest.mark.parametrize("b", [1, 3, 64, 130])
def test_lds_resident_forward_small_ragged_nets(b, activation):
    """The single-launch forward with activations in LDS: rectangular layers, ragged rows (some empty, some longer
    than a block's neighbours), a partial last group of samples; same bits as the per-layer kernels and the oracle."""
    sizes = (150, 333, 97, 210, 64)
    layers = [wl.random_layer(1200 + l, sizes[l + 1], sizes[l], 0.15, scale=0.5) for l in range(4)]
    layers[1] = wl.ragged_layer(1250, sizes[2], sizes[1], 0.05, 3, 200, 3, 60)
    x = wl.normal_inputs(1290, sizes[0], b)
    cap = float("inf") if activation == "sigmoid" else 1.3
    ref = P.ORACLES[activation].forward(layers, x, cap)[-1]
    outs = {}
    for mode in (sdnn.SDNN_LDS_ON, sdnn.SDNN_LDS_OFF):
        net = sdnn.Net(layers, cap, max(b, 4), training=False, activation=activation, lds_forward=mode)
        out = torch.full((sizes[-1], b), -3.0, device=P.DEV)
        net.sdnn_forward(P.dev(x), out)
        outs[mode] = P.host(out)
        net.close()
    P.assert_forward_close(outs[sdnn.SDNN_LDS_ON], ref, "lds forward")
    if activation == "relu":
        assert np.array_equal(outs[sdnn.SDNN_LDS_ON], ref)
    assert np.array_equal(outs[sdnn.SDNN_LDS_ON], outs[sdnn.SDNN_LDS_OFF])


def test_lds_resident_forward_benchmark_nets_and_replaced_weights():
    work = wl.make_config(2, n_layers=10, density=0.37, b_infer=260, b_train=64)
    ref = P.O32.forward(work.layers, work.x_infer, work.act_cap)
    assert 0.05 < (ref[-1] > 0).mean() and (ref[-1] < 32).any()
    net = sdnn.Net(work.layers, work.act_cap, 260, training=False, lds_forward=sdnn.SDNN_LDS_ON)
    out = torch.empty(4096, 260, device=P.DEV)
    net.sdnn_forward(P.dev(work.x_infer), out)
    assert np.array_equal(P.host(out), ref[-1])
    # new weights for two layers: the lane-major copy must follow
    rng = np.random.default_rng(5)
    for k in (1, 7):
        lay = work.layers[k - 1]
        lay.values = (lay.values * rng.uniform(0.5, 1.5, lay.nnz)).astype(np.float32)
        lay.bias = (lay.bias * 0.5).astype(np.float32)
        net.sdnn_set_weights(k, P.dev(lay.values), P.dev(lay.bias))
    ref2 = P.O32.forward(work.layers, work.x_infer, work.act_cap)[-1]
    assert not np.array_equal(ref2, ref[-1])
    net.sdnn_forward(P.dev(work.x_infer), out)
    assert np.array_equal(P.host(out), ref2)
    out2 = torch.empty(4096, 260, device=P.DEV)
    net.sdnn_forward_noalloc(P.dev(work.x_infer), out2)
    assert torch.equal(out, out2)
    net.close()
    # a net wider than LDS holds keeps the per-layer kernels, whatever the option says
    wide = [wl.regular_layer(77, 4100, 8, 0.125, -0.1)]
    net = sdnn.Net(wide, 32.0, 8, training=False, lds_forward=sdnn.SDNN_LDS_ON)
    x = wl.binary_inputs(78, 4100, 8, 0.5)
    out = torch.empty(4100, 8, device=P.DEV)
    net.sdnn_forward(P.dev(x), out)
    assert np.array_equal(P.host(out), P.O32.forward(wide, x, 32.0)[-1])
    net.close()


@pytest.mark.parametrize("n,b,opts", [(4096, 2304, dict(lds_forward=-1)),            # sub-blocks of 1024, 1024, 256
                                     (24576, 448, dict(panel_cols=4096)),           # panel sweep throughout: 128, 128, 128, 64
                                     (24576, 448, dict(panel_cols=-1))])            # 256, 192
def test_inference_in_sub_blocks_of_samples(n, b, opts):
    """Activation blocks of more than 32 MiB are taken through all layers in sub-blocks of samples (what a layer
    wrote is still on chip when the next one gathers it): every column of the result must be the oracle's."""
    layers = [wl.regular_layer(8400 + l, n, 32, 0.0625, -0.3) for l in range(3)]
    rng = np.random.default_rng(8410)
    for l in layers:
        l.values = (l.values * rng.uniform(0.5, 1.5, l.nnz)).astype(np.float32)
    assert 4 * n * b > 32 * 2 ** 20
    x = wl.binary_inputs(8411, n, b, 0.4)
    ref = P.O32.forward(layers, x, 32.0)[-1]
    assert 0.2 < (ref > 0).mean() and (ref < 32.0).mean() > 0.2
    net = sdnn.Net(layers, 32.0, b, training=False, **opts)
    out = torch.full((n, b), -1.0, device=P.DEV)
    net.sdnn_forward(P.dev(x), out)
    assert np.array_equal(P.host(out), ref)
    net.close()
