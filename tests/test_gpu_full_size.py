"""Configurations 3, 4 and 5 at their full size: every layer, full width, full batch, in the launch
configuration bench.py times (these are the first workspaces above 4 GiB).  Training: one step on the
nominal inputs, compared with the oracle layer by layer (activations, deltas, the gradient that the
step applies, updated weights).  Inference: all samples (config 4: streamed in blocks of 1024), the
oracle on sampled sample columns through all layers (forward columns are independent: the batch vectors
are the columns of X, Section 5.1), on the nominal inputs and on inputs dense enough that the net
stays alive and saturates at the cap (non-zero values in every layer's buffer).

The nominal nets of configs 3 and 4 die after the first layer (reported, not hidden: every later
activation and every gradient is exactly zero), so what these tests add to the live depth prefixes of
test_gpu_configs.py is the full-size workspace, its offsets and the deep launch chains."""
import sys
import time

import numpy as np
import pytest
import torch

from paper_2104_11805_amd import sdnn, workloads as wl
from tests import parity as P

pytestmark = pytest.mark.gpu


def _log(msg):
    print(f"[full-size] {msg}", file=sys.stderr, flush=True)


def _sample_cols(bi, seed, n=24):
    rng = np.random.default_rng(seed)
    extra = rng.choice(np.arange(n, bi), size=n, replace=False)
    return np.concatenate([np.arange(n), np.sort(extra)]).astype(np.int64)


def _inference(work, x_all, block, cols, what):
    """GPU: all samples of x_all in blocks; oracle: the sampled columns, every layer."""
    t0 = time.time()
    n_out, bi = work.layers[-1].n_out, x_all.shape[1]
    net = sdnn.Net(work.layers, work.act_cap, block, training=False)
    got = np.empty((n_out, bi), np.float32)
    out = torch.empty(n_out, block, device=P.DEV)
    for s in range(0, bi, block):
        w = min(block, bi - s)
        o = out[:, :w].contiguous() if w != block else out
        net.sdnn_forward(P.dev(x_all[:, s:s + w]), o)
        got[:, s:s + w] = P.host(o)
    ws = net.workspace_bytes
    net.close()
    _log(f"{what}: GPU inference of {bi} samples done, workspace {ws / 2 ** 30:.2f} GiB [{time.time() - t0:.1f} s]")
    ref = P.ORACLES[work.activation].forward(work.layers, np.ascontiguousarray(x_all[:, cols]), work.act_cap)[-1]
    _log(f"{what}: oracle on {len(cols)} columns done [{time.time() - t0:.1f} s]")
    P.assert_forward_close(got[:, cols], ref, what)
    assert np.array_equal(got[:, cols], ref), what
    assert (got >= 0).all() and (got <= work.act_cap).all()
    return got, ref


@pytest.fixture(scope="module")
def cfg3():
    return wl.make_config(3)


def test_config3_full_size_training_step(cfg3):
    """N=16384, all 480 layers, minibatch 128 (two half-batch launch chains, gradient formed in the backward sweep)."""
    assert len(cfg3.layers) == 480 and cfg3.x_train.shape == (16384, 128) and cfg3.total_nnz == 251658240
    st = P.full_step_compare(cfg3, cfg3.x_train, "cfg3 full", log=_log)
    assert st["bitexact_x"] == 480 and st["bitexact_d"] == 480
    assert st["workspace_bytes"] > 8 * 2 ** 30
    assert st["live_x"] <= 2, "the nominal net is expected to die after the first layers"


def test_config3_full_size_inference(cfg3):
    """All 4096 samples through all 480 layers in one block."""
    got, ref = _inference(cfg3, cfg3.x_infer, 4096, _sample_cols(4096, 3), "cfg3 inference")
    assert (got == 0).all()          # dead after layer 1: reported, not hidden
    x_live = wl.binary_inputs(3902, 16384, 1024, 0.40)
    got, ref = _inference(cfg3, x_live, 1024, _sample_cols(1024, 33), "cfg3 inference, live inputs")
    assert (ref == 32.0).mean() > 0.9, "expected a saturated net at full depth"


@pytest.fixture(scope="module")
def cfg4():
    return wl.make_config(4)


def test_config4_full_size_training_step(cfg4):
    """N=65536, all 120 layers, minibatch 64, every X_l and Delta_l resident."""
    assert len(cfg4.layers) == 120 and cfg4.x_train.shape == (65536, 64) and cfg4.total_nnz == 251658240
    st = P.full_step_compare(cfg4, cfg4.x_train, "cfg4 full", log=_log)
    assert st["bitexact_x"] == 120 and st["bitexact_d"] == 120
    assert st["workspace_bytes"] > 8 * 2 ** 30


def test_config4_full_size_inference_streamed(cfg4):
    """All 8192 samples, streamed in 8 activation blocks of 1024, through all 120 layers."""
    got, ref = _inference(cfg4, cfg4.x_infer, 1024, _sample_cols(8192, 4), "cfg4 inference")
    assert (got == 0).all()
    x_live = wl.binary_inputs(4902, 65536, 1024, 0.60)
    got, ref = _inference(cfg4, x_live, 1024, _sample_cols(1024, 44), "cfg4 inference, live inputs")
    assert (ref == 32.0).mean() > 0.9


@pytest.fixture(scope="module")
def cfg5():
    return wl.make_config(5)


def test_config5_full_size_training_step(cfg5):
    """N=8192, all 30 layers of heavy-tailed rows, minibatch 256, softmax cross-entropy; the loss gradient
    scaled by 2^12 (exact) so that the gradients clear the absolute floor of the tolerance."""
    assert len(cfg5.layers) == 30 and cfg5.x_train.shape == (8192, 256)
    st = P.full_step_compare(cfg5, cfg5.x_train, "cfg5 full", scale=4096.0, log=_log)
    assert st["bitexact_x"] == 30 and st["live_d"] == 30 and st["live_g"] == 30


def test_config5_full_size_inference(cfg5):
    got, ref = _inference(cfg5, cfg5.x_infer, 2048, _sample_cols(2048, 5), "cfg5 inference")
    assert 0.3 < (ref > 0).mean() < 0.7


def test_config4_full_size_sigmoid_training_step_is_live_in_every_layer(cfg4):
    """Config 4's nets and minibatch with the sigmoid of the paper's own training setup (Section 6.1): no neuron
    dies or saturates, so every layer of the full-size workspace carries non-zero activations, deltas (down to
    the subnormal range in the first layers: the delta shrinks by about 0.4 per layer going back) and gradients."""
    work = wl.Workload("cfg4-sigmoid", cfg4.layers, float("inf"), cfg4.x_infer[:, :64], 64, "mse", 0.01,
                       targets=cfg4.targets, activation="sigmoid")
    st = P.full_step_compare(work, work.x_train, "cfg4 sigmoid", log=_log)
    assert st["live_x"] == 120 and st["live_d"] >= 100 and st["live_g"] >= 100
    assert st["bitexact_d"] >= 100
