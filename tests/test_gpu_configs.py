"""The five benchmark configurations at their real widths and batch sizes
(depth reduced where a full-depth oracle run would take minutes), in the
launch configuration bench.py times.  Inference is checked on sampled sample
columns (forward columns are independent: the batch vectors are the columns of
X, Section 5.1); training always on the full minibatch, on the nominal inputs
and on "live" inputs whose gradients are not identically zero."""
import numpy as np
import pytest
import torch

from paper_2104_11805_amd import sdnn, workloads as wl
from tests import parity as P

pytestmark = pytest.mark.gpu


def _infer_columns(work, block, cols):
    """GPU inference over all samples in blocks of `block`; oracle on the sampled columns only."""
    n_out = work.layers[-1].n_out
    bi = work.x_infer.shape[1]
    net = sdnn.Net(work.layers, work.act_cap, block, training=False)
    got = np.empty((n_out, bi), np.float32)
    for s in range(0, bi, block):
        w = min(block, bi - s)
        out = torch.empty(n_out, w, device=P.DEV)
        net.sdnn_forward(P.dev(work.x_infer[:, s:s + w]), out)
        got[:, s:s + w] = P.host(out)
    net.close()
    ref = P.O32.forward(work.layers, work.x_infer[:, cols], work.act_cap)[-1]
    P.assert_forward_close(got[:, cols], ref, "inference")
    assert np.array_equal(got[:, cols], ref)
    assert (got >= 0).all() and (got <= work.act_cap).all()
    return got, ref


def _sample_cols(bi, seed):
    rng = np.random.default_rng(seed)
    extra = rng.choice(np.arange(32, bi), size=min(32, max(bi - 32, 0)), replace=False) if bi > 32 else []
    return np.concatenate([np.arange(min(32, bi)), np.sort(extra)]).astype(np.int64)


def _train(work, x0, what, scale=1.0, live_layers=None):
    g = P.gpu_train_step(work, x0, scale=scale)
    o = P.oracle_train_step(work, x0, scale=scale)
    st = P.compare_step(g, o, what)
    if live_layers is not None:
        assert st["live_g"] >= live_layers, st
    return st


def test_config2_full_depth_nominal():
    """N=4096, L=480, minibatch 128 and 1024 inference samples, exactly as benchmarked."""
    work = wl.make_config(2)
    assert len(work.layers) == 480 and work.x_train.shape == (4096, 128)
    st = _train(work, work.x_train, "cfg2")
    assert st["bitexact_d"] == 480
    got, ref = _infer_columns(work, 1024, _sample_cols(1024, 2))
    assert (got == 0).all()          # the nominal net is dead after layer 1: reported, not hidden


@pytest.mark.parametrize("cfg,n_layers,b,density", [(2, 6, 128, 0.40), (3, 6, 128, 0.40), (4, 6, 64, 0.60)])
def test_live_training_prefix_at_full_width(cfg, n_layers, b, density):
    """Depth-6 prefix at an input density above the net's dying point (-bias): all masks open,
    nothing clamped yet, dense gradients in every layer."""
    work = wl.make_config(cfg, n_layers=n_layers, density=density, b_infer=b, b_train=b)
    st = _train(work, work.x_train, f"cfg{cfg}-live", live_layers=n_layers)
    assert st["live_d"] == n_layers


@pytest.mark.parametrize("cfg,n_layers,b_infer,block,density", [(3, 12, 4096, 4096, 0.37), (4, 4, 2048, 1024, 0.50)])
def test_wide_configs_inference_blocks(cfg, n_layers, b_infer, block, density):
    """Configs 3 and 4 at full width; config 4 streamed in activation blocks of 1024."""
    work = wl.make_config(cfg, n_layers=n_layers, density=density, b_infer=b_infer, b_train=64)
    got, ref = _infer_columns(work, block, _sample_cols(b_infer, cfg))
    assert (ref > 0).mean() > 0.05, "dead outputs: the comparison would prove nothing"


def test_config5_irregular_full_width():
    """N=8192, heavy-tailed rows (12..2048 entries), mixed signs, no cap; minibatch 256 with
    softmax cross-entropy, also with the loss gradient scaled by 2^12; 2048 inference samples."""
    work = wl.make_config(5, n_layers=3)
    lens = np.diff(work.layers[0].row_ptr)
    assert lens.max() == 2048 and lens.min() < 64 and 800 < lens.mean() < 840
    _train(work, work.x_train, "cfg5", scale=1.0)
    st = _train(work, work.x_train, "cfg5 x4096", scale=4096.0, live_layers=3)
    got, ref = _infer_columns(work, 2048, _sample_cols(2048, 5))
    assert 0.3 < (ref > 0).mean() < 0.7


def test_config2_skip_dead_at_full_width():
    """Config 2's net (first 60 layers) at its inference batch of 1024 with inputs of mixed density,
    so that samples die at different depths: dropping them gives the bits of the plain pass, which
    the oracle confirms on sampled columns."""
    work = wl.make_config(2, n_layers=60)
    work.x_infer = wl.mixed_density_inputs(2950, 4096, 1024, (0.05, 0.25, 0.30, 0.33, 0.36, 0.45))
    net = sdnn.Net(work.layers, work.act_cap, 1024, training=False)
    x = P.dev(work.x_infer)
    plain = torch.empty(4096, 1024, device=P.DEV)
    skipped = torch.full((4096, 1024), -1.0, device=P.DEV)
    n_live = torch.zeros(1, dtype=torch.int32, device=P.DEV)
    net.sdnn_forward(x, plain)
    net.sdnn_forward_skip_dead(x, skipped, check_every=4, n_live=n_live)
    assert torch.equal(plain, skipped)
    cols = np.r_[0:12, 500:512, 1012:1024]
    ref = P.O32.forward(work.layers, work.x_infer[:, cols], work.act_cap)
    P.assert_forward_close(P.host(skipped)[:, cols], ref[-1], "skip-dead inference")
    alive = int((P.host(plain) != 0).any(axis=0).sum())
    assert 0 < alive < 1024 and alive <= int(n_live.item()) < 1024
    net.close()
