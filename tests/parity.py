"""Shared helpers of the GPU parity tests: run one workload through the HIP
library (via the binding) and through the CPU oracle, on the same arrays."""
import numpy as np
import torch

from oracle.sdnn_oracle import Oracle, mse_dloss, softmax_ce_dloss
from paper_2104_11805_amd import sdnn

O32 = Oracle(np.float32)
ORACLES = {"relu": O32, "sigmoid": Oracle(np.float32, "sigmoid")}
DEV = "cuda:0"


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def oracle_dloss_fn(work, scale=1.0):
    if work.loss == "mse":
        f = lambda xl: mse_dloss(xl, work.targets[:, :xl.shape[1]])
    else:
        f = lambda xl: softmax_ce_dloss(xl, work.labels, work.n_classes)
    if scale == 1.0:
        return f
    return lambda xl: (f(xl) * np.float32(scale)).astype(np.float32)   # power-of-two scale: exact


def gpu_dloss(work, xl, scale=1.0):
    if work.loss == "mse":
        d = sdnn.sdnn_mse_dloss(xl, dev(work.targets[:, :xl.shape[1]]))
    else:
        d = sdnn.sdnn_softmax_ce_dloss(xl, dev(work.labels, torch.int32), work.n_classes)
    if scale != 1.0:
        d = d * scale   # exact power-of-two scaling of an input of the backward pass
    return d


def gpu_train_step(work, x0, lr=None, scale=1.0, update_bias=True, max_batch=None, keep=True, fuse_gradient=0,
                   **net_options):
    """forward + backward + sgd_step through the C ABI; returns everything as numpy."""
    b = x0.shape[1]
    net = sdnn.Net(work.layers, work.act_cap, max_batch or b, training=True, update_bias=update_bias,
                   activation=work.activation, fuse_gradient=fuse_gradient, **net_options)
    L = net.n_layers
    xl = torch.empty(work.layers[-1].n_out, b, device=DEV)
    net.sdnn_forward(dev(x0), xl)
    dl = gpu_dloss(work, xl, scale)
    net.sdnn_backward(dl)
    out = dict(xl=host(xl), dloss=host(dl))
    if keep:
        out["xs"] = [host(net.sdnn_get_activation(k, b)) for k in range(L + 1)]
        out["deltas"] = [None] + [host(net.sdnn_get_delta(k, b)) for k in range(1, L + 1)]
        out["grads"] = [tuple(host(t) for t in net.sdnn_weight_grad(k)) for k in range(1, L + 1)]
    net.sdnn_sgd_step(work.lr if lr is None else lr)
    out["new"] = [tuple(host(t) for t in net.sdnn_get_weights(k)) for k in range(1, L + 1)]
    net.close()
    return out


def oracle_train_step(work, x0, lr=None, scale=1.0, update_bias=True):
    xs, deltas, grads, new = ORACLES[work.activation].train_step(work.layers, x0, work.act_cap, oracle_dloss_fn(work, scale),
                                            work.lr if lr is None else lr, update_bias)
    return dict(xs=xs, deltas=deltas, grads=grads, new=new, xl=xs[-1])


# ---- the parity bar ---------------------------------------------------------
FWD_RTOL = 1e-5                 # forward: max relative error
GRAD_RTOL, GRAD_ATOL = 1e-4, 1e-6   # gradients, deltas, updated weights


def assert_forward_close(got, ref, what=""):
    """max relative error <= 1e-5 and exactly the same set of active neurons."""
    assert got.shape == ref.shape and got.dtype == ref.dtype == np.float32, what
    assert np.array_equal(got > 0, ref > 0), f"{what}: active sets differ"
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    bound = FWD_RTOL * np.abs(ref.astype(np.float64))
    assert (err <= bound).all(), f"{what}: max rel err {np.max(err / np.maximum(np.abs(ref), 1e-300)):.3e}"


def assert_grad_close(got, ref, what=""):
    assert got.shape == ref.shape, what
    if ref.size == 0:
        return
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    bound = GRAD_ATOL + GRAD_RTOL * np.abs(ref.astype(np.float64))
    assert (err <= bound).all(), f"{what}: max err {err.max():.3e} (ref max {np.abs(ref).max():.3e})"


def assert_rel_close(got, ref, rtol, what=""):
    """Pure relative check against the largest reference magnitude (no absolute floor)."""
    if ref.size == 0:
        return
    scale = float(np.abs(ref).max())
    err = float(np.abs(got.astype(np.float64) - ref.astype(np.float64)).max())
    assert err <= rtol * scale, f"{what}: max err {err:.3e} vs scale {scale:.3e}"


def compare_step(g, o, what="", exact_fwd=True):
    L = len(o["xs"]) - 1
    stats = dict(bitexact_x=0, bitexact_d=0, layers=L, live_d=0, live_g=0)
    for k in range(L + 1):
        assert_forward_close(g["xs"][k], o["xs"][k], f"{what} X_{k}")
        stats["bitexact_x"] += int(np.array_equal(g["xs"][k], o["xs"][k]))
    for k in range(1, L + 1):
        assert_grad_close(g["deltas"][k], o["deltas"][k], f"{what} Delta_{k}")
        assert np.array_equal(g["deltas"][k] != 0, o["deltas"][k] != 0), f"{what} Delta_{k} support"
        stats["bitexact_d"] += int(np.array_equal(g["deltas"][k], o["deltas"][k]))
        stats["live_d"] += int((o["deltas"][k] != 0).any())
        for j, name in ((0, "g"), (1, "gb")):
            assert_grad_close(g["grads"][k - 1][j], o["grads"][k - 1][j], f"{what} {name}_{k}")
            if o["grads"][k - 1][j].size and np.abs(o["grads"][k - 1][j]).max() > 0:
                assert_rel_close(g["grads"][k - 1][j], o["grads"][k - 1][j], 1e-5, f"{what} {name}_{k} rel")
            assert_grad_close(g["new"][k - 1][j], o["new"][k - 1][j], f"{what} new {name}_{k}")
        stats["live_g"] += int((o["grads"][k - 1][0] != 0).any())
    if exact_fwd:
        assert stats["bitexact_x"] == L + 1, f"{what}: forward not bit-identical to the oracle: {stats}"
    return stats


def full_step_compare(work, x0, what="", scale=1.0, log=None):
    """One training step of a deep, wide net on the GPU and in the oracle, compared layer by layer as
    the oracle walks Algorithm 1, so that only the oracle's activations (which its backward sweep
    needs) and its updated weights are ever held on the host.  Same bar as compare_step."""
    import time
    t0 = time.time()
    say = (lambda m: log(f"{what}: {m} [{time.time() - t0:.1f} s]")) if log else (lambda m: None)
    orc = ORACLES[work.activation]
    b = x0.shape[1]
    L = len(work.layers)
    net = sdnn.Net(work.layers, work.act_cap, b, training=True, activation=work.activation)
    say(f"net created, workspace {net.workspace_bytes / 2 ** 30:.2f} GiB")
    xl = torch.empty(work.layers[-1].n_out, b, device=DEV)
    net.sdnn_forward(dev(x0), xl)
    dl = gpu_dloss(work, xl, scale)
    net.sdnn_backward(dl)
    torch.cuda.synchronize()
    say("GPU forward + backward done")
    stats = dict(layers=L, bitexact_x=0, bitexact_d=0, live_x=0, live_d=0, live_g=0, workspace_bytes=net.workspace_bytes)
    # feed-forward sweep (Eq. 3)
    xs = [np.ascontiguousarray(x0, dtype=np.float32)]
    assert np.array_equal(host(net.sdnn_get_activation(0, b)), xs[0])
    for k in range(1, L + 1):
        xs.append(orc.forward_layer(work.layers[k - 1], xs[-1], work.act_cap))
        got = host(net.sdnn_get_activation(k, b))
        assert_forward_close(got, xs[k], f"{what} X_{k}")
        stats["bitexact_x"] += int(np.array_equal(got, xs[k]))
        stats["live_x"] += int((xs[k] != 0).any())
    say("oracle forward sweep compared")
    # output delta (Eq. 6), then per layer: gradient (Eq. 4), descent step (Eq. 5), delta of the layer below (Eq. 7)
    dloss = oracle_dloss_fn(work, scale)(xs[L])
    assert_grad_close(host(dl), dloss, f"{what} dLoss")
    delta = orc.output_delta(dloss, xs[L], work.act_cap)
    new_vals = [None] * L
    lr = work.lr
    for k in range(L, 0, -1):
        got = host(net.sdnn_get_delta(k, b))
        assert_grad_close(got, delta, f"{what} Delta_{k}")
        assert np.array_equal(got != 0, delta != 0), f"{what} Delta_{k} support"
        stats["bitexact_d"] += int(np.array_equal(got, delta))
        stats["live_d"] += int((delta != 0).any())
        g, gb = orc.weight_grad(work.layers[k - 1], delta, xs[k - 1])
        gg, ggb = (host(t) for t in net.sdnn_weight_grad(k))
        for got_, ref_, name in ((gg, g, "g"), (ggb, gb, "gb")):
            assert_grad_close(got_, ref_, f"{what} {name}_{k}")
            if ref_.size and np.abs(ref_).max() > 0:
                assert_rel_close(got_, ref_, 1e-5, f"{what} {name}_{k} rel")
        stats["live_g"] += int((g != 0).any())
        new_vals[k - 1] = (orc.sgd_apply(work.layers[k - 1].values, g, lr), orc.sgd_apply(work.layers[k - 1].bias, gb, lr))
        if k > 1:
            delta = orc.backward_layer(work.layers[k - 1], delta, xs[k - 1], work.act_cap)
        xs[k] = None
    say("oracle backward sweep and gradients compared")
    net.sdnn_sgd_step(lr)
    for k in range(1, L + 1):
        v, bi = (host(t) for t in net.sdnn_get_weights(k))
        assert_grad_close(v, new_vals[k - 1][0], f"{what} new values_{k}")
        assert_grad_close(bi, new_vals[k - 1][1], f"{what} new bias_{k}")
        new_vals[k - 1] = None
    net.close()
    say(f"updated weights compared: {stats}")
    return stats
