"""CPU oracle driver: TEST INFRASTRUCTURE ONLY (tests, smoke check, CPU baseline).

Walks the layers in the order of Algorithm 1 (feed-forward sweep, output
delta, then the backward loop over the layers) and calls the plain C routines of
sdnn_oracle.c for every per-layer operation.  Nothing here is shared with the
HIP library, and nothing here may be imported by it.

Reading of the minibatch form (Section 5.1): a matrix Delta_l [N][B] is
back-propagated, one column per sample, each column obeying Eq. 7; the weight
gradient sums Eq. 4 over the samples.  Any 1/B averaging lives in the caller's
loss gradient.  The backward pass uses the weights as they were in the forward
pass (Algorithm 1 computes delta^{k-1} before it updates W^k) and delta^0 is
not formed (there is no z^0).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sdnn_oracle.c")
_LIBS = {}


def build(force: bool = False) -> None:
    """Compile sdnn_oracle.c twice: float storage and double storage."""
    for suffix, real in (("f32", "float"), ("f64", "double")):
        out = os.path.join(_HERE, f"libsdnn_oracle_{suffix}.so")
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
            continue
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-ffp-contract=off",
               f"-DREAL={real}", f"-DSUFFIX={suffix}", "-o", out, _SRC, "-lm"]
        subprocess.run(cmd, check=True)


def _lib(suffix: str):
    if suffix not in _LIBS:
        build()
        _LIBS[suffix] = ctypes.CDLL(os.path.join(_HERE, f"libsdnn_oracle_{suffix}.so"))
    return _LIBS[suffix]


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


class Oracle:
    """Oracle over one storage precision: np.float32 (default) or np.float64."""

    def __init__(self, dtype=np.float32, activation: str = "relu"):
        """activation: "relu" (clamped at the cap passed to each call) or "sigmoid" (cap ignored)."""
        self.kind = {"relu": 0, "sigmoid": 1}[activation]
        self.dtype = np.dtype(dtype)
        self.sfx = {"float32": "f32", "float64": "f64"}[self.dtype.name]
        self.lib = _lib(self.sfx)

    def _fn(self, name):
        return getattr(self.lib, f"{name}_{self.sfx}")

    def threads(self) -> int:
        return int(self._fn("oracle_threads")())

    def set_threads(self, n: int) -> None:
        """Thread count of the following calls (for timing; the results do not depend on it)."""
        self._fn("oracle_set_threads")(int(n))

    def _arr(self, a):
        return np.ascontiguousarray(a, dtype=self.dtype)

    def _cap(self, cap: float) -> float:
        """The cap is a number of the storage precision, like the activations
        clamped to it: only then does 'x < cap' on a stored output mean 'z < cap'."""
        return float(self.dtype.type(cap))

    # ---- per-layer operations -------------------------------------------
    def forward_layer(self, layer, x_in: np.ndarray, cap: float) -> np.ndarray:
        x_in = self._arr(x_in)
        assert x_in.shape[0] == layer.n_in
        b = x_in.shape[1]
        out = np.empty((layer.n_out, b), dtype=self.dtype)
        vals = self._arr(layer.values)
        bias = None if layer.bias is None else self._arr(layer.bias)
        self._fn("oracle_forward_layer")(
            ctypes.c_int32(layer.n_out), _ptr(layer.row_ptr), _ptr(layer.col_idx), _ptr(vals),
            _ptr(bias), _ptr(x_in), ctypes.c_int32(b), ctypes.c_int(self.kind), ctypes.c_double(self._cap(cap)),
            _ptr(out))
        return out

    def output_delta(self, dloss: np.ndarray, x_last: np.ndarray, cap: float) -> np.ndarray:
        dloss = self._arr(dloss)
        x_last = self._arr(x_last)
        assert dloss.shape == x_last.shape
        out = np.empty_like(x_last)
        self._fn("oracle_output_delta")(
            ctypes.c_int32(x_last.shape[0]), ctypes.c_int32(x_last.shape[1]), _ptr(dloss),
            _ptr(x_last), ctypes.c_int(self.kind), ctypes.c_double(self._cap(cap)), _ptr(out))
        return out

    def backward_layer(self, layer, delta: np.ndarray, x_prev: Optional[np.ndarray],
                       cap: float) -> np.ndarray:
        delta = self._arr(delta)
        assert delta.shape[0] == layer.n_out
        b = delta.shape[1]
        if x_prev is not None:
            x_prev = self._arr(x_prev)
            assert x_prev.shape == (layer.n_in, b)
        vals = self._arr(layer.values)
        out = np.empty((layer.n_in, b), dtype=self.dtype)
        self._fn("oracle_backward_layer")(
            ctypes.c_int32(layer.n_out), ctypes.c_int32(layer.n_in), _ptr(layer.row_ptr),
            _ptr(layer.col_idx), _ptr(vals), _ptr(delta), _ptr(x_prev), ctypes.c_int32(b),
            ctypes.c_int(self.kind), ctypes.c_double(self._cap(cap)), _ptr(out))
        return out

    def weight_grad(self, layer, delta: np.ndarray, x_prev: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
        delta = self._arr(delta)
        x_prev = self._arr(x_prev)
        b = delta.shape[1]
        assert delta.shape[0] == layer.n_out and x_prev.shape == (layer.n_in, b)
        g = np.empty(layer.nnz, dtype=self.dtype)
        gb = np.empty(layer.n_out, dtype=self.dtype)
        self._fn("oracle_weight_grad")(
            ctypes.c_int32(layer.n_out), _ptr(layer.row_ptr), _ptr(layer.col_idx), _ptr(delta),
            _ptr(x_prev), ctypes.c_int32(b), _ptr(g), _ptr(gb))
        return g, gb

    def sgd_apply(self, w: np.ndarray, g: np.ndarray, lr: float) -> np.ndarray:
        """Returns w - lr*g.  lr is first rounded to fp32: the library's ABI takes a float."""
        w = self._arr(w).copy()
        g = self._arr(g)
        assert w.shape == g.shape
        self._fn("oracle_sgd_apply")(ctypes.c_size_t(w.size), _ptr(w), _ptr(g),
                                     ctypes.c_double(float(np.float32(lr))))
        return w

    # ---- Algorithm 1 ----------------------------------------------------
    def forward(self, layers: Sequence, x0: np.ndarray, cap: float) -> List[np.ndarray]:
        """Feed-forward sweep (Eq. 3 for k = 1..L): returns [X_0, X_1, ..., X_L]."""
        xs = [self._arr(x0)]
        for layer in layers:
            xs.append(self.forward_layer(layer, xs[-1], cap))
        return xs

    def backward(self, layers: Sequence, xs: List[np.ndarray], dloss: np.ndarray,
                 cap: float) -> List[Optional[np.ndarray]]:
        """Output delta (Eq. 6), then Eq. 7 for k = L..2: returns [None, Delta_1, ..., Delta_L]."""
        L = len(layers)
        deltas: List[Optional[np.ndarray]] = [None] * (L + 1)
        deltas[L] = self.output_delta(dloss, xs[L], cap)
        for k in range(L, 1, -1):
            deltas[k - 1] = self.backward_layer(layers[k - 1], deltas[k], xs[k - 1], cap)
        return deltas

    def gradients(self, layers: Sequence, xs, deltas):
        """Eq. 4 for every layer: [(g_k, gb_k)] for k = 1..L (list index k-1)."""
        return [self.weight_grad(layers[k - 1], deltas[k], xs[k - 1]) for k in range(1, len(layers) + 1)]

    def sgd_step(self, layers: Sequence, grads, lr: float, update_bias: bool = True):
        """Eq. 5 (descent step): new (values, bias) per layer; the pattern is never touched."""
        out = []
        for layer, (g, gb) in zip(layers, grads):
            v = self.sgd_apply(layer.values, g, lr)
            b = self.sgd_apply(layer.bias, gb, lr) if update_bias else self._arr(layer.bias).copy()
            out.append((v, b))
        return out

    def train_step(self, layers, x0, cap, dloss_fn, lr, update_bias=True):
        """One full pass of Algorithm 1 on a minibatch.  dloss_fn(X_L) -> dJ/dX_L."""
        xs = self.forward(layers, x0, cap)
        deltas = self.backward(layers, xs, dloss_fn(xs[-1]), cap)
        grads = self.gradients(layers, xs, deltas)
        return xs, deltas, grads, self.sgd_step(layers, grads, lr, update_bias)


# ---- the caller's losses (outside the library: only dJ/dX_L enters, Eq. 6) ----

def mse_loss(x_last: np.ndarray, targets: np.ndarray) -> float:
    """J = 1/(2B) sum_s ||x_s - y_s||^2, in fp64."""
    d = x_last.astype(np.float64) - targets.astype(np.float64)
    return float((d * d).sum() / (2.0 * x_last.shape[1]))


def mse_dloss(x_last: np.ndarray, targets: np.ndarray) -> np.ndarray:
    """dJ/dX_L = (X_L - Y)/B, computed in fp64 and rounded to X_L's dtype."""
    b = x_last.shape[1]
    return ((x_last.astype(np.float64) - targets.astype(np.float64)) / b).astype(x_last.dtype)


def softmax_ce_loss(x_last: np.ndarray, labels: np.ndarray, n_classes: int) -> float:
    """J = -1/B sum_s log softmax(logits_s)[label_s]; logits = the last n_classes rows of X_L."""
    z = x_last[-n_classes:, :].astype(np.float64)
    z = z - z.max(axis=0, keepdims=True)
    logp = z - np.log(np.exp(z).sum(axis=0, keepdims=True))
    return float(-logp[labels, np.arange(z.shape[1])].mean())


def softmax_ce_dloss(x_last: np.ndarray, labels: np.ndarray, n_classes: int) -> np.ndarray:
    """dJ/dX_L = (softmax - onehot)/B on the last n_classes rows, zero elsewhere."""
    b = x_last.shape[1]
    z = x_last[-n_classes:, :].astype(np.float64)
    z = z - z.max(axis=0, keepdims=True)
    p = np.exp(z)
    p /= p.sum(axis=0, keepdims=True)
    p[labels, np.arange(b)] -= 1.0
    out = np.zeros(x_last.shape, dtype=np.float64)
    out[-n_classes:, :] = p / b
    return out.astype(x_last.dtype)
