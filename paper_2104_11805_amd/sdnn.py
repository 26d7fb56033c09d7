"""Thin ctypes binding of libsdnn.so: argument marshalling only.

Function names mirror include/sdnn.h.  torch is used for device memory (the
workspace and the I/O tensors) and for the current stream, nothing else; every
step of the three passes runs in the library's HIP kernels.  There is no CPU
fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsdnn.so")

SDNN_OK, SDNN_EINVAL, SDNN_ESTATE, SDNN_ENOMEM, SDNN_EHIP = 0, -1, -2, -3, -4
SDNN_ACT_RELU_CAP, SDNN_ACT_SIGMOID = 0, 1
SDNN_FUSE_AUTO, SDNN_FUSE_ON, SDNN_FUSE_OFF = 0, 1, -1
SDNN_NOALLOC_SCRATCH_BYTES = 16 << 20
SDNN_PANEL_AUTO, SDNN_PANEL_OFF = 0, -1
SDNN_LDS_AUTO, SDNN_LDS_ON, SDNN_LDS_OFF = 0, 1, -1


class SdnnError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"sdnn error {code}: {msg}")
        self.code = code


class sdnn_layer(C.Structure):
    _fields_ = [("n_out", C.c_int32), ("n_in", C.c_int32), ("row_ptr", C.c_void_p),
                ("col_idx", C.c_void_p), ("values", C.c_void_p), ("bias", C.c_void_p)]


class sdnn_config(C.Structure):
    _fields_ = [("act_cap", C.c_float), ("max_batch", C.c_int32), ("training", C.c_int32),
                ("update_bias", C.c_int32), ("activation", C.c_int32), ("fuse_gradient", C.c_int32),
                ("panel_cols", C.c_int32), ("reorder_rows", C.c_int32), ("lds_forward", C.c_int32)]


# name -> (restype, argtypes); every symbol include/sdnn.h declares
_P, _I32, _I64P, _SZ = C.c_void_p, C.c_int32, C.POINTER(C.c_int64), C.c_size_t
SIGNATURES = {
    "sdnn_workspace_bytes": (C.c_int, [C.POINTER(sdnn_layer), _I32, C.POINTER(sdnn_config), C.POINTER(_SZ)]),
    "sdnn_create": (C.c_int, [C.POINTER(sdnn_layer), _I32, C.POINTER(sdnn_config), _P, _SZ, _P, C.POINTER(_P)]),
    "sdnn_destroy": (None, [_P]),
    "sdnn_forward": (C.c_int, [_P, _P, _I32, _P, _P]),
    "sdnn_forward_noalloc": (C.c_int, [_P, _P, _I32, _P, _P]),
    "sdnn_forward_skip_dead": (C.c_int, [_P, _P, _I32, _P, _I32, _P, _P]),
    "sdnn_backward": (C.c_int, [_P, _P, _P]),
    "sdnn_sgd_step": (C.c_int, [_P, C.c_float, _P]),
    "sdnn_get_activation": (C.c_int, [_P, _I32, _P, _P]),
    "sdnn_get_delta": (C.c_int, [_P, _I32, _P, _P]),
    "sdnn_weight_grad": (C.c_int, [_P, _I32, _P, _P, _P]),
    "sdnn_get_weights": (C.c_int, [_P, _I32, _P, _P, _P]),
    "sdnn_set_weights": (C.c_int, [_P, _I32, _P, _P, _P]),
    "sdnn_layer_shape": (C.c_int, [_P, _I32, C.POINTER(_I32), C.POINTER(_I32), _I64P]),
    "sdnn_mse_dloss": (C.c_int, [_P, _P, _I32, _I32, _P, _P]),
    "sdnn_softmax_ce_dloss": (C.c_int, [_P, _P, _I32, _I32, _I32, _P, _P]),
    "sdnn_gather_probe": (C.c_int, [_P, _I32, _I32, _P, _I32, _I32, _P, _P]),
    "sdnn_check_csr": (C.c_int, [_I32, _I32, _P, _P]),
    "sdnn_transpose_pattern": (C.c_int, [_I32, _I32, _P, _P, _P, _P, _P]),
    "sdnn_row_schedule": (C.c_int, [_I32, _P, _P]),
    "sdnn_cluster_rows": (C.c_int, [_I32, _I32, _P, _P, _I32, _P, _P]),
    "sdnn_deal_rows_to_xcds": (C.c_int, [_I32, _P, _P, _P]),
    "sdnn_last_error": (C.c_char_p, [_P]),
    "sdnn_version": (C.c_char_p, []),
}

_lib = None


def lib():
    """Load libsdnn.so (built by paper_2104_11805_amd.build / __graft_entry__.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            # nothing built yet: compile once (hipcc cross-compiles for gfx950 without a GPU); no fallback exists
            try:
                from . import build as _build
                _build.build_lib()
            except Exception as e:
                raise ImportError(f"{LIB_PATH} is missing and could not be built ({e}): run "
                                  "`python -c 'import __graft_entry__ as g; g.build()'`") from e
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


def last_error(net=None) -> str:
    return (lib().sdnn_last_error(net) or b"").decode()


def _check(rc: int, net=None):
    if rc != SDNN_OK:
        raise SdnnError(rc, last_error(net))


def _np(a, dtype):
    return None if a is None else np.ascontiguousarray(a, dtype=dtype)


def _hp(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


# ---- host-only setup pieces ------------------------------------------------

def sdnn_check_csr(n_out, n_in, row_ptr, col_idx) -> int:
    rp, ci = _np(row_ptr, np.int32), _np(col_idx, np.int32)
    return lib().sdnn_check_csr(n_out, n_in, _hp(rp), _hp(ci))


def sdnn_transpose_pattern(n_out, n_in, row_ptr, col_idx):
    rp, ci = _np(row_ptr, np.int32), _np(col_idx, np.int32)
    nnz = int(rp[n_out])
    t_rp = np.empty(n_in + 1, np.int32)
    t_ri = np.empty(nnz, np.int32)
    t_pm = np.empty(nnz, np.int32)
    _check(lib().sdnn_transpose_pattern(n_out, n_in, _hp(rp), _hp(ci), _hp(t_rp), _hp(t_ri), _hp(t_pm)))
    return t_rp, t_ri, t_pm


def sdnn_row_schedule(n_rows, row_ptr):
    rp = _np(row_ptr, np.int32)
    order = np.empty(n_rows, np.int32)
    _check(lib().sdnn_row_schedule(n_rows, _hp(rp), _hp(order)))
    return order


def sdnn_cluster_rows(n_rows, n_cols, row_ptr, col_idx, max_cluster_rows=256):
    rp, ci = _np(row_ptr, np.int32), _np(col_idx, np.int32)
    order = np.empty(n_rows, np.int32)
    cluster_of = np.empty(n_rows, np.int32)
    _check(lib().sdnn_cluster_rows(n_rows, n_cols, _hp(rp), _hp(ci), max_cluster_rows, _hp(order), _hp(cluster_of)))
    return order, cluster_of


def sdnn_deal_rows_to_xcds(n_rows, row_ptr, order):
    rp, od = _np(row_ptr, np.int32), _np(order, np.int32)
    dealt = np.empty(n_rows, np.int32)
    _check(lib().sdnn_deal_rows_to_xcds(n_rows, _hp(rp), _hp(od), _hp(dealt)))
    return dealt


# ---- the network handle ------------------------------------------------------

def _stream_ptr(stream=None):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _dp(t):
    """Device pointer of a contiguous fp32/int32 CUDA tensor (None -> NULL)."""
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous CUDA tensors"
    return C.c_void_p(t.data_ptr())


class Net:
    """Owns the workspace tensor and the opaque sdnn_net handle."""

    def __init__(self, layers: Sequence, act_cap: float, max_batch: int, training: bool = True,
                 update_bias: bool = True, device: str = "cuda:0", activation: str = "relu",
                 fuse_gradient: int = 0, panel_cols: int = 0, reorder_rows: bool = False, lds_forward: int = 0):
        import torch
        self._handle = None
        self._keep = []
        arr = (sdnn_layer * len(layers))()
        for k, l in enumerate(layers):
            rp, ci = _np(l.row_ptr, np.int32), _np(l.col_idx, np.int32)
            va, bi = _np(l.values, np.float32), _np(l.bias, np.float32)
            self._keep += [rp, ci, va, bi]
            arr[k] = sdnn_layer(l.n_out, l.n_in, _hp(rp).value, _hp(ci).value,
                                _hp(va).value if va.size else None,
                                None if bi is None else _hp(bi).value)
        self.cfg = sdnn_config(float(act_cap), int(max_batch), int(training), int(update_bias),
                               {"relu": SDNN_ACT_RELU_CAP, "sigmoid": SDNN_ACT_SIGMOID}[activation],
                               int(fuse_gradient), int(panel_cols), int(reorder_rows), int(lds_forward))
        nbytes = C.c_size_t(0)
        _check(lib().sdnn_workspace_bytes(arr, len(layers), C.byref(self.cfg), C.byref(nbytes)))
        self.device = torch.device(device)
        self.workspace_bytes = nbytes.value
        # the library lays its large arrays out on multiples of up to 2 MiB relative to the workspace: hand it a
        # workspace that starts on a 2 MiB boundary itself (torch only promises 512 bytes)
        big = 2 << 20
        self.workspace = torch.empty(max(nbytes.value, 256) + big, dtype=torch.uint8, device=self.device)
        base = (self.workspace.data_ptr() + big - 1) // big * big
        h = C.c_void_p()
        with torch.cuda.device(self.device):
            _check(lib().sdnn_create(arr, len(layers), C.byref(self.cfg),
                                     C.c_void_p(base), nbytes.value,
                                     _stream_ptr(), C.byref(h)))
        self._handle = h
        self._keep = []
        self.n_layers = len(layers)
        self.shapes = [(l.n_out, l.n_in, int(l.row_ptr[l.n_out])) for l in layers]
        self.total_nnz = sum(s[2] for s in self.shapes)

    def close(self):
        if self._handle is not None:
            lib().sdnn_destroy(self._handle)
            self._handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- passes (names as in the header) --
    def sdnn_forward(self, x0, xl=None, stream=None):
        b = x0.shape[1]
        _check(lib().sdnn_forward(self._handle, _dp(x0), b, _dp(xl), _stream_ptr(stream)), self._handle)
        return xl

    def sdnn_forward_noalloc(self, x0, xl, stream=None):
        b = x0.shape[1]
        _check(lib().sdnn_forward_noalloc(self._handle, _dp(x0), b, _dp(xl), _stream_ptr(stream)), self._handle)
        return xl

    def sdnn_forward_skip_dead(self, x0, xl, check_every: int = 4, n_live=None, stream=None):
        """n_live: None or an int32 device tensor of one element that receives the live-sample count."""
        b = x0.shape[1]
        _check(lib().sdnn_forward_skip_dead(self._handle, _dp(x0), b, _dp(xl), int(check_every), _dp(n_live),
                                            _stream_ptr(stream)), self._handle)
        return xl

    def sdnn_backward(self, dloss, stream=None):
        _check(lib().sdnn_backward(self._handle, _dp(dloss), _stream_ptr(stream)), self._handle)

    def sdnn_sgd_step(self, lr: float, stream=None):
        _check(lib().sdnn_sgd_step(self._handle, C.c_float(lr), _stream_ptr(stream)), self._handle)

    # -- inspection --
    def _empty(self, *shape, dtype=None):
        import torch
        return torch.empty(*shape, dtype=dtype or torch.float32, device=self.device)

    def sdnn_get_activation(self, layer: int, b: int, stream=None):
        n = self.shapes[0][1] if layer == 0 else self.shapes[layer - 1][0]
        out = self._empty(n, b)
        _check(lib().sdnn_get_activation(self._handle, layer, _dp(out), _stream_ptr(stream)), self._handle)
        return out

    def sdnn_get_delta(self, layer: int, b: int, stream=None):
        out = self._empty(self.shapes[layer - 1][0], b)
        _check(lib().sdnn_get_delta(self._handle, layer, _dp(out), _stream_ptr(stream)), self._handle)
        return out

    def sdnn_weight_grad(self, layer: int, stream=None):
        n_out, _, nnz = self.shapes[layer - 1]
        g, gb = self._empty(nnz), self._empty(n_out)
        _check(lib().sdnn_weight_grad(self._handle, layer, _dp(g), _dp(gb), _stream_ptr(stream)), self._handle)
        return g, gb

    def sdnn_get_weights(self, layer: int, stream=None):
        n_out, _, nnz = self.shapes[layer - 1]
        v, b = self._empty(nnz), self._empty(n_out)
        _check(lib().sdnn_get_weights(self._handle, layer, _dp(v), _dp(b), _stream_ptr(stream)), self._handle)
        return v, b

    def sdnn_set_weights(self, layer: int, values=None, bias=None, stream=None):
        _check(lib().sdnn_set_weights(self._handle, layer, _dp(values), _dp(bias), _stream_ptr(stream)), self._handle)


def sdnn_mse_dloss(xl, y, out=None, stream=None):
    import torch
    out = torch.empty_like(xl) if out is None else out
    _check(lib().sdnn_mse_dloss(_dp(xl), _dp(y), xl.shape[0], xl.shape[1], _dp(out), _stream_ptr(stream)))
    return out


def sdnn_softmax_ce_dloss(xl, labels_i32, n_classes: int, out=None, stream=None):
    import torch
    out = torch.empty_like(xl) if out is None else out
    _check(lib().sdnn_softmax_ce_dloss(_dp(xl), _dp(labels_i32), xl.shape[0], xl.shape[1], n_classes,
                                       _dp(out), _stream_ptr(stream)))
    return out


def sdnn_gather_probe(table, v: int, idx_i32, n_waves: int, per_wave: int, out, stream=None):
    """table [rows][64*v] fp32, idx int32 [n_waves*per_wave], out fp32 [n_waves*64]: all device tensors."""
    _check(lib().sdnn_gather_probe(_dp(table), table.shape[0], int(v), _dp(idx_i32), int(n_waves), int(per_wave), _dp(out),
                                   _stream_ptr(stream)))
