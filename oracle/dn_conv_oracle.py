"""ctypes front end of the CPU checker's convolutional and max-pooling layers
(oracle/dn_conv_oracle.c).

TEST INFRASTRUCTURE: imported only by tests, the smoke check and the
benchmark's CPU-baseline leg.  It never imports the device library.

mode "o32": fp32 storage, fp64 accumulation (the parity reference of an fp32
device path); mode "o64": all fp64 (finite differences, closed forms).
Arrays are C-contiguous: images [batch][channel][row][column], filters
[out channel][in channel][filter row][filter column].
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from .dn_oracle import _load


def _dtype(mode):
    assert mode in ("o32", "o64")
    return np.float32 if mode == "o32" else np.float64


def _p(a, dt):
    assert a.dtype == dt and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.c_void_p)


def out_size(n: int, k: int, stride: int, pad: int) -> int:
    return (n + 2 * pad - k) // stride + 1


def conv_forward(mode, X, Wt, bias, stride, pad, act):
    dt = _dtype(mode)
    B, Cin, H, W = X.shape
    Cout, Cin2, KH, KW = Wt.shape
    assert Cin2 == Cin and bias.shape == (Cout,)
    Y = np.zeros((B, Cout, out_size(H, KH, stride, pad), out_size(W, KW, stride, pad)), dtype=dt)
    f = getattr(_load(), mode + "_conv_forward")
    f.restype = None
    f(B, Cin, H, W, Cout, KH, KW, int(stride), int(pad), int(act), _p(X, dt), _p(Wt, dt), _p(bias, dt), _p(Y, dt))
    return Y


def conv_backward(mode, X, Wt, Y, dA, stride, pad, act, want_dx=True):
    """Returns (delta, dX or None, dW, dbias)."""
    dt = _dtype(mode)
    B, Cin, H, W = X.shape
    Cout, _, KH, KW = Wt.shape
    assert Y.shape == dA.shape == (B, Cout, out_size(H, KH, stride, pad), out_size(W, KW, stride, pad))
    delta = np.zeros_like(Y)
    dX = np.zeros_like(X) if want_dx else None
    dW = np.zeros_like(Wt)
    db = np.zeros(Cout, dtype=dt)
    f = getattr(_load(), mode + "_conv_backward")
    f.restype = None
    f(B, Cin, H, W, Cout, KH, KW, int(stride), int(pad), int(act), _p(X, dt), _p(Wt, dt), _p(Y, dt), _p(dA, dt),
      _p(delta, dt), _p(dX, dt) if want_dx else None, _p(dW, dt), _p(db, dt))
    return delta, dX, dW, db


def maxpool_forward(mode, X, k, stride):
    dt = _dtype(mode)
    B, Cn, H, W = X.shape
    Y = np.zeros((B, Cn, (H - k) // stride + 1, (W - k) // stride + 1), dtype=dt)
    f = getattr(_load(), mode + "_maxpool_forward")
    f.restype = None
    f(B, Cn, H, W, int(k), int(stride), _p(X, dt), _p(Y, dt))
    return Y


def maxpool_backward(mode, X, dY, k, stride):
    dt = _dtype(mode)
    B, Cn, H, W = X.shape
    assert dY.shape == (B, Cn, (H - k) // stride + 1, (W - k) // stride + 1)
    dX = np.zeros_like(X)
    f = getattr(_load(), mode + "_maxpool_backward")
    f.restype = None
    f(B, Cn, H, W, int(k), int(stride), _p(X, dt), _p(dY, dt), _p(dX, dt))
    return dX
