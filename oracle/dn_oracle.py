"""ctypes front end of the CPU checker (oracle/dn_oracle.c).

TEST INFRASTRUCTURE: imported only by tests, the smoke check and the
benchmark's CPU-baseline leg.  It never imports the device library.

Two precisions of the same C code:
  Oracle("o32") : fp32 storage, fp64 accumulation, one rounding per stored
                  element -- the parity reference for an fp32 device path.
  Oracle("o64") : all fp64 -- for finite differences and closed forms.
  Oracle("o32a"): fp32 storage, fp32 accumulation -- NOT a reference: a second valid fp32
                  evaluation, used to measure how far rounding alone moves ill-conditioned results.
Parameters, velocities and gradients live in flat numpy vectors laid out as
W_1, b_1, W_2, b_2, ... (row-major W_l [n_l, n_{l-1}]).
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libdn_oracle.so")
_lib = None


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build_oracle  # compile on first use
            build_oracle.build(force=True)
        _lib = C.CDLL(_LIB_PATH)
    return _lib


def threads() -> int:
    """Threads the checker's loops run on (OpenMP max threads)."""
    f = _load().o32_threads
    f.restype = C.c_int
    return int(f())


def set_threads(n: int) -> None:
    """Threads for the checker's loops from now on (its results do not depend on the count)."""
    lib = _load()
    lib.o32_set_threads(C.c_int(int(n)))   # one OpenMP runtime: this sets it for every build of the checker


class Oracle:
    def __init__(self, mode: str, widths: Sequence[int], acts: Sequence[int], loss: int):
        assert mode in ("o32", "o64", "o32a")
        lib = _load()
        self.mode = mode
        self.dtype = np.float64 if mode == "o64" else np.float32
        self._real = C.c_double if mode == "o64" else C.c_float
        self.widths = np.asarray(widths, dtype=np.int32)
        self.acts = np.asarray(acts, dtype=np.int32)
        self.L = len(widths) - 1
        assert len(acts) == self.L
        self.loss = int(loss)
        f = lambda name: getattr(lib, mode + "_" + name)
        self._param_count = f("param_count"); self._param_count.restype = C.c_size_t
        self._act_count = f("act_count"); self._act_count.restype = C.c_size_t
        self._forward = f("forward"); self._forward.restype = None
        self._forward_census = f("forward_census"); self._forward_census.restype = C.c_int64
        self._backward = f("backward"); self._backward.restype = C.c_double
        self._update = f("update"); self._update.restype = None
        self._input_gradient = f("input_gradient"); self._input_gradient.restype = None
        self._train_epoch = f("train_epoch"); self._train_epoch.restype = C.c_double
        self._evaluate = f("evaluate"); self._evaluate.restype = C.c_double
        self.P = int(self._param_count(C.c_int(self.L), self._ip(self.widths)))
        self.params = np.zeros(self.P, dtype=self.dtype)
        self.vel = np.zeros(self.P, dtype=self.dtype)
        self.grads = np.zeros(self.P, dtype=self.dtype)
        self.A = None
        self.D = None
        self._B = 0
        self._X = None

    # -- helpers -------------------------------------------------------------
    @staticmethod
    def _ip(a):
        return a.ctypes.data_as(C.POINTER(C.c_int32))

    def _rp(self, a):
        assert a.dtype == self.dtype and a.flags["C_CONTIGUOUS"]
        return a.ctypes.data_as(C.c_void_p)

    def _slices(self) -> List[Tuple[slice, slice]]:
        out, p = [], 0
        for l in range(self.L):
            nw = int(self.widths[l + 1]) * int(self.widths[l])
            nb = int(self.widths[l + 1])
            out.append((slice(p, p + nw), slice(p + nw, p + nw + nb)))
            p += nw + nb
        return out

    def set_params(self, W: Sequence[np.ndarray], b: Sequence[np.ndarray]):
        for (sw, sb), Wl, bl in zip(self._slices(), W, b):
            self.params[sw] = np.asarray(Wl, dtype=self.dtype).reshape(-1)
            self.params[sb] = np.asarray(bl, dtype=self.dtype).reshape(-1)
        self.vel[:] = 0

    def _split(self, flat):
        Ws, bs = [], []
        for l, (sw, sb) in enumerate(self._slices()):
            Ws.append(flat[sw].reshape(int(self.widths[l + 1]), int(self.widths[l])).copy())
            bs.append(flat[sb].copy())
        return Ws, bs

    def get_params(self):
        return self._split(self.params)

    def get_grads(self):
        return self._split(self.grads)

    def _acts_split(self, flat, B):
        out, p = [], 0
        for l in range(1, self.L + 1):
            n = int(self.widths[l])
            out.append(flat[p:p + B * n].reshape(B, n).copy())
            p += B * n
        return out

    # -- the steps -------------------------------------------------------------
    def forward(self, X: np.ndarray, kink_eps: float = 0.0, kink_cap: int = 0) -> List[np.ndarray]:
        """Activations A_1..A_L of the batch.  With kink_eps > 0 the batch's kink census is taken as
        well: self.kinks = its count, self.kink_list = the first kink_cap hits as rows (row, layer, unit)."""
        X = np.ascontiguousarray(X, dtype=self.dtype)
        B = X.shape[0]
        na = int(self._act_count(C.c_int(self.L), self._ip(self.widths), C.c_int(B)))
        self.A = np.zeros(na, dtype=self.dtype)
        self.D = np.zeros(na, dtype=self.dtype)
        self._B, self._X = B, X
        if kink_eps > 0.0:
            buf = np.zeros((max(kink_cap, 1), 3), dtype=np.int64)
            self.kinks = int(self._forward_census(
                C.c_int(self.L), self._ip(self.widths), self._ip(self.acts), self._rp(self.params), self._rp(X),
                C.c_int(B), self._rp(self.A), C.c_double(kink_eps),
                buf.ctypes.data_as(C.c_void_p) if kink_cap > 0 else None, C.c_int64(kink_cap)))
            self.kink_list = buf[:min(self.kinks, kink_cap)]
        else:
            self._forward(C.c_int(self.L), self._ip(self.widths), self._ip(self.acts),
                          self._rp(self.params), self._rp(X), C.c_int(B), self._rp(self.A))
        return self._acts_split(self.A, B)

    def backward(self, labels: np.ndarray) -> float:
        labels = np.ascontiguousarray(labels, dtype=np.int32)
        assert self.A is not None and labels.shape[0] == self._B
        return float(self._backward(C.c_int(self.L), self._ip(self.widths), self._ip(self.acts),
                                    C.c_int(self.loss), self._rp(self.params), self._rp(self._X),
                                    self._ip(labels), C.c_int(self._B), self._rp(self.A),
                                    self._rp(self.D), self._rp(self.grads)))

    def deltas(self) -> List[np.ndarray]:
        return self._acts_split(self.D, self._B)

    def input_gradient(self) -> np.ndarray:
        """dE_s/dx_s for every sample of the last backward(), [B][n_0]."""
        dX = np.zeros((self._B, int(self.widths[0])), dtype=self.dtype)
        self._input_gradient(C.c_int(self.L), self._ip(self.widths), self._rp(self.params),
                             self._rp(self.D), C.c_int(self._B), self._rp(dX))
        return dX

    def update(self, lr: float, momentum: float):
        self._update(C.c_size_t(self.P), self._rp(self.params), self._rp(self.vel),
                     self._rp(self.grads), self._real(lr), self._real(momentum))

    def train_epoch(self, X: np.ndarray, labels: np.ndarray, batch: int, lr: float,
                    momentum: float, steps_limit: int = 0, kink_eps: float = 0.0, kink_cap: int = 0):
        """Returns (epoch loss, count of ReLU units with |z| < kink_eps).  With kink_cap > 0 the
        first kink_cap of those units are kept in self.kink_list as rows (sample, layer, unit)."""
        X = np.ascontiguousarray(X, dtype=self.dtype)
        labels = np.ascontiguousarray(labels, dtype=np.int32)
        kinks = C.c_int64(0)
        buf = np.zeros((max(kink_cap, 1), 3), dtype=np.int64)
        loss = self._train_epoch(C.c_int(self.L), self._ip(self.widths), self._ip(self.acts),
                                 C.c_int(self.loss), self._rp(self.params), self._rp(self.vel),
                                 self._rp(X), self._ip(labels), C.c_int64(X.shape[0]),
                                 C.c_int(batch), self._real(lr), self._real(momentum),
                                 C.c_int64(steps_limit), C.c_double(kink_eps), C.byref(kinks),
                                 buf.ctypes.data_as(C.c_void_p) if kink_cap > 0 else None, C.c_int64(kink_cap))
        self.kink_list = buf[:min(int(kinks.value), kink_cap)] if kink_cap > 0 else buf[:0]
        return float(loss), int(kinks.value)

    def evaluate(self, X: np.ndarray, labels: np.ndarray) -> Tuple[float, int]:
        """(mean loss, number of samples whose largest output is at the label) at the current parameters."""
        X = np.ascontiguousarray(X, dtype=self.dtype)
        labels = np.ascontiguousarray(labels, dtype=np.int32)
        correct = C.c_int64(0)
        loss = self._evaluate(C.c_int(self.L), self._ip(self.widths), self._ip(self.acts), C.c_int(self.loss),
                              self._rp(self.params), self._rp(X), self._ip(labels), C.c_int64(X.shape[0]),
                              C.byref(correct))
        return float(loss), int(correct.value)

    def train(self, X: np.ndarray, labels: np.ndarray, batch: int, lr: float, momentum: float,
              max_error: float, max_epochs: int) -> Tuple[int, float, List[float]]:
        """Epochs until the epoch loss is at most max_error (the work-flow's maximum-error
        parameter) or max_epochs have run: (epochs run, last epoch loss, all epoch losses)."""
        losses = []
        for _ in range(max_epochs):
            losses.append(self.train_epoch(X, labels, batch, lr, momentum)[0])
            if losses[-1] <= max_error:
                break
        return len(losses), losses[-1], losses

    def loss_value(self, X: np.ndarray, labels: np.ndarray) -> float:
        """Batch-mean loss at the current parameters (forward + loss only)."""
        self.forward(X)
        saved = self.grads.copy()
        val = self.backward(labels)
        self.grads[:] = saved
        return val
