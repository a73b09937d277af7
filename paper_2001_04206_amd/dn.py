"""ctypes binding of libdn: same names as include/dn.h, argument marshalling only.

PyTorch-ROCm is used for device memory (the arena and the data tensors) and for
the HIP stream handle; no torch operator takes part in a training step.  The
library must be built (``python -m paper_2001_04206_amd.build``); a missing
library is an error, there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdn.so")

DN_OK, DN_ERR_INVALID_ARG, DN_ERR_SHAPE, DN_ERR_UNSUPPORTED, DN_ERR_OOM, DN_ERR_DEVICE = range(6)
DN_ACT_LINEAR, DN_ACT_SIGMOID, DN_ACT_TANH, DN_ACT_RELU, DN_ACT_SOFTMAX = range(5)
DN_LOSS_MSE, DN_LOSS_CROSS_ENTROPY = 0, 1
DN_K_FORWARD, DN_K_DELTA, DN_K_GRAD_UPDATE, DN_K_OUTPUT, DN_K_ONLINE = range(5)
KERNEL_CLASS_NAMES = ["forward", "delta", "grad_update", "output", "online"]
(DN_SCHED_NONE, DN_SCHED_LAUNCHES, DN_SCHED_PER_SAMPLE, DN_SCHED_TWO_COPY, DN_SCHED_MINIBATCH,
 DN_SCHED_MINIBATCH_DEEP, DN_SCHED_ONE_WAVE, DN_SCHED_WIDE_HIDDEN, DN_SCHED_ONE_WAVE_REGISTERS,
 DN_SCHED_ONE_WORKGROUP) = range(10)
# the kernel behind each persistent schedule
SCHEDULE_KERNELS = {DN_SCHED_PER_SAMPLE: "online_epoch_kernel", DN_SCHED_TWO_COPY: "twin_epoch_kernel",
                    DN_SCHED_MINIBATCH: "batch_epoch_kernel", DN_SCHED_MINIBATCH_DEEP: "deep_batch_epoch_kernel",
                    DN_SCHED_ONE_WAVE: "tiny_epoch_kernel", DN_SCHED_WIDE_HIDDEN: "wide_epoch_kernel",
                    DN_SCHED_ONE_WAVE_REGISTERS: "tiny_regs_epoch_kernel", DN_SCHED_ONE_WORKGROUP: "solo_epoch_kernel"}

EXPORTS = [
    "dn_status_string", "dn_net_arena_bytes", "dn_net_create", "dn_net_destroy", "dn_set_params",
    "dn_get_params", "dn_get_grads", "dn_forward", "dn_backward", "dn_update", "dn_train_epoch",
    "dn_train", "dn_evaluate", "dn_layer_backward_workspace_bytes", "dn_layer_backward_host",
    "dn_last_epoch_ms", "dn_last_schedule", "dn_kernel_time", "dn_kernel_flops", "dn_set_option",
    "dn_conv_forward", "dn_conv_backward_workspace_bytes", "dn_conv_backward", "dn_maxpool_forward",
    "dn_maxpool_backward", "dn_input_gradient", "dn_sgd_step",
    "dn_conv_backward_static", "dn_conv_backward_static_limit",
    "dn_cnn_arena_bytes", "dn_cnn_create", "dn_cnn_destroy", "dn_cnn_dense", "dn_cnn_flat_size",
    "dn_cnn_set_filters", "dn_cnn_get_filters", "dn_cnn_get_filter_grads", "dn_cnn_forward", "dn_cnn_train_epoch",
]

_lib = None


class DnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (status %d)" % (where, status_string(status), status))


def lib():
    """Load libdn.so (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libdn.so is missing: build it with `python -m paper_2001_04206_amd.build`")
        # PyTorch ships its own HIP runtime (same soname as the system one).  Import it
        # first so that libdn binds to that copy: device pointers and streams handed
        # over from torch are only meaningful inside the runtime that created them.
        import torch  # noqa: F401
        l = C.CDLL(LIB_PATH)
        vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
        l.dn_status_string.restype = C.c_char_p
        l.dn_status_string.argtypes = [C.c_int]
        l.dn_net_arena_bytes.restype = C.c_size_t
        l.dn_net_arena_bytes.argtypes = [vp, i32, i32]
        l.dn_net_create.argtypes = [vp, i32, vp, C.c_int, i32, vp, C.c_size_t, vp, C.POINTER(vp)]
        l.dn_net_destroy.argtypes = [vp]
        for f in (l.dn_set_params, l.dn_get_params, l.dn_get_grads):
            f.argtypes = [vp, i32, vp, vp]
        l.dn_forward.argtypes = [vp, vp, i32, vp]
        l.dn_backward.argtypes = [vp, vp, i32, vp]
        l.dn_update.argtypes = [vp, f32, f32]
        l.dn_input_gradient.argtypes = [vp, i32, vp]
        l.dn_sgd_step.argtypes = [vp, vp, vp, i64, f32, f32, vp]
        l.dn_train_epoch.argtypes = [vp, vp, vp, i64, i32, f32, f32, C.POINTER(f32)]
        l.dn_train.argtypes = [vp, vp, vp, i64, i32, f32, f32, f32, i32, C.POINTER(i32), C.POINTER(f32)]
        l.dn_evaluate.argtypes = [vp, vp, vp, i64, i32, C.POINTER(f32), C.POINTER(i64)]
        l.dn_layer_backward_workspace_bytes.restype = C.c_size_t
        l.dn_layer_backward_workspace_bytes.argtypes = [i32, i32]
        l.dn_layer_backward_host.argtypes = [vp, vp, f32, i32, i32, vp, vp, vp, vp, C.c_size_t, vp,
                                             C.POINTER(f32), C.POINTER(f32), C.POINTER(f32)]
        l.dn_last_epoch_ms.argtypes = [vp, C.POINTER(f32)]
        l.dn_last_schedule.argtypes = [vp, C.POINTER(i32)]
        l.dn_kernel_time.argtypes = [vp, i32, C.POINTER(f32), C.POINTER(i64)]
        l.dn_kernel_flops.argtypes = [vp, i32, C.POINTER(C.c_double)]
        l.dn_set_option.argtypes = [vp, C.c_char_p, i64]
        l.dn_cnn_arena_bytes.argtypes = [i32, i32, i32, vp, i32, vp, i32, i32]
        l.dn_cnn_create.argtypes = [i32, i32, i32, vp, i32, vp, i32, vp, C.c_int, i32, vp, C.c_size_t, vp, C.POINTER(vp)]
        l.dn_cnn_destroy.argtypes = [vp]
        l.dn_cnn_dense.argtypes = [vp]
        l.dn_cnn_flat_size.argtypes = [vp]
        for f in (l.dn_cnn_set_filters, l.dn_cnn_get_filters, l.dn_cnn_get_filter_grads):
            f.argtypes = [vp, i32, vp, vp]
        l.dn_cnn_forward.argtypes = [vp, vp, i32, vp]
        l.dn_cnn_train_epoch.argtypes = [vp, vp, vp, i64, i32, f32, f32, C.POINTER(f32)]
        for name in EXPORTS[2:]:
            if name.endswith("_workspace_bytes") or name.endswith("_static_limit") or name.endswith("_arena_bytes"):
                getattr(l, name).restype = C.c_size_t
            elif name == "dn_cnn_dense":
                getattr(l, name).restype = vp
            elif name == "dn_cnn_flat_size":
                getattr(l, name).restype = i32
            else:
                getattr(l, name).restype = C.c_int
        _lib = l
    return _lib


def status_string(status: int) -> str:
    return lib().dn_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != DN_OK:
        raise DnError(status, where)


def _i32(a: Sequence[int]):
    arr = np.ascontiguousarray(a, dtype=np.int32)
    return arr, arr.ctypes.data_as(C.c_void_p)


def dn_net_arena_bytes(widths: Sequence[int], max_batch: int) -> int:
    arr, p = _i32(widths)
    return int(lib().dn_net_arena_bytes(p, len(arr), int(max_batch)))


def _dev_ptr(t, dtype, what: str):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError("%s must be a contiguous device tensor of dtype %s" % (what, dtype))
    return C.c_void_p(t.data_ptr())


def dn_layer_backward_host(deltas, inputs, learning_rate: float, gradients, delta_weights, delta_biases,
                           workspace=None):
    """One layer's backward step for one sample with host buffers copied in and out around the
    kernel.  All arrays are host tensors (torch CPU float32, pinned or not) or numpy float32
    arrays; `workspace` is a device uint8 tensor (allocated here if None).  Returns the device
    milliseconds of (copy in, kernel, copy out)."""
    import torch

    def host_ptr(a, n, what):
        if isinstance(a, torch.Tensor):
            if a.is_cuda or a.dtype != torch.float32 or not a.is_contiguous() or a.numel() != n:
                raise TypeError("%s must be a contiguous host float32 tensor of %d elements" % (what, n))
            return C.c_void_p(a.data_ptr())
        if not isinstance(a, np.ndarray) or a.dtype != np.float32 or not a.flags["C_CONTIGUOUS"] or a.size != n:
            raise TypeError("%s must be a contiguous float32 array of %d elements" % (what, n))
        return a.ctypes.data_as(C.c_void_p)

    cols_out = int(deltas.shape[0])
    cols_in = int(inputs.shape[0])
    need = int(lib().dn_layer_backward_workspace_bytes(cols_out, cols_in))
    if need == 0:
        raise DnError(DN_ERR_SHAPE, "dn_layer_backward_workspace_bytes")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    stream = torch.cuda.current_stream(workspace.device)
    t = [C.c_float(0.0), C.c_float(0.0), C.c_float(0.0)]
    with torch.cuda.device(workspace.device):
        st = lib().dn_layer_backward_host(
            host_ptr(deltas, cols_out, "deltas"), host_ptr(inputs, cols_in, "inputs"), float(learning_rate),
            cols_out, cols_in, host_ptr(gradients, cols_out * cols_in, "gradients"),
            host_ptr(delta_weights, cols_out * cols_in, "delta_weights"),
            host_ptr(delta_biases, cols_out, "delta_biases"), C.c_void_p(workspace.data_ptr()),
            int(workspace.numel()), C.c_void_p(stream.cuda_stream), C.byref(t[0]), C.byref(t[1]), C.byref(t[2]))
    _check(st, "dn_layer_backward_host")
    return t[0].value, t[1].value, t[2].value


def _shape_check(t, shape, what):
    if tuple(t.shape) != tuple(shape):
        raise TypeError("%s must have shape %s, not %s" % (what, tuple(shape), tuple(t.shape)))


def conv_out_size(n: int, k: int, stride: int, pad: int) -> int:
    return (n + 2 * pad - k) // stride + 1


def dn_conv_forward(X, W, bias, Y, stride: int, pad: int, act: int):
    """Y = f(conv(X, W) + bias).  X [B][Cin][H][W], W [Cout][Cin][KH][KW], bias [Cout],
    Y [B][Cout][Ho][Wo]: contiguous float32 device tensors.  Enqueued on torch's current stream."""
    import torch
    B, Cin, H, Wd = (int(v) for v in X.shape)
    Cout, Cin2, KH, KW = (int(v) for v in W.shape)
    if Cin2 != Cin:
        raise TypeError("filter channels do not match the input")
    _shape_check(bias, (Cout,), "bias")
    _shape_check(Y, (B, Cout, conv_out_size(H, KH, stride, pad), conv_out_size(Wd, KW, stride, pad)), "Y")
    f32 = torch.float32
    with torch.cuda.device(X.device):
        stream = torch.cuda.current_stream(X.device)
        _check(lib().dn_conv_forward(_dev_ptr(X, f32, "X"), _dev_ptr(W, f32, "W"), _dev_ptr(bias, f32, "bias"),
                                     _dev_ptr(Y, f32, "Y"), B, Cin, H, Wd, Cout, KH, KW, int(stride), int(pad),
                                     int(act), C.c_void_p(stream.cuda_stream)), "dn_conv_forward")


def dn_conv_backward(X, W, Y, dA, delta, dX, dW, dbias, stride: int, pad: int, act: int, workspace=None):
    """delta = dA * f'(Y); dW, dbias = batch means of the parameter gradients; dX (or None) = dE/dX.
    `workspace`: a device uint8 tensor of dn_conv_backward_workspace_bytes(...) bytes (allocated here if None)."""
    import torch
    B, Cin, H, Wd = (int(v) for v in X.shape)
    Cout, Cin2, KH, KW = (int(v) for v in W.shape)
    if Cin2 != Cin:
        raise TypeError("filter channels do not match the input")
    yshape = (B, Cout, conv_out_size(H, KH, stride, pad), conv_out_size(Wd, KW, stride, pad))
    for t, name in ((Y, "Y"), (dA, "dA"), (delta, "delta")):
        _shape_check(t, yshape, name)
    _shape_check(dW, W.shape, "dW")
    _shape_check(dbias, (Cout,), "dbias")
    if dX is not None:
        _shape_check(dX, X.shape, "dX")
    f32 = torch.float32
    need = int(lib().dn_conv_backward_workspace_bytes(B, Cin, H, Wd, Cout, KH, KW, int(stride), int(pad)))
    if need == 0:
        raise DnError(DN_ERR_INVALID_ARG, "dn_conv_backward_workspace_bytes")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
    with torch.cuda.device(X.device):
        stream = torch.cuda.current_stream(X.device)
        _check(lib().dn_conv_backward(_dev_ptr(X, f32, "X"), _dev_ptr(W, f32, "W"), _dev_ptr(Y, f32, "Y"),
                                      _dev_ptr(dA, f32, "dA"), _dev_ptr(delta, f32, "delta"),
                                      None if dX is None else _dev_ptr(dX, f32, "dX"), _dev_ptr(dW, f32, "dW"),
                                      _dev_ptr(dbias, f32, "dbias"), _dev_ptr(workspace, torch.uint8, "workspace"),
                                      C.c_size_t(int(workspace.numel())), B, Cin, H, Wd, Cout, KH, KW, int(stride),
                                      int(pad), int(act), C.c_void_p(stream.cuda_stream)), "dn_conv_backward")


def dn_conv_backward_static_limit() -> int:
    return int(lib().dn_conv_backward_static_limit())


def dn_conv_backward_static(X, W, Y, dA, delta, dX, dW, dbias, stride: int, pad: int, act: int):
    """dn_conv_backward with the library's fixed scratch array in place of a workspace: nothing is
    allocated, here or in the library."""
    import torch
    B, Cin, H, Wd = (int(v) for v in X.shape)
    Cout, Cin2, KH, KW = (int(v) for v in W.shape)
    if Cin2 != Cin:
        raise TypeError("filter channels do not match the input")
    yshape = (B, Cout, conv_out_size(H, KH, stride, pad), conv_out_size(Wd, KW, stride, pad))
    for t, name in ((Y, "Y"), (dA, "dA"), (delta, "delta")):
        _shape_check(t, yshape, name)
    _shape_check(dW, W.shape, "dW")
    _shape_check(dbias, (Cout,), "dbias")
    if dX is not None:
        _shape_check(dX, X.shape, "dX")
    f32 = torch.float32
    with torch.cuda.device(X.device):
        stream = torch.cuda.current_stream(X.device)
        _check(lib().dn_conv_backward_static(_dev_ptr(X, f32, "X"), _dev_ptr(W, f32, "W"), _dev_ptr(Y, f32, "Y"),
                                             _dev_ptr(dA, f32, "dA"), _dev_ptr(delta, f32, "delta"),
                                             None if dX is None else _dev_ptr(dX, f32, "dX"),
                                             _dev_ptr(dW, f32, "dW"), _dev_ptr(dbias, f32, "dbias"), B, Cin, H, Wd,
                                             Cout, KH, KW, int(stride), int(pad), int(act),
                                             C.c_void_p(stream.cuda_stream)), "dn_conv_backward_static")


def dn_maxpool_forward(X, Y, k: int, stride: int):
    import torch
    B, Cn, H, Wd = (int(v) for v in X.shape)
    _shape_check(Y, (B, Cn, (H - k) // stride + 1, (Wd - k) // stride + 1), "Y")
    f32 = torch.float32
    with torch.cuda.device(X.device):
        stream = torch.cuda.current_stream(X.device)
        _check(lib().dn_maxpool_forward(_dev_ptr(X, f32, "X"), _dev_ptr(Y, f32, "Y"), B, Cn, H, Wd, int(k),
                                        int(stride), C.c_void_p(stream.cuda_stream)), "dn_maxpool_forward")


def dn_maxpool_backward(X, dY, dX, k: int, stride: int):
    import torch
    B, Cn, H, Wd = (int(v) for v in X.shape)
    _shape_check(dY, (B, Cn, (H - k) // stride + 1, (Wd - k) // stride + 1), "dY")
    _shape_check(dX, X.shape, "dX")
    f32 = torch.float32
    with torch.cuda.device(X.device):
        stream = torch.cuda.current_stream(X.device)
        _check(lib().dn_maxpool_backward(_dev_ptr(X, f32, "X"), _dev_ptr(dY, f32, "dY"), _dev_ptr(dX, f32, "dX"),
                                         B, Cn, H, Wd, int(k), int(stride), C.c_void_p(stream.cuda_stream)),
               "dn_maxpool_backward")


def dn_sgd_step(param, grad, velocity, lr: float, momentum: float):
    """The update rule of Net.dn_update for a parameter tensor the caller owns."""
    import torch
    f32 = torch.float32
    _shape_check(grad, param.shape, "grad")
    if velocity is not None:
        _shape_check(velocity, param.shape, "velocity")
    with torch.cuda.device(param.device):
        stream = torch.cuda.current_stream(param.device)
        _check(lib().dn_sgd_step(_dev_ptr(param, f32, "param"), _dev_ptr(grad, f32, "grad"),
                                 None if velocity is None else _dev_ptr(velocity, f32, "velocity"),
                                 int(param.numel()), float(lr), float(momentum), C.c_void_p(stream.cuda_stream)),
               "dn_sgd_step")


class Net:
    """One network on the current device.  Owns the arena tensor (torch
    allocation) and the library handle; method names follow include/dn.h."""

    def __init__(self, widths: Sequence[int], acts: Sequence[int], loss: int, max_batch: int,
                 device: str = "cuda:0", _borrowed=None):
        import torch
        self._torch = torch
        self.widths = [int(w) for w in widths]
        self.L = len(self.widths) - 1
        self.max_batch = int(max_batch)
        self.device = torch.device(device)
        self._owned = _borrowed is None
        if _borrowed is not None:      # a handle that another object (Cnn) owns and destroys
            self._h = _borrowed
            return
        nbytes = dn_net_arena_bytes(self.widths, self.max_batch)
        if nbytes == 0:
            raise DnError(DN_ERR_SHAPE, "dn_net_arena_bytes")
        self.arena = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.stream = torch.cuda.current_stream(self.device)
        w_arr, w_p = _i32(self.widths)
        a_arr, a_p = _i32(acts)
        handle = C.c_void_p()
        with torch.cuda.device(self.device):
            st = lib().dn_net_create(w_p, len(w_arr), a_p, int(loss), self.max_batch,
                                     C.c_void_p(self.arena.data_ptr()), nbytes,
                                     C.c_void_p(self.stream.cuda_stream), C.byref(handle))
        _check(st, "dn_net_create")
        self._h = handle

    def close(self):
        if getattr(self, "_h", None):
            if self._owned:
                lib().dn_net_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- parameters ------------------------------------------------------------
    def dn_set_params(self, layer: int, W: Optional[np.ndarray], b: Optional[np.ndarray]):
        if not 1 <= layer <= self.L:
            raise DnError(DN_ERR_INVALID_ARG, "dn_set_params")
        Wc = None if W is None else np.ascontiguousarray(W, dtype=np.float32)
        bc = None if b is None else np.ascontiguousarray(b, dtype=np.float32)
        if Wc is not None and Wc.shape != (self.widths[layer], self.widths[layer - 1]):
            raise DnError(DN_ERR_SHAPE, "dn_set_params")
        if bc is not None and bc.shape != (self.widths[layer],):
            raise DnError(DN_ERR_SHAPE, "dn_set_params")
        _check(lib().dn_set_params(self._h, layer,
                                   None if Wc is None else Wc.ctypes.data_as(C.c_void_p),
                                   None if bc is None else bc.ctypes.data_as(C.c_void_p)), "dn_set_params")

    def _get(self, fn, name, layer) -> Tuple[np.ndarray, np.ndarray]:
        if not 1 <= layer <= self.L:          # the host buffers below are sized from the layer's widths
            raise DnError(DN_ERR_INVALID_ARG, name)
        W = np.empty((self.widths[layer], self.widths[layer - 1]), dtype=np.float32)
        b = np.empty(self.widths[layer], dtype=np.float32)
        _check(fn(self._h, layer, W.ctypes.data_as(C.c_void_p), b.ctypes.data_as(C.c_void_p)), name)
        return W, b

    def dn_get_params(self, layer: int):
        return self._get(lib().dn_get_params, "dn_get_params", layer)

    def dn_get_grads(self, layer: int):
        return self._get(lib().dn_get_grads, "dn_get_grads", layer)

    def set_all(self, W: Sequence[np.ndarray], b: Sequence[np.ndarray]):
        for l in range(1, self.L + 1):
            self.dn_set_params(l, W[l - 1], b[l - 1])

    def get_all(self) -> Tuple[List[np.ndarray], List[np.ndarray]]:
        pairs = [self.dn_get_params(l) for l in range(1, self.L + 1)]
        return [p[0] for p in pairs], [p[1] for p in pairs]

    def get_all_grads(self):
        pairs = [self.dn_get_grads(l) for l in range(1, self.L + 1)]
        return [p[0] for p in pairs], [p[1] for p in pairs]

    # -- the steps ---------------------------------------------------------------
    def dn_forward(self, X, out=None):
        t = self._torch
        batch = int(X.shape[0])
        _check(lib().dn_forward(self._h, _dev_ptr(X, t.float32, "X"), batch,
                                None if out is None else _dev_ptr(out, t.float32, "out")), "dn_forward")

    def dn_backward(self, labels, loss_out=None):
        t = self._torch
        _check(lib().dn_backward(self._h, _dev_ptr(labels, t.int32, "labels"), int(labels.shape[0]),
                                 None if loss_out is None else _dev_ptr(loss_out, t.float32, "loss")),
               "dn_backward")

    def dn_input_gradient(self, dX):
        t = self._torch
        _shape_check(dX, (int(dX.shape[0]), self.widths[0]), "dX")
        _check(lib().dn_input_gradient(self._h, int(dX.shape[0]), _dev_ptr(dX, t.float32, "dX")),
               "dn_input_gradient")

    def dn_update(self, lr: float, momentum: float):
        _check(lib().dn_update(self._h, float(lr), float(momentum)), "dn_update")

    def dn_train_epoch(self, X, labels, batch: int, lr: float, momentum: float,
                       n_samples: Optional[int] = None) -> float:
        t = self._torch
        n = int(X.shape[0]) if n_samples is None else int(n_samples)
        loss = C.c_float(0.0)
        _check(lib().dn_train_epoch(self._h, _dev_ptr(X, t.float32, "X"), _dev_ptr(labels, t.int32, "labels"),
                                    n, int(batch), float(lr), float(momentum), C.byref(loss)),
               "dn_train_epoch")
        return float(loss.value)

    def dn_train(self, X, labels, batch: int, lr: float, momentum: float, max_error: float,
                 max_epochs: int, n_samples: Optional[int] = None) -> Tuple[int, float]:
        """(epochs run, last epoch loss)."""
        t = self._torch
        n = int(X.shape[0]) if n_samples is None else int(n_samples)
        epochs, loss = C.c_int32(0), C.c_float(0.0)
        _check(lib().dn_train(self._h, _dev_ptr(X, t.float32, "X"), _dev_ptr(labels, t.int32, "labels"), n,
                              int(batch), float(lr), float(momentum), float(max_error), int(max_epochs),
                              C.byref(epochs), C.byref(loss)), "dn_train")
        return int(epochs.value), float(loss.value)

    def dn_evaluate(self, X, labels, batch: int, n_samples: Optional[int] = None) -> Tuple[float, int]:
        """(mean loss, number of samples whose largest output is at the label)."""
        t = self._torch
        n = int(X.shape[0]) if n_samples is None else int(n_samples)
        loss, correct = C.c_float(0.0), C.c_int64(0)
        _check(lib().dn_evaluate(self._h, _dev_ptr(X, t.float32, "X"), _dev_ptr(labels, t.int32, "labels"), n,
                                 int(batch), C.byref(loss), C.byref(correct)), "dn_evaluate")
        return float(loss.value), int(correct.value)

    # -- measurement ---------------------------------------------------------------
    def dn_last_epoch_ms(self) -> float:
        ms = C.c_float(0.0)
        _check(lib().dn_last_epoch_ms(self._h, C.byref(ms)), "dn_last_epoch_ms")
        return float(ms.value)

    def dn_last_schedule(self) -> int:
        v = C.c_int32(0)
        _check(lib().dn_last_schedule(self._h, C.byref(v)), "dn_last_schedule")
        return int(v.value)

    def dn_kernel_time(self, kernel_class: int) -> Tuple[float, int]:
        ms, n = C.c_float(0.0), C.c_int64(0)
        _check(lib().dn_kernel_time(self._h, kernel_class, C.byref(ms), C.byref(n)), "dn_kernel_time")
        return float(ms.value), int(n.value)

    def dn_kernel_flops(self, kernel_class: int) -> float:
        f = C.c_double(0.0)
        _check(lib().dn_kernel_flops(self._h, kernel_class, C.byref(f)), "dn_kernel_flops")
        return float(f.value)

    def dn_set_option(self, name: str, value: int):
        _check(lib().dn_set_option(self._h, name.encode(), int(value)), "dn_set_option")


class Cnn:
    """A convolutional classifier on the current device (dn_cnn_* of include/dn.h): blocks of
    (c_out, k, stride, pad, act, pool_k, pool_stride) in front of a fully connected net.  Owns
    the arena tensor and the library handle; `dense` is the fully connected part as a Net."""

    def __init__(self, c: int, h: int, w: int, blocks: Sequence[Sequence[int]], dense_widths: Sequence[int],
                 dense_acts: Sequence[int], loss: int, max_batch: int, device: str = "cuda:0"):
        import torch
        self._torch = torch
        self.shape = (int(c), int(h), int(w))
        self.blocks = [tuple(int(v) for v in b) for b in blocks]
        if any(len(b) != 7 for b in self.blocks):
            raise DnError(DN_ERR_INVALID_ARG, "dn_cnn_create")
        self.max_batch = int(max_batch)
        self.device = torch.device(device)
        b_arr, b_p = _i32([v for b in self.blocks for v in b])
        w_arr, w_p = _i32(dense_widths)
        a_arr, a_p = _i32(dense_acts)
        nbytes = int(lib().dn_cnn_arena_bytes(c, h, w, b_p, len(self.blocks), w_p, len(w_arr), self.max_batch))
        if nbytes == 0:
            raise DnError(DN_ERR_SHAPE, "dn_cnn_arena_bytes")
        self.arena = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.stream = torch.cuda.current_stream(self.device)
        handle = C.c_void_p()
        with torch.cuda.device(self.device):
            st = lib().dn_cnn_create(c, h, w, b_p, len(self.blocks), w_p, len(w_arr), a_p, int(loss), self.max_batch,
                                     C.c_void_p(self.arena.data_ptr()), nbytes, C.c_void_p(self.stream.cuda_stream),
                                     C.byref(handle))
        _check(st, "dn_cnn_create")
        self._h = handle
        self.flat = int(lib().dn_cnn_flat_size(self._h))
        self.dense = Net([self.flat] + [int(v) for v in dense_widths], dense_acts, loss, self.max_batch, device,
                         _borrowed=C.c_void_p(lib().dn_cnn_dense(self._h)))
        # filter shapes, block by block
        self.filter_shapes, cin = [], int(c)
        for b in self.blocks:
            self.filter_shapes.append((b[0], cin, b[1], b[1]))
            cin = b[0]

    def close(self):
        if getattr(self, "_h", None):
            self.dense.close()
            lib().dn_cnn_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def dn_cnn_set_filters(self, block: int, W: Optional[np.ndarray], bias: Optional[np.ndarray]):
        if not 0 <= block < len(self.blocks):
            raise DnError(DN_ERR_INVALID_ARG, "dn_cnn_set_filters")
        Wc = None if W is None else np.ascontiguousarray(W, dtype=np.float32)
        bc = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
        if Wc is not None and Wc.shape != self.filter_shapes[block]:
            raise DnError(DN_ERR_SHAPE, "dn_cnn_set_filters")
        if bc is not None and bc.shape != (self.filter_shapes[block][0],):
            raise DnError(DN_ERR_SHAPE, "dn_cnn_set_filters")
        _check(lib().dn_cnn_set_filters(self._h, block, None if Wc is None else Wc.ctypes.data_as(C.c_void_p),
                                        None if bc is None else bc.ctypes.data_as(C.c_void_p)), "dn_cnn_set_filters")

    def _get(self, fn, name, block):
        if not 0 <= block < len(self.blocks):      # the host buffers below are sized from the block's shape
            raise DnError(DN_ERR_INVALID_ARG, name)
        W = np.empty(self.filter_shapes[block], dtype=np.float32)
        b = np.empty(self.filter_shapes[block][0], dtype=np.float32)
        _check(fn(self._h, block, W.ctypes.data_as(C.c_void_p), b.ctypes.data_as(C.c_void_p)), name)
        return W, b

    def dn_cnn_get_filters(self, block: int):
        return self._get(lib().dn_cnn_get_filters, "dn_cnn_get_filters", block)

    def dn_cnn_get_filter_grads(self, block: int):
        return self._get(lib().dn_cnn_get_filter_grads, "dn_cnn_get_filter_grads", block)

    def dn_cnn_forward(self, X, out=None):
        t = self._torch
        _shape_check(X, (int(X.shape[0]),) + self.shape, "X")
        _check(lib().dn_cnn_forward(self._h, _dev_ptr(X, t.float32, "X"), int(X.shape[0]),
                                    None if out is None else _dev_ptr(out, t.float32, "out")), "dn_cnn_forward")

    def dn_cnn_train_epoch(self, X, labels, batch: int, lr: float, momentum: float,
                           n_samples: Optional[int] = None) -> float:
        t = self._torch
        _shape_check(X, (int(X.shape[0]),) + self.shape, "X")
        n = int(X.shape[0]) if n_samples is None else int(n_samples)
        if n > int(X.shape[0]) or n > int(labels.shape[0]):
            raise DnError(DN_ERR_SHAPE, "dn_cnn_train_epoch")
        loss = C.c_float(0.0)
        _check(lib().dn_cnn_train_epoch(self._h, _dev_ptr(X, t.float32, "X"), _dev_ptr(labels, t.int32, "labels"), n,
                                        int(batch), float(lr), float(momentum), C.byref(loss)), "dn_cnn_train_epoch")
        return float(loss.value)
