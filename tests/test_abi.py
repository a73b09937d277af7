"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol include/dn.h declares, sizes arenas sanely and rejects bad
arguments with status codes before touching the device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2001_04206_amd import dn

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(dn.LIB_PATH):
        from paper_2001_04206_amd import build
        build.build()
    return dn.lib()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "dn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dn_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(lib):
    names = declared_functions()
    assert set(names) == set(dn.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_status_strings(lib):
    seen = {dn.status_string(s) for s in range(6)}
    assert len(seen) == 6 and dn.status_string(99) == "unknown status"


def test_arena_bytes(lib):
    assert dn.dn_net_arena_bytes([4, 16, 3], 1) > 3 * 4 * (4 * 16 + 16 + 16 * 3 + 3)
    small, big = dn.dn_net_arena_bytes([784, 128, 10], 1), dn.dn_net_arena_bytes([784, 128, 10], 128)
    assert big > small and small % 256 == 0 and big % 256 == 0
    # activations and deltas of every layer scale with the batch
    assert big - small >= 127 * 2 * 4 * 128
    assert dn.dn_net_arena_bytes([4], 1) == 0
    assert dn.dn_net_arena_bytes([4, 0, 3], 1) == 0
    assert dn.dn_net_arena_bytes([4, -1], 1) == 0
    assert dn.dn_net_arena_bytes([4, 3], 0) == 0
    assert lib.dn_net_arena_bytes(None, 3, 1) == 0
    assert dn.dn_net_arena_bytes([2 ** 31 - 1, 2 ** 31 - 1], 1) == 0      # absurd size is refused


def _create(lib, widths, acts, loss, max_batch=4, arena=0x10000, nbytes=1 << 40, out=True):
    w = np.asarray(widths, dtype=np.int32)
    a = np.asarray(acts, dtype=np.int32)
    h = C.c_void_p()
    st = lib.dn_net_create(w.ctypes.data_as(C.c_void_p), len(w), a.ctypes.data_as(C.c_void_p), loss,
                           max_batch, C.c_void_p(arena), nbytes, None, C.byref(h) if out else None)
    return st, h


def test_create_rejects_bad_arguments_before_touching_the_device(lib):
    S, T, R, SM = dn.DN_ACT_SIGMOID, dn.DN_ACT_TANH, dn.DN_ACT_RELU, dn.DN_ACT_SOFTMAX
    assert _create(lib, [4, 3], [S], dn.DN_LOSS_MSE, out=False)[0] == dn.DN_ERR_INVALID_ARG
    assert _create(lib, [4, 3], [S], dn.DN_LOSS_MSE, arena=0)[0] == dn.DN_ERR_INVALID_ARG
    assert _create(lib, [4, 3], [S], dn.DN_LOSS_MSE, arena=0x10010)[0] == dn.DN_ERR_INVALID_ARG   # misaligned
    assert _create(lib, [4, 3], [S], 7)[0] == dn.DN_ERR_INVALID_ARG
    assert _create(lib, [4, 3], [9], dn.DN_LOSS_MSE)[0] == dn.DN_ERR_INVALID_ARG
    assert _create(lib, [4], [], dn.DN_LOSS_MSE)[0] == dn.DN_ERR_SHAPE
    assert _create(lib, [4, 0, 3], [S, S], dn.DN_LOSS_MSE)[0] == dn.DN_ERR_SHAPE
    assert _create(lib, [4, 3], [S], dn.DN_LOSS_MSE, max_batch=0)[0] == dn.DN_ERR_SHAPE
    assert _create(lib, [4, 3], [S], dn.DN_LOSS_MSE, nbytes=16)[0] == dn.DN_ERR_SHAPE            # arena too small
    assert _create(lib, [4, 5, 3], [SM, S], dn.DN_LOSS_MSE)[0] == dn.DN_ERR_UNSUPPORTED          # softmax not last
    assert _create(lib, [4, 5, 3], [T, SM], dn.DN_LOSS_MSE)[0] == dn.DN_ERR_UNSUPPORTED          # softmax w/o CE
    assert _create(lib, [4, 5, 3], [T, R], dn.DN_LOSS_CROSS_ENTROPY)[0] == dn.DN_ERR_UNSUPPORTED  # CE w/o softmax
    st, h = _create(lib, [4, 3], [S], dn.DN_LOSS_MSE, out=True, arena=0)
    assert h.value is None


def test_null_handles_are_rejected(lib):
    f = C.c_float(0)
    assert lib.dn_net_destroy(None) == dn.DN_ERR_INVALID_ARG
    assert lib.dn_forward(None, None, 1, None) == dn.DN_ERR_INVALID_ARG
    assert lib.dn_backward(None, None, 1, None) == dn.DN_ERR_INVALID_ARG
    assert lib.dn_update(None, 0.1, 0.0) == dn.DN_ERR_INVALID_ARG
    assert lib.dn_train_epoch(None, None, None, 1, 1, 0.1, 0.0, C.byref(f)) == dn.DN_ERR_INVALID_ARG
    assert lib.dn_set_params(None, 1, None, None) == dn.DN_ERR_INVALID_ARG
    assert lib.dn_get_params(None, 1, None, None) == dn.DN_ERR_INVALID_ARG
    assert lib.dn_get_grads(None, 1, None, None) == dn.DN_ERR_INVALID_ARG
    assert lib.dn_last_epoch_ms(None, C.byref(f)) == dn.DN_ERR_INVALID_ARG
    assert lib.dn_last_schedule(None, None) == dn.DN_ERR_INVALID_ARG
    assert lib.dn_kernel_time(None, 0, C.byref(f), None) == dn.DN_ERR_INVALID_ARG
    assert lib.dn_set_option(None, b"time_kernels", 1) == dn.DN_ERR_INVALID_ARG


def test_binding_refuses_host_tensors(lib):
    import torch
    with pytest.raises(TypeError):
        dn._dev_ptr(torch.zeros(3), torch.float32, "X")


def test_layer_backward_host_argument_checks(lib):
    assert lib.dn_layer_backward_workspace_bytes(0, 5) == 0
    assert lib.dn_layer_backward_workspace_bytes(5, -1) == 0
    assert lib.dn_layer_backward_workspace_bytes(1 << 20, 1 << 20) == 0          # more than 2^31 weights
    need = lib.dn_layer_backward_workspace_bytes(10, 340)
    assert need >= 4 * (10 + 10 + 340 + 2 * 3400) and need % 256 == 0
    buf = (C.c_float * 3400)()
    vp = lambda a: C.cast(a, C.c_void_p)
    args = lambda ws, nbytes, co=10, ci=340, lr=0.1, d=buf: (
        vp(d) if d is not None else None, vp(buf), C.c_float(lr), co, ci, vp(buf), vp(buf), vp(buf), C.c_void_p(ws),
        nbytes, None, None, None, None)
    f = lib.dn_layer_backward_host
    assert f(*args(0x10000, need, d=None)) == dn.DN_ERR_INVALID_ARG               # NULL operand
    assert f(*args(0, need)) == dn.DN_ERR_INVALID_ARG                             # NULL workspace
    assert f(*args(0x10000, need, lr=float("nan"))) == dn.DN_ERR_INVALID_ARG
    assert f(*args(0x10000, need - 1)) == dn.DN_ERR_SHAPE                         # workspace too small
    assert f(*args(0x10000, need, co=0)) == dn.DN_ERR_SHAPE
    assert f(*args(0x10010, need)) == dn.DN_ERR_INVALID_ARG                       # misaligned workspace


def test_conv_and_pool_argument_checks(lib):
    """Bad arguments are refused before anything is enqueued (dummy non-NULL pointers)."""
    p = C.c_void_p(0x1000)
    conv = lambda **k: lib.dn_conv_forward(p, p, p, p, k.get("B", 2), k.get("Cin", 3), k.get("H", 8), k.get("W", 8),
                                           k.get("Cout", 4), k.get("KH", 3), k.get("KW", 3), k.get("stride", 1),
                                           k.get("pad", 1), k.get("act", 2), None)
    assert lib.dn_conv_forward(None, p, p, p, 2, 3, 8, 8, 4, 3, 3, 1, 1, 2, None) == dn.DN_ERR_INVALID_ARG
    assert conv(B=0) == dn.DN_ERR_INVALID_ARG
    assert conv(KH=8) == dn.DN_ERR_INVALID_ARG            # filter edge above 7
    assert conv(pad=3) == dn.DN_ERR_INVALID_ARG           # padding as wide as the filter
    assert conv(stride=0) == dn.DN_ERR_INVALID_ARG
    assert conv(H=1, pad=0) == dn.DN_ERR_INVALID_ARG      # empty output
    assert conv(act=4) == dn.DN_ERR_UNSUPPORTED           # softmax is not a convolutional activation
    assert conv(B=60000, Cin=64, H=64, W=64) == dn.DN_ERR_INVALID_ARG   # more than 2^31 - 1 elements
    need = lib.dn_conv_backward_workspace_bytes(2, 3, 8, 8, 4, 3, 3, 1, 1)
    assert need >= 4 * 4 * 3 * 3 * 3 and need % 4 == 0
    assert lib.dn_conv_backward_workspace_bytes(2, 3, 8, 8, 4, 9, 3, 1, 1) == 0
    back = lambda dW, **k: lib.dn_conv_backward(p, p, p, p, p, None, dW, p, k.get("ws", p), C.c_size_t(k.get("nbytes", need)),
                                                2, 3, 8, 8, 4, k.get("KH", 3), 3, 1, 1, 2, None)
    assert back(None) == dn.DN_ERR_INVALID_ARG
    assert back(p, KH=9) == dn.DN_ERR_INVALID_ARG
    assert back(p, ws=None) == dn.DN_ERR_INVALID_ARG
    assert back(p, nbytes=need - 4) == dn.DN_ERR_SHAPE        # workspace too small
    pool = lambda **k: lib.dn_maxpool_forward(p, p, k.get("B", 2), 3, k.get("H", 8), 8, k.get("k", 2),
                                              k.get("stride", 2), None)
    assert lib.dn_maxpool_forward(p, None, 2, 3, 8, 8, 2, 2, None) == dn.DN_ERR_INVALID_ARG
    assert pool(k=9) == dn.DN_ERR_INVALID_ARG             # window larger than the image
    assert pool(stride=0) == dn.DN_ERR_INVALID_ARG
    assert pool(B=40000) == dn.DN_ERR_INVALID_ARG         # more planes than the launch grid holds
    assert lib.dn_maxpool_backward(p, p, None, 2, 3, 8, 8, 2, 2, None) == dn.DN_ERR_INVALID_ARG
    # the stand-alone update rule and the input gradient
    assert lib.dn_sgd_step(None, p, None, 10, 0.1, 0.0, None) == dn.DN_ERR_INVALID_ARG
    assert lib.dn_sgd_step(p, None, None, 10, 0.1, 0.0, None) == dn.DN_ERR_INVALID_ARG
    assert lib.dn_sgd_step(p, p, None, 10, 0.1, 0.5, None) == dn.DN_ERR_INVALID_ARG    # momentum without velocity
    assert lib.dn_sgd_step(p, p, p, 10, -0.1, 0.0, None) == dn.DN_ERR_INVALID_ARG
    assert lib.dn_sgd_step(p, p, p, 10, 0.1, 1.0, None) == dn.DN_ERR_INVALID_ARG
    assert lib.dn_sgd_step(p, p, p, 10, float("nan"), 0.0, None) == dn.DN_ERR_INVALID_ARG
    assert lib.dn_sgd_step(p, p, p, 0, 0.1, 0.0, None) == dn.DN_ERR_SHAPE
    assert lib.dn_input_gradient(None, 4, p) == dn.DN_ERR_INVALID_ARG


def test_cnn_object_argument_checks(lib):
    """Sizes of a convolutional classifier are checked on the host: the arena query returns 0 for
    invalid ones, creation refuses bad arguments before anything is enqueued."""
    def blocks(*rows):
        arr = np.ascontiguousarray(rows, dtype=np.int32)
        return arr, arr.ctypes.data_as(C.c_void_p), len(rows)
    dense = np.array([16, 5], dtype=np.int32)
    dp = dense.ctypes.data_as(C.c_void_p)
    acts = np.array([2, 4], dtype=np.int32)
    ap = acts.ctypes.data_as(C.c_void_p)
    good, gp, gn = blocks((8, 3, 1, 1, 3, 2, 2), (4, 3, 1, 1, 2, 0, 0))
    need = lib.dn_cnn_arena_bytes(3, 12, 12, gp, gn, dp, 2, 16)
    # at least the filters three times over, the two convolution outputs twice, and the dense net
    dense_widths = np.array([4 * 6 * 6, 16, 5], dtype=np.int32)
    dense_need = lib.dn_net_arena_bytes(dense_widths.ctypes.data_as(C.c_void_p), 3, 16)
    assert need >= 3 * 4 * (8 * 3 * 9 + 4 * 8 * 9) + 2 * 4 * 16 * (8 * 12 * 12 + 4 * 6 * 6) + dense_need and need % 256 == 0
    assert lib.dn_cnn_arena_bytes(3, 12, 12, gp, gn, dp, 2, 32) > need                    # grows with the batch
    for bad in ((8, 9, 1, 1, 3, 2, 2),      # 9 x 9 filters
                (8, 3, 1, 3, 3, 2, 2),      # padding as wide as the filter
                (8, 3, 0, 1, 3, 2, 2),      # stride 0
                (8, 3, 1, 1, 4, 2, 2),      # softmax inside a block
                (8, 3, 1, 1, 3, 13, 2),     # pooling window larger than the image
                (0, 3, 1, 1, 3, 2, 2)):     # no output channels
        _, bp, bn = blocks(bad)
        assert lib.dn_cnn_arena_bytes(3, 12, 12, bp, bn, dp, 2, 16) == 0, bad
    assert lib.dn_cnn_arena_bytes(3, 12, 12, gp, 0, dp, 2, 16) == 0
    assert lib.dn_cnn_arena_bytes(3, 12, 12, gp, gn, dp, 0, 16) == 0
    assert lib.dn_cnn_arena_bytes(3, 12, 12, gp, gn, dp, 2, 0) == 0
    assert lib.dn_cnn_arena_bytes(3, 12, 12, None, gn, dp, 2, 16) == 0
    out = C.c_void_p()
    create = lambda arena, nbytes, o=C.byref(out): lib.dn_cnn_create(3, 12, 12, gp, gn, dp, 2, ap, 1, 16, C.c_void_p(arena),
                                                                     C.c_size_t(nbytes), None, o)
    assert create(0x10000, need, None) == dn.DN_ERR_INVALID_ARG
    assert create(0, need) == dn.DN_ERR_INVALID_ARG
    assert create(0x10010, need) == dn.DN_ERR_INVALID_ARG          # misaligned arena
    assert create(0x10000, need - 1) == dn.DN_ERR_SHAPE            # arena too small
    assert out.value is None
    assert lib.dn_cnn_destroy(None) == dn.DN_ERR_INVALID_ARG
    assert lib.dn_cnn_dense(None) is None and lib.dn_cnn_flat_size(None) == 0
    assert lib.dn_cnn_forward(None, None, 1, None) == dn.DN_ERR_INVALID_ARG
    assert lib.dn_cnn_train_epoch(None, None, None, 1, 1, 0.1, 0.0, None) == dn.DN_ERR_INVALID_ARG
    assert lib.dn_cnn_set_filters(None, 0, None, None) == dn.DN_ERR_INVALID_ARG
