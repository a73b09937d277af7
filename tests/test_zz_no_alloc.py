"""dn_conv_backward_static (the entry point that allocates nothing: its workspace is a fixed array in
the library's device image) against dn_conv_backward on the same inputs, through the C ABI: two
calls in a row on one device, the second with a smaller layer, so the second call finds the first
one's contents in the shared array.  Both run the same launches, so the results must be the same
bits; the larger case is also held against the CPU checker."""
import ctypes as C
import gc

import numpy as np
import pytest
import torch

from oracle import dn_conv_oracle as co
from paper_2001_04206_amd import dn
from parity_util import announce, assert_close

pytestmark = pytest.mark.gpu

TANH, RELU = 2, 3


def _case(B, Cin, H, W, Cout, K, pad, act, seed):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((B, Cin, H, W)).astype(np.float32)
    Wt = (rng.standard_normal((Cout, Cin, K, K)) / np.sqrt(Cin * K * K)).astype(np.float32)
    b = (rng.standard_normal(Cout) * 0.1).astype(np.float32)
    Y = co.conv_forward("o32", X, Wt, b, 1, pad, act)
    dA = rng.standard_normal(Y.shape).astype(np.float32)
    return X, Wt, Y, dA


def _raw_call(static, t, shape, stride, pad, act, workspace=None):
    """Straight through the C ABI (ctypes on the loaded library), no helper in between."""
    lib = dn.lib()
    B, Cin, H, W, Cout, K = shape
    p = lambda x: C.c_void_p(x.data_ptr())
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    if static:
        return lib.dn_conv_backward_static(p(t["X"]), p(t["W"]), p(t["Y"]), p(t["dA"]), p(t["delta"]), p(t["dX"]),
                                           p(t["dW"]), p(t["db"]), B, Cin, H, W, Cout, K, K, stride, pad, act, stream)
    return lib.dn_conv_backward(p(t["X"]), p(t["W"]), p(t["Y"]), p(t["dA"]), p(t["delta"]), p(t["dX"]), p(t["dW"]),
                                p(t["db"]), p(workspace), C.c_size_t(workspace.numel()), B, Cin, H, W, Cout, K, K,
                                stride, pad, act, stream)


def _buffers(X, Wt, Y, dA):
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    nan = lambda shape: torch.full(shape, float("nan"), dtype=torch.float32, device="cuda:0")
    return {"X": d(X), "W": d(Wt), "Y": d(Y), "dA": d(dA), "delta": nan(Y.shape), "dX": nan(X.shape),
            "dW": nan(Wt.shape), "db": nan((Wt.shape[0],))}


def test_static_scratch_matches_workspace_entry_point_twice():
    lib = dn.lib()
    limit = dn.dn_conv_backward_static_limit()
    assert limit == 32 << 20
    # first call: a layer on the matrix-core path with a multi-megabyte workspace; second: a smaller one
    cases = [((64, 16, 20, 20, 40, 3), 1, TANH, 31), ((6, 5, 11, 9, 7, 3), 1, RELU, 32)]
    prepared = []
    for shape, pad, act, seed in cases:
        B, Cin, H, W, Cout, K = shape
        X, Wt, Y, dA = _case(B, Cin, H, W, Cout, K, pad, act, seed)
        need = int(lib.dn_conv_backward_workspace_bytes(B, Cin, H, W, Cout, K, K, 1, pad))
        assert 0 < need <= limit
        ref = _buffers(X, Wt, Y, dA)
        ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
        announce("no-alloc: workspace entry point, shape %s (%d workspace bytes)" % (shape, need))
        assert _raw_call(False, ref, shape, 1, pad, act, ws) == dn.DN_OK
        prepared.append((shape, pad, act, (X, Wt, Y, dA), ref))
    torch.cuda.synchronize()
    # everything is allocated before the two static calls; they run back to back on one stream
    outs = [_buffers(*c[3]) for c in prepared]
    torch.cuda.synchronize()
    # Allocations between here and the second call's end are counted, not bytes in use: the collector may
    # free tensors of earlier tests at any moment, which lowers the bytes in use but never the count.
    gc.collect()
    allocs_before = torch.cuda.memory_stats()["allocation.all.allocated"]
    free_before = torch.cuda.mem_get_info()[0]
    for (shape, pad, act, _, _), got in zip(prepared, outs):
        announce("no-alloc: static entry point, shape %s" % (shape,))
        assert _raw_call(True, got, shape, 1, pad, act) == dn.DN_OK
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == allocs_before   # none through torch
    assert torch.cuda.mem_get_info()[0] >= free_before                                # none from the device either
    for (shape, pad, act, host, ref), got in zip(prepared, outs):
        for name in ("delta", "dX", "dW", "db"):
            assert torch.equal(got[name], ref[name]), "%s differs at shape %s" % (name, shape)
    # and the first case against the CPU checker, to the same tolerance as the other layer tests
    (shape, pad, act, (X, Wt, Y, dA), _), got = prepared[0], outs[0]
    delta_r, dX_r, dW_r, db_r = co.conv_backward("o32", X, Wt, Y, dA, 1, pad, act)
    assert_close(got["delta"].cpu().numpy(), delta_r, 1e-4, "delta")
    assert_close(got["dW"].cpu().numpy(), dW_r, 1e-4, "dW")
    assert_close(got["db"].cpu().numpy(), db_r, 1e-4, "dbias")
    assert_close(got["dX"].cpu().numpy(), dX_r, 1e-4, "dX")


def test_static_scratch_rejects_layers_beyond_its_limit():
    announce("no-alloc: layer larger than the fixed array is refused")
    lib = dn.lib()
    B, Cin, H, W, Cout, K = 64, 512, 16, 16, 512, 3
    need = int(lib.dn_conv_backward_workspace_bytes(B, Cin, H, W, Cout, K, K, 1, 1))
    assert need > dn.dn_conv_backward_static_limit()
    one = torch.zeros(4, dtype=torch.float32, device="cuda:0")     # never touched: the size check comes first
    p = C.c_void_p(one.data_ptr())
    st = lib.dn_conv_backward_static(p, p, p, p, p, None, p, p, B, Cin, H, W, Cout, K, K, 1, 1, TANH, None)
    assert st == dn.DN_ERR_SHAPE
    assert lib.dn_conv_backward_static(None, p, p, p, p, None, p, p, 1, 1, 4, 4, 1, 3, 3, 1, 1, TANH, None) == dn.DN_ERR_INVALID_ARG
