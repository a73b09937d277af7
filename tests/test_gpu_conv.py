"""GPU parity of the convolutional and max-pooling layers against the CPU checker
(fp32 storage, fp64 accumulation), element by element, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import dn_conv_oracle as co
from paper_2001_04206_amd import dn
from parity_util import announce, assert_close

pytestmark = pytest.mark.gpu

LIN, SIG, TANH, RELU = 0, 1, 2, 3
TOL = 1e-4

CONV_CASES = [
    # B, Cin, H, W, Cout, KH, KW, stride, pad, act
    (2, 3, 7, 6, 4, 3, 2, 1, 0, TANH),
    (1, 1, 5, 5, 1, 3, 3, 1, 1, LIN),
    (3, 2, 9, 8, 5, 3, 3, 2, 1, SIG),            # stride 2, channel count not a multiple of the group of 4
    (2, 4, 6, 10, 3, 5, 5, 1, 2, RELU),
    (5, 6, 19, 23, 7, 7, 7, 1, 3, TANH),          # largest filter, several workgroups per image
    (4, 3, 33, 31, 9, 3, 3, 3, 0, TANH),          # stride 3, ragged
    (1, 16, 1, 1, 8, 1, 1, 1, 0, SIG),            # one-pixel images: a dense layer
    (16, 8, 28, 28, 16, 5, 5, 1, 0, RELU),        # the size of a small image classifier's second layer
    # wide enough for the matrix-core form (>= 32 output channels, >= 8 input channels, >= 16 columns, >= 12 for 3 x 3 filters):
    (2, 9, 21, 19, 35, 3, 3, 1, 1, TANH),         # forward on the matrix cores; ragged channels, rows and columns
    (2, 40, 18, 37, 33, 5, 3, 1, 2, SIG),         # forward and input gradient; non-square filter, two column tiles
    (1, 8, 20, 40, 32, 7, 7, 1, 3, TANH),         # largest filter: the biggest LDS stage
    (3, 64, 16, 16, 64, 3, 3, 1, 0, RELU),        # no padding: the input gradient pads by kh - 1
    # 3 x 3, stride 1, output width a multiple of 4 and enough workgroups: the filter gradient on the matrix cores
    (16, 20, 22, 20, 35, 3, 3, 1, 1, TANH),       # two channel groups of 10 (no fifth tile), ragged bands and channels
    (16, 33, 9, 36, 70, 3, 3, 1, 1, SIG),         # groups of 17 and 16, two channel blocks, two column blocks
    (96, 16, 18, 18, 64, 3, 3, 1, 0, RELU),       # no padding, one group of 16; 16 x 16 outputs: pixel blocks 16 columns wide
    (96, 16, 16, 44, 64, 3, 3, 1, 1, TANH),       # 16-column blocks, three per row, the last ragged
    (96, 16, 16, 16, 64, 3, 3, 1, 0, TANH),       # 14 x 14 outputs: rows are not whole 16-byte pieces, 16-column blocks
    (16, 20, 24, 32, 35, 3, 3, 1, 0, SIG),        # 22 x 30 outputs: the same with 32-column blocks
    (96, 16, 15, 15, 64, 3, 3, 1, 0, RELU),       # 13 x 13 outputs: close to the narrowest images the matrix-core kernels take
    (4, 40, 20, 24, 36, 5, 5, 1, 2, RELU),        # 5 x 5 forward product and input gradient with stages requested ahead, 64-channel tiles
    (4, 33, 17, 20, 32, 5, 5, 1, 2, TANH),        # the same with 32-channel tiles forward; a last stage of one channel
    (64, 12, 20, 20, 40, 5, 5, 1, 2, TANH),       # 5 x 5 filter gradient on the matrix cores: two groups of 6 channels, 32-column blocks
    (96, 8, 18, 18, 33, 5, 5, 1, 0, SIG),         # 5 x 5, 14 x 14 outputs: 16-column blocks, ragged pieces
    (64, 9, 20, 20, 40, 7, 7, 1, 3, SIG),         # 7 x 7 filter gradient on the matrix cores: three groups of 3 channels
    (128, 8, 16, 16, 256, 3, 3, 1, 1, RELU),      # 16 x 16 pixel tiles at full height (enough workgroups), 64-channel tiles
    (512, 8, 16, 16, 32, 3, 3, 1, 1, TANH),       # the same with 32-channel tiles
    (97, 68, 4, 16, 256, 3, 3, 1, 1, TANH),       # two images per chunk, the last chunk has one
    (64, 8, 17, 16, 32, 3, 3, 1, 1, SIG),         # the narrowest layer that takes this form: one half-filled channel tile, 17 rows in bands of 8
]


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("B,Cin,H,W,Cout,KH,KW,stride,pad,act", CONV_CASES)
def test_conv_forward_and_backward(B, Cin, H, W, Cout, KH, KW, stride, pad, act):
    announce("conv B=%d Cin=%d %dx%d Cout=%d k=%dx%d stride=%d pad=%d act=%d" % (B, Cin, H, W, Cout, KH, KW, stride, pad, act))
    rng = np.random.default_rng(21)
    X = rng.standard_normal((B, Cin, H, W)).astype(np.float32)
    Wt = (rng.standard_normal((Cout, Cin, KH, KW)) / np.sqrt(Cin * KH * KW)).astype(np.float32)
    b = (rng.standard_normal(Cout) * 0.1).astype(np.float32)
    Yr = co.conv_forward("o32", X, Wt, b, stride, pad, act)
    dA = rng.standard_normal(Yr.shape).astype(np.float32)
    delta_r, dX_r, dW_r, db_r = co.conv_backward("o32", X, Wt, Yr, dA, stride, pad, act)

    Xd, Wd, bd = dev(X), dev(Wt), dev(b)
    Y = torch.full(Yr.shape, float("nan"), dtype=torch.float32, device="cuda:0")
    dn.dn_conv_forward(Xd, Wd, bd, Y, stride, pad, act)
    assert_close(Y.cpu().numpy(), Yr, TOL, "Y")
    # backward from the checker's own output, so both sides differentiate at the same point
    Yd, dAd = dev(Yr), dev(dA)
    delta = torch.full(Yr.shape, float("nan"), dtype=torch.float32, device="cuda:0")
    dX = torch.full(X.shape, float("nan"), dtype=torch.float32, device="cuda:0")
    dW = torch.full(Wt.shape, float("nan"), dtype=torch.float32, device="cuda:0")
    db = torch.full((Cout,), float("nan"), dtype=torch.float32, device="cuda:0")
    dn.dn_conv_backward(Xd, Wd, Yd, dAd, delta, dX, dW, db, stride, pad, act)
    assert_close(delta.cpu().numpy(), delta_r, TOL, "delta")
    assert_close(dW.cpu().numpy(), dW_r, TOL, "dW")
    assert_close(db.cpu().numpy(), db_r, TOL, "dbias")
    assert_close(dX.cpu().numpy(), dX_r, TOL, "dX")
    # without an input gradient the other outputs are the same bits
    dW2 = torch.zeros_like(dW)
    db2 = torch.zeros_like(db)
    dn.dn_conv_backward(Xd, Wd, Yd, dAd, delta, None, dW2, db2, stride, pad, act)
    assert torch.equal(dW2, dW) and torch.equal(db2, db)


def test_conv_filter_gradient_with_unaligned_delta():
    """The matrix-core filter gradient reads delta 16 bytes at a time only if the caller's buffer
    allows it: a delta buffer that starts 4 bytes past an aligned address gives the same bits."""
    announce("conv filter gradient, delta buffer not 16-byte aligned")
    B, Cin, H, W, Cout, K = 16, 20, 22, 20, 35, 3
    rng = np.random.default_rng(5)
    X = rng.standard_normal((B, Cin, H, W)).astype(np.float32)
    Wt = (rng.standard_normal((Cout, Cin, K, K)) / np.sqrt(Cin * K * K)).astype(np.float32)
    Y = rng.standard_normal((B, Cout, H, W)).astype(np.float32)
    dA = rng.standard_normal(Y.shape).astype(np.float32)
    Xd, Wd, Yd, dAd = dev(X), dev(Wt), dev(Y), dev(dA)
    outs = []
    for shift in (0, 1):
        buf = torch.zeros(Y.size + 4, dtype=torch.float32, device="cuda:0")
        delta = buf[shift:shift + Y.size].view(Y.shape)
        assert delta.data_ptr() % 16 == 4 * shift
        dW = torch.zeros(Wt.shape, dtype=torch.float32, device="cuda:0")
        db = torch.zeros((Cout,), dtype=torch.float32, device="cuda:0")
        dn.dn_conv_backward(Xd, Wd, Yd, dAd, delta, None, dW, db, 1, 1, TANH)
        outs.append((delta.clone(), dW, db))
    for a, b in zip(outs[0], outs[1]):
        assert torch.equal(a, b)


def test_conv_and_pool_at_the_benchmark_shape():
    """The layer pair bench.py times (128 x 32 x 32 x 32 -> 64 channels, 3x3, pad 1, ReLU, then 2x2
    pooling), in the same launch configuration, every element against the checker."""
    announce("conv + pool at the benchmark shape")
    B, Cin, H, W, Cout, K = 128, 32, 32, 32, 64, 3
    rng = np.random.default_rng(0)
    X = rng.standard_normal((B, Cin, H, W)).astype(np.float32)
    Wt = (rng.standard_normal((Cout, Cin, K, K)) * np.sqrt(2.0 / (Cin * K * K))).astype(np.float32)
    b = (rng.standard_normal(Cout) * 0.1).astype(np.float32)
    dP = rng.standard_normal((B, Cout, H // 2, W // 2)).astype(np.float32)
    Yr = co.conv_forward("o32", X, Wt, b, 1, 1, RELU)
    Pr = co.maxpool_forward("o32", Yr, 2, 2)
    dYr = co.maxpool_backward("o32", Yr, dP, 2, 2)
    delta_r, dX_r, dW_r, db_r = co.conv_backward("o32", X, Wt, Yr, dYr, 1, 1, RELU)
    Xd, Wd = dev(X), dev(Wt)
    Y = torch.empty(Yr.shape, dtype=torch.float32, device="cuda:0")
    dn.dn_conv_forward(Xd, Wd, dev(b), Y, 1, 1, RELU)
    assert_close(Y.cpu().numpy(), Yr, TOL, "Y")
    # pooling and the backward pass from the checker's activations: a ReLU output within rounding
    # of zero would otherwise put the two sides on different branches
    Yd = dev(Yr)
    P, dY = torch.empty(Pr.shape, dtype=torch.float32, device="cuda:0"), torch.empty_like(Yd)
    dn.dn_maxpool_forward(Yd, P, 2, 2)
    assert np.array_equal(P.cpu().numpy(), Pr)
    dn.dn_maxpool_backward(Yd, dev(dP), dY, 2, 2)
    assert np.array_equal(dY.cpu().numpy(), dYr)
    delta, dX, dW, db = torch.empty_like(Yd), torch.empty_like(Xd), torch.empty_like(Wd), torch.empty(Cout, device="cuda:0")
    dn.dn_conv_backward(Xd, Wd, Yd, dY, delta, dX, dW, db, 1, 1, RELU)
    assert_close(delta.cpu().numpy(), delta_r, TOL, "delta")
    assert_close(dW.cpu().numpy(), dW_r, TOL, "dW")
    assert_close(db.cpu().numpy(), db_r, TOL, "dbias")
    assert_close(dX.cpu().numpy(), dX_r, TOL, "dX")


POOL_CASES = [((2, 3, 8, 8), 2, 2), ((1, 2, 7, 9), 3, 2), ((2, 1, 6, 6), 3, 1), ((1, 1, 5, 5), 5, 1),
              ((2, 2, 9, 7), 2, 3), ((3, 5, 33, 47), 3, 2), ((16, 16, 24, 24), 2, 2), ((2, 2, 4, 5), 1, 1)]


@pytest.mark.parametrize("shape,k,s", POOL_CASES)
def test_maxpool_forward_and_backward(shape, k, s):
    announce("maxpool shape=%s k=%d stride=%d" % (shape, k, s))
    rng = np.random.default_rng(22)
    # few distinct values: many windows hold equal maxima, so the tie rule is exercised
    X = rng.integers(-3, 4, size=shape).astype(np.float32)
    Yr = co.maxpool_forward("o32", X, k, s)
    dY = rng.standard_normal(Yr.shape).astype(np.float32)
    dXr = co.maxpool_backward("o32", X, dY, k, s)
    Xd = dev(X)
    Y = torch.full(Yr.shape, float("nan"), dtype=torch.float32, device="cuda:0")
    dn.dn_maxpool_forward(Xd, Y, k, s)
    assert np.array_equal(Y.cpu().numpy(), Yr)                    # a selection: exact
    dX = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda:0")
    dn.dn_maxpool_backward(Xd, dev(dY), dX, k, s)
    got = dX.cpu().numpy()
    assert np.array_equal(got != 0, dXr != 0)                     # the same positions receive gradient
    if s >= k:
        assert np.array_equal(got, dXr)                           # windows do not overlap: values are moved, not added
    else:
        np.testing.assert_allclose(got, dXr, rtol=1e-6, atol=1e-6)   # sums of up to ceil(k/s)^2 terms


def test_conv_backward_is_bitwise_reproducible():
    announce("conv determinism")
    rng = np.random.default_rng(23)
    X = dev(rng.standard_normal((8, 6, 20, 20)).astype(np.float32))
    Wt = dev(rng.standard_normal((10, 6, 3, 3)).astype(np.float32))
    Y = dev(rng.standard_normal((8, 10, 20, 20)).astype(np.float32))
    dA = dev(rng.standard_normal((8, 10, 20, 20)).astype(np.float32))
    outs = []
    for _ in range(2):
        delta, dX, dW, db = torch.empty_like(Y), torch.empty_like(X), torch.empty_like(Wt), torch.empty(10, device="cuda:0")
        dn.dn_conv_backward(X, Wt, Y, dA, delta, dX, dW, db, 1, 1, TANH)
        outs.append((dX.clone(), dW.clone(), db.clone()))
    for a, b in zip(*outs):
        assert torch.equal(a, b)
