"""Pins of the CPU checker's convolutional and max-pooling layers against things
other than itself: a library correlation routine, central finite differences,
the dense layer they reduce to, brute-force Python loops, closed-form special
cases and invariants.  The paper prints no formulas or numbers for these layers
(it only lists them, "Deep Netts Deep Learning Engine", and names them as the
next to accelerate, "Summary"), so nothing here comes from it."""
import numpy as np
import pytest
from scipy.signal import correlate2d

from oracle import dn_conv_oracle as co
from oracle.dn_oracle import Oracle

LIN, SIG, TANH, RELU = 0, 1, 2, 3
ACT = {LIN: lambda z: z, SIG: lambda z: 1 / (1 + np.exp(-z)), TANH: np.tanh, RELU: lambda z: np.maximum(z, 0)}


def rand_case(seed, B, Cin, H, W, Cout, KH, KW):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((B, Cin, H, W)), rng.standard_normal((Cout, Cin, KH, KW)) * 0.3,
            rng.standard_normal(Cout) * 0.1)


CASES = [
    # B, Cin, H, W, Cout, KH, KW, stride, pad
    (2, 3, 7, 6, 4, 3, 2, 1, 0),
    (1, 1, 5, 5, 1, 3, 3, 1, 1),
    (3, 2, 9, 8, 5, 3, 3, 2, 1),
    (2, 4, 6, 10, 3, 5, 5, 1, 2),
    (2, 2, 8, 8, 2, 2, 2, 2, 0),
    (1, 3, 7, 7, 2, 1, 1, 3, 0),
]


@pytest.mark.parametrize("B,Cin,H,W,Cout,KH,KW,stride,pad", CASES)
@pytest.mark.parametrize("act", [LIN, TANH, SIG, RELU])
def test_conv_forward_is_a_library_correlation(B, Cin, H, W, Cout, KH, KW, stride, pad, act):
    X, Wt, b = rand_case(1, B, Cin, H, W, Cout, KH, KW)
    Y = co.conv_forward("o64", X, Wt, b, stride, pad, act)
    Xp = np.pad(X, ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    for s in range(B):
        for o in range(Cout):
            z = sum(correlate2d(Xp[s, c], Wt[o, c], mode="valid") for c in range(Cin)) + b[o]
            np.testing.assert_allclose(Y[s, o], ACT[act](z[::stride, ::stride]), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("B,Cin,H,W,Cout,KH,KW,stride,pad", CASES)
@pytest.mark.parametrize("act", [LIN, TANH, SIG])
def test_conv_backward_matches_finite_differences(B, Cin, H, W, Cout, KH, KW, stride, pad, act):
    """E = sum_b sum c . y_b for a fixed random c: dA = c for every sample; parameter
    gradients are the mean over the batch of dE_b/dparam, dX is dE/dX."""
    X, Wt, b = rand_case(2, B, Cin, H, W, Cout, KH, KW)
    Y = co.conv_forward("o64", X, Wt, b, stride, pad, act)
    c = np.random.default_rng(3).standard_normal(Y.shape)
    _, dX, dW, db = co.conv_backward("o64", X, Wt, Y, c, stride, pad, act)
    E = lambda X_, W_, b_: float((c * co.conv_forward("o64", X_, W_, b_, stride, pad, act)).sum())
    h = 1e-6
    rng = np.random.default_rng(4)

    def fd(arr, idx, which):
        p, m = arr.copy(), arr.copy()
        p[idx] += h
        m[idx] -= h
        args_p = {"X": (p, Wt, b), "W": (X, p, b), "b": (X, Wt, p)}[which]
        args_m = {"X": (m, Wt, b), "W": (X, m, b), "b": (X, Wt, m)}[which]
        return (E(*args_p) - E(*args_m)) / (2 * h)

    for _ in range(12):
        i = tuple(rng.integers(0, n) for n in Wt.shape)
        assert abs(fd(Wt, i, "W") / B - dW[i]) <= 1e-6 * max(1.0, abs(dW[i]))
        i = tuple(rng.integers(0, n) for n in X.shape)
        assert abs(fd(X, i, "X") - dX[i]) <= 1e-6 * max(1.0, abs(dX[i]))
    for o in range(Cout):
        assert abs(fd(b, (o,), "b") / B - db[o]) <= 1e-6 * max(1.0, abs(db[o]))


def test_conv_on_one_pixel_images_is_a_dense_layer():
    """1x1 images and a 1x1 filter: the layer is a fully connected one; forward, parameter
    gradients and input gradient must be those of the dense checker (linear regression on
    a squared error with targets folded into dA)."""
    rng = np.random.default_rng(5)
    B, Cin, Cout = 6, 5, 4
    X = rng.standard_normal((B, Cin, 1, 1))
    Wt = rng.standard_normal((Cout, Cin, 1, 1))
    b = rng.standard_normal(Cout)
    labels = rng.integers(0, Cout, B).astype(np.int32)
    Y = co.conv_forward("o64", X, Wt, b, 1, 0, TANH)
    dense = Oracle("o64", [Cin, Cout], [TANH], 0)     # squared error
    dense.set_params([Wt[:, :, 0, 0].copy()], [b.copy()])
    A = dense.forward(X[:, :, 0, 0].copy())
    np.testing.assert_allclose(Y[:, :, 0, 0], A[-1], rtol=1e-13, atol=1e-13)
    dense.backward(labels)
    G, g = dense.get_grads()
    onehot = np.eye(Cout)[labels]
    dA = (Y[:, :, 0, 0] - onehot)[:, :, None, None]    # dE/dy of the squared error
    delta, dX, dW, db = co.conv_backward("o64", X, Wt, Y, np.ascontiguousarray(dA), 1, 0, TANH)
    np.testing.assert_allclose(dW[:, :, 0, 0], G[0], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(db, g[0], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dX[:, :, 0, 0], delta[:, :, 0, 0] @ Wt[:, :, 0, 0], rtol=1e-12, atol=1e-13)


def test_conv_parameter_gradients_are_batch_means():
    X1, Wt, b = rand_case(6, 1, 2, 6, 6, 3, 3, 3)
    X = np.ascontiguousarray(np.repeat(X1, 4, axis=0))
    for act in (LIN, SIG):
        Y1 = co.conv_forward("o64", X1, Wt, b, 1, 1, act)
        Y = co.conv_forward("o64", X, Wt, b, 1, 1, act)
        dA1 = np.random.default_rng(7).standard_normal(Y1.shape)
        dA = np.ascontiguousarray(np.repeat(dA1, 4, axis=0))
        _, dX1, dW1, db1 = co.conv_backward("o64", X1, Wt, Y1, dA1, 1, 1, act)
        _, dX, dW, db = co.conv_backward("o64", X, Wt, Y, dA, 1, 1, act)
        np.testing.assert_allclose(dW, dW1, rtol=1e-13)
        np.testing.assert_allclose(db, db1, rtol=1e-13)
        np.testing.assert_allclose(dX[2], dX1[0], rtol=1e-13)


def test_conv_identity_filter_and_relu_derivative_at_zero():
    # a 3x3 filter that is 1 in the middle, padding 1: y = relu(x); dX = dA where x > 0, else 0
    X = np.array([[[[1.0, -2.0, 0.0], [3.0, 0.5, -1.0], [0.0, 2.0, -0.5]]]])
    Wt = np.zeros((1, 1, 3, 3)); Wt[0, 0, 1, 1] = 1.0
    Y = co.conv_forward("o64", X, Wt, np.zeros(1), 1, 1, RELU)
    np.testing.assert_array_equal(Y, np.maximum(X, 0))
    dA = np.full_like(Y, 2.0)
    delta, dX, dW, db = co.conv_backward("o64", X, Wt, Y, dA, 1, 1, RELU)
    np.testing.assert_array_equal(dX, np.where(X > 0, 2.0, 0.0))
    assert db[0] == 2.0 * (X > 0).sum()
    assert dW[0, 0, 1, 1] == 2.0 * X[X > 0].sum()


def test_o32_conv_is_the_rounded_o64():
    X, Wt, b = rand_case(8, 2, 3, 9, 9, 4, 3, 3)
    X32, W32, b32 = X.astype(np.float32), Wt.astype(np.float32), b.astype(np.float32)
    Y32 = co.conv_forward("o32", X32, W32, b32, 2, 1, TANH)
    Y64 = co.conv_forward("o64", X32.astype(np.float64), W32.astype(np.float64), b32.astype(np.float64), 2, 1, TANH)
    np.testing.assert_allclose(Y32, Y64, rtol=2e-7, atol=1e-7)
    dA = np.random.default_rng(9).standard_normal(Y32.shape).astype(np.float32)
    r32 = co.conv_backward("o32", X32, W32, Y32, dA, 2, 1, TANH)
    r64 = co.conv_backward("o64", X32.astype(np.float64), W32.astype(np.float64), Y32.astype(np.float64),
                           dA.astype(np.float64), 2, 1, TANH)
    for a, e in zip(r32, r64):
        np.testing.assert_allclose(a, e, rtol=1e-5, atol=1e-6)


# ----------------------------------------------------------------- max pooling ----

def brute_pool(X, k, s):
    B, C, H, W = X.shape
    Ho, Wo = (H - k) // s + 1, (W - k) // s + 1
    Y = np.empty((B, C, Ho, Wo))
    arg = np.empty((B, C, Ho, Wo, 2), dtype=int)
    for b in range(B):
        for c in range(C):
            for i in range(Ho):
                for j in range(Wo):
                    win = X[b, c, i * s:i * s + k, j * s:j * s + k]
                    f = int(np.argmax(win))            # first maximum in row-major order
                    Y[b, c, i, j] = win.flat[f]
                    arg[b, c, i, j] = (i * s + f // k, j * s + f % k)
    return Y, arg


@pytest.mark.parametrize("shape,k,s", [((2, 3, 8, 8), 2, 2), ((1, 2, 7, 9), 3, 2), ((2, 1, 6, 6), 3, 1),
                                       ((1, 1, 5, 5), 5, 1), ((2, 2, 9, 7), 2, 3)])
def test_maxpool_matches_brute_force(shape, k, s):
    rng = np.random.default_rng(10)
    X = rng.standard_normal(shape)
    X[0, 0, :2, :2] = 1.5          # ties inside the first window
    Y = co.maxpool_forward("o64", X, k, s)
    Yb, arg = brute_pool(X, k, s)
    np.testing.assert_array_equal(Y, Yb)
    dY = rng.standard_normal(Y.shape)
    dX = co.maxpool_backward("o64", X, dY, k, s)
    ref = np.zeros_like(X)
    for idx in np.ndindex(*Y.shape):
        r, c = arg[idx]
        ref[idx[0], idx[1], r, c] += dY[idx]
    np.testing.assert_allclose(dX, ref, rtol=1e-14, atol=1e-14)
    assert abs(dX.sum() - dY.sum()) < 1e-10        # every output gradient lands exactly once


def test_maxpool_non_overlapping_is_a_reshape_max():
    X = np.random.default_rng(11).standard_normal((3, 2, 8, 6))
    Y = co.maxpool_forward("o64", X, 2, 2)
    np.testing.assert_array_equal(Y, X.reshape(3, 2, 4, 2, 3, 2).max(axis=(3, 5)))


def test_maxpool_window_of_one_is_the_identity():
    X = np.random.default_rng(12).standard_normal((2, 2, 4, 5))
    np.testing.assert_array_equal(co.maxpool_forward("o64", X, 1, 1), X)
    dY = np.random.default_rng(13).standard_normal(X.shape)
    np.testing.assert_array_equal(co.maxpool_backward("o64", X, dY, 1, 1), dY)


def test_maxpool_tie_goes_to_the_first_maximum():
    X = np.zeros((1, 1, 2, 2))
    dX = co.maxpool_backward("o64", X, np.array([[[[3.0]]]]), 2, 1)
    np.testing.assert_array_equal(dX, np.array([[[[3.0, 0.0], [0.0, 0.0]]]]))
    X[0, 0, 1, 0] = X[0, 0, 1, 1] = 2.0
    dX = co.maxpool_backward("o64", X, np.array([[[[3.0]]]]), 2, 1)
    np.testing.assert_array_equal(dX, np.array([[[[0.0, 0.0], [3.0, 0.0]]]]))
