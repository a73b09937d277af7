"""Pins for the CPU checker: each test ties oracle/dn_oracle.c to something
other than itself -- a closed form, a library routine on a textbook special
case, central finite differences, or an invariant of the method.  The paper
prints no worked numerical example, so none of the expected values come from
it; its role here is the list of steps (feed forward, loss, back propagation,
update -- section "The Deep Netts Work-flow") and the rank-1 shape of the
per-sample weight gradient (section "How Deep Netts is parallelized with
TornadoVM?").
"""
import itertools

import numpy as np
import pytest
import torch
from scipy.special import softmax as sp_softmax

from oracle.dn_oracle import Oracle

LIN, SIG, TANH, RELU, SOFTMAX = 0, 1, 2, 3, 4
MSE, CE = 0, 1


def rand_net(rng, widths, scale=0.7):
    W = [rng.standard_normal((widths[l + 1], widths[l])) * scale for l in range(len(widths) - 1)]
    b = [rng.standard_normal(widths[l + 1]) * 0.3 for l in range(len(widths) - 1)]
    return W, b


def onehot(labels, n):
    y = np.zeros((len(labels), n))
    y[np.arange(len(labels)), labels] = 1.0
    return y


# ---------------------------------------------------------------- forward ----

def np_forward(W, b, acts, X):
    """Textbook forward pass with numpy/scipy library calls."""
    a = X
    out = []
    for Wl, bl, act in zip(W, b, acts):
        z = a @ Wl.T + bl
        if act == SIG:
            a = 1.0 / (1.0 + np.exp(-z))
        elif act == TANH:
            a = np.tanh(z)
        elif act == RELU:
            a = np.maximum(z, 0.0)
        elif act == SOFTMAX:
            a = sp_softmax(z, axis=1)
        else:
            a = z
        out.append(a)
    return out


@pytest.mark.parametrize("acts", [[SIG, SIG], [TANH, LIN], [RELU, SOFTMAX], [TANH, TANH, SOFTMAX]])
def test_forward_matches_library_matmul(acts):
    rng = np.random.default_rng(1)
    widths = [5, 7, 4] if len(acts) == 2 else [5, 7, 6, 4]
    W, b = rand_net(rng, widths)
    X = rng.standard_normal((9, widths[0]))
    o = Oracle("o64", widths, acts, CE if acts[-1] == SOFTMAX else MSE)
    o.set_params(W, b)
    got = o.forward(X)
    want = np_forward(W, b, acts, X)
    for g, w in zip(got, want):
        np.testing.assert_allclose(g, w, rtol=1e-13, atol=1e-14)


# ------------------------------------------------------------ closed forms ----

def test_single_linear_layer_mse_closed_form():
    # G = (W x + b - y) x^T, g = W x + b - y ; loss = 1/2 |W x + b - y|^2
    rng = np.random.default_rng(2)
    W, b = rand_net(rng, [6, 4])
    x = rng.standard_normal((1, 6))
    label = np.array([2], dtype=np.int32)
    o = Oracle("o64", [6, 4], [LIN], MSE)
    o.set_params(W, b)
    o.forward(x)
    loss = o.backward(label)
    r = W[0] @ x[0] + b[0] - onehot(label, 4)[0]
    G, g = o.get_grads()
    np.testing.assert_allclose(G[0], np.outer(r, x[0]), rtol=1e-14, atol=1e-15)
    np.testing.assert_allclose(g[0], r, rtol=1e-14, atol=1e-15)
    assert abs(loss - 0.5 * r @ r) < 1e-14


def test_softmax_regression_closed_form():
    # one softmax layer + cross-entropy: G = mean_s (p - y) x^T, loss = -log p_label
    rng = np.random.default_rng(3)
    W, b = rand_net(rng, [5, 3])
    X = rng.standard_normal((4, 5))
    labels = np.array([0, 2, 1, 2], dtype=np.int32)
    o = Oracle("o64", [5, 3], [SOFTMAX], CE)
    o.set_params(W, b)
    o.forward(X)
    loss = o.backward(labels)
    p = sp_softmax(X @ W[0].T + b[0], axis=1)
    d = p - onehot(labels, 3)
    G, g = o.get_grads()
    np.testing.assert_allclose(G[0], d.T @ X / 4, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(g[0], d.mean(axis=0), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(o.deltas()[0], d, rtol=1e-13, atol=1e-15)
    assert abs(loss - (-np.log(p[np.arange(4), labels])).mean()) < 1e-13
    assert np.abs(o.deltas()[0].sum(axis=1)).max() < 1e-15   # rows of p - y sum to zero


def test_linear_regression_converges_to_normal_equations():
    # Linear net + squared error + full-batch gradient descent is least squares
    # on one-hot targets: the fixed point is numpy.linalg.lstsq's solution.
    rng = np.random.default_rng(4)
    N, d, c = 40, 3, 2
    X = rng.standard_normal((N, d))
    labels = rng.integers(0, c, N).astype(np.int32)
    o = Oracle("o64", [d, c], [LIN], MSE)
    o.set_params([np.zeros((c, d))], [np.zeros(c)])
    for _ in range(3000):
        o.train_epoch(X, labels, batch=N, lr=0.1, momentum=0.0)
    Xa = np.hstack([X, np.ones((N, 1))])
    sol, *_ = np.linalg.lstsq(Xa, onehot(labels, c), rcond=None)
    W, b = o.get_params()
    np.testing.assert_allclose(W[0], sol[:d].T, atol=1e-9)
    np.testing.assert_allclose(b[0], sol[d], atol=1e-9)


# ------------------------------------------------------ finite differences ----

FD_CASES = [
    ([3, 4, 2], [SIG, SIG], MSE),
    ([3, 4, 2], [TANH, LIN], MSE),
    ([3, 4, 2], [RELU, SIG], MSE),
    ([3, 4, 2], [RELU, TANH], MSE),
    ([3, 4, 2], [LIN, RELU], MSE),
    ([3, 5, 4, 2], [TANH, SIG, SOFTMAX], CE),
    ([3, 5, 4, 2], [RELU, RELU, SOFTMAX], CE),
    ([3, 5, 4, 2], [SIG, TANH, LIN], MSE),
    ([4, 3], [SOFTMAX], CE),
]


@pytest.mark.parametrize("widths,acts,loss", FD_CASES)
def test_gradients_match_central_finite_differences(widths, acts, loss):
    rng = np.random.default_rng(10 + len(widths) + sum(acts))
    B = 3
    for attempt in range(20):   # redraw until every ReLU net input is away from its kink
        W, b = rand_net(rng, widths)
        X = rng.standard_normal((B, widths[0]))
        a = X
        ok = True
        for Wl, bl, act in zip(W, b, acts):
            z = a @ Wl.T + bl
            if act == RELU and np.abs(z).min() < 1e-2:
                ok = False
            a = np_forward([Wl], [bl], [act], a)[0]
        if ok:
            break
    assert ok
    labels = rng.integers(0, widths[-1], B).astype(np.int32)
    o = Oracle("o64", widths, acts, loss)
    o.set_params(W, b)
    o.forward(X)
    o.backward(labels)
    analytic = o.grads.copy()
    h = 1e-5
    fd = np.zeros_like(analytic)
    base = o.params.copy()
    for p in range(o.P):
        o.params[:] = base
        o.params[p] = base[p] + h
        up = o.loss_value(X, labels)
        o.params[p] = base[p] - h
        dn = o.loss_value(X, labels)
        fd[p] = (up - dn) / (2 * h)
    o.params[:] = base
    err = np.linalg.norm(fd - analytic) / max(np.linalg.norm(fd), 1e-30)
    assert err < 1e-7, err
    assert np.abs(fd - analytic).max() < 1e-7 * max(1.0, np.abs(fd).max())


# ------------------------------------------------ library autograd cross-check ----

def torch_net(W, b, acts, X, labels, loss):
    Wt = [torch.tensor(w, dtype=torch.float64, requires_grad=True) for w in W]
    bt = [torch.tensor(v, dtype=torch.float64, requires_grad=True) for v in b]

    def closure(Xb, yb):
        a = Xb if torch.is_tensor(Xb) else torch.tensor(Xb, dtype=torch.float64)
        for Wl, bl, act in zip(Wt, bt, acts):
            z = a @ Wl.T + bl
            if act == SIG:
                a = torch.sigmoid(z)
            elif act == TANH:
                a = torch.tanh(z)
            elif act == RELU:
                a = torch.relu(z)
            elif act == SOFTMAX:
                a = z           # folded into cross_entropy below
            else:
                a = z
        yb = torch.tensor(yb, dtype=torch.long)
        if loss == CE:
            return torch.nn.functional.cross_entropy(a, yb, reduction="mean")
        tgt = torch.nn.functional.one_hot(yb, a.shape[1]).to(torch.float64)
        return 0.5 * ((a - tgt) ** 2).sum(dim=1).mean()
    return Wt, bt, closure


@pytest.mark.parametrize("widths,acts,loss,mu", [
    ([4, 16, 3], [SIG, SIG], MSE, 0.0),
    ([6, 8, 5], [RELU, SOFTMAX], CE, 0.9),
    ([6, 8, 7, 5], [TANH, TANH, SOFTMAX], CE, 0.5),
])
def test_training_epochs_match_torch_sgd(widths, acts, loss, mu):
    # torch.optim.SGD keeps v <- mu v + g, p <- p - lr v; for a constant rate that is
    # the same trajectory as dW <- mu dW - lr g, W <- W + dW with dW = -lr v.
    rng = np.random.default_rng(20)
    N, B, lr = 23, 5, 0.05          # last batch is short (3 samples)
    W, b = rand_net(rng, widths, scale=0.5)
    X = rng.standard_normal((N, widths[0]))
    labels = rng.integers(0, widths[-1], N).astype(np.int32)
    o = Oracle("o64", widths, acts, loss)
    o.set_params(W, b)
    Wt, bt, closure = torch_net(W, b, acts, X, labels, loss)
    opt = torch.optim.SGD(Wt + bt, lr=lr, momentum=mu)
    for epoch in range(3):
        tot = 0.0
        for s0 in range(0, N, B):
            opt.zero_grad()
            l = closure(X[s0:s0 + B], labels[s0:s0 + B])
            l.backward()
            tot += float(l.detach()) * len(X[s0:s0 + B])
            opt.step()
        got, _ = o.train_epoch(X, labels, batch=B, lr=lr, momentum=mu)
        assert abs(got - tot / N) < 1e-12 * max(1.0, abs(tot / N))
    Wo, bo = o.get_params()
    for a_, t_ in zip(Wo + bo, Wt + bt):
        np.testing.assert_allclose(a_, t_.detach().numpy(), rtol=1e-10, atol=1e-12)


def test_one_step_gradients_match_torch_autograd():
    rng = np.random.default_rng(21)
    widths, acts = [5, 6, 4, 3], [SIG, RELU, SOFTMAX]
    W, b = rand_net(rng, widths)
    X = rng.standard_normal((7, 5))
    labels = rng.integers(0, 3, 7).astype(np.int32)
    o = Oracle("o64", widths, acts, CE)
    o.set_params(W, b)
    o.forward(X)
    loss = o.backward(labels)
    Wt, bt, closure = torch_net(W, b, acts, X, labels, CE)
    l = closure(X, labels)
    l.backward()
    assert abs(loss - float(l)) < 1e-13
    G, g = o.get_grads()
    for a_, t_ in zip(G + g, Wt + bt):
        np.testing.assert_allclose(a_, t_.grad.numpy(), rtol=1e-11, atol=1e-14)


@pytest.mark.parametrize("widths,acts,loss", [
    ([5, 6, 3], [TANH, SOFTMAX], CE),
    ([4, 3, 5, 2], [SIG, RELU, SIG], MSE),
    ([6, 4], [SOFTMAX], CE),
])
def test_input_gradient_matches_finite_differences_and_library_autograd(widths, acts, loss):
    """dE_s/dx_s per sample: central differences of the checker's own per-sample loss (forward
    and loss only, one sample at a time), and torch's autograd on the textbook net (the batch-mean
    loss's input gradient times B, since every sample's loss depends on its own input only)."""
    rng = np.random.default_rng(33)
    W, b = rand_net(rng, widths)
    B = 5
    X = rng.standard_normal((B, widths[0]))
    labels = rng.integers(0, widths[-1], B).astype(np.int32)
    o = Oracle("o64", widths, acts, loss)
    o.set_params(W, b)
    o.forward(X)
    o.backward(labels)
    dX = o.input_gradient()
    assert dX.shape == X.shape
    h = 1e-6
    for s in range(B):
        for i in range(widths[0]):
            xp, xm = X[s:s + 1].copy(), X[s:s + 1].copy()
            xp[0, i] += h
            xm[0, i] -= h
            fd = (o.loss_value(xp, labels[s:s + 1]) - o.loss_value(xm, labels[s:s + 1])) / (2 * h)
            assert abs(dX[s, i] - fd) < 1e-7 * max(1.0, abs(fd)), (s, i, dX[s, i], fd)
    Wt, bt, closure = torch_net(W, b, acts, X, labels, loss)
    Xt = torch.tensor(X, dtype=torch.float64, requires_grad=True)
    closure(Xt, labels).backward()
    np.testing.assert_allclose(dX, Xt.grad.numpy() * B, rtol=1e-10, atol=1e-13)


def test_input_gradient_of_one_linear_layer_is_delta_times_weights():
    """One linear layer with squared error: dE/dx = (W x + b - y) W, written out."""
    rng = np.random.default_rng(34)
    W, b = rand_net(rng, [4, 3])
    X = rng.standard_normal((2, 4))
    labels = np.array([2, 0], dtype=np.int32)
    o = Oracle("o64", [4, 3], [LIN], MSE)
    o.set_params(W, b)
    o.forward(X)
    o.backward(labels)
    expect = (X @ W[0].T + b[0] - onehot(labels, 3)) @ W[0]
    np.testing.assert_allclose(o.input_gradient(), expect, rtol=1e-13, atol=1e-15)


# ---------------------------------------------------------------- invariants ----

def test_zero_gradient_at_exact_fit():
    # identity weights on one-hot inputs reproduce the one-hot target exactly:
    # all gradients vanish and any number of steps leaves the parameters alone.
    n = 4
    labels = np.array([0, 3, 1, 2, 2], dtype=np.int32)
    X = onehot(labels, n)
    for mode in ("o64", "o32"):
        o = Oracle(mode, [n, n], [LIN], MSE)
        o.set_params([np.eye(n)], [np.zeros(n)])
        o.forward(X)
        assert o.backward(labels) == 0.0
        assert not o.grads.any()
        before = o.params.copy()
        for _ in range(3):
            loss, _ = o.train_epoch(X, labels, batch=2, lr=0.1, momentum=0.9)
            assert loss == 0.0
        assert np.array_equal(before, o.params)


@pytest.mark.parametrize("mu", [0.0, 0.9])
def test_softmax_ce_conserves_output_bias_sum_and_column_sums(mu):
    # delta_L = p - y sums to zero over the classes, so sum_k b_L[k] and every
    # column sum of W_L never move, with or without momentum.
    rng = np.random.default_rng(30)
    widths, acts = [6, 9, 4], [TANH, SOFTMAX]
    W, b = rand_net(rng, widths)
    b[1] = rng.standard_normal(4)
    X = rng.standard_normal((50, 6))
    labels = rng.integers(0, 4, 50).astype(np.int32)
    o = Oracle("o64", widths, acts, CE)
    o.set_params(W, b)
    o.train_epoch(X, labels, batch=8, lr=0.1, momentum=mu)
    o.train_epoch(X, labels, batch=8, lr=0.1, momentum=mu)
    W2, b2 = o.get_params()
    assert abs(b2[1].sum() - b[1].sum()) < 1e-13
    np.testing.assert_allclose(W2[1].sum(axis=0), W[1].sum(axis=0), atol=1e-13)
    assert np.abs(W2[0] - W[0]).max() > 1e-3          # ... while training did move the net


def test_batch_gradient_is_mean_of_per_sample_gradients_and_copies_collapse():
    rng = np.random.default_rng(31)
    widths, acts = [5, 6, 3], [SIG, SOFTMAX]
    W, b = rand_net(rng, widths)
    X = rng.standard_normal((6, 5))
    labels = rng.integers(0, 3, 6).astype(np.int32)
    o = Oracle("o64", widths, acts, CE)
    o.set_params(W, b)
    o.forward(X); lb = o.backward(labels)
    batch_grad = o.grads.copy()
    acc = np.zeros_like(batch_grad); ls = 0.0
    for s in range(6):
        o.forward(X[s:s + 1]); ls += o.backward(labels[s:s + 1]); acc += o.grads
    np.testing.assert_allclose(batch_grad, acc / 6, rtol=1e-12, atol=1e-15)
    assert abs(lb - ls / 6) < 1e-13
    # permuting the samples of a batch changes nothing beyond rounding
    perm = rng.permutation(6)
    o.forward(X[perm]); o.backward(labels[perm])
    np.testing.assert_allclose(o.grads, batch_grad, rtol=1e-12, atol=1e-15)
    # B copies of one sample are one sample
    o.forward(np.repeat(X[:1], 4, axis=0)); o.backward(np.repeat(labels[:1], 4))
    rep = o.grads.copy()
    o.forward(X[:1]); o.backward(labels[:1])
    np.testing.assert_allclose(rep, o.grads, rtol=1e-13, atol=1e-16)


def test_batch1_weight_gradient_is_rank1_outer_product():
    # per-sample gradient of a layer = delta (x) input: the two-index loop the paper offloads
    rng = np.random.default_rng(32)
    widths, acts = [5, 6, 3], [TANH, SOFTMAX]
    W, b = rand_net(rng, widths)
    x = rng.standard_normal((1, 5))
    o = Oracle("o64", widths, acts, CE)
    o.set_params(W, b)
    A = o.forward(x); o.backward(np.array([1], dtype=np.int32))
    D = o.deltas(); G, g = o.get_grads()
    np.testing.assert_allclose(G[1], np.outer(D[1][0], A[0][0]), rtol=1e-14)
    np.testing.assert_allclose(G[0], np.outer(D[0][0], x[0]), rtol=1e-14)
    np.testing.assert_allclose(g[0], D[0][0], rtol=1e-15)
    assert np.linalg.matrix_rank(G[0]) == 1


def test_momentum_zero_is_plain_sgd_bitwise():
    rng = np.random.default_rng(33)
    widths, acts = [6, 8, 4], [RELU, SOFTMAX]
    W, b = rand_net(rng, widths)
    X = rng.standard_normal((12, 6)).astype(np.float32)
    labels = rng.integers(0, 4, 12).astype(np.int32)
    o = Oracle("o32", widths, acts, CE)
    o.set_params(W, b)
    ref = Oracle("o32", widths, acts, CE)
    ref.set_params(W, b)
    o.train_epoch(X, labels, batch=4, lr=0.05, momentum=0.0)
    lr32 = np.float32(0.05)
    for s0 in range(0, 12, 4):                       # hand-rolled W <- W - lr G
        ref.forward(X[s0:s0 + 4]); ref.backward(labels[s0:s0 + 4])
        step = (-(lr32.astype(np.float64)) * ref.grads.astype(np.float64)).astype(np.float32)
        ref.params[:] = (ref.params.astype(np.float64) + step.astype(np.float64)).astype(np.float32)
    assert np.array_equal(o.params, ref.params)


def test_dead_relu_unit_has_zero_gradient_row_and_derivatives_at_zero():
    rng = np.random.default_rng(34)
    widths = [4, 5, 3]
    W, b = rand_net(rng, widths)
    W[0][2, :] = 0.0; b[0][2] = -1.0                 # hidden unit 2 never fires
    X = np.abs(rng.standard_normal((3, 4)))
    labels = np.array([0, 1, 2], dtype=np.int32)
    o = Oracle("o64", widths, [RELU, SOFTMAX], CE)
    o.set_params(W, b)
    A = o.forward(X); o.backward(labels)
    G, g = o.get_grads()
    assert not A[0][:, 2].any() and not G[0][2].any() and g[0][2] == 0.0
    assert not G[1][:, 2].any()                      # and it feeds nothing forward
    # f'(0): tanh 1, sigmoid 1/4, ReLU 0 (net input exactly zero)
    for act, want in ((TANH, 1.0), (SIG, 0.25), (RELU, 0.0)):
        o = Oracle("o64", [2, 1, 1], [act, LIN], MSE)
        o.set_params([np.zeros((1, 2)), np.ones((1, 1))], [np.zeros(1), np.zeros(1)])
        o.forward(np.ones((1, 2))); o.backward(np.array([0], dtype=np.int32))
        a1 = 0.5 if act == SIG else 0.0
        dL = a1 - 1.0                                # linear output a_2 = a_1, target 1
        np.testing.assert_allclose(o.deltas()[0][0, 0], dL * want, rtol=1e-15, atol=0)


def test_fp32_storage_mode_tracks_fp64_mode():
    # noise floor of the parity reference itself: one step and a short run
    rng = np.random.default_rng(35)
    widths, acts = [20, 30, 10], [TANH, SOFTMAX]
    W, b = rand_net(rng, widths, scale=0.3)
    W = [w.astype(np.float32) for w in W]; b = [v.astype(np.float32) for v in b]
    X = rng.standard_normal((64, 20)).astype(np.float32)
    labels = rng.integers(0, 10, 64).astype(np.int32)
    a, c = Oracle("o32", widths, acts, CE), Oracle("o64", widths, acts, CE)
    a.set_params(W, b); c.set_params(W, b)
    a.forward(X); c.forward(X)
    la, lc = a.backward(labels), c.backward(labels)
    assert abs(la - lc) < 1e-6
    assert np.linalg.norm(a.grads - c.grads) < 1e-6 * np.linalg.norm(c.grads)
    for _ in range(5):
        l32, _ = a.train_epoch(X, labels, batch=1, lr=0.01, momentum=0.0)
        l64, _ = c.train_epoch(X, labels, batch=1, lr=np.float32(0.01), momentum=0.0)
    assert abs(l32 - l64) < 1e-5
    assert np.linalg.norm(a.params - c.params) < 1e-5 * np.linalg.norm(c.params)


def test_fp32_accumulating_build_is_the_same_definition_up_to_fp32_rounding():
    """The o32a build (fp32 storage and fp32 sums) is only used to measure rounding drift; it must
    still be the same computation: gradients and a short training run agree with the reference
    build to fp32 rounding of the sums, on every activation / loss pair."""
    for acts, loss in [([RELU, SOFTMAX], CE), ([TANH, SIG], MSE), ([SIG, LIN], MSE)]:
        rng = np.random.default_rng(4)
        widths = [19, 33, 6]
        W = [rng.standard_normal((widths[l + 1], widths[l])).astype(np.float32) * 0.3 for l in range(2)]
        b = [rng.standard_normal(widths[l + 1]).astype(np.float32) * 0.1 for l in range(2)]
        X = rng.standard_normal((24, 19)).astype(np.float32)
        y = rng.integers(0, 6, 24).astype(np.int32)
        a, c = Oracle("o32", widths, acts, loss), Oracle("o32a", widths, acts, loss)
        a.set_params(W, b); c.set_params(W, b)
        a.forward(X); c.forward(X)
        la, lc = a.backward(y), c.backward(y)
        assert abs(la - lc) <= 1e-5 * abs(la)
        assert np.linalg.norm(a.grads.astype(np.float64) - c.grads) <= 1e-5 * np.linalg.norm(a.grads)
        ea, _ = a.train_epoch(X, y, 5, 0.05, 0.9)
        ec, _ = c.train_epoch(X, y, 5, 0.05, 0.9)
        assert abs(ea - ec) <= 1e-5 * abs(ea)
        assert np.linalg.norm(a.params.astype(np.float64) - c.params) <= 1e-5 * np.linalg.norm(a.params)


def test_kink_census_counts_small_relu_net_inputs():
    o = Oracle("o64", [1, 2, 2], [RELU, SOFTMAX], CE)
    o.set_params([np.array([[1.0], [1.0]]), np.zeros((2, 2))], [np.array([0.0, 5.0]), np.zeros(2)])
    X = np.array([[1e-7], [1.0], [-1e-8]])
    _, kinks = o.train_epoch(X, np.zeros(3, dtype=np.int32), batch=1, lr=0.0, momentum=0.0,
                             kink_eps=1e-5)
    assert kinks == 2       # hidden unit 0 on samples 0 and 2
    # the same census with the hits listed as (sample, layer, unit); a short list keeps the count
    for batch in (1, 2):
        _, kinks = o.train_epoch(X, np.zeros(3, dtype=np.int32), batch=batch, lr=0.0, momentum=0.0,
                                 kink_eps=1e-5, kink_cap=8)
        assert kinks == 2
        assert sorted(map(tuple, o.kink_list.tolist())) == [(0, 1, 0), (2, 1, 0)]
    # the census of a single forward pass: same hits, same activations as the plain forward pass
    plain = o.forward(X)
    with_census = o.forward(X, kink_eps=1e-5, kink_cap=8)
    assert o.kinks == 2 and sorted(map(tuple, o.kink_list.tolist())) == [(0, 1, 0), (2, 1, 0)]
    for a, c in zip(plain, with_census):
        assert np.array_equal(a, c)
    _, kinks = o.train_epoch(X, np.zeros(3, dtype=np.int32), batch=3, lr=0.0, momentum=0.0, kink_eps=1e-5, kink_cap=1)
    assert kinks == 2 and len(o.kink_list) == 1 and tuple(o.kink_list[0]) in [(0, 1, 0), (2, 1, 0)]


# ------------------------------------------------- evaluation and stopping rule ----

@pytest.mark.parametrize("acts,loss", [([TANH, SOFTMAX], CE), ([SIG, SIG], MSE), ([SOFTMAX], CE)])
def test_evaluate_matches_library_loss_and_argmax(acts, loss):
    """Mean loss from scipy's log-sum-exp / a direct squared-error formula, hits from numpy's
    argmax, both on a library forward pass; 157 samples span several of the checker's chunks."""
    from scipy.special import logsumexp
    rng = np.random.default_rng(21)
    widths = [6, 9, 5] if len(acts) == 2 else [6, 5]
    W, b = rand_net(rng, widths)
    X = rng.standard_normal((157, widths[0]))
    labels = rng.integers(0, widths[-1], size=157).astype(np.int32)
    o = Oracle("o64", widths, acts, loss)
    o.set_params(W, b)
    got_loss, got_hits = o.evaluate(X, labels)
    outs = np_forward(W, b, acts, X)
    if loss == CE:
        a_prev = outs[-2] if len(acts) > 1 else X
        z = a_prev @ W[-1].T + b[-1]
        want = float(np.mean(logsumexp(z, axis=1) - z[np.arange(157), labels]))
    else:
        want = float(np.mean(0.5 * np.sum((outs[-1] - onehot(labels, widths[-1])) ** 2, axis=1)))
    assert abs(got_loss - want) <= 1e-12 * max(1.0, abs(want))
    assert got_hits == int(np.sum(np.argmax(outs[-1], axis=1) == labels))


def test_evaluate_counts_ties_for_the_lowest_index_and_leaves_parameters_alone():
    o = Oracle("o64", [2, 3], [LIN], MSE)
    o.set_params([np.zeros((3, 2))], [np.array([0.5, 0.5, 0.1])])      # outputs 0.5, 0.5, 0.1 for any input
    before = o.params.copy()
    X = np.ones((3, 2))
    loss, hits = o.evaluate(X, np.array([0, 1, 2], dtype=np.int32))
    assert hits == 1                                                    # only label 0 is the (first) largest
    want = np.mean([0.5 * (0.25 + 0.25 + 0.01), 0.5 * (0.25 + 0.25 + 0.01), 0.5 * (0.25 + 0.25 + 0.81)])
    assert abs(loss - want) < 1e-15
    assert np.array_equal(before, o.params)


def test_training_until_max_error_stops_at_the_first_epoch_below_it():
    from paper_2001_04206_amd import synth
    w = synth.learnable()
    o = Oracle("o64", w.widths, w.acts, w.loss)
    o.set_params(w.W, w.b)
    _, _, losses = o.train(w.X, w.labels, w.batch, w.lr, w.momentum, max_error=-1.0, max_epochs=12)
    assert len(losses) == 12 and losses[-1] < 0.5 * losses[0]           # the labels carry signal: the loss falls
    k = next(i for i in range(1, 12) if losses[i] < losses[i - 1] and losses[i] < min(losses[:i]))
    threshold = 0.5 * (losses[k] + min(losses[:k]))                     # first crossed by epoch k+1
    o.set_params(w.W, w.b)
    epochs, last, again = o.train(w.X, w.labels, w.batch, w.lr, w.momentum, threshold, 12)
    assert epochs == k + 1 and last == losses[k] and again == losses[:k + 1]
    # the held-out part is predicted better than chance after training
    o.set_params(w.W, w.b)
    o.train(w.X[:360], w.labels[:360], w.batch, w.lr, w.momentum, -1.0, 12)
    _, hits = o.evaluate(w.X[360:], w.labels[360:])
    assert hits > 40 * 0.5


# ----------------------------------------------- what the paper itself prints ----

def _paper_numbers():
    import os
    kv = {}
    for line in open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_benchmark.txt")):
        if not line.startswith("#") and "=" in line:
            k, v = line.split("=", 1)
            kv[k.strip()] = v.strip()
    return kv


def test_paper_shape_workload_is_the_papers_network():
    """The synthetic stand-in for the paper's benchmark has the shape, activations and loss the paper
    states, and the per-sample weight gradients of its two layers have the sizes of the two offloaded
    methods' outputs (outputs x inputs: 10 x 100000 and 100000 x 340)."""
    from paper_2001_04206_amd import synth
    kv = _paper_numbers()
    w = synth.paper_shape(n_samples=2)
    assert w.widths == [int(kv["input_features"]), int(kv["fully_connected_neurons"]), int(kv["output_categories"])]
    assert w.acts == [TANH, SOFTMAX] and kv["fully_connected_activation"] == "tanh" and kv["output_activation"] == "softmax"
    assert w.loss == CE and kv["loss"] == "cross_entropy" and w.batch == 1
    o = Oracle("o32", w.widths, w.acts, w.loss)
    o.set_params(w.W, w.b)
    o.forward(w.X[:1]); o.backward(w.labels[:1])
    G, _ = o.get_grads()
    assert G[1].shape == (10, 100000) and G[0].shape == (100000, 340)
    # rank-1: the softmax layer's gradient is its delta times the hidden activations
    d = o.deltas()
    np.testing.assert_allclose(G[1], np.outer(d[1][0], o.forward(w.X[:1])[0][0]), rtol=1e-6, atol=1e-12)


def test_paper_timings_are_consistent_with_its_stated_speedups():
    kv = _paper_numbers()
    assert round(float(kv["softmax_backward_original_ms"]) / float(kv["softmax_backward_offloaded_ms"])) == int(kv["softmax_backward_speedup"])
    ratio = float(kv["fully_connected_backward_original_ms"]) / float(kv["fully_connected_backward_offloaded_ms"])
    assert abs(ratio - float(kv["fully_connected_backward_speedup"])) < 0.01
    assert abs(float(kv["large_dataset_bytes"]) / float(kv["small_dataset_bytes"]) - float(kv["large_dataset_factor"])) < 0.5
