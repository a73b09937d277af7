"""GPU parity for the pieces that let convolutional and pooling layers train in front of a fully
connected net: the net's per-sample input gradient (dn_input_gradient), the stand-alone update
rule (dn_sgd_step), and one whole training step of a small convolutional classifier composed
from the C-ABI calls, each against the CPU checker composed the same way."""
import ctypes as C

import numpy as np
import pytest

from oracle import dn_conv_oracle as co
from oracle.dn_oracle import Oracle
from paper_2001_04206_amd import synth
from parity_util import announce, assert_close

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

LIN, SIG, TANH, RELU, SOFTMAX = 0, 1, 2, 3, 4
MSE, CE = 0, 1
TOL = 1e-4


@pytest.fixture(scope="module")
def dn():
    from paper_2001_04206_amd import dn as mod
    assert torch.cuda.is_available(), "these tests need the GPU"
    mod.lib()      # raises if the HIP library has not been built: no fallback
    return mod


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


INPUT_GRADIENT_CASES = [
    # widths, activations, loss, batch
    ([7, 5, 3], [TANH, SOFTMAX], CE, 3),                 # tiny and ragged
    ([20, 10], [SOFTMAX], CE, 9),                         # one layer of at most 16 outputs: the narrow kernels
    ([300, 12, 4], [RELU, SIG], MSE, 130),   # narrow first layer, several row tiles
    ([150, 200, 10], [TANH, SOFTMAX], CE, 70),            # the contraction kernels, ragged tiles
    ([1024, 2048, 10], [RELU, SOFTMAX], CE, 256),         # full tiles, long k
    ([4096, 300, 10], [SIG, SOFTMAX], CE, 8),             # few output tiles and a long k: the k-split form
]


@pytest.mark.parametrize("widths,acts,loss,B", INPUT_GRADIENT_CASES)
def test_input_gradient(dn, widths, acts, loss, B):
    announce("input gradient widths=%s B=%d" % (widths, B))
    w = synth.make("dx", widths, acts, loss, n_samples=B, features="normal", init="xavier_uniform", batch=B,
                   lr=0.05, momentum=0.0, seed=11)
    net = dn.Net(w.widths, w.acts, w.loss, B)
    net.set_all(w.W, w.b)
    o = Oracle("o32", w.widths, w.acts, w.loss)
    o.set_params(w.W, w.b)
    X, y = dev(w.X), dev(w.labels)
    net.dn_forward(X)
    net.dn_backward(y)
    dX = torch.full((B, widths[0]), float("nan"), dtype=torch.float32, device="cuda:0")
    net.dn_input_gradient(dX)
    o.forward(w.X)
    o.backward(w.labels)
    assert_close(dX.cpu().numpy(), o.input_gradient(), TOL, "dX")
    # the call is read-only on the net: gradients and a second call are unchanged
    dX2 = torch.zeros_like(dX)
    net.dn_input_gradient(dX2)
    assert torch.equal(dX, dX2)
    G, g = o.get_grads()
    for l in range(1, len(widths)):
        Gd, gd = net.dn_get_grads(l)
        assert_close(Gd, G[l - 1], TOL, "G_%d" % l)
    net.close()


def test_input_gradient_argument_errors(dn):
    announce("input gradient: argument errors")
    w = synth.make("edge", [8, 5, 3], [TANH, SOFTMAX], CE, n_samples=8, features="normal",
                   init="xavier_uniform", batch=4, lr=0.05, momentum=0.0, seed=1)
    net = dn.Net(w.widths, w.acts, w.loss, 4)
    net.set_all(w.W, w.b)
    X, y = dev(w.X), dev(w.labels)
    dX = torch.zeros((4, 8), dtype=torch.float32, device="cuda:0")

    def status(fn, *a):
        with pytest.raises(dn.DnError) as e:
            fn(*a)
        return e.value.status
    assert status(net.dn_input_gradient, dX) == dn.DN_ERR_INVALID_ARG          # before any backward
    net.dn_forward(X[:4].contiguous())
    assert status(net.dn_input_gradient, dX) == dn.DN_ERR_INVALID_ARG          # forward alone is not enough
    net.dn_backward(y[:4].contiguous())
    assert status(net.dn_input_gradient, dX[:3].contiguous()) == dn.DN_ERR_SHAPE   # another batch size
    net.dn_input_gradient(dX)
    net.dn_update(0.1, 0.0)
    assert status(net.dn_input_gradient, dX) == dn.DN_ERR_INVALID_ARG          # W_1 has moved on
    net.dn_forward(X[:4].contiguous())
    net.dn_backward(y[:4].contiguous())
    net.set_all(w.W, w.b)
    assert status(net.dn_input_gradient, dX) == dn.DN_ERR_INVALID_ARG          # W_1 was replaced
    net.close()


@pytest.mark.parametrize("n,mu", [(1, 0.0), (1000, 0.0), (70001, 0.9)])
def test_sgd_step(dn, n, mu):
    announce("sgd step n=%d momentum=%g" % (n, mu))
    rng = np.random.default_rng(3)
    p = rng.standard_normal(n).astype(np.float32)
    o = Oracle("o32", [1, 1], [LIN], MSE)    # only its update rule is used, on arrays of our own
    P, V = dev(p), torch.zeros(n, dtype=torch.float32, device="cuda:0")
    p_ref, v_ref = p.copy(), np.zeros(n, dtype=np.float32)
    for step in range(3):
        g = rng.standard_normal(n).astype(np.float32)
        dn.dn_sgd_step(P, dev(g), V if mu > 0 else None, 0.05, mu)
        o._update(C.c_size_t(n), o._rp(p_ref), o._rp(v_ref), o._rp(g), o._real(0.05), o._real(mu))
    assert_close(P.cpu().numpy(), p_ref, 1e-6, "parameters")
    if mu > 0:
        assert_close(V.cpu().numpy(), v_ref, 1e-6, "velocity")
    with pytest.raises(dn.DnError) as e:
        dn.dn_sgd_step(P, dev(np.zeros(n, np.float32)), None, 0.05, 0.5)       # momentum without a velocity buffer
    assert e.value.status == dn.DN_ERR_INVALID_ARG


def run_classifier(dn, B, C0, H0, W0, chans, dense, steps, seed, lr=0.05):
    """conv 3x3 (ReLU) + 2x2 pooling blocks, then a dense net (tanh hidden layers, softmax,
    cross-entropy); `steps` plain gradient-descent steps on one batch.  Every gradient and every
    updated parameter is compared with the checker's convolution, pooling and dense-net functions
    chained in the same order."""
    K, pad = 3, 1
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((B, C0, H0, W0)).astype(np.float32)
    labels = rng.integers(0, dense[-1], B).astype(np.int32)
    f32 = dict(dtype=torch.float32, device="cuda:0")
    blocks, cin, h, w = [], C0, H0, W0
    for cout in chans:
        blk = {"W_ref": (rng.standard_normal((cout, cin, K, K)) * np.sqrt(2.0 / (cin * K * K))).astype(np.float32),
               "b_ref": (rng.standard_normal(cout) * 0.1).astype(np.float32)}
        blk["W"], blk["b"] = dev(blk["W_ref"]), dev(blk["b_ref"])
        blk["Y"] = torch.empty((B, cout, h, w), **f32)
        blk["P"] = torch.empty((B, cout, h // 2, w // 2), **f32)
        blk["dP"], blk["dY"], blk["delta"] = torch.empty_like(blk["P"]), torch.empty_like(blk["Y"]), torch.empty_like(blk["Y"])
        blk["dW"], blk["db"] = torch.empty_like(blk["W"]), torch.empty_like(blk["b"])
        blocks.append(blk)
        cin, h, w = cout, h // 2, w // 2
    flat = cin * h * w
    widths = [flat] + list(dense)
    acts = [TANH] * (len(dense) - 1) + [SOFTMAX]
    Wd = [(rng.standard_normal((widths[l + 1], widths[l])) / np.sqrt(widths[l])).astype(np.float32) for l in range(len(dense))]
    bd = [(rng.standard_normal(widths[l + 1]) * 0.1).astype(np.float32) for l in range(len(dense))]
    net = dn.Net(widths, acts, CE, B)
    net.set_all(Wd, bd)
    o = Oracle("o32", widths, acts, CE)
    o.set_params(Wd, bd)
    Xd, yd = dev(X), dev(labels)
    dX0 = torch.empty_like(Xd)
    loss = torch.zeros(1, **f32)
    for step in range(steps):
        # device: forward through all layers, backward in reverse, then the updates
        a = Xd
        for blk in blocks:
            dn.dn_conv_forward(a, blk["W"], blk["b"], blk["Y"], 1, pad, RELU)
            dn.dn_maxpool_forward(blk["Y"], blk["P"], 2, 2)
            a = blk["P"]
        net.dn_forward(a.view(B, flat))
        net.dn_backward(yd, loss)
        net.dn_input_gradient(blocks[-1]["dP"].view(B, flat))
        for i in range(len(blocks) - 1, -1, -1):
            blk = blocks[i]
            dn.dn_maxpool_backward(blk["Y"], blk["dP"], blk["dY"], 2, 2)
            dn.dn_conv_backward(Xd if i == 0 else blocks[i - 1]["P"], blk["W"], blk["Y"], blk["dY"], blk["delta"],
                                dX0 if i == 0 else blocks[i - 1]["dP"], blk["dW"], blk["db"], 1, pad, RELU)
        net.dn_update(lr, 0.0)
        for blk in blocks:
            dn.dn_sgd_step(blk["W"], blk["dW"], None, lr, 0.0)
            dn.dn_sgd_step(blk["b"], blk["db"], None, lr, 0.0)
        # checker
        a_ref, kept = X, []
        for blk in blocks:
            Yr = co.conv_forward("o32", a_ref, blk["W_ref"], blk["b_ref"], 1, pad, RELU)
            kept.append((a_ref, Yr))
            a_ref = co.maxpool_forward("o32", Yr, 2, 2)
        o.forward(a_ref.reshape(B, flat))
        loss_r = o.backward(labels)
        d_ref = o.input_gradient().reshape(a_ref.shape)
        note = " step %d" % step
        assert abs(float(loss.cpu()[0]) - loss_r) <= TOL * max(1.0, abs(loss_r)), (float(loss.cpu()[0]), loss_r)
        assert_close(blocks[-1]["P"].cpu().numpy(), a_ref, TOL, "pooled" + note)
        for i in range(len(blocks) - 1, -1, -1):
            blk, (in_ref, Yr) = blocks[i], kept[i]
            assert_close(blk["dP"].cpu().numpy(), d_ref, TOL, "dP block %d%s" % (i, note))
            dYr = co.maxpool_backward("o32", Yr, d_ref, 2, 2)
            _, d_ref, dWr, dbr = co.conv_backward("o32", in_ref, blk["W_ref"], Yr, dYr, 1, pad, RELU)
            assert_close(blk["dW"].cpu().numpy(), dWr, TOL, "dW block %d%s" % (i, note))
            assert_close(blk["db"].cpu().numpy(), dbr, TOL, "db block %d%s" % (i, note))
            blk["W_ref"] = (blk["W_ref"] - np.float32(lr) * dWr).astype(np.float32)
            blk["b_ref"] = (blk["b_ref"] - np.float32(lr) * dbr).astype(np.float32)
            assert_close(blk["W"].cpu().numpy(), blk["W_ref"], TOL, "W block %d%s" % (i, note))
        assert_close(dX0.cpu().numpy(), d_ref, TOL, "dX" + note)
        o.update(lr, 0.0)
        Wr, br = o.get_params()
        for l in range(1, len(widths)):
            Wg, bg = net.dn_get_params(l)
            assert_close(Wg, Wr[l - 1], TOL, "W_%d%s" % (l, note))
            assert_close(bg, br[l - 1], TOL, "b_%d%s" % (l, note))
    net.close()


def test_convolutional_classifier_training_steps(dn):
    announce("convolutional classifier: two training steps")
    run_classifier(dn, 16, 3, 12, 12, (8,), (24, 5), steps=2, seed=17)


def test_two_block_classifier_training_steps(dn):
    announce("convolutional classifier with two blocks: two training steps")
    run_classifier(dn, 6, 2, 16, 20, (5, 9), (12, 10, 4), steps=2, seed=18)


def test_classifier_at_the_benchmark_shape(dn):
    """The classifier bench.py times (128 x 3 x 32 x 32, blocks of 32 and 64 channels, dense
    4096-512-10), one step in the same launch configuration."""
    announce("convolutional classifier at the benchmark shape")
    run_classifier(dn, 128, 3, 32, 32, (32, 64), (512, 10), steps=1, seed=19, lr=0.01)


def reference_cnn_epoch(shape, blocks, filters, biases, o, X, labels, batch, lr, mu, vel):
    """One epoch of the classifier on the CPU checker's functions, in the order of the chain
    rule: per batch forward through every block and the dense net, backward, then the update
    v <- mu v - lr g, p <- p + v of every parameter.  filters / biases / vel are updated in
    place; returns the epoch's mean loss."""
    n, acc = X.shape[0], 0.0
    for s0 in range(0, n, batch):
        xb, yb = X[s0:s0 + batch], labels[s0:s0 + batch]
        B = xb.shape[0]
        a, kept = xb, []
        for i, (cout, k, stride, pad, act, pk, ps) in enumerate(blocks):
            Y = co.conv_forward("o32", a, filters[i], biases[i], stride, pad, act)
            out = co.maxpool_forward("o32", Y, pk, ps) if pk > 0 else Y
            kept.append((a, Y))
            a = out
        o.forward(a.reshape(B, -1))
        acc += o.backward(yb) * B
        d = o.input_gradient().reshape(a.shape)
        grads = [None] * len(blocks)
        for i in range(len(blocks) - 1, -1, -1):
            cout, k, stride, pad, act, pk, ps = blocks[i]
            a_in, Y = kept[i]
            dA = co.maxpool_backward("o32", Y, d, pk, ps) if pk > 0 else d
            _, d, dW, db = co.conv_backward("o32", a_in, filters[i], Y, dA, stride, pad, act)
            grads[i] = (dW, db)
        o.update(lr, mu)
        for i, (dW, db) in enumerate(grads):
            for p, g, v in ((filters[i], dW, vel[i][0]), (biases[i], db, vel[i][1])):
                v[...] = (np.float32(mu) * v - np.float32(lr) * g).astype(np.float32)
                p[...] = (p + v).astype(np.float32)
    return acc / n


CNN_OBJECT_CASES = [
    # (c, h, w), blocks (c_out, k, stride, pad, act, pool_k, pool_stride), dense widths, n, batch, momentum
    ((3, 12, 12), [(8, 3, 1, 1, RELU, 2, 2)], (24, 5), 40, 16, 0.0),                       # ragged last batch
    ((2, 16, 20), [(5, 3, 1, 1, RELU, 2, 2), (9, 3, 1, 1, TANH, 0, 0)], (12, 4), 18, 6, 0.9),   # a block without pooling, momentum
    ((1, 28, 28), [(6, 5, 1, 0, RELU, 2, 2), (16, 5, 1, 0, RELU, 2, 2)], (32, 10), 20, 10, 0.5),  # 5 x 5 filters, no padding
    ((4, 9, 11), [(7, 3, 2, 1, SIG, 3, 2)], (10, 3), 9, 4, 0.0),                           # stride 2, overlapping 3 x 3 pooling
]


@pytest.mark.parametrize("shape,blocks,dense,n,batch,mu", CNN_OBJECT_CASES)
def test_cnn_object_epochs_match_checker(dn, shape, blocks, dense, n, batch, mu):
    """dn_cnn_train_epoch (every layer's forward, backward and update enqueued by the library,
    two epochs) against the checker's functions chained by reference_cnn_epoch: loss of each
    epoch, every filter, bias and dense parameter, then dn_cnn_forward's output."""
    announce("cnn object shape=%s blocks=%s dense=%s n=%d batch=%d momentum=%g" % (shape, blocks, dense, n, batch, mu))
    c, h, w = shape
    rng = np.random.default_rng(23)
    X = rng.standard_normal((n, c, h, w)).astype(np.float32)
    labels = rng.integers(0, dense[-1], n).astype(np.int32)
    acts = [TANH] * (len(dense) - 1) + [SOFTMAX]
    net = dn.Cnn(c, h, w, blocks, dense, acts, CE, batch)
    filters, biases, vel, cin = [], [], [], c
    for i, (cout, k, stride, pad, act, pk, ps) in enumerate(blocks):
        filters.append((rng.standard_normal((cout, cin, k, k)) * np.sqrt(2.0 / (cin * k * k))).astype(np.float32))
        biases.append((rng.standard_normal(cout) * 0.1).astype(np.float32))
        vel.append((np.zeros_like(filters[i]), np.zeros_like(biases[i])))
        net.dn_cnn_set_filters(i, filters[i], biases[i])
        cin = cout
    widths = [net.flat] + list(dense)
    Wd = [(rng.standard_normal((widths[l + 1], widths[l])) / np.sqrt(widths[l])).astype(np.float32) for l in range(len(dense))]
    bd = [(rng.standard_normal(widths[l + 1]) * 0.1).astype(np.float32) for l in range(len(dense))]
    net.dense.set_all(Wd, bd)
    o = Oracle("o32", widths, acts, CE)
    o.set_params(Wd, bd)
    Xd, yd = dev(X), dev(labels)
    lr = 0.05
    for epoch in range(2):
        loss = net.dn_cnn_train_epoch(Xd, yd, batch, lr, mu)
        loss_r = reference_cnn_epoch(shape, blocks, filters, biases, o, X, labels, batch, lr, mu, vel)
        assert abs(loss - loss_r) <= TOL * max(1.0, abs(loss_r)), (epoch, loss, loss_r)
        for i in range(len(blocks)):
            Wg, bg = net.dn_cnn_get_filters(i)
            assert_close(Wg, filters[i], TOL, "filters of block %d, epoch %d" % (i, epoch))
            assert_close(bg, biases[i], TOL, "biases of block %d, epoch %d" % (i, epoch))
        Wr, br = o.get_params()
        for l in range(1, len(widths)):
            Wg, bg = net.dense.dn_get_params(l)
            assert_close(Wg, Wr[l - 1], TOL, "W_%d, epoch %d" % (l, epoch))
            assert_close(bg, br[l - 1], TOL, "b_%d, epoch %d" % (l, epoch))
    # inference through the whole stack
    B = min(batch, n)
    out = torch.empty((B, dense[-1]), dtype=torch.float32, device="cuda:0")
    net.dn_cnn_forward(Xd[:B].contiguous(), out)
    a = X[:B]
    for i, (cout, k, stride, pad, act, pk, ps) in enumerate(blocks):
        a = co.conv_forward("o32", a, filters[i], biases[i], stride, pad, act)
        if pk > 0:
            a = co.maxpool_forward("o32", a, pk, ps)
    assert_close(out.cpu().numpy(), o.forward(a.reshape(B, -1))[-1], TOL, "network output")
    net.close()


def test_cnn_object_equals_the_composed_calls(dn):
    """The epoch loop adds nothing of its own: one dn_cnn_train_epoch step leaves the same bits as
    the same calls made one by one from here (run_classifier's order)."""
    announce("cnn object against the composed calls, bit for bit")
    B, c, h, w, cout, K, pad, lr = 8, 3, 10, 10, 6, 3, 1, 0.05
    rng = np.random.default_rng(5)
    X = rng.standard_normal((B, c, h, w)).astype(np.float32)
    labels = rng.integers(0, 4, B).astype(np.int32)
    Wf = (rng.standard_normal((cout, c, K, K)) * 0.3).astype(np.float32)
    bf = (rng.standard_normal(cout) * 0.1).astype(np.float32)
    flat = cout * (h // 2) * (w // 2)
    Wd = [(rng.standard_normal((4, flat)) / np.sqrt(flat)).astype(np.float32)]
    bd = [np.zeros(4, dtype=np.float32)]
    net = dn.Cnn(c, h, w, [(cout, K, 1, pad, RELU, 2, 2)], (4,), [SOFTMAX], CE, B)
    net.dn_cnn_set_filters(0, Wf, bf)
    net.dense.set_all(Wd, bd)
    Xd, yd = dev(X), dev(labels)
    net.dn_cnn_train_epoch(Xd, yd, B, lr, 0.0)
    # the same step from single calls
    f32 = dict(dtype=torch.float32, device="cuda:0")
    W, b = dev(Wf), dev(bf)
    Y, P = torch.empty((B, cout, h, w), **f32), torch.empty((B, cout, h // 2, w // 2), **f32)
    dP, dY, delta = torch.empty_like(P), torch.empty_like(Y), torch.empty_like(Y)
    dW, db = torch.empty_like(W), torch.empty_like(b)
    dense = dn.Net([flat, 4], [SOFTMAX], CE, B)
    dense.set_all(Wd, bd)
    dn.dn_conv_forward(Xd, W, b, Y, 1, pad, RELU)
    dn.dn_maxpool_forward(Y, P, 2, 2)
    dense.dn_forward(P.view(B, flat))
    dense.dn_backward(yd)
    dense.dn_input_gradient(dP.view(B, flat))
    dn.dn_maxpool_backward(Y, dP, dY, 2, 2)
    dn.dn_conv_backward(Xd, W, Y, dY, delta, None, dW, db, 1, pad, RELU)
    dense.dn_update(lr, 0.0)
    dn.dn_sgd_step(W, dW, None, lr, 0.0)
    dn.dn_sgd_step(b, db, None, lr, 0.0)
    Wg, bg = net.dn_cnn_get_filters(0)
    assert np.array_equal(Wg, W.cpu().numpy()) and np.array_equal(bg, b.cpu().numpy())
    W1, b1 = net.dense.dn_get_params(1)
    W2, b2 = dense.dn_get_params(1)
    assert np.array_equal(W1, W2) and np.array_equal(b1, b2)
    dense.close()
    net.close()


def test_cnn_object_argument_errors(dn):
    announce("cnn object: argument errors")
    with pytest.raises(dn.DnError) as e:
        dn.Cnn(3, 8, 8, [(4, 9, 1, 1, RELU, 2, 2)], (5,), [SOFTMAX], CE, 4)          # 9 x 9 filters
    assert e.value.status == dn.DN_ERR_SHAPE
    with pytest.raises(dn.DnError) as e:
        dn.Cnn(3, 8, 8, [(4, 3, 1, 1, SOFTMAX, 2, 2)], (5,), [SOFTMAX], CE, 4)       # softmax inside a block
    assert e.value.status == dn.DN_ERR_SHAPE
    with pytest.raises(dn.DnError) as e:
        dn.Cnn(3, 8, 8, [(4, 3, 1, 1, RELU, 2, 2)], (5,), [TANH], CE, 4)             # cross-entropy without softmax
    assert e.value.status == dn.DN_ERR_UNSUPPORTED
    net = dn.Cnn(3, 8, 8, [(4, 3, 1, 1, RELU, 2, 2)], (5,), [SOFTMAX], CE, 4)
    X = torch.zeros((6, 3, 8, 8), dtype=torch.float32, device="cuda:0")
    y = torch.zeros(6, dtype=torch.int32, device="cuda:0")
    with pytest.raises(dn.DnError) as e:
        net.dn_cnn_train_epoch(X, y, 5, 0.1, 0.0)                                     # batch above max_batch
    assert e.value.status == dn.DN_ERR_SHAPE
    with pytest.raises(dn.DnError) as e:
        net.dn_cnn_train_epoch(X, y, 4, 0.1, 1.0)                                     # momentum outside [0, 1)
    assert e.value.status == dn.DN_ERR_INVALID_ARG
    with pytest.raises(dn.DnError) as e:
        net.dn_cnn_set_filters(1, None, None)                                         # no such block
    assert e.value.status == dn.DN_ERR_INVALID_ARG
    assert net.dn_cnn_train_epoch(X, y, 4, 0.0, 0.0) == pytest.approx(np.log(5.0), rel=1e-5)   # zero parameters, zero rate: uniform output
    net.close()
