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
