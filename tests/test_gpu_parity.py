"""GPU parity: libdn (through its C ABI) against the CPU checker on the same
seeded inputs.  Tolerances: relative error 1e-4 on
gradients and on weights after one step, 1e-3 on weights and loss after an
epoch (relative L2 per tensor and max-abs relative to the tensor's max).
The reference is the checker's fp32-storage / fp64-accumulate mode."""
import numpy as np
import pytest

from oracle.dn_oracle import Oracle
from paper_2001_04206_amd import synth
from parity_util import announce, assert_close, rel_err

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

LIN, SIG, TANH, RELU, SOFTMAX = 0, 1, 2, 3, 4
MSE, CE = 0, 1
STEP_TOL, EPOCH_TOL = 1e-4, 1e-3


@pytest.fixture(scope="module")
def dnlib():
    from paper_2001_04206_amd import dn
    assert torch.cuda.is_available(), "these tests need the GPU"
    dn.lib()      # raises if the HIP library has not been built: no fallback
    return dn


def to_dev(w):
    X = torch.from_numpy(w.X).to("cuda:0")
    y = torch.from_numpy(w.labels).to("cuda:0")
    return X, y


def make_pair(dn, w, max_batch):
    net = dn.Net(w.widths, w.acts, w.loss, max_batch)
    net.set_all(w.W, w.b)
    o = Oracle("o32", w.widths, w.acts, w.loss)
    o.set_params(w.W, w.b)
    return net, o


def check_one_step(dn, w, B, lr, mu, tol=STEP_TOL, variant=-1, second_step=True, split_k=1):
    """forward / backward / update through the split API, compared tensor by tensor."""
    net, o = make_pair(dn, w, B)
    if variant >= 0:
        net.dn_set_option("gemm_variant", variant)
    net.dn_set_option("split_k", split_k)
    X, y = to_dev(w)
    nL = w.widths[-1]
    for step in range(2 if second_step else 1):
        Xb, yb = X[step * B:(step + 1) * B].contiguous(), y[step * B:(step + 1) * B].contiguous()
        out = torch.empty((B, nL), dtype=torch.float32, device="cuda:0")
        loss = torch.zeros(1, dtype=torch.float32, device="cuda:0")
        net.dn_forward(Xb, out)
        net.dn_backward(yb, loss)
        A = o.forward(w.X[step * B:(step + 1) * B])
        ref_loss = o.backward(w.labels[step * B:(step + 1) * B])
        assert_close(out.cpu().numpy(), A[-1], tol, "A_L step %d" % step)
        got_loss = float(loss.cpu()[0])
        assert abs(got_loss - ref_loss) <= tol * max(abs(ref_loss), 1e-6), (got_loss, ref_loss)
        G, g = net.get_all_grads()
        Gr, gr = o.get_grads()
        for l in range(net.L):
            assert_close(G[l], Gr[l], tol, "G_%d step %d" % (l + 1, step))
            assert_close(g[l], gr[l], tol, "g_%d step %d" % (l + 1, step))
        net.dn_update(lr, mu)
        o.update(lr, mu)
        W, b = net.get_all()
        Wr, br = o.get_params()
        for l in range(net.L):
            assert_close(W[l], Wr[l], tol, "W_%d step %d" % (l + 1, step))
            assert_close(b[l], br[l], tol, "b_%d step %d" % (l + 1, step))
    net.close()


def check_epochs(dn, w, n_samples, epochs=1, tol=EPOCH_TOL, steps_note=""):
    net, o = make_pair(dn, w, w.batch)
    X, y = to_dev(w)
    X, y = X[:n_samples].contiguous(), y[:n_samples].contiguous()
    for e in range(epochs):
        got = net.dn_train_epoch(X, y, w.batch, w.lr, w.momentum)
        ref, kinks = o.train_epoch(w.X[:n_samples], w.labels[:n_samples], w.batch, w.lr, w.momentum,
                                   kink_eps=1e-5)
        assert np.isfinite(got)
        assert abs(got - ref) <= tol * abs(ref), "epoch %d loss %r vs %r (kink census %d)" % (e, got, ref, kinks)
    W, b = net.get_all()
    Wr, br = o.get_params()
    for l in range(net.L):
        assert_close(W[l], Wr[l], tol, "W_%d after %d epoch(s) %s (kink census %d)" % (l + 1, epochs, steps_note, kinks))
        assert_close(b[l], br[l], tol, "b_%d after %d epoch(s) %s (kink census %d)" % (l + 1, epochs, steps_note, kinks))
    net.close()
    return W, b


# ------------------------------------------------------------ small and ragged ----

SMALL_CASES = [
    # widths, acts, loss, B  (several tiles + ragged tails in every dimension)
    ([4, 16, 3], [SIG, SIG], MSE, 1),
    ([4, 16, 3], [SIG, SIG], MSE, 7),
    ([37, 70, 5], [TANH, LIN], MSE, 3),
    ([37, 70, 5], [RELU, TANH], MSE, 33),
    ([130, 67, 129, 11], [RELU, SIG, SOFTMAX], CE, 1),
    ([130, 67, 129, 11], [TANH, RELU, SOFTMAX], CE, 65),
    ([200, 257, 10], [TANH, SOFTMAX], CE, 130),
    ([1, 1, 2], [TANH, SOFTMAX], CE, 1),            # degenerate widths
    ([9, 1], [SIG], MSE, 5),                        # single layer, single output
    ([300, 10], [SOFTMAX], CE, 260),                # single layer softmax regression
]


@pytest.mark.parametrize("widths,acts,loss,B", SMALL_CASES)
@pytest.mark.parametrize("variant", [-1, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12])
def test_one_step_small_and_ragged(dnlib, widths, acts, loss, B, variant):
    announce("one_step_small widths=%s acts=%s loss=%d B=%d variant=%d" % (widths, acts, loss, B, variant))
    w = synth.make("small", widths, acts, loss, n_samples=2 * B, features="normal",
                   init="xavier_uniform", batch=B, lr=0.1, momentum=0.9, seed=3)
    rng = np.random.default_rng(5)
    w.b = [rng.standard_normal(n).astype(np.float32) * 0.1 for n in widths[1:]]   # non-zero biases
    check_one_step(dnlib, w, B, lr=0.1, mu=0.9, variant=variant)


SPLIT_K_CASES = [
    # long contractions with few output tiles: forward / delta products split k across workgroups
    ([1000, 300, 52, 10], [TANH, RELU, SOFTMAX], CE, 40),
    ([517, 259, 33, 7], [SIG, TANH, SOFTMAX], CE, 5),        # scalar-load path, ragged everywhere
    ([2048, 96, 10], [TANH, SOFTMAX], CE, 64),
    ([1536, 1024, 3], [RELU, LIN], MSE, 16),
]


@pytest.mark.parametrize("widths,acts,loss,B", SPLIT_K_CASES)
@pytest.mark.parametrize("variant", [-1, 2, 4, 5, 6, 9])
@pytest.mark.parametrize("split_k", [1, 0])
def test_one_step_split_k(dnlib, widths, acts, loss, B, variant, split_k):
    announce("one_step_split_k widths=%s B=%d variant=%d split_k=%d" % (widths, B, variant, split_k))
    w = synth.make("splitk", widths, acts, loss, n_samples=2 * B, features="normal",
                   init="xavier_uniform", batch=B, lr=0.05, momentum=0.9, seed=7)
    check_one_step(dnlib, w, B, lr=0.05, mu=0.9, variant=variant, split_k=split_k)


PAIR_CASES = [
    # weight matrices of at least 64 tiles of 64 x 64 with widths that are multiples of 4: the gradient /
    # update products of all layers share one launch, and a narrow last layer's gradient rides with the
    # delta product below it.  Ragged against every tile size involved.
    ([1040, 1028, 1100, 24], [TANH, RELU, SOFTMAX], CE, 40, 0.9),
    ([1028, 1092, 1032, 1040, 20], [RELU, TANH, SIG, LIN], MSE, 132, 0.0),
    ([1024, 1024, 1024, 10], [TANH, TANH, SOFTMAX], CE, 516, 0.9),     # batch beyond the limit of 512: one launch per product
    ([1028, 1040, 1100, 12], [TANH, TANH, SOFTMAX], CE, 136, 0.9),     # narrow last layer: its gradient rides with the delta product below it
    ([516, 1040, 1100, 16], [RELU, SIG, SIG], MSE, 50, 0.0),           # the same with squared error and 16 outputs
    ([2052, 2060, 2100, 24], [TANH, RELU, SOFTMAX], CE, 24, 0.9),      # 33 x 33 tiles and more per layer, an odd count
]


@pytest.mark.parametrize("widths,acts,loss,B,mu", PAIR_CASES)
@pytest.mark.parametrize("pair", [1, 0])
def test_merged_backward_launches(dnlib, widths, acts, loss, B, mu, pair):
    announce("merged backward launches widths=%s B=%d mu=%g merge_launches=%d" % (widths, B, mu, pair))
    w = synth.make("pair", widths, acts, loss, n_samples=3 * B - 7, features="normal",
                   init="xavier_uniform", batch=B, lr=0.05, momentum=mu, seed=23)
    rng = np.random.default_rng(29)
    w.b = [rng.standard_normal(n).astype(np.float32) * 0.1 for n in widths[1:]]
    # the split API (gradients stored), then fused epochs (plain / last-step / momentum updates, short last batch)
    net, o = make_pair(dnlib, w, B)
    net.dn_set_option("merge_launches", pair)
    X, y = to_dev(w)
    out = torch.empty((B, widths[-1]), dtype=torch.float32, device="cuda:0")
    net.dn_forward(X[:B].contiguous(), out)
    net.dn_backward(y[:B].contiguous())
    o.forward(w.X[:B]); o.backward(w.labels[:B])
    G, g = net.get_all_grads()
    Gr, gr = o.get_grads()
    for l in range(net.L):
        assert_close(G[l], Gr[l], STEP_TOL, "G_%d" % (l + 1))
        assert_close(g[l], gr[l], STEP_TOL, "g_%d" % (l + 1))
    for e in range(2):
        got = net.dn_train_epoch(X, y, B, w.lr, mu)
        ref, _ = o.train_epoch(w.X, w.labels, B, w.lr, mu)
        assert abs(got - ref) <= EPOCH_TOL * abs(ref), (e, got, ref)
    W, b = net.get_all()
    Wr, br = o.get_params()
    for l in range(net.L):
        assert_close(W[l], Wr[l], EPOCH_TOL, "W_%d" % (l + 1))
        assert_close(b[l], br[l], EPOCH_TOL, "b_%d" % (l + 1))
    net.close()


NARROW_CASES = [
    # layers of at most 16 outputs take plain-FMA kernels for their delta and gradient products:
    # vector (width % 4 == 0) and scalar paths, batches beyond one row per thread, ragged
    ([64, 128, 10], [TANH, SOFTMAX], CE, 512),
    ([33, 70, 5], [RELU, LIN], MSE, 515),
    ([40, 16, 16], [SIG, SIG], MSE, 777),          # both layers narrow
    ([130, 67, 3], [TANH, SOFTMAX], CE, 1030),     # scalar path, several rows per thread
]


@pytest.mark.parametrize("widths,acts,loss,B", NARROW_CASES)
def test_one_step_narrow_layers(dnlib, widths, acts, loss, B):
    announce("one_step_narrow widths=%s acts=%s loss=%d B=%d" % (widths, acts, loss, B))
    w = synth.make("narrow", widths, acts, loss, n_samples=2 * B, features="normal",
                   init="xavier_uniform", batch=B, lr=0.1, momentum=0.9, seed=11)
    rng = np.random.default_rng(13)
    w.b = [rng.standard_normal(n).astype(np.float32) * 0.1 for n in widths[1:]]
    check_one_step(dnlib, w, B, lr=0.1, mu=0.9)


NARROW_EPOCHS = [
    # widths, acts, loss, batch, samples, momentum: training steps through the fused forward + output
    # kernel of a narrow last layer and the fused update modes of the narrow gradient kernel
    # (plain steps, the last step that leaves the velocity behind, momentum), short last batches
    ([48, 96, 10], [TANH, SOFTMAX], CE, 600, 2000, 0.0),
    ([48, 96, 10], [TANH, SOFTMAX], CE, 600, 2000, 0.9),
    ([30, 50, 7], [RELU, SIG], MSE, 64, 300, 0.9),            # squared error, several rows per workgroup
    ([21, 33, 16], [TANH, TANH], MSE, 1100, 2500, 0.0),       # four rows per wave, scalar loads
    ([24, 5], [SOFTMAX], CE, 1500, 4000, 0.9),                # single layer: the input is the batch itself
]


@pytest.mark.parametrize("widths,acts,loss,batch,n,momentum", NARROW_EPOCHS)
def test_epoch_narrow_layers(dnlib, widths, acts, loss, batch, n, momentum):
    announce("epoch narrow widths=%s loss=%d B=%d n=%d momentum=%g" % (widths, loss, batch, n, momentum))
    w = synth.make("narrow_epoch", widths, acts, loss, n_samples=n, features="normal",
                   init="xavier_uniform", batch=batch, lr=0.05, momentum=momentum, seed=17)
    net, o = make_pair(dnlib, w, w.batch)
    net.dn_set_option("batch_mode", 1)      # one launch per product, not the persistent kernels
    X, y = to_dev(w)
    for e in range(2):
        got = net.dn_train_epoch(X, y, w.batch, w.lr, w.momentum)
        ref, kinks = o.train_epoch(w.X, w.labels, w.batch, w.lr, w.momentum, kink_eps=1e-5)
        assert abs(got - ref) <= EPOCH_TOL * abs(ref), "epoch %d loss %r vs %r" % (e, got, ref)
    W, b = net.get_all()
    Wr, br = o.get_params()
    for l in range(net.L):
        assert_close(W[l], Wr[l], EPOCH_TOL, "W_%d (kink census %d)" % (l + 1, kinks))
        assert_close(b[l], br[l], EPOCH_TOL, "b_%d (kink census %d)" % (l + 1, kinks))
    net.close()


def _epoch_params(dnlib, w, split_k):
    net = dnlib.Net(w.widths, w.acts, w.loss, w.batch)
    net.set_all(w.W, w.b)
    net.dn_set_option("split_k", split_k)
    net.dn_set_option("batch_mode", 1)          # one launch per product: the path that splits k
    X, y = to_dev(w)
    loss = net.dn_train_epoch(X, y, w.batch, w.lr, w.momentum)
    W, b = net.get_all()
    net.close()
    return loss, W + b


def test_split_k_is_bitwise_reproducible(dnlib):
    announce("determinism: k split across workgroups, two runs")
    w = synth.tanh_sweep(32, n_samples=256)
    a, b = _epoch_params(dnlib, w, 1), _epoch_params(dnlib, w, 1)
    assert a[0] == b[0]
    for x, y in zip(a[1], b[1]):
        assert np.array_equal(x, y)


@pytest.mark.parametrize("widths,acts,loss,B", SPLIT_K_CASES)
def test_split_k_order_is_fixed(dnlib, widths, acts, loss, B):
    """The partial tiles of a k split are added in split order by whichever workgroup arrives last,
    so two epochs with the split give the same bits whatever the arrival order was; the same epoch
    without the split adds the same terms in another order and agrees to rounding."""
    announce("determinism: k split, widths=%s B=%d, two runs and against no split" % (widths, B))
    w = synth.make("splitk", widths, acts, loss, n_samples=6 * B + 3, features="normal",
                   init="xavier_uniform", batch=B, lr=0.002, momentum=0.5, seed=7)
    a, b, c = _epoch_params(dnlib, w, 1), _epoch_params(dnlib, w, 1), _epoch_params(dnlib, w, 0)
    assert np.isfinite(a[0]) and all(np.all(np.isfinite(x)) for x in a[1])
    assert a[0] == b[0]
    for x, y in zip(a[1], b[1]):
        assert np.array_equal(x, y)
    assert abs(a[0] - c[0]) <= 1e-5 * abs(c[0])
    for x, y in zip(a[1], c[1]):
        assert_close(x, y, 1e-5, "k split against no split")


# --------------------------------------------------- the five named workloads ----

def test_one_step_iris_like(dnlib):
    announce("one_step cfg1 4-16-3 B=1")
    w = synth.iris_like()
    check_one_step(dnlib, w, 1, w.lr, w.momentum)


@pytest.mark.parametrize("B,mu,lr", [(1, 0.0, 0.01), (128, 0.9, 0.05)])
def test_one_step_digits_like(dnlib, B, mu, lr):
    announce("one_step cfg2/3 784-128-10 B=%d" % B)
    w = synth.digits_like_online(n_samples=2 * B)
    check_one_step(dnlib, w, B, lr, mu)


@pytest.mark.parametrize("B", [1, 8, 32, 128, 512, 2048])
def test_one_step_tanh_sweep(dnlib, B):
    announce("one_step cfg5 1024x4-10 B=%d" % B)
    w = synth.tanh_sweep(B, n_samples=2 * B if B < 512 else B)
    check_one_step(dnlib, w, B, w.lr, w.momentum, second_step=B < 512)


def test_one_step_wide_relu_full_size(dnlib):
    announce("one_step cfg4 4096-4096-4096-1000 B=256 (full size, every element)")
    w = synth.wide_relu(n_samples=256)
    check_one_step(dnlib, w, 256, w.lr, w.momentum, second_step=False)


# ----------------------------------------------------------------- whole epochs ----

def test_epochs_iris_like(dnlib):
    announce("epochs cfg1 4-16-3 B=1 x10 epochs")
    w = synth.iris_like()
    check_epochs(dnlib, w, w.n_samples, epochs=10)


def test_epoch_digits_like_online(dnlib):
    # ReLU at batch 1: a hidden net input within rounding of zero can take a different
    # derivative on the two sides; the failure message carries the checker's census of
    # such near-kink units so a miss can be told from a real defect.
    announce("epoch cfg2 784-128-10 B=1, 60000 steps")
    w = synth.digits_like_online()
    check_epochs(dnlib, w, w.n_samples)


def test_epoch_digits_like_minibatch(dnlib):
    announce("epoch cfg3 784-128-10 B=128 momentum (469 steps, short last batch)")
    w = synth.digits_like_minibatch()
    W, b = check_epochs(dnlib, w, w.n_samples)
    # softmax + cross-entropy conserves the output layer's bias sum and column sums
    assert abs(float(b[-1].sum())) < 1e-4
    np.testing.assert_allclose(W[-1].sum(axis=0), w.W[-1].sum(axis=0), atol=2e-4)


@pytest.mark.parametrize("B", [1, 8, 32, 128, 512, 2048])
def test_epoch_tanh_sweep_full(dnlib, B):
    """The whole 16384-sample pass of the batch-size sweep, in the configuration bench.py times:
    every weight, every bias and the epoch loss against the checker."""
    announce("epoch cfg5 1024x4-10 B=%d, all 16384 samples" % B)
    w = synth.tanh_sweep(B)
    W, b = check_epochs(dnlib, w, w.n_samples, steps_note="(full pass)")
    # softmax + cross-entropy conserves the output layer's bias sum and column sums
    assert abs(float(b[-1].sum())) < 1e-4
    np.testing.assert_allclose(W[-1].sum(axis=0), w.W[-1].sum(axis=0), atol=5e-4)


# the 4096-4096-4096-1000 workload (first 16 steps against the checker, then the invariants of its
# full 256-step epoch) has a file of its own: test_gpu_wide_relu.py


# ------------------------------------------------------------------- edge cases ----

def test_short_last_batch_and_momentum_zero_velocity(dnlib):
    announce("edge: N=10, B=4 (short last batch), mu=0 epoch then mu=0.9 epoch")
    w = synth.make("edge", [20, 33, 6], [TANH, SOFTMAX], CE, n_samples=10, features="normal",
                   init="xavier_uniform", batch=4, lr=0.05, momentum=0.0, seed=9)
    net, o = make_pair(dnlib, w, 4)
    X, y = to_dev(w)
    for mu in (0.0, 0.9):       # the second epoch starts from the velocity the first one left
        got = net.dn_train_epoch(X, y, 4, 0.05, mu)
        ref, _ = o.train_epoch(w.X, w.labels, 4, 0.05, mu)
        assert abs(got - ref) <= STEP_TOL * abs(ref)
    W, b = net.get_all(); Wr, br = o.get_params()
    for l in range(2):
        assert_close(W[l], Wr[l], STEP_TOL, "W_%d" % (l + 1))
        assert_close(b[l], br[l], STEP_TOL, "b_%d" % (l + 1))
    net.close()


def test_runtime_argument_errors(dnlib):
    announce("edge: runtime argument errors")
    dn = dnlib
    w = synth.make("edge", [8, 5, 3], [TANH, SOFTMAX], CE, n_samples=8, features="normal",
                   init="xavier_uniform", batch=4, lr=0.05, momentum=0.0, seed=1)
    net = dn.Net(w.widths, w.acts, w.loss, 4)
    net.set_all(w.W, w.b)
    X, y = to_dev(w)

    def status(fn, *a):
        with pytest.raises(dn.DnError) as e:
            fn(*a)
        return e.value.status
    assert status(net.dn_backward, y[:4].contiguous()) == dn.DN_ERR_INVALID_ARG       # before forward
    assert status(net.dn_update, 0.1, 0.0) == dn.DN_ERR_INVALID_ARG                  # before backward
    assert status(net.dn_forward, X[:8].contiguous()) == dn.DN_ERR_SHAPE             # batch > max_batch
    net.dn_forward(X[:4].contiguous())
    assert status(net.dn_backward, y[:3].contiguous()) == dn.DN_ERR_SHAPE            # batch mismatch
    net.dn_backward(y[:4].contiguous())
    assert status(net.dn_update, -1.0, 0.0) == dn.DN_ERR_INVALID_ARG
    assert status(net.dn_update, 0.1, 1.0) == dn.DN_ERR_INVALID_ARG
    assert status(net.dn_update, float("nan"), 0.0) == dn.DN_ERR_INVALID_ARG
    assert status(net.dn_train_epoch, X, y, 5, 0.1, 0.0) == dn.DN_ERR_SHAPE
    assert status(net.dn_train_epoch, X, y, 4, 0.1, 0.0, 0) == dn.DN_ERR_INVALID_ARG  # no samples
    assert status(net.dn_set_option, "no_such_option", 1) == dn.DN_ERR_INVALID_ARG
    assert status(net.dn_get_params, 3) == dn.DN_ERR_INVALID_ARG
    net.close()


def test_same_seed_twice_is_bitwise_identical(dnlib):
    announce("determinism: two runs of the same epoch")
    w = synth.digits_like_minibatch(n_samples=1000)
    outs = []
    for _ in range(2):
        net = dnlib.Net(w.widths, w.acts, w.loss, w.batch)
        net.set_all(w.W, w.b)
        X, y = to_dev(w)
        net.dn_train_epoch(X, y, w.batch, w.lr, w.momentum)
        outs.append(net.get_all())
        net.close()
    for a, b in zip(outs[0][0] + outs[0][1], outs[1][0] + outs[1][1]):
        assert np.array_equal(a, b)


# ---------------------------------------------- evaluation and the stopping rule ----

@pytest.mark.parametrize("widths,acts,loss", [([20, 32, 4], [TANH, SOFTMAX], CE), ([37, 70, 5], [RELU, SIG], MSE),
                                              ([300, 10], [SOFTMAX], CE), ([64, 200, 300], [TANH, SOFTMAX], CE)])
def test_evaluate_matches_checker(dnlib, widths, acts, loss):
    announce("evaluate widths=%s" % (widths,))
    w = synth.make("eval", widths, acts, loss, n_samples=333, features="normal", init="xavier_uniform",
                   batch=50, lr=0.1, momentum=0.0, seed=12)
    net, o = make_pair(dnlib, w, 50)
    X, y = to_dev(w)
    before = net.get_all()
    got_loss, got_hits = net.dn_evaluate(X, y, 50)          # 6 chunks of 50 and one of 33
    ref_loss, ref_hits = o.evaluate(w.X, w.labels)
    assert abs(got_loss - ref_loss) <= STEP_TOL * abs(ref_loss)
    # a hit is an argmax: samples whose two largest outputs are closer than rounding may fall either way
    out = np.sort(o.forward(w.X)[-1].astype(np.float64), axis=1)
    near_ties = int(np.sum(out[:, -1] - out[:, -2] < 1e-5 * np.abs(out[:, -1])))
    assert abs(got_hits - ref_hits) <= near_ties, (got_hits, ref_hits, near_ties)
    after = net.get_all()
    for a, b in zip(before[0] + before[1], after[0] + after[1]):
        assert np.array_equal(a, b)
    net.close()


@pytest.mark.parametrize("batch", [1, 8])
def test_train_until_max_error_matches_checker(dnlib, batch):
    announce("train until max error, batch %d" % batch)
    w = synth.learnable(batch=batch)
    net, o = make_pair(dnlib, w, batch)
    X, y = to_dev(w)
    _, _, losses = o.train(w.X, w.labels, batch, w.lr, w.momentum, -1.0, 10)
    k = next(i for i in range(1, 10) if losses[i] < min(losses[:i]))
    threshold = 0.5 * (losses[k] + min(losses[:k]))         # midway: rounding cannot move the stopping epoch
    epochs, last = net.dn_train(X, y, batch, w.lr, w.momentum, threshold, 10)
    assert epochs == k + 1
    assert abs(last - losses[k]) <= EPOCH_TOL * abs(losses[k])
    o.set_params(w.W, w.b)
    o.train(w.X, w.labels, batch, w.lr, w.momentum, threshold, 10)
    W, b = net.get_all(); Wr, br = o.get_params()
    for l in range(net.L):
        assert_close(W[l], Wr[l], EPOCH_TOL, "W_%d" % (l + 1))
        assert_close(b[l], br[l], EPOCH_TOL, "b_%d" % (l + 1))
    # never reaching the threshold runs max_epochs; bad arguments are refused
    assert net.dn_train(X, y, batch, w.lr, w.momentum, -1.0, 2)[0] == 2
    with pytest.raises(dnlib.DnError) as e:
        net.dn_train(X, y, batch, w.lr, w.momentum, 0.1, 0)
    assert e.value.status == dnlib.DN_ERR_INVALID_ARG
    net.close()
