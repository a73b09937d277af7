"""GPU parity of per-sample (batch 1) training through dn_train_epoch, in both of its
schedules: the persistent whole-epoch kernel ("online_mode" 2) and one launch per
phase ("online_mode" 1), each against the CPU checker (fp32 storage, fp64 sums) on the
same seeded inputs.  Tolerances: 1e-4 after the first steps, 1e-3 after an epoch."""
import numpy as np
import pytest

from oracle.dn_oracle import Oracle
from paper_2001_04206_amd import synth
from parity_util import announce, assert_close

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

LIN, SIG, TANH, RELU, SOFTMAX = 0, 1, 2, 3, 4
MSE, CE = 0, 1
PER_PHASE, PERSISTENT = 1, 2


@pytest.fixture(scope="module")
def dnlib():
    from paper_2001_04206_amd import dn
    assert torch.cuda.is_available(), "these tests need the GPU"
    dn.lib()
    return dn


def run_pair(dn, w, n, passes, mode, min_tile=None, tol=1e-4, biases=True, resident=1, twin=1, twin_expected=None, tiny=0,
             wide=0, solo=0):
    """`passes` = list of momenta; one pass over the first n samples per entry.  twin=0 keeps
    plain-gradient-descent passes of deeper nets on the general persistent kernel; tiny=1 or 2 lets nets
    with no layer wider than 64 run on one wavefront (1: plain passes of two-layer nets keep the net in
    registers, 2: every pass keeps it in LDS); wide=1 lets two-layer nets with a
    hidden layer beyond LDS run on the kernel that keeps rows of W_1 in LDS and registers (every
    pass must then report that schedule); solo=1 lets plain passes of two-layer nets whose W_1 fits one
    compute unit's registers run on one workgroup (solo=2: ... but this call has too few samples for it)."""
    if biases:
        rng = np.random.default_rng(11)
        w.b = [rng.standard_normal(k).astype(np.float32) * 0.1 for k in w.widths[1:]]
    net = dn.Net(w.widths, w.acts, w.loss, 1)
    net.set_all(w.W, w.b)
    net.dn_set_option("online_mode", mode)
    if min_tile is not None:
        net.dn_set_option("online_min_tile", min_tile)
    net.dn_set_option("online_resident", resident)
    net.dn_set_option("online_twin", twin)
    net.dn_set_option("online_tiny", tiny)
    net.dn_set_option("online_wide", wide)
    net.dn_set_option("online_solo", 1 if solo else 0)
    o = Oracle("o32", w.widths, w.acts, w.loss)
    o.set_params(w.W, w.b)
    X = torch.from_numpy(w.X[:n]).to("cuda:0")
    y = torch.from_numpy(w.labels[:n]).to("cuda:0")
    for mu in passes:
        got = net.dn_train_epoch(X, y, 1, w.lr, mu)
        if tiny:
            regs = tiny == 1 and len(w.widths) == 3 and mu == 0.0
            want = dn.DN_SCHED_ONE_WAVE_REGISTERS if regs else dn.DN_SCHED_ONE_WAVE
            assert net.dn_last_schedule() == want, (net.dn_last_schedule(), want)
        elif solo:
            one = solo == 1 and mu == 0.0
            assert (net.dn_last_schedule() == dn.DN_SCHED_ONE_WORKGROUP) == one, (net.dn_last_schedule(), mu)
        elif wide:
            assert net.dn_last_schedule() == dn.DN_SCHED_WIDE_HIDDEN, net.dn_last_schedule()
        elif mode == PERSISTENT and twin_expected is not None:
            want = dn.DN_SCHED_TWO_COPY if (twin_expected and mu == 0.0) else dn.DN_SCHED_PER_SAMPLE
            assert net.dn_last_schedule() == want, (net.dn_last_schedule(), want)
        ref, _ = o.train_epoch(w.X[:n], w.labels[:n], 1, w.lr, mu)
        assert np.isfinite(got)
        assert abs(got - ref) <= tol * max(abs(ref), 1e-6), (got, ref)
    W, b = net.get_all()
    Wr, br = o.get_params()
    for l in range(net.L):
        assert_close(W[l], Wr[l], tol, "W_%d" % (l + 1))
        assert_close(b[l], br[l], tol, "b_%d" % (l + 1))
    net.close()
    return W, b


SHAPES = [
    # widths, acts, loss
    ([4, 16, 3], [SIG, SIG], MSE),
    ([37, 70, 5], [TANH, LIN], MSE),                        # rows that are not whole float4s
    ([130, 67, 129, 11], [RELU, SIG, SOFTMAX], CE),
    ([20, 40, 30, 50, 24, 6], [TANH, SIG, RELU, TANH, SOFTMAX], CE),
    ([300, 10], [SOFTMAX], CE),                             # one layer
    ([9, 1], [SIG], MSE),
    ([1, 1, 2], [TANH, SOFTMAX], CE),
    ([64, 2048, 1024, 10], [TANH, TANH, SOFTMAX], CE),      # column chunks < waves: rows split across waves
    ([16, 4100, 24, 10], [TANH, RELU, SOFTMAX], CE),        # column chunks >= waves (float4 rows)
    ([16, 1030, 24, 128], [SIG, TANH, SOFTMAX], CE),        # column chunks >= waves (scalar rows), widest output
    ([340, 3000, 10], [TANH, SOFTMAX], CE),                 # the paper's benchmark shape, narrower hidden layer
    ([2000, 5000, 10], [TANH, SOFTMAX], CE),                # first layer beyond LDS: part of each block resident, the rest streamed
    ([2000, 5000, 40, 10], [SIG, TANH, SOFTMAX], CE),       # the same under a middle layer
    ([1999, 5003, 7], [TANH, LIN], MSE),                    # the same with rows that are not whole float4s
    ([400, 30000, 10], [TANH, SOFTMAX], CE),                # streamed first layer with short rows: update and next forward product in one sweep
    ([256, 20000, 24, 10], [SIG, TANH, SOFTMAX], CE),       # the same under a middle layer
    ([36, 70000, 3], [RELU, SIG], MSE),                     # very short rows (fewer float4s than the sixteen lanes of a row)
]


@pytest.mark.parametrize("widths,acts,loss", SHAPES)
@pytest.mark.parametrize("min_tile", [None, 16])
@pytest.mark.parametrize("resident", [1, 0])
def test_persistent_epochs_match_checker(dnlib, widths, acts, loss, min_tile, resident):
    """resident=1 keeps the workgroups' weight slices in LDS where they fit (all of these shapes
    except the widest); resident=0 streams them from device memory."""
    announce("online persistent widths=%s min_tile=%s resident=%d" % (widths, min_tile, resident))
    # (thousands of inputs and outputs per unit: a smaller rate keeps the 48 steps from driving the loss to rounding level)
    w = synth.make("online", widths, acts, loss, n_samples=48, features="normal", init="xavier_uniform",
                   batch=1, lr=0.0001 if max(widths) >= 5000 else 0.005, momentum=0.0, seed=4)
    # plain SGD pass (leaves velocity = last step's delta), then two momentum passes on top of it
    run_pair(dnlib, w, 48, [0.0, 0.5, 0.5], PERSISTENT, min_tile, resident=resident, twin=0)


TWIN_SHAPES = [
    # two or more layers, every width but the last a multiple of 4, slices that fit in LDS twice
    ([784, 128, 10], [RELU, SOFTMAX], CE),                            # two layers: one exchange per step
    ([4, 16, 3], [SIG, SIG], MSE),                                    # one workgroup owns the whole net
    ([340, 3000, 10], [TANH, SOFTMAX], CE),
    ([32, 64, 48, 10], [TANH, SIG, SOFTMAX], CE),
    ([20, 40, 32, 52, 24, 6], [TANH, SIG, RELU, TANH, SOFTMAX], CE),   # five layers
    ([64, 2048, 1024, 10], [TANH, TANH, SOFTMAX], CE),                # fits with 16-weight tiles only
    ([16, 4100, 24, 10], [TANH, RELU, SOFTMAX], CE),                  # layers owned by different numbers of workgroups
    ([12, 8, 4, 3], [SIG, TANH, SIG], MSE),                           # squared error, one workgroup
    ([256, 512, 512, 7], [RELU, TANH, LIN], MSE),
    ([1024, 1024, 1024, 1024, 10], [TANH, TANH, TANH, SOFTMAX], CE),  # the shape of the batch sweep
    # the kernel is compiled per depth: six, seven and eight layers
    ([16, 24, 32, 24, 16, 12, 5], [TANH, SIG, RELU, TANH, SIG, SOFTMAX], CE),
    ([12, 20, 16, 28, 16, 20, 12, 4], [SIG, TANH, SIG, TANH, RELU, TANH, LIN], MSE),
    ([8, 16, 12, 16, 20, 16, 12, 8, 3], [TANH, SIG, TANH, SIG, TANH, RELU, TANH, SOFTMAX], CE),
]


@pytest.mark.parametrize("widths,acts,loss", TWIN_SHAPES)
@pytest.mark.parametrize("min_tile", [None, 16])
def test_two_copy_persistent_epochs_match_checker(dnlib, widths, acts, loss, min_tile):
    """Plain-gradient-descent passes run on the kernel that keeps row and column copies of the
    inner weights; the momentum pass that follows (general kernel) starts from the velocity the
    last plain step left, so that state is checked too; then a plain pass again."""
    announce("online two-copy persistent widths=%s min_tile=%s" % (widths, min_tile))
    w = synth.make("online", widths, acts, loss, n_samples=48, features="normal", init="xavier_uniform",
                   batch=1, lr=0.005, momentum=0.0, seed=4)
    fits = not (widths == [64, 2048, 1024, 10] and min_tile is None)   # 64-row tiles of that net exceed LDS
    run_pair(dnlib, w, 48, [0.0, 0.0, 0.5, 0.0], PERSISTENT, min_tile, twin_expected=fits)


TINY_SHAPES = [
    # no layer wider than 64
    ([4, 16, 3], [SIG, SIG], MSE),
    ([37, 64, 5], [TANH, LIN], MSE),
    ([20, 40, 30, 50, 24, 6], [TANH, SIG, RELU, TANH, SOFTMAX], CE),
    ([64, 64, 64, 64], [RELU, TANH, SOFTMAX], CE),
    ([9, 1], [SIG], MSE),
    ([1, 1, 2], [TANH, SOFTMAX], CE),
    ([3, 5, 7, 2, 9, 4, 6, 8, 10], [TANH, SIG, TANH, LIN, RELU, SIG, TANH, SOFTMAX], CE),   # eight layers
    # two layers at and around the sizes the register-resident form is built for
    ([64, 64, 64], [TANH, SOFTMAX], CE),
    ([5, 17, 16], [RELU, SIG], MSE),
    ([16, 16, 4], [SIG, LIN], MSE),
    ([17, 3, 17], [TANH, TANH], MSE),
]


@pytest.mark.parametrize("form", [1, 2], ids=["registers", "lds"])
@pytest.mark.parametrize("widths,acts,loss", TINY_SHAPES)
def test_one_wave_epochs_match_checker(dnlib, widths, acts, loss, form):
    """Nets with no layer wider than 64 run whole epochs on one wavefront: a plain pass (which
    leaves the last step's change as velocity), two momentum passes, a plain pass again.  Form 1
    lets plain passes of two-layer nets keep the whole net in registers; form 2 keeps every
    pass on the kernel that holds the net in LDS."""
    announce("online one-wave widths=%s form=%d" % (widths, form))
    w = synth.make("online", widths, acts, loss, n_samples=48, features="normal", init="xavier_uniform",
                   batch=1, lr=0.005, momentum=0.0, seed=4)
    run_pair(dnlib, w, 48, [0.0, 0.5, 0.5, 0.0], PERSISTENT, tiny=form)


SOLO_SHAPES = [
    # two layers, W_1 within one compute unit's registers; (unit groups, columns per lane, samples left to other kernels)
    ([784, 128, 10], [SIG, SOFTMAX], CE),      # 2, 196, 0: the 784-128-10 benchmark shape
    ([100, 100, 10], [TANH, SOFTMAX], CE),     # 2, 32, 1
    ([1500, 50, 16], [RELU, SOFTMAX], CE),     # 1, 196, 1
    ([300, 256, 3], [SIG, SIG], MSE),          # 4, 196, 1
    ([5, 200, 2], [TANH, LIN], MSE),           # 4, 32, 12
    ([65, 70, 16], [SIG, TANH], MSE),          # 2, 32, 1
    ([392, 129, 1], [TANH, SIG], MSE),         # 4, 196, 0
    ([512, 64, 12], [RELU, SOFTMAX], CE),      # 1, 64, 0
    ([200, 40, 5], [SIG, SOFTMAX], CE),        # 1, 32, 1
    ([1000, 30, 4], [TANH, LIN], MSE),         # 1, 128, 1
    ([250, 120, 7], [RELU, SOFTMAX], CE),      # 2, 64, 1
    ([500, 90, 10], [SIG, SOFTMAX], CE),       # 2, 128, 1
    ([128, 250, 16], [TANH, SOFTMAX], CE),     # 4, 64, 0
    ([255, 130, 2], [SIG, SIG], MSE),          # 4, 128, 1
]


@pytest.mark.parametrize("widths,acts,loss", SOLO_SHAPES)
def test_one_workgroup_epochs_match_checker(dnlib, widths, acts, loss):
    """Two-layer nets whose first weight matrix fits one compute unit's registers: a plain pass on one
    workgroup (which leaves the last step's change as velocity), a momentum pass (another kernel), a
    plain pass again."""
    announce("online one-workgroup widths=%s" % (widths,))
    w = synth.make("online", widths, acts, loss, n_samples=40, features="normal", init="xavier_uniform",
                   batch=1, lr=0.005, momentum=0.0, seed=6)
    run_pair(dnlib, w, 40, [0.0, 0.5, 0.0], PERSISTENT, solo=1)


def test_one_workgroup_edges(dnlib):
    announce("online one-workgroup: one sample; fewer samples than the kernel leaves to others; not two layers")
    w = synth.make("online", [784, 128, 10], [SIG, SOFTMAX], CE, n_samples=1, features="normal",
                   init="xavier_uniform", batch=1, lr=0.05, momentum=0.0, seed=2)
    run_pair(dnlib, w, 1, [0.0, 0.0], PERSISTENT, solo=1)
    w = synth.make("online", [5, 200, 2], [TANH, LIN], MSE, n_samples=12, features="normal",
                   init="xavier_uniform", batch=1, lr=0.05, momentum=0.0, seed=2)
    run_pair(dnlib, w, 12, [0.0], PERSISTENT, solo=2)      # 12 samples, all 12 would be left over
    run_pair(dnlib, w, 12, [0.0], 0, solo=2)               # (automatic mode)
    w = synth.make("online", [100, 80, 70, 10], [TANH, TANH, SOFTMAX], CE, n_samples=8, features="normal",
                   init="xavier_uniform", batch=1, lr=0.05, momentum=0.0, seed=2)
    run_pair(dnlib, w, 8, [0.0], PERSISTENT, solo=2)


def test_one_wave_single_sample_and_refusal(dnlib):
    announce("online one-wave: one sample; a 65-wide layer goes elsewhere")
    w = synth.make("online", [12, 20, 4], [TANH, SOFTMAX], CE, n_samples=1, features="normal",
                   init="xavier_uniform", batch=1, lr=0.05, momentum=0.0, seed=2)
    run_pair(dnlib, w, 1, [0.0, 0.5], PERSISTENT, tiny=1)
    w = synth.make("online", [12, 65, 4], [TANH, SOFTMAX], CE, n_samples=8, features="normal",
                   init="xavier_uniform", batch=1, lr=0.05, momentum=0.0, seed=2)
    net = dnlib.Net(w.widths, w.acts, w.loss, 1)
    net.set_all(w.W, w.b)
    X = torch.from_numpy(w.X).to("cuda:0")
    y = torch.from_numpy(w.labels).to("cuda:0")
    assert np.isfinite(net.dn_train_epoch(X, y, 1, w.lr, 0.0))
    assert net.dn_last_schedule() not in (dnlib.DN_SCHED_ONE_WAVE, dnlib.DN_SCHED_ONE_WAVE_REGISTERS)
    net.close()


def test_two_copy_and_general_kernel_agree(dnlib):
    """The same plain pass on both persistent kernels: results within rounding of each other."""
    announce("online two-copy against the general persistent kernel")
    w = synth.make("online", [64, 128, 96, 10], [TANH, TANH, SOFTMAX], CE, n_samples=64, features="normal",
                   init="xavier_uniform", batch=1, lr=0.01, momentum=0.0, seed=9)
    outs = []
    for twin in (1, 0):
        net = dnlib.Net(w.widths, w.acts, w.loss, 1)
        net.set_all(w.W, w.b)
        net.dn_set_option("online_mode", PERSISTENT)
        net.dn_set_option("online_twin", twin)
        X = torch.from_numpy(w.X).to("cuda:0")
        y = torch.from_numpy(w.labels).to("cuda:0")
        loss = net.dn_train_epoch(X, y, 1, w.lr, 0.0)
        outs.append((loss, net.get_all()))
        net.close()
    assert abs(outs[0][0] - outs[1][0]) <= 1e-5 * abs(outs[1][0])
    for a, b in zip(outs[0][1][0] + outs[0][1][1], outs[1][1][0] + outs[1][1][1]):
        assert_close(a, b, 1e-5, "two-copy vs general")


@pytest.mark.parametrize("widths,acts,loss", SHAPES[:6])
def test_per_phase_epochs_match_checker(dnlib, widths, acts, loss):
    announce("online per-phase widths=%s" % (widths,))
    w = synth.make("online", widths, acts, loss, n_samples=48, features="normal", init="xavier_uniform",
                   batch=1, lr=0.005, momentum=0.0, seed=4)
    run_pair(dnlib, w, 48, [0.0, 0.5, 0.5], PER_PHASE)


def test_single_sample_epoch(dnlib):
    announce("online persistent, one sample")
    w = synth.make("online", [12, 20, 4], [TANH, SOFTMAX], CE, n_samples=1, features="normal",
                   init="xavier_uniform", batch=1, lr=0.05, momentum=0.0, seed=2)
    run_pair(dnlib, w, 1, [0.0, 0.5], PERSISTENT, 16)


def test_persistent_is_bitwise_reproducible(dnlib):
    announce("online persistent determinism")
    w = synth.tanh_sweep(1, n_samples=300)
    outs = []
    for _ in range(2):
        net = dnlib.Net(w.widths, w.acts, w.loss, 1)
        net.set_all(w.W, w.b)
        net.dn_set_option("online_mode", PERSISTENT)
        X = torch.from_numpy(w.X).to("cuda:0")
        y = torch.from_numpy(w.labels).to("cuda:0")
        loss = net.dn_train_epoch(X, y, 1, w.lr, w.momentum)
        outs.append((loss, net.get_all()))
        net.close()
    assert outs[0][0] == outs[1][0]
    for a, b in zip(outs[0][1][0] + outs[0][1][1], outs[1][1][0] + outs[1][1][1]):
        assert np.array_equal(a, b)


def test_persistent_not_available_is_reported(dnlib):
    announce("online persistent refused for a wide output layer")
    w = synth.make("online", [8, 12, 300], [TANH, SOFTMAX], CE, n_samples=4, features="normal",
                   init="xavier_uniform", batch=1, lr=0.05, momentum=0.0, seed=2)
    net = dnlib.Net(w.widths, w.acts, w.loss, 1)
    net.set_all(w.W, w.b)
    net.dn_set_option("online_mode", PERSISTENT)
    X = torch.from_numpy(w.X).to("cuda:0")
    y = torch.from_numpy(w.labels).to("cuda:0")
    with pytest.raises(dnlib.DnError) as e:
        net.dn_train_epoch(X, y, 1, 0.05, 0.0)
    assert e.value.status == dnlib.DN_ERR_UNSUPPORTED
    net.dn_set_option("online_mode", 0)          # automatic choice falls back to per-phase launches
    assert np.isfinite(net.dn_train_epoch(X, y, 1, 0.05, 0.0))
    net.close()


# ------------------------------------------------- the named batch-1 workloads ----

def test_iris_like_ten_epochs_persistent(dnlib):
    announce("cfg1 4-16-3 B=1, 10 epochs, persistent")
    w = synth.iris_like()
    run_pair(dnlib, w, w.n_samples, [0.0] * 10, PERSISTENT, tol=1e-3, biases=False)


@pytest.mark.parametrize("form", [1, 2], ids=["registers", "lds"])
def test_iris_like_ten_epochs_one_wave(dnlib, form):
    announce("cfg1 4-16-3 B=1, 10 epochs, one wavefront (the default schedule for this net), form %d" % form)
    w = synth.iris_like()
    run_pair(dnlib, w, w.n_samples, [0.0] * 10, PERSISTENT, tol=1e-3, biases=False, tiny=form)


def test_digits_like_online_prefix_per_phase(dnlib):
    announce("cfg2 784-128-10 B=1, first 1500 steps, per-phase launches")
    w = synth.digits_like_online(n_samples=1500)
    run_pair(dnlib, w, 1500, [0.0], PER_PHASE, tol=1e-3, biases=False)


def test_tanh_sweep_b1_prefix_persistent(dnlib):
    announce("cfg5 1024x4-10 B=1, first 2048 steps, persistent")
    w = synth.tanh_sweep(1, n_samples=2048)
    W, b = run_pair(dnlib, w, 2048, [0.0], PERSISTENT, tol=1e-3, biases=False, twin_expected=True)
    assert abs(float(b[-1].sum())) < 1e-4      # softmax + cross-entropy conserves the output bias sum


@pytest.mark.parametrize("wide", [0, 1])
def test_paper_shape_first_steps(dnlib, wide):
    """340 -> 100000 (tanh) -> 10 softmax, the network of the paper's benchmark application,
    full size, every weight compared after 24 steps: on the general persistent kernel (wide=0) and
    on the kernel for wide hidden layers, which is what the library picks for it."""
    announce("paper shape 340-100000-10 B=1, 24 steps, persistent, wide=%d" % wide)
    w = synth.paper_shape(n_samples=24)
    run_pair(dnlib, w, 24, [0.0], PERSISTENT, tol=1e-4, biases=False, wide=wide)


WIDE_SHAPES = [
    # two layers, inputs a multiple of 4 and at most 384, at most 16 outputs, a hidden layer beyond LDS
    ([340, 100000, 10], [TANH, SOFTMAX], CE),     # the paper's network: rows in LDS, in registers and streamed
    ([340, 99991, 10], [TANH, SOFTMAX], CE),      # a last workgroup with fewer rows than the others
    ([384, 50000, 16], [SIG, SOFTMAX], CE),       # the longest rows and the widest output the kernel takes
    ([128, 90000, 7], [RELU, SIG], MSE),          # short rows: without momentum LDS and registers hold the whole block
    ([64, 700000, 3], [TANH, SIG], MSE),          # many rows per workgroup: most of them streamed
    ([8, 1000000, 2], [TANH, SOFTMAX], CE),       # rows of two float4s: fourteen of a row's sixteen lanes idle
]


@pytest.mark.parametrize("widths,acts,loss", WIDE_SHAPES)
def test_wide_hidden_layer_epochs_match_checker(dnlib, widths, acts, loss):
    """Four passes on the wide-hidden-layer kernel against the checker: plain gradient descent (its last
    step leaves the applied change as velocity), two momentum passes that start from it (rows and
    velocities side by side in LDS and registers), plain gradient descent again."""
    announce("online wide-hidden-layer kernel widths=%s" % (widths,))
    w = synth.make("wide", widths, acts, loss, n_samples=20, features="normal", init="xavier_uniform",
                   batch=1, lr=0.0005, momentum=0.0, seed=6)
    run_pair(dnlib, w, 20, [0.0, 0.5, 0.9, 0.0], PERSISTENT, wide=1)


def test_wide_hidden_layer_kernel_edges(dnlib):
    """One sample (no next sample to take products with); two epochs in a row (the stamps of the
    second continue the first's); and nets the kernel must leave to the others."""
    announce("online wide-hidden-layer kernel: single sample, consecutive epochs, refusals")
    w = synth.make("wide1", [340, 100000, 10], [TANH, SOFTMAX], CE, n_samples=5, features="normal", init="xavier_uniform",
                   batch=1, lr=0.0005, momentum=0.0, seed=8)
    run_pair(dnlib, w, 1, [0.0, 0.5], PERSISTENT, wide=1)
    run_pair(dnlib, w, 5, [0.0, 0.0, 0.5, 0.5], PERSISTENT, wide=1)
    for widths, acts in (([340, 3000, 10], [TANH, SOFTMAX]),            # the hidden layer fits in LDS
                         ([400, 100000, 10], [TANH, SOFTMAX]),          # more than 384 inputs
                         ([338, 100000, 10], [TANH, SOFTMAX]),          # inputs not a multiple of 4
                         ([340, 100000, 24], [TANH, SOFTMAX]),          # more than 16 outputs
                         ([340, 100000, 64, 10], [TANH, TANH, SOFTMAX])):   # three layers
        v = synth.make("notwide", widths, acts, CE, n_samples=2, features="normal", init="xavier_uniform",
                       batch=1, lr=0.0005, momentum=0.0, seed=9)
        net = dnlib.Net(v.widths, v.acts, v.loss, 1)
        net.set_all(v.W, v.b)      # (automatic choice of the schedule: whatever takes the net, only not this kernel)
        net.dn_train_epoch(torch.from_numpy(v.X).to("cuda:0"), torch.from_numpy(v.labels).to("cuda:0"), 1, v.lr, 0.0)
        assert net.dn_last_schedule() not in (dnlib.DN_SCHED_NONE, dnlib.DN_SCHED_WIDE_HIDDEN), widths
        net.close()


# ------------------------------- the paper's per-call execution model (copies around every call) ----

@pytest.mark.parametrize("cols_out,cols_in,pinned", [(10, 1000, False), (340, 1001, True), (3, 4, False), (1, 1, True)])
def test_layer_backward_host_matches_checker(dnlib, cols_out, cols_in, pinned):
    """One sample's backward outputs of one layer.  Reference: the checker's batch-1 gradient of a
    one-layer linear net whose output delta is the given vector (squared error with targets
    chosen so that a - y = deltas), i.e. the pinned rank-1 outer product delta x input."""
    announce("layer_backward_host %dx%d pinned=%s" % (cols_out, cols_in, pinned))
    rng = np.random.default_rng(3)
    deltas = rng.standard_normal(cols_out).astype(np.float32)
    inputs = rng.standard_normal(cols_in).astype(np.float32)
    lr = np.float32(0.05)
    # checker: linear layer, squared error; with W = 0 and b = deltas + onehot(label) the output
    # delta (a - y) f' is exactly `deltas`
    o = Oracle("o32", [cols_in, cols_out], [LIN], MSE)
    b = deltas.astype(np.float64).copy(); b[0] += 1.0
    o.set_params([np.zeros((cols_out, cols_in))], [b])
    o.forward(inputs[None, :]); o.backward(np.zeros(1, dtype=np.int32))
    if not np.allclose(o.deltas()[0][0], deltas, rtol=0, atol=1e-6):       # fp32 rounding of b - 1
        pytest.skip("checker delta does not reproduce the given vector exactly enough")
    Gr, gr = o.get_grads()
    mk = (lambda n: torch.empty(n, dtype=torch.float32).pin_memory()) if pinned else (lambda n: np.empty(n, dtype=np.float32))
    G, dW, dB = mk(cols_out * cols_in), mk(cols_out * cols_in), mk(cols_out)
    d_in = torch.from_numpy(o.deltas()[0][0].copy()) if pinned else o.deltas()[0][0].copy()
    ms = dnlib.dn_layer_backward_host(d_in, torch.from_numpy(inputs) if pinned else inputs, float(lr), G, dW, dB)
    assert all(t >= 0.0 for t in ms)
    G, dW, dB = (np.asarray(t).reshape(-1) for t in (G, dW, dB))
    assert_close(G.reshape(cols_out, cols_in), Gr[0], 1e-6, "gradients")
    assert_close(dW.reshape(cols_out, cols_in), -np.float64(lr) * Gr[0].astype(np.float64), 1e-6, "deltaWeights")
    assert_close(dB, -np.float64(lr) * gr[0].astype(np.float64), 1e-6, "deltaBiases")


# ------------------------------ minibatches of one- and two-layer nets: persistent kernel ----

BATCH_SHAPES = [
    # widths, acts, loss, batch, samples
    ([4, 16, 3], [SIG, SIG], MSE, 7, 30),                  # short last batch (30 = 4 x 7 + 2)
    ([784, 128, 10], [RELU, SOFTMAX], CE, 128, 300),       # the 784-128-10 minibatch workload, short last batch
    ([36, 70, 5], [TANH, LIN], MSE, 33, 99),
    ([300, 10], [SOFTMAX], CE, 64, 200),                   # one layer: input features split over workgroups
    ([12, 1], [SIG], MSE, 5, 23),
    ([2048, 40, 128], [TANH, SOFTMAX], CE, 16, 48),        # widest input and output the kernel takes
    ([8, 1000, 7], [SIG, SOFTMAX], CE, 256, 512),          # many hidden units, largest batch
]


@pytest.mark.parametrize("widths,acts,loss,B,n", BATCH_SHAPES)
@pytest.mark.parametrize("min_tile", [None, 64])
def test_persistent_minibatch_epochs_match_checker(dnlib, widths, acts, loss, B, n, min_tile):
    announce("persistent minibatch widths=%s B=%d min_tile=%s" % (widths, B, min_tile))
    w = synth.make("pbatch", widths, acts, loss, n_samples=n, features="normal", init="xavier_uniform",
                   batch=B, lr=0.02, momentum=0.0, seed=6)
    rng = np.random.default_rng(13)
    w.b = [rng.standard_normal(k).astype(np.float32) * 0.1 for k in w.widths[1:]]
    net = dnlib.Net(w.widths, w.acts, w.loss, B)
    net.set_all(w.W, w.b)
    net.dn_set_option("batch_mode", 2)
    if min_tile is not None:
        net.dn_set_option("online_min_tile", min_tile)
    o = Oracle("o32", w.widths, w.acts, w.loss)
    o.set_params(w.W, w.b)
    X = torch.from_numpy(w.X).to("cuda:0")
    y = torch.from_numpy(w.labels).to("cuda:0")
    for mu in (0.0, 0.7, 0.7):       # plain pass (leaves the last step's velocity), then momentum on top of it
        got = net.dn_train_epoch(X, y, B, w.lr, mu)
        ref, _ = o.train_epoch(w.X, w.labels, B, w.lr, mu)
        assert abs(got - ref) <= 1e-4 * max(abs(ref), 1e-6), (got, ref)
    W, b = net.get_all()
    Wr, br = o.get_params()
    for l in range(net.L):
        assert_close(W[l], Wr[l], 1e-4, "W_%d" % (l + 1))
        assert_close(b[l], br[l], 1e-4, "b_%d" % (l + 1))
    net.close()


def test_tile_option_refits_the_minibatch_kernel(dnlib):
    """Slices as large as "online_min_tile" asks for can exceed LDS: the automatic choice then runs
    the epoch with one launch per product (same result) instead of failing, and a forced
    persistent kernel is refused."""
    announce("persistent minibatch: tile option beyond LDS falls back to launches")
    w = synth.make("batch", [2048, 64, 10], [TANH, SOFTMAX], CE, n_samples=40, features="normal",
                   init="xavier_uniform", batch=8, lr=0.05, momentum=0.9, seed=5)
    X = torch.from_numpy(w.X).to("cuda:0")
    y = torch.from_numpy(w.labels).to("cuda:0")
    outs = []
    for tile in (None, 1 << 22):
        net = dnlib.Net(w.widths, w.acts, w.loss, 8)
        net.set_all(w.W, w.b)
        if tile is not None:
            net.dn_set_option("online_min_tile", tile)
        loss = net.dn_train_epoch(X, y, 8, w.lr, w.momentum)
        assert net.dn_last_schedule() == (dnlib.DN_SCHED_MINIBATCH if tile is None else dnlib.DN_SCHED_LAUNCHES)
        outs.append((loss, net.get_all()))
        if tile is not None:
            net.dn_set_option("batch_mode", 2)
            with pytest.raises(dnlib.DnError) as e:
                net.dn_train_epoch(X, y, 8, w.lr, w.momentum)
            assert e.value.status == dnlib.DN_ERR_UNSUPPORTED
        net.close()
    assert abs(outs[0][0] - outs[1][0]) <= 1e-5 * abs(outs[1][0])
    for a, b in zip(outs[0][1][0] + outs[0][1][1], outs[1][1][0] + outs[1][1][1]):
        assert_close(a, b, 1e-5, "persistent minibatch vs launches")


def test_persistent_minibatch_refused_for_three_layers(dnlib):
    announce("persistent minibatch refused for a three-layer net")
    w = synth.make("pbatch", [8, 12, 9, 4], [TANH, TANH, SOFTMAX], CE, n_samples=8, features="normal",
                   init="xavier_uniform", batch=4, lr=0.05, momentum=0.0, seed=2)
    net = dnlib.Net(w.widths, w.acts, w.loss, 4)
    net.set_all(w.W, w.b)
    net.dn_set_option("batch_mode", 2)
    X = torch.from_numpy(w.X).to("cuda:0")
    y = torch.from_numpy(w.labels).to("cuda:0")
    with pytest.raises(dnlib.DnError) as e:
        net.dn_train_epoch(X, y, 4, 0.05, 0.0)
    assert e.value.status == dnlib.DN_ERR_UNSUPPORTED
    net.dn_set_option("batch_mode", 0)
    assert np.isfinite(net.dn_train_epoch(X, y, 4, 0.05, 0.0))
    net.close()


def test_persistent_minibatch_is_bitwise_reproducible_and_close_to_per_launch(dnlib):
    announce("persistent minibatch determinism, and agreement with one launch per product")
    w = synth.digits_like_minibatch(n_samples=1000)
    outs = []
    for mode in (2, 2, 1):
        net = dnlib.Net(w.widths, w.acts, w.loss, w.batch)
        net.set_all(w.W, w.b)
        net.dn_set_option("batch_mode", mode)
        X = torch.from_numpy(w.X).to("cuda:0")
        y = torch.from_numpy(w.labels).to("cuda:0")
        loss = net.dn_train_epoch(X, y, w.batch, w.lr, w.momentum)
        outs.append((loss, net.get_all()))
        net.close()
    assert outs[0][0] == outs[1][0]
    for a, b in zip(outs[0][1][0] + outs[0][1][1], outs[1][1][0] + outs[1][1][1]):
        assert np.array_equal(a, b)
    for a, b in zip(outs[0][1][0] + outs[0][1][1], outs[2][1][0] + outs[2][1][1]):
        assert_close(a, b, 1e-4, "persistent vs per-launch")


# ------------------------------ minibatches of deeper nets, plain gradient descent: persistent kernel ----

DEEP_SHAPES = [
    # widths, acts, loss, batch, samples
    ([64, 96, 80, 10], [TANH, RELU, SOFTMAX], CE, 8, 44),               # short last batch
    ([20, 40, 32, 52, 24, 6], [TANH, SIG, RELU, TANH, SOFTMAX], CE, 5, 25),
    ([1024, 1024, 1024, 1024, 10], [TANH, TANH, TANH, SOFTMAX], CE, 8, 24),   # the batch-size sweep's net
    ([128, 2048, 64, 3], [SIG, TANH, SIG], MSE, 64, 128),               # widest batch; rows longer than 1024
    ([16, 1000, 24, 128], [RELU, TANH, SOFTMAX], CE, 32, 64),
]


@pytest.mark.parametrize("widths,acts,loss,B,n", DEEP_SHAPES)
@pytest.mark.parametrize("min_tile", [None, 64])
def test_persistent_deep_minibatch_epochs_match_checker(dnlib, widths, acts, loss, B, n, min_tile):
    announce("persistent deep minibatch widths=%s B=%d min_tile=%s" % (widths, B, min_tile))
    w = synth.make("pdeep", widths, acts, loss, n_samples=n, features="normal", init="xavier_uniform",
                   batch=B, lr=0.02, momentum=0.0, seed=8)
    rng = np.random.default_rng(17)
    w.b = [rng.standard_normal(k).astype(np.float32) * 0.1 for k in w.widths[1:]]
    net = dnlib.Net(w.widths, w.acts, w.loss, B)
    net.set_all(w.W, w.b)
    net.dn_set_option("batch_mode", 2)
    if min_tile is not None:
        net.dn_set_option("online_min_tile", min_tile)
    o = Oracle("o32", w.widths, w.acts, w.loss)
    o.set_params(w.W, w.b)
    X = torch.from_numpy(w.X).to("cuda:0")
    y = torch.from_numpy(w.labels).to("cuda:0")
    for _ in range(2):
        got = net.dn_train_epoch(X, y, B, w.lr, 0.0)
        ref, _ = o.train_epoch(w.X, w.labels, B, w.lr, 0.0)
        assert abs(got - ref) <= 1e-4 * max(abs(ref), 1e-6), (got, ref)
    # a momentum pass afterwards (one launch per product) starts from the velocity the plain pass left
    net.dn_set_option("batch_mode", 0)
    got = net.dn_train_epoch(X, y, B, w.lr, 0.5)
    ref, _ = o.train_epoch(w.X, w.labels, B, w.lr, 0.5)
    assert abs(got - ref) <= 1e-4 * max(abs(ref), 1e-6), (got, ref)
    W, b = net.get_all()
    Wr, br = o.get_params()
    for l in range(net.L):
        assert_close(W[l], Wr[l], 1e-4, "W_%d" % (l + 1))
        assert_close(b[l], br[l], 1e-4, "b_%d" % (l + 1))
    net.close()


def test_persistent_deep_minibatch_is_bitwise_reproducible(dnlib):
    announce("persistent deep minibatch determinism")
    w = synth.tanh_sweep(8, n_samples=320)
    outs = []
    for _ in range(2):
        net = dnlib.Net(w.widths, w.acts, w.loss, 8)
        net.set_all(w.W, w.b)
        net.dn_set_option("batch_mode", 2)
        X = torch.from_numpy(w.X).to("cuda:0")
        y = torch.from_numpy(w.labels).to("cuda:0")
        loss = net.dn_train_epoch(X, y, 8, w.lr, 0.0)
        outs.append((loss, net.get_all()))
        net.close()
    assert outs[0][0] == outs[1][0]
    for a, b in zip(outs[0][1][0] + outs[0][1][1], outs[1][1][0] + outs[1][1][1]):
        assert np.array_equal(a, b)


def test_every_benchmark_workload_takes_its_intended_schedule(dnlib):
    """The automatic choice of dn_train_epoch for the shapes bench.py times (a few steps of each):
    a silent fall-back to a slower schedule would still pass every parity test."""
    announce("schedules of the benchmark workloads")
    S = dnlib
    cases = [
        (synth.iris_like(), S.DN_SCHED_ONE_WAVE_REGISTERS),
        (synth.digits_like_online(n_samples=8), S.DN_SCHED_ONE_WORKGROUP),
        (synth.digits_like_minibatch(n_samples=256), S.DN_SCHED_MINIBATCH),
        (synth.wide_relu(n_samples=512), S.DN_SCHED_LAUNCHES),
        (synth.tanh_sweep(1, n_samples=8), S.DN_SCHED_TWO_COPY),
        (synth.tanh_sweep(8, n_samples=32), S.DN_SCHED_MINIBATCH_DEEP),
        (synth.tanh_sweep(32, n_samples=64), S.DN_SCHED_MINIBATCH_DEEP),
        (synth.tanh_sweep(128, n_samples=256), S.DN_SCHED_LAUNCHES),
        (synth.tanh_sweep(512, n_samples=1024), S.DN_SCHED_LAUNCHES),
        (synth.tanh_sweep(2048, n_samples=2048), S.DN_SCHED_LAUNCHES),
        (synth.paper_shape(n_samples=4), S.DN_SCHED_WIDE_HIDDEN),
    ]
    for w, want in cases:
        net = S.Net(w.widths, w.acts, w.loss, w.batch)
        net.set_all(w.W, w.b)
        assert net.dn_last_schedule() == S.DN_SCHED_NONE
        loss = net.dn_train_epoch(torch.from_numpy(w.X).to("cuda:0"), torch.from_numpy(w.labels).to("cuda:0"), w.batch,
                                  w.lr, w.momentum)
        assert np.isfinite(loss), w.name
        assert net.dn_last_schedule() == want, (w.name, net.dn_last_schedule(), want)
        net.close()
