#!/usr/bin/env python3
"""Throughput of dense-network training (forward + back propagation + update)
on one MI355X, with the roofline fraction of the dominant kernel and the CPU
checker timed beside it.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A step is one training step (one batch) of the chosen workload; inputs and
parameters are resident in device memory before the timed region starts.
Protocol: one repeat of K steps straight after the host-side parameter upload
(`value_after_idle`), then untimed steps until the device has worked for
--settle-ms, W warm-up steps, and at least five timed repeats of exactly K
steps, back to back (training simply goes on from one repeat to the next), each
bracketed by device synchronisation; `value` and `ms_per_step` are the median
repeat, `value_min` / `value_max` the slowest and fastest.  The settling is
there because the chip, once it has idled even for the length of a host copy,
runs its next ~30 ms of work some 15 % slower (measured: the same 20 steps take
0.56 ms each straight after a copy and 0.48 ms once 60 steps of any work have
gone before); a training run lives in the settled state, a 10 ms timed region
after a copy does not.  The same steps then run once more with every kernel
launch bracketed by HIP events on the library's stream: the `roofline` object
comes from those durations and from the algorithmic flop counts the library
keeps per launch.  The CPU checker is then timed on a bounded sample of the same
workload with all host threads and with one.  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0        # MI355X HBM3E
PEAK_MFMA_F32_TFLOPS = 157.3  # dense fp32 matrix rate: 256 CUs x 256 flop/clk x 2.4 GHz


def workloads():
    from paper_2001_04206_amd import synth
    w = {
        "cfg1_4_16_3_b1": (synth.iris_like, "latency"),
        "cfg2_784_128_10_b1": (synth.digits_like_online, "hbm"),
        "cfg3_784_128_10_b128": (synth.digits_like_minibatch, "mfma"),
        "cfg4_4096x3_1000_b256": (synth.wide_relu, "mfma"),
        "paper_340_100000_10_b1": (lambda: synth.paper_shape(n_samples=512), "hbm"),
    }
    for b in (1, 8, 32, 128, 512, 2048):
        w["cfg5_1024x4_10_b%d" % b] = ((lambda b=b: synth.tanh_sweep(b)), "hbm" if b <= 32 else "mfma")
    return w


PEAK_VALU_F32_TFLOPS = 78.6  # fp32 vector rate of this build: 256 CUs x 64 lanes x 2 flop x 2.4 GHz (plain v_fma_f32; the
                             # library is compiled without packed fp32 instructions, which would double it)

# A convolutional layer followed by 2x2 max pooling, batch of images resident on the device.
# name: (batch, c_in, h, w, c_out, k, stride, pad)
CONV_WORKLOADS = {
    "conv_32x32x32_to_64_k3_b128": (128, 32, 32, 32, 64, 3, 1, 1),
    "conv_1x28x28_to_6_k5_b128": (128, 1, 28, 28, 6, 5, 1, 0),
}


# A small convolutional classifier trained by plain gradient descent, every layer's forward,
# backward and update on the device: conv 3x3 (ReLU) + 2x2 pooling blocks, then a dense net.
# name: (batch, (c, h, w) of the input, output channels of the blocks, dense widths after the flatten)
CNN_WORKLOADS = {
    "cnn_3x32x32_c32_c64_fc512_10_b128": (128, (3, 32, 32), (32, 64), (512, 10)),
}


def bench_cnn(args, spec):
    """One step = forward, backward and update of the whole classifier on one batch."""
    import numpy as np
    import torch
    from paper_2001_04206_amd import dn
    B, (C0, H0, W0), chans, dense = spec
    RELU, SOFTMAX, CE, K, pad, lr = 3, 4, 1, 3, 1, 0.01
    rng = np.random.default_rng(0)
    Xh = rng.standard_normal((B, C0, H0, W0)).astype(np.float32)
    labels_h = rng.integers(0, dense[-1], B).astype(np.int32)
    dev = lambda a: torch.from_numpy(a).to("cuda:0")
    f32 = dict(dtype=torch.float32, device="cuda:0")
    blocks, cin, h, w = [], C0, H0, W0
    for cout in chans:
        Wh = (rng.standard_normal((cout, cin, K, K)) * np.sqrt(2.0 / (cin * K * K))).astype(np.float32)
        blk = {"cin": cin, "cout": cout, "h": h, "w": w, "Wh": Wh, "bh": np.zeros(cout, dtype=np.float32)}
        blk["W"], blk["b"] = dev(Wh), dev(blk["bh"])
        blk["Y"] = torch.empty(B, cout, h, w, **f32)
        blk["P"] = torch.empty(B, cout, h // 2, w // 2, **f32)
        blk["dP"], blk["dY"], blk["delta"] = torch.empty_like(blk["P"]), torch.empty_like(blk["Y"]), torch.empty_like(blk["Y"])
        blk["dW"], blk["db"] = torch.empty_like(blk["W"]), torch.empty_like(blk["b"])
        blk["ws"] = torch.empty(dn.lib().dn_conv_backward_workspace_bytes(B, cin, h, w, cout, K, K, 1, pad),
                                dtype=torch.uint8, device="cuda:0")
        blocks.append(blk)
        cin, h, w = cout, h // 2, w // 2
    for i in range(1, len(blocks)):
        blocks[i]["dX"] = blocks[i - 1]["dP"]    # a block's input gradient is the pooling gradient of the one before
    blocks[0]["dX"] = None
    flat = cin * h * w
    widths = [flat] + list(dense)
    acts = [RELU] * (len(dense) - 1) + [SOFTMAX]
    Wd = [(rng.standard_normal((widths[l + 1], widths[l])) * np.sqrt(2.0 / widths[l])).astype(np.float32)
          for l in range(len(dense))]
    bd = [np.zeros(widths[l + 1], dtype=np.float32) for l in range(len(dense))]
    net = dn.Net(widths, acts, CE, B)
    net.set_all(Wd, bd)
    X, labels = dev(Xh), dev(labels_h)

    def forward():
        a = X
        for blk in blocks:
            dn.dn_conv_forward(a, blk["W"], blk["b"], blk["Y"], 1, pad, RELU)
            dn.dn_maxpool_forward(blk["Y"], blk["P"], 2, 2)
            a = blk["P"]
        net.dn_forward(a.view(B, flat))

    def backward():
        net.dn_backward(labels)
        net.dn_input_gradient(blocks[-1]["dP"].view(B, flat))
        for i in range(len(blocks) - 1, -1, -1):
            blk = blocks[i]
            a = X if i == 0 else blocks[i - 1]["P"]
            dn.dn_maxpool_backward(blk["Y"], blk["dP"], blk["dY"], 2, 2)
            dn.dn_conv_backward(a, blk["W"], blk["Y"], blk["dY"], blk["delta"], blk["dX"], blk["dW"], blk["db"], 1, pad,
                                RELU, workspace=blk["ws"])

    def update():
        net.dn_update(lr, 0.0)
        for blk in blocks:
            dn.dn_sgd_step(blk["W"], blk["dW"], None, lr, 0.0)
            dn.dn_sgd_step(blk["b"], blk["db"], None, lr, 0.0)

    def step():
        forward(); backward(); update()

    steps = args.steps if args.steps > 0 else 200
    warmup = args.warmup if args.warmup >= 0 else 10
    # The timed steps: the same classifier as one library object (dn_cnn_*), whose epoch call enqueues
    # every step's launches itself; the batch is repeated so that one call covers up to 50 steps.
    cnn = dn.Cnn(C0, H0, W0, [(cout, K, 1, pad, RELU, 2, 2) for cout in chans], dense, acts, CE, B)
    for i, blk in enumerate(blocks):
        cnn.dn_cnn_set_filters(i, blk["Wh"], blk["bh"])
    cnn.dense.set_all(Wd, bd)
    per_call = min(50, max(steps, 1))
    Xrep, yrep = X.repeat(per_call, 1, 1, 1).contiguous(), labels.repeat(per_call).contiguous()

    def run_steps(n):
        done = 0
        while done < n:
            k = min(per_call, n - done)
            cnn.dn_cnn_train_epoch(Xrep, yrep, B, lr, 0.0, n_samples=k * B)
            done += k
    run_steps(max(warmup, 1))
    t_settle = time.perf_counter()
    while (time.perf_counter() - t_settle) * 1e3 < args.settle_ms:     # see main(): a device at work, not one coming out of idle
        run_steps(per_call)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(steps)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    # the same steps driven call by call from here (what the phase times below are taken from)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    wall_composed = time.perf_counter() - t0
    # algorithmic flops of a step: three products per convolution (two for the first block, whose
    # input gradient nobody needs) and three per dense layer (the first one's input gradient feeds the blocks)
    conv_flop = [2.0 * B * b_["cout"] * b_["h"] * b_["w"] * b_["cin"] * K * K for b_ in blocks]
    dense_flop = [2.0 * B * widths[l] * widths[l + 1] for l in range(len(dense))]
    step_flop = sum(f * (2 if i == 0 else 3) for i, f in enumerate(conv_flop)) + 3.0 * sum(dense_flop)
    # the phases bracketed by events on the stream they are enqueued on
    ms = {"forward": 0.0, "backward": 0.0, "update": 0.0}
    roofline = None
    if not args.no_kernel_timing:
        n_ev = min(steps, 50)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        for _ in range(n_ev):
            ev[0].record(); forward()
            ev[1].record(); backward()
            ev[2].record(); update()
            ev[3].record(); torch.cuda.synchronize()
            for i, n in enumerate(ms):
                ms[n] += ev[i].elapsed_time(ev[i + 1]) / n_ev
        bwd_flop = sum(f * (1 if i == 0 else 2) for i, f in enumerate(conv_flop)) + 2.0 * sum(dense_flop)
        ach = bwd_flop / (ms["backward"] * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": "backward phase (loss, dense deltas and gradients, input gradient, pooling and "
                    "convolution gradients: all launches between the forward pass and the update)",
                    "achieved": ach, "peak": PEAK_MFMA_F32_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_MFMA_F32_TFLOPS,
                    "traffic": None, "avg_launch_us": ms["backward"] * 1e3}
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import dn_conv_oracle as co
        from oracle.dn_oracle import Oracle
        o = Oracle("o32", widths, acts, CE)
        o.set_params(Wd, bd)
        n = 1
        while True:   # grow the sample until the checker works for about ten seconds
            t1 = time.perf_counter()
            a, Ys = Xh[:n], []
            for blk in blocks:
                Yo = co.conv_forward("o32", a, blk["Wh"], blk["bh"], 1, pad, RELU)
                Ys.append((a, Yo))
                a = co.maxpool_forward("o32", Yo, 2, 2)
            o.forward(a.reshape(n, flat))
            o.backward(labels_h[:n])
            d = o.input_gradient().reshape(a.shape)
            for blk, (a_in, Yo) in zip(reversed(blocks), reversed(Ys)):
                dYo = co.maxpool_backward("o32", Yo, d, 2, 2)
                _, d, _, _ = co.conv_backward("o32", a_in, blk["Wh"], Yo, dYo, 1, pad, RELU)
            dt = time.perf_counter() - t1
            if dt >= 5.0 or n >= B:
                break
            n = min(B, max(n + 1, int(n * min(8.0, 10.0 / max(dt, 1e-3)))))
        cpu = {"value": n / dt, "unit": "samples/s", "cores": 1, "kind": "oracle",
               "sample": "forward and backward of the first %d images of the same batch (no update), %.1f s" % (n, dt)}
    net.close()
    cnn.close()
    return {"metric": "training samples/sec (fwd+bwd+update)", "value": B * steps / wall,
            "unit": "samples/s", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": wall / steps * 1e3,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": args.workload, "batch": B, "input": [C0, H0, W0], "conv_channels": list(chans),
                       "filter": K, "pad": pad, "pool": "2x2 stride 2", "dense_widths": widths, "activation": "relu",
                       "loss": "softmax + cross-entropy", "lr": lr, "momentum": 0.0},
            "roofline": roofline, "cpu_baseline": cpu,
            "phase_ms": ms, "ms_per_step_call_by_call": wall_composed / steps * 1e3,
            "total_tflops": step_flop * steps / wall / 1e12}


def bench_conv(args, shape):
    """One step = forward and backward of the layer pair on one batch: convolution (ReLU), pooling,
    pooling backward, convolution backward (delta, filter / bias gradients, input gradient)."""
    import numpy as np
    import torch
    from paper_2001_04206_amd import dn
    B, Cin, H, W, Cout, K, stride, pad = shape
    act = 3   # ReLU
    rng = np.random.default_rng(0)
    Xh = rng.standard_normal((B, Cin, H, W)).astype(np.float32)
    Wh = (rng.standard_normal((Cout, Cin, K, K)) * np.sqrt(2.0 / (Cin * K * K))).astype(np.float32)
    bh = np.zeros(Cout, dtype=np.float32)
    Ho, Wo = dn.conv_out_size(H, K, stride, pad), dn.conv_out_size(W, K, stride, pad)
    dPh = rng.standard_normal((B, Cout, Ho // 2, Wo // 2)).astype(np.float32)
    dev = lambda a: torch.from_numpy(a).to("cuda:0")
    X, Wt, b, dP = dev(Xh), dev(Wh), dev(bh), dev(dPh)
    Y = torch.empty(B, Cout, Ho, Wo, device="cuda:0")
    P = torch.empty(B, Cout, Ho // 2, Wo // 2, device="cuda:0")
    dY, delta, dX, dW, db = torch.empty_like(Y), torch.empty_like(Y), torch.empty_like(X), torch.empty_like(Wt), torch.empty_like(b)
    ws = torch.empty(dn.lib().dn_conv_backward_workspace_bytes(B, Cin, H, W, Cout, K, K, stride, pad), dtype=torch.uint8,
                     device="cuda:0")

    def step():
        dn.dn_conv_forward(X, Wt, b, Y, stride, pad, act)
        dn.dn_maxpool_forward(Y, P, 2, 2)
        dn.dn_maxpool_backward(Y, dP, dY, 2, 2)
        dn.dn_conv_backward(X, Wt, Y, dY, delta, dX, dW, db, stride, pad, act, workspace=ws)

    steps = args.steps if args.steps > 0 else 200
    warmup = args.warmup if args.warmup >= 0 else 10
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    # the same steps with the four calls bracketed by events on the stream they are enqueued on
    names = ["conv_forward", "maxpool_forward", "maxpool_backward", "conv_backward"]
    ms = dict.fromkeys(names, 0.0)
    if not args.no_kernel_timing:
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(5)]
        for _ in range(min(steps, 50)):
            ev[0].record(); dn.dn_conv_forward(X, Wt, b, Y, stride, pad, act)
            ev[1].record(); dn.dn_maxpool_forward(Y, P, 2, 2)
            ev[2].record(); dn.dn_maxpool_backward(Y, dP, dY, 2, 2)
            ev[3].record(); dn.dn_conv_backward(X, Wt, Y, dY, delta, dX, dW, db, stride, pad, act, workspace=ws)
            ev[4].record(); torch.cuda.synchronize()
            for i, n in enumerate(names):
                ms[n] += ev[i].elapsed_time(ev[i + 1]) / min(steps, 50)
    fwd_flop = 2.0 * B * Cout * Ho * Wo * Cin * K * K
    roofline = None
    if not args.no_kernel_timing:
        ach = 2.0 * fwd_flop / (ms["conv_backward"] * 1e-3) / 1e12   # filter gradient + input gradient
        # wide 3 x 3 layers take the matrix-core kernels for both gradients, the others plain vector kernels
        on_mfma = Cout >= 32 and Cin >= 8 and Wo >= 12 and K == 3 and stride == 1
        peak = PEAK_MFMA_F32_TFLOPS if on_mfma else PEAK_VALU_F32_TFLOPS
        roofline = {"bound": "mfma" if on_mfma else "alu",
                    "kernel": "conv_backward (delta, filter / bias gradient, chunk sum, input gradient: four launches)",
                    "achieved": ach, "peak": peak, "unit": "TFLOP/s", "frac": ach / peak,
                    "traffic": None, "avg_launch_us": ms["conv_backward"] * 1e3}
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import dn_conv_oracle as co
        n = 1
        while True:   # grow the sample until the checker works for about ten seconds
            t1 = time.perf_counter()
            Yo = co.conv_forward("o32", Xh[:n], Wh, bh, stride, pad, act)
            Po = co.maxpool_forward("o32", Yo, 2, 2)
            dYo = co.maxpool_backward("o32", Yo, dPh[:n], 2, 2)
            co.conv_backward("o32", Xh[:n], Wh, Yo, dYo, stride, pad, act)
            dt = time.perf_counter() - t1
            if dt >= 5.0 or n >= B:
                break
            n = min(B, max(n + 1, int(n * min(8.0, 10.0 / max(dt, 1e-3)))))
        cpu = {"value": n / dt, "unit": "samples/s", "cores": 1, "kind": "oracle",
               "sample": "first %d images of the same batch, %.1f s" % (n, dt)}
    return {"metric": "layer-pair samples/sec (convolution + max pooling, fwd+bwd)", "value": B * steps / wall,
            "unit": "samples/s", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": wall / steps * 1e3,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": args.workload, "batch": B, "c_in": Cin, "h": H, "w": W, "c_out": Cout, "filter": K,
                       "stride": stride, "pad": pad, "pool": "2x2 stride 2", "activation": "relu"},
            "roofline": roofline, "cpu_baseline": cpu,
            "call_ms": ms, "total_tflops": 3.0 * fwd_flop * steps / wall / 1e12}


def step_costs(widths, batch, momentum):
    """Algorithmic flops and bytes of one training step (fp32)."""
    pw = sum(widths[l + 1] * widths[l] for l in range(len(widths) - 1))
    p = pw + sum(widths[1:])
    flops = {
        "forward": 2.0 * batch * pw,
        "delta": 2.0 * batch * (pw - widths[1] * widths[0]),
        "grad_update": 2.0 * batch * pw,
    }
    if widths[-1] <= 16:
        # a last layer of at most 16 outputs: its forward product runs inside the output-error launch
        last = 2.0 * batch * widths[-1] * widths[-2]
        flops["forward"] -= last
        flops["output"] = last
    # weights: forward read + backward read + write (+ velocity read + write);
    # activations / deltas: written once, read by the next product and by the gradient
    per_param = 20.0 if momentum != 0.0 else 12.0
    act_bytes = 4.0 * batch * (widths[0] + 3 * sum(widths[1:]))
    return flops, per_param * p + act_bytes


def hbm_traffic(workload):
    """HBM bytes of the workload's dominant kernel from the committed profiler counter summary
    (profiles/<workload>_hbm_traffic.txt): (bytes, 'launch' | 'step'), or None when there is no
    summary or the kernel's source has changed since the counters were taken."""
    import hashlib
    path = os.path.join(ROOT, "profiles", workload + "_hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    kv = {}
    for line in open(path):
        if not line.startswith("#") and ":" in line:
            k, v = line.split(":", 1)
            kv[k.strip()] = v.strip()
    try:
        src = os.path.join(ROOT, kv["source_file"])
        if hashlib.sha256(open(src, "rb").read()).hexdigest() != kv["source_sha256"]:
            return None
        return float(kv["traffic_bytes"]), kv["per"]
    except (KeyError, OSError, ValueError):
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed training steps (0: one pass over the data)")
    ap.add_argument("--warmup", type=int, default=-1, help="untimed steps (-1: workload default)")
    ap.add_argument("--workload", default="cfg4_4096x3_1000_b256")
    ap.add_argument("--repeats", type=int, default=0,
                    help="timed repeats of the --steps steps, back to back; value is the median "
                         "(0: at least 5, more while a repeat is short, up to 25)")
    ap.add_argument("--settle-ms", type=float, default=100.0,
                    help="untimed steps run for this long before the warm-up steps and before the event-bracketed "
                         "pass, so that the timed steps see the clocks of a device at work (0: none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--per-call-offload", action="store_true",
                    help="instead of a workload: time the paper's execution model (host operands copied in, one "
                         "layer's backward step for one sample, results copied out) on the two layers of its "
                         "340-100000-10 network, and exit")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                    help="instead of a workload: copy MIB mebibytes device to device three times and exit "
                         "(a plain copy of known size, to scale the profiler's HBM byte counters)")
    ap.add_argument("--no-kernel-timing", action="store_true",
                    help="skip the second, event-bracketed pass over the same steps (roofline becomes null)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: the library has no multi-GPU path (run with --gpus 1)")

    import numpy as np
    import torch
    from paper_2001_04206_amd import dn

    if args.calibrate_copy > 0:
        assert torch.cuda.is_available(), "bench.py needs the GPU"
        n = args.calibrate_copy * (1 << 20)
        src = torch.ones(n, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes": n, "copies": 3}))
        return

    if args.per_call_offload:
        assert torch.cuda.is_available(), "bench.py needs the GPU"
        dn.lib()
        calls = args.steps if args.steps > 0 else 20
        out = {"mode": "per-call offload of one layer's backward step (copy in, kernel, copy out)",
               "calls": calls, "host_memory": "pinned", "layers": {}}
        rng = np.random.default_rng(0)
        for name, (co, ci) in {"softmax_output_10x100000": (10, 100000), "fully_connected_100000x340": (100000, 340)}.items():
            pin = lambda a: torch.from_numpy(a).pin_memory()
            d, x = pin(rng.standard_normal(co).astype(np.float32)), pin(rng.random(ci, dtype=np.float32))
            G, dW, dB = (torch.empty(n, dtype=torch.float32).pin_memory() for n in (co * ci, co * ci, co))
            ws = torch.empty(dn.lib().dn_layer_backward_workspace_bytes(co, ci), dtype=torch.uint8, device="cuda:0")
            for _ in range(3):
                dn.dn_layer_backward_host(d, x, 0.01, G, dW, dB, ws)
            t = np.array([dn.dn_layer_backward_host(d, x, 0.01, G, dW, dB, ws) for _ in range(calls)])
            t0 = time.perf_counter()
            for _ in range(calls):
                dn.dn_layer_backward_host(d, x, 0.01, G, dW, dB, ws)
            wall = (time.perf_counter() - t0) / calls
            mean = t.mean(axis=0)
            out["layers"][name] = {"copy_in_ms": float(mean[0]), "kernel_ms": float(mean[1]), "copy_out_ms": float(mean[2]),
                                   "wall_ms_per_call": wall * 1e3, "bytes_out": 4 * (2 * co * ci + co),
                                   "kernel_GBps": 4 * (2 * co * ci) / (mean[1] * 1e-3) / 1e9,
                                   "copy_out_GBps": 4 * (2 * co * ci + co) / (mean[2] * 1e-3) / 1e9}
        print(json.dumps(out))
        return

    if args.workload in CONV_WORKLOADS:
        assert torch.cuda.is_available(), "bench.py needs the GPU"
        dn.lib()
        print(json.dumps(bench_conv(args, CONV_WORKLOADS[args.workload])))
        return

    if args.workload in CNN_WORKLOADS:
        assert torch.cuda.is_available(), "bench.py needs the GPU"
        dn.lib()
        print(json.dumps(bench_cnn(args, CNN_WORKLOADS[args.workload])))
        return

    table = workloads()
    if args.workload not in table:
        sys.exit("unknown workload %r; choose from %s"
                 % (args.workload, ", ".join(sorted(list(table) + list(CONV_WORKLOADS) + list(CNN_WORKLOADS)))))
    make, bound = table[args.workload]
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dn.lib()   # fails loudly if libdn.so has not been built

    t0 = time.time()
    w = make()
    B, N = w.batch, w.n_samples
    steps_per_pass = (N + B - 1) // B
    steps = args.steps if args.steps > 0 else steps_per_pass
    warmup = args.warmup if args.warmup >= 0 else min(steps_per_pass, 100 if B == 1 else 16)
    sys.stderr.write("[bench] %s: %d samples, batch %d, %d timed steps, %d warm-up (inputs drawn in %.1fs)\n"
                     % (w.name, N, B, steps, warmup, time.time() - t0))
    sys.stderr.flush()

    torch.cuda.set_device(0)
    th = time.time()
    X = torch.from_numpy(w.X).to("cuda:0")
    y = torch.from_numpy(w.labels).to("cuda:0")
    torch.cuda.synchronize()
    h2d_s = time.time() - th
    net = dn.Net(w.widths, w.acts, w.loss, B)

    def run(n_steps):
        """n_steps training steps, walking the data set in order and wrapping around."""
        done, dev_ms, loss = 0, 0.0, float("nan")
        while done < n_steps:
            k = min(n_steps - done, steps_per_pass)
            n = min(k * B, N)
            loss = net.dn_train_epoch(X, y, B, w.lr, w.momentum, n_samples=n)
            dev_ms += net.dn_last_epoch_ms()
            done += k
        return dev_ms, loss

    def settle():
        """Untimed steps until the device has been at work for --settle-ms."""
        t = time.perf_counter()
        while (time.perf_counter() - t) * 1e3 < args.settle_ms:
            run(min(steps_per_pass, 64))
            torch.cuda.synchronize()

    samples = sum(min(B, N - ((s % steps_per_pass) * B)) for s in range(steps))
    # the requested steps once, straight after the upload of the parameters (a device that has idled)
    net.set_all(w.W, w.b)
    run(1)                                   # first-launch set-up (kernel attributes, code upload) stays out of it
    net.set_all(w.W, w.b)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    run(steps)
    torch.cuda.synchronize()
    wall_idle = time.perf_counter() - t1

    net.set_all(w.W, w.b)
    settle()
    if warmup:
        run(warmup)
    net.dn_set_option("time_kernels", 0)
    # Timed repeats: each runs exactly `steps` steps, bracketed by device synchronisation on both
    # sides; they follow one another without a host copy between them (the parameters go on from
    # where the last repeat left them, the samples start over); the figure reported is the median.
    walls, dev_mss, loss = [], [], float("nan")
    repeats = args.repeats if args.repeats > 0 else 5
    r = 0
    while r < repeats:
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        dev_ms_r, loss = run(steps)
        torch.cuda.synchronize()
        walls.append(time.perf_counter() - t1)
        dev_mss.append(dev_ms_r)
        r += 1
        if r == 1 and args.repeats <= 0 and walls[0] < 0.1:      # short repeats: take more of them (about half a second in all)
            repeats = max(5, min(25, int(0.5 / max(walls[0], 1e-6))))
    order = sorted(range(len(walls)), key=lambda i: walls[i])
    mid = order[len(order) // 2]
    wall, dev_ms = walls[mid], dev_mss[mid]
    value = samples / wall

    # The same steps once more with every kernel launch bracketed by HIP events on the library's
    # stream: per-kernel durations for the roofline.  (Kept out of the throughput figure above: an
    # event pair per launch costs microseconds, which is most of a step for the small workloads.)
    if not args.no_kernel_timing:
        settle()
        net.dn_set_option("time_kernels", 1)
        torch.cuda.synchronize()
        run(steps)
        torch.cuda.synchronize()
        net.dn_set_option("time_kernels", 0)

    flops, step_bytes = step_costs(w.widths, B, w.momentum)
    schedule = net.dn_last_schedule()
    roofline = None
    classes = {}
    if not args.no_kernel_timing:
        for cid, cname in enumerate(dn.KERNEL_CLASS_NAMES):
            ms, n = net.dn_kernel_time(cid)
            if n:
                classes[cname] = {"ms": ms, "launches": n, "flop": net.dn_kernel_flops(cid)}
        # per-launch figures of the last dn_train_epoch call (one pass or the remainder)
        last_steps = steps % steps_per_pass or min(steps, steps_per_pass)
        if "online" in classes:      # a persistent whole-epoch kernel ran: no matrix instructions, one launch
            bound = "hbm"
        if bound == "mfma":
            # the class of matrix-product launches with the largest summed time; its algorithmic flops
            # (2 M N K per product, counted by the library per timed launch) / that time
            dom = max((c for c in classes if classes[c]["flop"] > 0 and c != "output"), key=lambda c: classes[c]["ms"],
                      default=None)
            if dom:
                per_launch_ms = classes[dom]["ms"] / classes[dom]["launches"]
                flop_per_launch = classes[dom]["flop"] / classes[dom]["launches"]
                ach = flop_per_launch / (per_launch_ms * 1e-3) / 1e12
                roofline = {"bound": "mfma", "kernel": dom, "achieved": ach, "peak": PEAK_MFMA_F32_TFLOPS,
                            "unit": "TFLOP/s", "frac": ach / PEAK_MFMA_F32_TFLOPS, "traffic": None,
                            "avg_launch_us": per_launch_ms * 1e3, "launches": classes[dom]["launches"]}
        else:
            # every kernel of a step streams the parameters, so the whole step is the unit:
            # algorithmic bytes of the timed steps / summed duration of their launches
            total_ms = sum(c["ms"] for c in classes.values())
            if "online" in classes:          # one persistent launch covers the whole pass
                timed_steps = last_steps
            else:                            # per-launch events stop after a fixed number of launches
                timed_steps = min(last_steps, classes["output"]["launches"])   # one output-error launch per step
            if total_ms > 0:
                ach = step_bytes * timed_steps / (total_ms * 1e-3) / 1e9
                roofline = {"bound": "hbm", "kernel": dn.SCHEDULE_KERNELS.get(schedule, "persistent kernel") if "online" in classes
                            else "all kernels of a step", "achieved": ach,
                            "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS, "traffic": None,
                            "avg_launch_us": total_ms * 1e3 / sum(c["launches"] for c in classes.values()),
                            "timed_steps": timed_steps}

    if roofline is not None:
        t = hbm_traffic(args.workload)
        if t is not None:     # per launch, like `achieved`: a persistent launch covers timed_steps steps
            roofline["traffic"] = t[0] * (roofline.get("timed_steps", 1) if t[1] == "step" else 1)
            if roofline["bound"] == "hbm" and roofline.get("avg_launch_us"):
                # what the counters saw moving, as a rate: `achieved` is the algorithmic figure (three
                # trips per weight and step at batch 1), which a kernel that keeps weights on chip or
                # fuses two of the trips undercuts -- it can then exceed the peak; this one cannot
                roofline["traffic_rate"] = roofline["traffic"] / (roofline["avg_launch_us"] * 1e-6) / 1e9
                roofline["traffic_frac"] = roofline["traffic_rate"] / PEAK_HBM_GBS

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import dn_oracle
        o = dn_oracle.Oracle("o32", w.widths, w.acts, w.loss)
        o.set_params(w.W, w.b)
        total_flop_per_sample = sum(flops.values()) / B
        budget_flop = 1.0e11                      # ~10-30 s of the checker on a host of this class
        n_cpu = int(max(B, min(N, budget_flop / total_flop_per_sample)) // B * B) or B
        n_cpu = min(n_cpu, N)
        tc = time.perf_counter()
        o.train_epoch(w.X[:n_cpu], w.labels[:n_cpu], B, w.lr, w.momentum)
        dtc = time.perf_counter() - tc
        cpu = {"value": n_cpu / dtc, "unit": "samples/s", "cores": dn_oracle.threads(), "kind": "oracle",
               "sample": "first %d samples (%d steps) of the same workload, %.1f s" % (n_cpu, (n_cpu + B - 1) // B, dtc)}
        # the same checker on one thread, on about a sixteenth of that work: whole steps where a step
        # is small, else the first samples as one short batch (the per-sample work is the same)
        all_threads = dn_oracle.threads()
        n_one = n_cpu if dtc < 2.0 else max(1, n_cpu // 16)     # a sample that took under two seconds is taken whole
        n_one = n_one // B * B if n_one >= B else n_one
        o.set_params(w.W, w.b)
        dn_oracle.set_threads(1)
        tc = time.perf_counter()
        o.train_epoch(w.X[:n_one], w.labels[:n_one], B, w.lr, w.momentum)
        dt1 = time.perf_counter() - tc
        dn_oracle.set_threads(all_threads)
        cpu["value_1thread"] = n_one / dt1
        cpu["sample_1thread"] = ("first %d samples (%d steps), %.1f s" % (n_one, n_one // B, dt1) if n_one >= B
                                 else "first %d samples as one short batch, %.1f s" % (n_one, dt1))

    out = {
        "metric": "training samples/sec (fwd+bwd+update)", "value": value, "unit": "samples/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": wall * 1e3 / steps,
        "repeats": len(walls), "value_min": samples / max(walls), "value_max": samples / min(walls),
        "ms_per_step_min": min(walls) * 1e3 / steps, "ms_per_step_max": max(walls) * 1e3 / steps,
        "settle_ms": args.settle_ms, "value_after_idle": samples / wall_idle,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": args.workload, "widths": w.widths, "batch": B, "lr": w.lr,
                   "momentum": w.momentum, "samples": N},
        "roofline": roofline, "cpu_baseline": cpu,
        "device_ms_per_step": dev_ms / steps, "kernel_classes": classes,
        "total_tflops": sum(flops.values()) * steps / wall / 1e12,
        "step_algorithmic_bytes": step_bytes, "final_loss": loss, "h2d_seconds_once": h2d_s,
    }
    net.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
