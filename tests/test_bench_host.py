"""Host-side checks of bench.py that need no GPU: the workload table, the algorithmic flop and
byte counts the roofline figures are built from, the reader of the committed counter summaries,
and the refusal of more than one GPU."""
import os
import subprocess
import sys

import pytest

import bench

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)
    assert not r.stdout.strip().startswith("{")       # no result line


def test_workload_table_names_every_configuration():
    table = bench.workloads()
    for name in ("cfg1_4_16_3_b1", "cfg2_784_128_10_b1", "cfg3_784_128_10_b128", "cfg4_4096x3_1000_b256",
                 "paper_340_100000_10_b1"):
        assert name in table
    for b in (1, 8, 32, 128, 512, 2048):
        assert "cfg5_1024x4_10_b%d" % b in table
    w = table["cfg5_1024x4_10_b32"][0]()
    assert (w.widths, w.batch, w.n_samples) == ([1024, 1024, 1024, 1024, 10], 32, 16384)
    # features and labels have the shapes the device calls take
    assert w.X.shape == (w.n_samples, 1024) and w.labels.shape == (w.n_samples,)


def test_step_costs_are_the_products_of_the_shapes():
    """cfg4 (4096-4096-4096-1000, batch 256): 2 B n_l n_{l-1} per product, written out."""
    widths, B = [4096, 4096, 4096, 1000], 256
    flops, nbytes = bench.step_costs(widths, B, 0.9)
    pw = 4096 * 4096 + 4096 * 4096 + 1000 * 4096
    assert flops["forward"] == 2.0 * B * pw                          # the last layer is wider than 16: no fused output launch
    assert flops["grad_update"] == 2.0 * B * pw
    assert flops["delta"] == 2.0 * B * (pw - 4096 * 4096)            # no delta below the first layer
    assert "output" not in flops
    assert abs(sum(flops.values()) / 1e9 - 49.24) < 0.01             # GFLOP per step
    p = pw + 4096 + 4096 + 1000
    assert nbytes == 20.0 * p + 4.0 * B * (4096 + 3 * (4096 + 4096 + 1000))
    # a narrow last layer: its forward product is counted with the output launch; plain gradient descent: 12 bytes per parameter
    flops, nbytes = bench.step_costs([1024, 1024, 10], 8, 0.0)
    assert flops["output"] == 2.0 * 8 * 10 * 1024
    assert flops["forward"] == 2.0 * 8 * 1024 * 1024
    assert nbytes == 12.0 * (1024 * 1024 + 10 * 1024 + 1024 + 10) + 4.0 * 8 * (1024 + 3 * (1024 + 10))


def test_counter_summaries_are_read_or_declared_stale():
    """Every committed traffic summary parses; bench.py uses it only while the kernel's source is the
    one the counters were taken from (otherwise the figure is null, never a stale number)."""
    import hashlib
    pdir = os.path.join(ROOT, "profiles")
    names = [f[:-len("_hbm_traffic.txt")] for f in os.listdir(pdir) if f.endswith("_hbm_traffic.txt")]
    assert names
    for wl in names:
        kv = {}
        for line in open(os.path.join(pdir, wl + "_hbm_traffic.txt")):
            if not line.startswith("#") and ":" in line:
                k, v = line.split(":", 1)
                kv[k.strip()] = v.strip()
        for key in ("workload", "kernel", "per", "traffic_bytes", "source_file", "source_sha256"):
            assert key in kv, (wl, key)
        assert kv["workload"] == wl and kv["per"] in ("launch", "step") and float(kv["traffic_bytes"]) > 0
        fresh = hashlib.sha256(open(os.path.join(ROOT, kv["source_file"]), "rb").read()).hexdigest() == kv["source_sha256"]
        got = bench.hbm_traffic(wl)
        if fresh:
            assert got == (float(kv["traffic_bytes"]), kv["per"])
        else:
            assert got is None
    assert bench.hbm_traffic("no_such_workload") is None


def test_peaks_are_the_published_ones():
    assert bench.PEAK_HBM_GBS == 8000.0
    assert bench.PEAK_MFMA_F32_TFLOPS == pytest.approx(256 * 256 * 2.4e9 / 1e12, rel=1e-3)   # 256 CUs x 256 flop per clock
    assert bench.PEAK_VALU_F32_TFLOPS == pytest.approx(256 * 64 * 2 * 2.4e9 / 1e12, rel=1e-3)
