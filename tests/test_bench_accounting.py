"""Host-side accounting of bench.py: the algorithmic work per kernel launch that the roofline figures divide by, the
rule that withholds the measured-traffic figure once a kernel's sources have changed, and the one-GPU guard."""
import os
import subprocess
import sys

import numpy as np

import bench
from datagen import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# output pixels of the three conv layers for an 84 x 84 input (Section 5: the Nature-DQN setup): (84 - 8) / 4 + 1 = 20,
# (20 - 4) / 2 + 1 = 9, (9 - 3) / 1 + 1 = 7
OUT_PIXELS = {"conv1": 20 * 20, "conv2": 9 * 9, "conv3": 7 * 7}


def macs_per_sample(A):
    """Multiply-accumulates of one forward pass of one sample, layer by layer, from the layer shapes alone."""
    m = {}
    for name, shape, fan_in in synth.layer_shapes(A):
        m[name] = shape[0] * fan_in * OUT_PIXELS.get(name, 1)
    return m


def test_forward_flops_match_the_layer_shapes():
    A, B, G = 18, 256, 2
    m = macs_per_sample(A)
    tower, _ = bench.kernel_work("conv_tower", B, A, G, "bf16")
    assert tower == 2.0 * G * B * (m["conv1"] + m["conv2"] + m["conv3"])
    fc1, _ = bench.kernel_work("fc1_fwd", B, A, G, "bf16")
    assert fc1 == 2.0 * G * B * m["fc1"]
    head, _ = bench.kernel_work("head_td", B, A, G, "bf16")
    assert head == 2.0 * G * B * m["fc2"]


def test_backward_flops_are_the_methods_own_macs():
    # a data gradient and a weight gradient of a layer each cost the layer's forward MACs (no zero-padded taps counted)
    A, B = 18, 128
    m = macs_per_sample(A)
    bwd, _ = bench.kernel_work("conv_tower_bwd", B, A, 2, "bf16")
    assert bwd == 2.0 * B * (m["conv3"] + m["conv2"])
    dg, _ = bench.kernel_work("fc1_dgrad", B, A, 2, "bf16")
    assert dg == 2.0 * B * m["fc1"]
    wg, _ = bench.kernel_work("wgrad_all", B, A, 2, "bf16")
    small, _ = bench.kernel_work("small_grads", B, A, 2, "bf16")
    assert wg - small == 2.0 * B * (m["conv1"] + m["conv2"] + m["conv3"] + m["fc1"])


def test_optimiser_bytes_per_parameter():
    # centered RMSProp reads theta, g, v, m and writes theta, v, m: 28 bytes per fp32 parameter, + 2 for the 16-bit copy
    A = 18
    n = synth.num_params(A)
    assert n == bench.N_PARAMS_BASE + 513 * A
    _, b16 = bench.kernel_work("rmsprop", 32, A, 2, "bf16")
    _, b32 = bench.kernel_work("rmsprop", 32, A, 2, "fp32")
    assert b16 == 30 * n and b32 == 28 * n


def test_roofline_object_fields_and_bound():
    r = bench.roofline_for("rmsprop", 0.0125, 32, 18, 2, "bf16")
    assert r["bound"] == "hbm" and r["unit"] == "GB/s" and r["peak"] == 8000.0
    assert np.isclose(r["achieved"], 30 * synth.num_params(18) / 12.5e-6 / 1e9)
    assert np.isclose(r["frac"], r["achieved"] / r["peak"])
    t = bench.roofline_for("conv_tower", 0.020, 256, 18, 2, "bf16")
    assert t["bound"] == "mfma" and t["unit"] == "TFLOP/s" and t["peak"] == 2500.0
    assert np.isclose(t["frac"], bench.kernel_work("conv_tower", 256, 18, 2, "bf16")[0] / 20e-6 / 1e12 / 2500.0)


def test_measured_traffic_is_withheld_when_sources_changed(monkeypatch):
    assert bench.measured_traffic("no_such_kernel", 32, "bf16") == (None, None)
    key = ("rmsprop", 32, "bf16")
    nbytes, srcs, sha, where = bench.TRAFFIC[key]
    for src in srcs:
        assert os.path.exists(os.path.join(ROOT, src))
    assert os.path.exists(os.path.join(ROOT, where))
    stale = dict(bench.TRAFFIC)
    stale[key] = (nbytes, srcs, "0" * 40, where)
    monkeypatch.setattr(bench, "TRAFFIC", stale)
    assert bench.measured_traffic(*key) == (None, None)


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
