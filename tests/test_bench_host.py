"""Host-side checks of bench.py: the byte counts behind its roofline line and its refusal of
more than one GPU.  No GPU is touched."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import bench          # noqa: E402
import workloads      # noqa: E402


def test_forward_launch_bytes_at_the_headline_shape():
    """700-128-128-20, T=128, B=256: the one forward launch reads the raster (1 byte per element)
    and the three rounded weight matrices (2 bytes), writes V (4) and S (1) of both layers and
    the readout's currents, trace and current gradients (4 bytes per padded class each)."""
    wl = workloads.CONFIGS["shd_ff128"]
    M = 128 * 256
    expect = M * 700 + 2 * (700 * 128 + 128 * 128 + 128 * 20) + 2 * M * 128 * 5 + 3 * M * 24 * 4
    assert expect == 74534912
    assert bench.forward_chain(wl, 1) == ([1, 2], True)
    assert bench.algorithmic_bytes(wl, "lif_forward", 1) == expect


def test_scan_and_weight_gradient_bytes_at_the_headline_shape():
    wl = workloads.CONFIGS["shd_ff128"]
    M = 128 * 256
    # reverse scans read the current gradients above (hi/lo words, padded columns) and V, write dI
    assert bench.algorithmic_bytes(wl, "lif_reverse", 2) == M * (24 * 4 + 128 * 8)
    assert bench.algorithmic_bytes(wl, "lif_reverse", 1) == M * (128 * 4 + 128 * 8)
    # weight gradients: spikes below (1 byte) and current gradients (4) of every layer, dW written
    expect = (M * 700 + M * 128 * 4 + 700 * 128 * 4) + (M * 128 + M * 128 * 4 + 128 * 128 * 4) + \
             (M * 128 + M * 20 * 4 + 128 * 20 * 4)
    assert bench.algorithmic_bytes(wl, "weight_grad", 0) == expect


def test_which_layers_run_as_one_forward_launch():
    """Mirrors the library's rule: feed-forward layers of a multiple of 64 and at most 1024
    neurons (fan-in too) on bf16 products; pairs of exactly 128; the readout rides along below
    128 neurons and at most 32 padded classes."""
    assert bench.forward_chain(workloads.CONFIGS["table1_ff512"], 1) == ([1], False)
    assert bench.forward_chain(workloads.CONFIGS["wide_ff1024"], 2) == ([2], False)
    assert bench.forward_chain(workloads.CONFIGS["deep_rec2048"], 2) == ([], False)
    assert bench.forward_chain(workloads.CONFIGS["shd_rec128"], 1) == ([], False)
    assert bench.forward_chain(workloads.CONFIGS["tiny_ff"], 1) == ([], False)     # fp32 products


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
