#!/usr/bin/env python3
"""Benchmark: training samples/s (forward + backward BPTT + SGD step) of the 700-128-128-20
LIF network at T=128, B=256 on one MI355X, with a roofline line for the dominant kernel and
the CPU oracle timed beside it.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload shd_ff128] [--no-cpu]

Prints ONE JSON line on stdout; diagnostics go to stderr.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0

# HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE run, then WRITE_SIZE run; KiB
# per dispatch, each scaled by what the same counter reads for the 256 MiB device copy this
# script issues first: FETCH_SIZE reads half the bytes of that copy, WRITE_SIZE all of them).
# The runs and their figures are in profiles/train_step_shd_ff128.txt.
MEASURED_TRAFFIC = {("shd_ff128", "weight_grad"): (33302.9 * 2.0 + 27136.0) * 1024.0,
                    ("shd_ff128", "lif_forward"): (15234.7 * 2.0 + 50256.0) * 1024.0}

# rocprofv3's duration of the calibration kernel that waits CALIBRATE_US on the device clock: the
# difference is the start and end of a dispatch, which the profiler counts as kernel time.  The
# event timer is calibrated against this figure so that its kernel times are the profiler's.
CALIBRATE_KERNEL_PROFILED_US = 10.96


def algorithmic_bytes(wl, kernel, layer):
    """HBM bytes one launch of `kernel` for text layer `layer` has to move (compulsory traffic
    of its operands and results, each touched once), in the formats this build stores."""
    M = wl.T * wl.B
    bf = wl.precision == "bf16"
    di = 4                           # current gradients are 4 bytes in memory in both modes
    planes = 1 if bf else 3
    L = len(wl.sizes) - 1
    if kernel == "weight_grad" and layer == 0:   # the merged launch: every layer's spikes below, dI and dW (+ dR)
        return sum(algorithmic_bytes(wl, kernel, l) for l in range(1, L + 1))
    n_in, n_out = wl.sizes[layer - 1], wl.sizes[layer]
    pad8 = lambda n: (n + 7) // 8 * 8
    # a feed-forward layer a multiple of 64 wide under a layer of at most 128 padded columns forms dS
    # in its reverse scan from that layer's current gradients (bf16 products)
    fused_rev = (bf and layer < L and not wl.recurrent[layer - 1] and n_out % 64 == 0
                 and pad8(wl.sizes[layer + 1]) <= 128)
    fused_fwd = fused_rev and layer == L - 1 and n_out in (64, 128, 256) and pad8(wl.sizes[L]) <= 32
    # a feed-forward layer of 64..1024 padded neurons runs product and scan as one launch (rasters beyond 256
    # steps: from 64 samples on); two consecutive such layers of exactly 128 neurons share a launch, and the
    # last spiking layer's launch (128 neurons, at most 32 padded classes) runs the whole readout
    chain, with_readout = forward_chain(wl, layer)
    if kernel == "lif_forward" and chain:
        # the launch that starts at `layer`: spikes below (1 B) and W (2 B) read; V (4) and S (1) written per
        # layer; with the readout its currents, its trace and its current gradients (4 B each)
        total = M * n_in
        for l in chain:
            total += 2 * wl.sizes[l - 1] * wl.sizes[l] + M * wl.sizes[l] * (4 + 1)
        if with_readout:
            total += 2 * wl.sizes[chain[-1]] * wl.sizes[L] + 3 * M * pad8(wl.sizes[L]) * 4
        return total
    if kernel == "lif_forward":      # read I (4), write V (4) and S (1 byte) [+ the readout's currents]
        return M * n_out * (4 + 4 + 1) + (M * pad8(wl.sizes[L]) * 4 if fused_fwd else 0)
    if kernel == "lif_reverse":      # read dS (4) [or the current gradients above] and V (4), write dI (4)
        above = pad8(wl.sizes[layer + 1]) if fused_rev else n_out
        return M * (above * 4 + n_out * (4 + di))
    if kernel == "current_gemm":     # read spikes (1 byte) and the weight planes, write I (4)
        return M * n_in + planes * 2 * n_in * n_out + M * n_out * 4
    if kernel == "weight_grad":      # read spikes and dI, write dW (recurrent: own spikes too, and dR)
        rec = layer < L and wl.recurrent[layer - 1]
        return M * n_in + M * n_out * di + n_in * n_out * 4 + (M * n_out + n_out * n_out * 4 if rec else 0)
    if kernel == "input_grad":       # read dI and the weight planes, write dS
        return M * n_out * di + planes * 2 * n_in * n_out + M * n_in * 4
    raise KeyError(kernel)


def forward_chain(wl, layer):
    """The spiking layers that the forward launch starting at text layer `layer` covers, and whether it
    runs the readout too; ([], False) if that layer runs as separate product and scan launches."""
    L = len(wl.sizes) - 1
    pad8 = lambda n: (n + 7) // 8 * 8

    def whole(l):
        n, k = pad8(wl.sizes[l]), wl.sizes[l - 1] if l >= 1 else 0
        return (wl.precision == "bf16" and 1 <= l < L and not wl.recurrent[l - 1] and n % 64 == 0 and n <= 1024
                and pad8(k) <= 1024 and (wl.T <= 256 or wl.B >= 64))
    if not whole(layer):
        return [], False
    chain = [layer]
    if pad8(wl.sizes[layer]) == 128 and whole(layer + 1) and pad8(wl.sizes[layer + 1]) == 128:
        chain.append(layer + 1)
    top = chain[-1]
    return chain, top == L - 1 and pad8(wl.sizes[top]) == 128 and pad8(wl.sizes[L]) <= 32


def gemm_flops(wl):
    M = wl.T * wl.B
    f = 0
    for l in range(1, len(wl.sizes)):
        k, n = wl.sizes[l - 1], wl.sizes[l]
        f += 2 * M * k * n            # current product
        f += 2 * M * k * n            # weight gradient
        if l > 1:
            f += 2 * M * k * n        # input gradient
    for l, rec in enumerate(wl.recurrent):
        if rec:
            n = wl.sizes[l + 1]
            f += 3 * 2 * M * n * n    # S R, g R^T, dR
    return f


def cpu_baseline(wl, inp, budget_s=12.0):
    """The oracle as it stands, whole training steps on the host cores."""
    import numpy as np
    from oracle import snn_oracle as O
    from tests.helpers import net_of
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    net = net_of(wl)
    W, R = [w.astype(np.float64) for w in inp.W], inp.R
    O.train_step(net, inp.X, W, R, inp.labels, 0.01)          # warm-up
    t0 = time.perf_counter()
    n = 0
    while True:
        _, _, W, R = O.train_step(net, inp.X, W, R, inp.labels, 0.01)
        n += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s or n >= 50:
            break
    return {"value": wl.B * n / dt, "unit": "samples/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{n} full training steps (forward+backward+SGD) of the same batch, "
                      f"T={wl.T} B={wl.B}, NumPy float64, {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="shd_ff128")
    ap.add_argument("--dominant", default=None,
                    help="kernel:layer bracketed for the roofline line (layer 0 = every layer)")
    ap.add_argument("--traffic", type=float, default=None,
                    help="measured HBM bytes per launch of the dominant kernel (from the rocprofv3 --pmc runs); "
                         "default: the committed measurement for the default workload and kernel")
    ap.add_argument("--breakdown", action="store_true", help="time every kernel class first (stderr)")
    ap.add_argument("--packed", action="store_true",
                    help="feed the raster packed along time (eight spikes per byte) through snn_forward_packed")
    ap.add_argument("--no-cpu", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only; --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads
    from paper_2402_18994_amd.binding import from_workload, KERNELS, CALIBRATE_US

    if not torch.cuda.is_available():
        print("bench.py: no HIP device; there is no CPU path to time", file=sys.stderr)
        sys.exit(3)
    wl = workloads.CONFIGS[args.workload]
    inp = workloads.generate(wl)
    dev = torch.device("cuda:0")
    snn = from_workload(wl, inp, device="cuda:0")
    x = torch.from_numpy(inp.X).to(dev)
    y = torch.from_numpy(inp.labels).to(dev)
    lr = 1e-3

    if args.packed:
        import numpy as np
        xp = torch.from_numpy(np.packbits(inp.X, axis=0)).to(dev)

    def step():
        if args.packed:
            snn.forward_packed(xp, y, want_loss=False)
        else:
            snn.forward(x, y, want_loss=False)
        snn.backward()
        snn.sgd_step(lr)

    # A plain device copy of known size: the reference the FETCH_SIZE / WRITE_SIZE counters of a
    # rocprofv3 --pmc run are scaled by (256 MiB read, 256 MiB written; the source is pushed out
    # of the caches first by writing 512 MiB elsewhere).
    cal_src = torch.zeros(256 << 20, dtype=torch.uint8, device=dev)
    cal_dst = torch.empty_like(cal_src)
    torch.empty(512 << 20, dtype=torch.uint8, device=dev).zero_()
    cal_dst.copy_(cal_src)
    del cal_src, cal_dst
    torch.cuda.synchronize()
    torch.cuda.empty_cache()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # What a bracket adds to the kernel it times: the library brackets a kernel that waits a
    # known time on the device clock, in the middle of a step; the excess is subtracted from
    # the bracketed launches below.
    snn.profile_select("calibrate", 0)
    for _ in range(50):
        step()
    e_ms, e_n = snn.profile_read()
    ev_overhead_us = e_ms / max(1, e_n) * 1e3 - CALIBRATE_KERNEL_PROFILED_US
    assert abs(CALIBRATE_KERNEL_PROFILED_US - CALIBRATE_US) < 2.0

    # every kernel class once, outside the timed region: microseconds per step, bracket cost removed
    per_class = {}
    for name in KERNELS:
        if name in ("none", "calibrate"):
            continue
        snn.profile_select(name, 0)
        for _ in range(10):
            step()
        ms, n = snn.profile_read()
        if n:
            per_class[name] = {"us_per_step": round((ms * 1e3 - n * ev_overhead_us) / 10, 2), "launches_per_step": n // 10}
    snn.profile_select("none", 0)
    # where the class is one kind of launch with a byte formula and every spiking layer is feed-forward:
    # algorithmic GB/s over all its launches of a step
    L = len(wl.sizes) - 1
    if not any(wl.recurrent):
        class_bytes = {"weight_grad": algorithmic_bytes(wl, "weight_grad", 0),
                       "lif_reverse": sum(algorithmic_bytes(wl, "lif_reverse", l) for l in range(1, L)),
                       "lif_forward": 0}
        l = 1
        while l < L:                                   # one term per forward launch of the class
            class_bytes["lif_forward"] += algorithmic_bytes(wl, "lif_forward", l)
            l += max(1, len(forward_chain(wl, l)[0]))
        for k, nbytes in class_bytes.items():
            if k in per_class and per_class[k]["us_per_step"] > 0:
                per_class[k]["algorithmic_gb_per_s"] = round(nbytes / per_class[k]["us_per_step"] / 1e3, 1)
    if args.breakdown:
        for k, v in per_class.items():
            print(f"[breakdown] {k:16s} {v['us_per_step']:9.1f} us/step over {v['launches_per_step']} launches/step",
                  file=sys.stderr)

    if args.dominant is None:
        # the launch with the largest share of the step: where the forward pass of all spiking layers and the
        # readout is one launch, that one; else the merged weight-gradient launch
        chain, with_readout = forward_chain(wl, 1)
        args.dominant = "lif_forward:1" if with_readout and len(chain) == len(wl.sizes) - 2 else "weight_grad:0"
    kname, klayer = args.dominant.split(":")
    klayer = int(klayer)
    # the weight-gradient products of all layers are one launch (layer 0); for the scans, layers of
    # equal width move equal bytes per launch
    blayer = klayer if (klayer or kname == "weight_grad") else 1
    # The dominant kernel is bracketed by events inside the timed steps, at every 8th step: an
    # event pair costs the stream about 3 us (calibrated above), which at every step would be
    # several per cent of a 90 us step.
    snn.profile_every(max(1, min(8, args.steps // 16)))
    snn.profile_select(kname, klayer)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    k_ms, k_n = snn.profile_read()
    snn.profile_every(1)
    snn.profile_select("none", 0)
    loss = snn.forward(x, y)

    ms_per_step = dt / args.steps * 1e3
    value = wl.B * args.steps / dt
    abytes = algorithmic_bytes(wl, kname, blayer)
    k_raw_us = k_ms / max(1, k_n) * 1e3
    k_avg_s = max(k_raw_us - ev_overhead_us, 1e-3) * 1e-6
    achieved = abytes / k_avg_s / 1e9 if k_n else 0.0
    out = {
        "metric": "training samples/sec (fwd+bwd BPTT + SGD step), T=%d, B=%d" % (wl.T, wl.B),
        "value": value, "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if wl.precision == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: {'-'.join(map(str, wl.sizes))} LIF, T={wl.T}, B={wl.B}, "
                               f"recurrent={list(map(int, wl.recurrent))}, {wl.surrogate}({wl.slope:g}), "
                               f"bf16 products / fp32 state" + (", input packed along time" if args.packed else "")
                               if wl.precision == "bf16" else
                               f"{wl.name}: {'-'.join(map(str, wl.sizes))}, T={wl.T}, B={wl.B}, fp32",
                   "final_loss": loss},
        "roofline": {"bound": "hbm", "kernel": f"{kname}" + (f" layer {klayer}" if klayer else " (all layers)"),
                     "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": args.traffic if args.traffic is not None else MEASURED_TRAFFIC.get((wl.name, kname)),
                     "algorithmic_bytes_per_launch": abytes,
                     "avg_launch_us": k_avg_s * 1e6, "avg_launch_us_with_events": k_raw_us,
                     "event_pair_overhead_us": ev_overhead_us, "launches": k_n},
        "gemm_tflops_whole_step": gemm_flops(wl) / (dt / args.steps) / 1e12,
        "kernel_classes": per_class,
    }
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(wl, inp)
    snn.destroy()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
