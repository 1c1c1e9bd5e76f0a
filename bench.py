#!/usr/bin/env python3
"""Benchmark: training samples/s (forward + backward BPTT + SGD step) of the 700-128-128-20
LIF network at T=128, B=256 on one MI355X, with a roofline line for the dominant kernel, every
launch of the step against its own roof, and the CPU oracle timed beside it.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload shd_ff128] [--no-cpu]

Prints ONE JSON line on stdout; diagnostics go to stderr.

Order of the run: warm-up; the timed region (K steps, nothing bracketed: `value`); then, outside
it, K more steps with the dominant kernel bracketed by HIP events on the library's stream
(`roofline`), a few steps per kernel class and layer (`kernels`), forward + backward without the
optimiser step (`forward_backward_only`), the same shape with fp32 products (`fp32_products`), and
the oracle on the host cores (`cpu_baseline`).
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
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA

# HBM bytes per launch of the dominant kernel as counted by rocprofv3 --pmc (FETCH_SIZE run, then
# WRITE_SIZE run; KiB per dispatch, each scaled by what the same counter reads for the 256 MiB
# device copy this script issues first: FETCH_SIZE reads half the bytes of that copy, WRITE_SIZE
# all of them).  Not measured by this run: the figure is the one in the named summary, which the
# same command produced under the profiler; --traffic replaces it.
PROFILED_TRAFFIC = {           # (workload, kernel, input packed along time)
    ("shd_ff128", "lif_forward", False): ((15841.0 * 2.0 + 50256.0) * 1024.0, "profiles/train_step_shd_ff128.txt"),
    ("shd_ff128", "lif_forward", True): ((4523.0 * 2.0 + 50256.0) * 1024.0, "profiles/train_step_shd_ff128.txt"),
}


def pad8(n):
    return (n + 7) // 8 * 8


def forward_chain(wl, layer):
    """The spiking layers that the forward launch starting at text layer `layer` covers, and whether it
    runs the readout too; ([], False) if that layer runs as separate product and scan launches."""
    L = len(wl.sizes) - 1

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


def reverse_forms_ds(wl, layer):
    """Whether the reverse scan of text layer `layer` forms dS from the current gradients above itself
    (bf16 products, feed-forward, a multiple of 64 wide, at most 128 padded columns above)."""
    L = len(wl.sizes) - 1
    if not (wl.precision == "bf16" and 1 <= layer < L and not wl.recurrent[layer - 1]):
        return False
    return wl.sizes[layer] % 64 == 0 and pad8(wl.sizes[layer + 1]) <= 128


def algorithmic_bytes(wl, kernel, layer, packed=False):
    """HBM bytes one launch of `kernel` for text layer `layer` has to move (compulsory traffic
    of its operands and results, each touched once), in the formats this build stores; `packed`:
    the input raster is read as eight steps per byte."""
    M = wl.T * wl.B
    # rows of the raster as the launches of layer 1 read it (they read the bits themselves where layer 1
    # runs as one launch and, for the weight gradient, the batch is a multiple of 8; else a pre-pass unpacks)
    x_rows = (wl.T + 7) // 8 * wl.B if packed and forward_chain(wl, 1)[0] and wl.B % 8 == 0 else M
    bf = wl.precision == "bf16"
    di = 4                           # current gradients are 4 bytes in memory in both modes
    planes = 1 if bf else 3
    L = len(wl.sizes) - 1
    if kernel == "weight_grad" and layer == 0:   # the merged launch: every layer's spikes below, dI and dW (+ dR)
        return sum(algorithmic_bytes(wl, kernel, l, packed) for l in range(1, L + 1))
    n_in, n_out = wl.sizes[layer - 1], wl.sizes[layer]
    fused_rev = reverse_forms_ds(wl, layer)
    fused_fwd = fused_rev and layer == L - 1 and n_out in (64, 128, 256) and pad8(wl.sizes[L]) <= 32
    chain, with_readout = forward_chain(wl, layer)
    if kernel == "lif_forward" and chain:
        # the launch that starts at `layer`: spikes below (1 B) and W (2 B) read; V (4) and S (1) written per
        # layer; with the readout its currents, its trace and its current gradients (4 B each)
        total = (x_rows if layer == 1 else M) * n_in
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
        return (x_rows if layer == 1 else M) * n_in + M * n_out * di + n_in * n_out * 4 + (M * n_out + n_out * n_out * 4 if rec else 0)
    if kernel == "input_grad":       # read dI and the weight planes, write dS
        return M * n_out * di + planes * 2 * n_in * n_out + M * n_in * 4
    if kernel == "readout_forward":  # J read, Y and dJ written (4 B per padded class)
        return 3 * M * pad8(wl.sizes[L]) * 4
    if kernel == "readout_reverse":
        return M * pad8(wl.sizes[L]) * 4
    raise KeyError(kernel)


def method_flops(wl, kernel, layer):
    """Multiply-add flops of the method (one pass over the operands; a hi+lo or three-piece operand
    is still one product) that one launch of `kernel` for text layer `layer` contains."""
    M = wl.T * wl.B
    L = len(wl.sizes) - 1
    if kernel == "weight_grad" and layer == 0:
        return sum(method_flops(wl, kernel, l) for l in range(1, L + 1))
    n_in, n_out = wl.sizes[layer - 1], wl.sizes[layer]
    if kernel == "lif_forward":
        chain, with_readout = forward_chain(wl, layer)
        f = sum(2 * M * wl.sizes[l - 1] * wl.sizes[l] for l in chain)
        if with_readout or (not chain and reverse_forms_ds(wl, layer) and layer == L - 1
                            and n_out in (64, 128, 256) and pad8(wl.sizes[L]) <= 32):
            f += 2 * M * n_out * wl.sizes[L]
        return f
    if kernel == "lif_reverse":
        return 2 * M * n_out * wl.sizes[layer + 1] if reverse_forms_ds(wl, layer) else 0
    if kernel in ("current_gemm", "input_grad"):
        return 2 * M * n_in * n_out
    if kernel == "weight_grad":
        rec = layer < L and wl.recurrent[layer - 1]
        return 2 * M * n_in * n_out + (2 * M * n_out * n_out if rec else 0)
    if kernel in ("rlif_forward", "rlif_reverse"):
        return 2 * M * n_out * n_out
    return 0


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


def roof_entry(us, nbytes, flops):
    """One launch against its own roof: min(MFMA peak, arithmetic intensity x HBM peak)."""
    e = {"us": round(us, 2)}
    if nbytes:
        e["algorithmic_bytes"] = int(nbytes)
        e["gb_per_s"] = round(nbytes / us / 1e3, 1)
        e["hbm_frac"] = round(nbytes / us / 1e3 / HBM_PEAK_GBS, 3)
    if flops:
        e["method_flops"] = int(flops)
        e["tflop_per_s"] = round(flops / us / 1e6, 1)
        e["mfma_frac"] = round(flops / us / 1e6 / MFMA_BF16_PEAK_TFLOPS, 3)
    if nbytes or flops:
        floor_us = max(nbytes / (HBM_PEAK_GBS * 1e3), flops / (MFMA_BF16_PEAK_TFLOPS * 1e6))
        e["bound"] = "mfma" if flops / (MFMA_BF16_PEAK_TFLOPS * 1e6) > nbytes / (HBM_PEAK_GBS * 1e3) else "hbm"
        e["roof_frac"] = round(floor_us / us, 3)
    return e


def cpu_baseline(wl, inp, budget_s=12.0):
    """The oracle as it stands, whole training steps on the host cores."""
    import numpy as np
    from oracle import snn_oracle as O
    from tests.helpers import net_of
    blas = None
    try:
        from threadpoolctl import threadpool_info
        blas = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        pass
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
    return {"value": wl.B * n / dt, "unit": "samples/s", "cores": int(os.cpu_count() or 1),
            "blas_threads": blas, "kind": "oracle",
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
                    help="HBM bytes per launch of the dominant kernel from rocprofv3 --pmc runs of this command")
    ap.add_argument("--packed", action="store_true",
                    help="feed the raster packed along time (eight spikes per byte) through snn_forward_packed")
    ap.add_argument("--option", action="append", default=[], metavar="NAME=VALUE",
                    help="kernel-selection option of the context (binding.OPTIONS), repeatable")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the per-launch table and the fp32-products run (profiler runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only; --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import workloads
    from paper_2402_18994_amd.binding import from_workload, CALIBRATE_US

    if not torch.cuda.is_available():
        print("bench.py: no HIP device; there is no CPU path to time", file=sys.stderr)
        sys.exit(3)
    wl = workloads.CONFIGS[args.workload]
    inp = workloads.generate(wl)
    dev = torch.device("cuda:0")
    options = {k: int(v) for k, v in (o.split("=", 1) for o in args.option)}
    snn = from_workload(wl, inp, device="cuda:0", options=options or None)
    x = torch.from_numpy(inp.X).to(dev)
    y = torch.from_numpy(inp.labels).to(dev)
    lr = 1e-3
    L = len(wl.sizes) - 1

    if args.packed:
        xp = torch.from_numpy(np.packbits(inp.X, axis=0)).to(dev)

    def step(net=snn):
        if args.packed:
            net.forward_packed(xp, y, want_loss=False)
        else:
            net.forward(x, y, want_loss=False)
        net.backward()
        net.sgd_step(lr)

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

    # ------------------------------------------------------------ the timed region: nothing bracketed
    snn.profile_select("none", 0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    value = wl.B * args.steps / dt

    # ------------------------------------------------------------ kernel durations, outside the timed region
    # An event pair brackets a launch on the library's stream.  What the pair adds to the launch it
    # brackets is measured in this run: the library brackets a one-wavefront kernel that waits
    # CALIBRATE_US on the device clock, once per step, in the middle of the backward pass; the excess
    # over CALIBRATE_US is subtracted from every bracketed launch.  Durations are therefore on the
    # device clock's scale: the calibration kernel counts as exactly its wait (rocprofv3 reports
    # about 1 us more for it, the start and end of a dispatch, which its durations include).
    # (A bracket around nothing costs more than it adds to a launch, so it is only reported.)
    def bracketed(name, layer, n):
        snn.profile_select(name, layer)
        for _ in range(n):
            step()
        ms, launches = snn.profile_read()
        return ms * 1e3, launches                      # microseconds in all, launches in all

    us, n = bracketed("event_pair", 0, 50)
    empty_pair_us = us / max(1, n)
    us, n = bracketed("calibrate", 0, 50)
    cal_raw_us = us / max(1, n)
    pair_us = cal_raw_us - CALIBRATE_US                 # what a bracket adds to the launch inside it

    if args.dominant is None:
        # the launch with the largest share of the step: where the forward pass of all spiking layers and the
        # readout is one launch, that one; else the merged weight-gradient launch
        chain, with_readout = forward_chain(wl, 1)
        args.dominant = "lif_forward:1" if with_readout and len(chain) == L - 1 else "weight_grad:0"
    kname, klayer = args.dominant.split(":")
    klayer = int(klayer)
    blayer = klayer if (klayer or kname == "weight_grad") else 1
    k_us, k_n = bracketed(kname, klayer, args.steps)   # the same number of steps as the timed region
    k_raw_us = k_us / max(1, k_n)
    k_avg_us = max(k_raw_us - pair_us, 1e-3)
    abytes = algorithmic_bytes(wl, kname, blayer, args.packed)
    achieved = abytes / k_avg_us / 1e3 if k_n else 0.0

    kernels = []
    if not args.no_extras:
        todo = [("lif_forward", l) for l in range(1, L)] + [("rlif_forward", l) for l in range(1, L)]
        todo += [("current_gemm", l) for l in range(1, L + 1)] + [("readout_forward", L), ("readout_reverse", L)]
        todo += [("lif_reverse", l) for l in range(L - 1, 0, -1)] + [("rlif_reverse", l) for l in range(L - 1, 0, -1)]
        todo += [("input_grad", l) for l in range(L, 1, -1)] + [("weight_grad", 0), ("grad_reduce", 0), ("sgd", 0)]
        reps = 10
        for name, layer in todo:
            us, n = bracketed(name, layer, reps)
            if not n:
                continue
            per_launch = us / n - pair_us
            nb = fl = 0
            try:
                nb = algorithmic_bytes(wl, name, layer if layer else 0, args.packed) if name not in ("rlif_forward", "rlif_reverse", "grad_reduce", "sgd") else 0
            except KeyError:
                nb = 0
            fl = method_flops(wl, name, layer)
            e = {"kernel": name, "layer": layer, "launches_per_step": n // reps}
            if n // reps > 1:                           # one launch per time step: no roof claimed (latency-bound)
                e["us"] = round(per_launch, 2)
                e["us_per_step_all_launches"] = round(per_launch * (n // reps), 1)
            else:
                e.update(roof_entry(max(per_launch, 1e-3), nb, fl))
            kernels.append(e)
    snn.profile_select("none", 0)

    # Forward + backward alone (the metric as BASELINE words it, without the optimiser step): the
    # backward pass then adds the weight gradients' partial sums itself instead of leaving them to
    # snn_sgd_step, so the gradients are complete when it returns.
    fwd_bwd = None
    if not args.no_extras:
        snn.set_option("defer_reduce", 0)
        nfb = max(20, args.steps // 2)

        def fb():
            if args.packed:
                snn.forward_packed(xp, y, want_loss=False)
            else:
                snn.forward(x, y, want_loss=False)
            snn.backward()
        for _ in range(5):
            fb()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(nfb):
            fb()
        torch.cuda.synchronize()
        dfb = time.perf_counter() - t0
        fwd_bwd = {"value": wl.B * nfb / dfb, "unit": "samples/s", "ms_per_step": dfb / nfb * 1e3, "steps": nfb,
                   "what": "snn_forward + snn_backward, gradients reduced, no snn_sgd_step"}
        snn.set_option("defer_reduce", options.get("defer_reduce", 1))

    loss = snn.forward(x, y)
    spike_rate = [float(snn.get_tensor("spikes", l).mean()) for l in range(1, L)]
    snn.destroy()

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
                   "options": options, "final_loss": loss, "spike_rate": spike_rate,
                   "note": "weights N(0, 1/sqrt(fan_in)) as the configuration states them: the hidden layers are "
                           "almost silent; no kernel branches on a spike, so the time per step does not depend on it"},
        "roofline": {"bound": "hbm", "kernel": f"{kname}" + (f" layer {klayer}" if klayer else " (all layers)"),
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": None, "traffic_source": None,
                     "algorithmic_bytes_per_launch": abytes,
                     "avg_launch_us": k_avg_us, "avg_launch_us_with_events": k_raw_us,
                     "event_pair_overhead_us": pair_us, "launches": k_n,
                     "calibration_kernel_with_events_us": cal_raw_us, "calibration_kernel_waits_us": CALIBRATE_US,
                     "empty_event_pair_us": empty_pair_us,
                     "timed": "HIP events on the library's stream, %d steps after the timed region" % args.steps},
        "gemm_tflops_whole_step": gemm_flops(wl) / (dt / args.steps) / 1e12,
        "kernels": kernels,
    }
    if fwd_bwd:
        out["forward_backward_only"] = fwd_bwd
    if args.traffic is not None:
        out["roofline"]["traffic"] = args.traffic
        out["roofline"]["traffic_source"] = "--traffic"
    elif (wl.name, kname, args.packed) in PROFILED_TRAFFIC and not options:
        out["roofline"]["traffic"], out["roofline"]["traffic_source"] = PROFILED_TRAFFIC[(wl.name, kname, args.packed)]

    if not args.no_extras and wl.precision == "bf16":
        # The same shape with fp32 products (the arithmetic of the paper's timing runs, Section 3.1): every
        # real operand enters the MFMA units as three bfloat16 pieces.
        wl32 = wl.scaled(precision="fp32")
        snn32 = from_workload(wl32, inp, device="cuda:0")
        n32 = max(5, args.steps // 4)
        for _ in range(3):
            step(snn32)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n32):
            step(snn32)
        torch.cuda.synchronize()
        d32 = time.perf_counter() - t0
        out["fp32_products"] = {"value": wl.B * n32 / d32, "unit": "samples/s", "ms_per_step": d32 / n32 * 1e3,
                                "steps": n32, "final_loss": snn32.forward(x, y)}
        snn32.destroy()

    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(wl, inp)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
