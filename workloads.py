"""Seeded synthetic workloads for the LIF-SNN training path.

This module only draws random inputs (spike rasters, weights, labels) and
names the five benchmark networks.  It holds none of the method's arithmetic:
no membrane update, no surrogate, no loss.  Both the CPU oracle's tests and the
HIP path's tests / bench take their inputs from here, so the two sides see the
same bytes without sharing any code of the method itself.

The rasters stand in for the paper's Spiking Heidelberg Digits workload
(Section 3.2: 700 input channels, feed-forward LIF network of width 128 or
512): 700 channels whose firing rates are drawn once per workload, then
independent Bernoulli draws per time step and sample.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import List, Optional, Tuple

import numpy as np

BASE_SEED = 20240218


@dataclass(frozen=True)
class Workload:
    name: str
    index: int                      # position in the benchmark list (1-based)
    T: int
    B: int
    sizes: Tuple[int, ...]          # N_0 (input) .. N_L (classes)
    recurrent: Tuple[bool, ...]     # one flag per spiking layer (L-1 entries)
    beta: Tuple[float, ...]         # one decay per layer (L entries, last = readout)
    theta: float
    surrogate: str                  # "superspike" | "arctan" | "sigmoid" | "triangular"
    slope: float
    precision: str                  # "fp32" | "bf16"
    rate_lo: float
    rate_hi: float
    rec_gain: float = 0.5           # recurrent weights ~ N(0, rec_gain / sqrt(N))
    loss: str = "max"               # "max" (over time) | "integral" (sum over time) of the readout trace
    adapt_decay: Optional[Tuple[float, ...]] = None   # per spiking layer: decay of the threshold adaptation
    adapt_step: Optional[Tuple[float, ...]] = None    # per spiking layer: rise of the threshold per spike (0: plain LIF)

    @property
    def n_layers(self) -> int:
        return len(self.sizes) - 1

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    def scaled(self, **kw) -> "Workload":
        """A copy with some fields replaced (used for reduced-size test cases)."""
        return replace(self, **kw)


def _wl(name, index, T, B, sizes, recurrent, beta, surrogate, slope, precision,
        rate_lo=0.005, rate_hi=0.04):
    L = len(sizes) - 1
    return Workload(name=name, index=index, T=T, B=B, sizes=tuple(sizes),
                    recurrent=tuple(bool(r) for r in recurrent),
                    beta=tuple([float(beta)] * L), theta=1.0,
                    surrogate=surrogate, slope=float(slope), precision=precision,
                    rate_lo=rate_lo, rate_hi=rate_hi)


CONFIGS = {
    # 1: tiny feed-forward, fp32
    "tiny_ff": _wl("tiny_ff", 1, 32, 16, (100, 64, 10), (0,), 0.9, "arctan", 2.0,
                   "fp32", rate_lo=0.05, rate_hi=0.05),
    # 2: the headline configuration
    "shd_ff128": _wl("shd_ff128", 2, 128, 256, (700, 128, 128, 20), (0, 0), 0.95,
                     "superspike", 25.0, "bf16"),
    # 3: recurrent variant of 2
    "shd_rec128": _wl("shd_rec128", 3, 128, 256, (700, 128, 128, 20), (1, 1), 0.95,
                      "superspike", 25.0, "bf16"),
    # 4: wide feed-forward
    "wide_ff1024": _wl("wide_ff1024", 4, 256, 512, (700, 1024, 1024, 20), (0, 0), 0.95,
                       "superspike", 25.0, "bf16"),
    # 5: deep, long horizon, first hidden layer recurrent
    "deep_rec2048": _wl("deep_rec2048", 5, 512, 128, (700, 2048, 2048, 2048, 20),
                        (1, 0, 0), 0.97, "arctan", 2.0, "bf16"),
    # beyond the five configurations: the shapes of the paper's own timing runs (Table 1: hidden
    # width 128 or 512, rasters of 256 steps, batch 256), with the input statistics of config 2
    "table1_ff128": _wl("table1_ff128", 6, 256, 256, (700, 128, 128, 20), (0, 0), 0.95,
                        "superspike", 25.0, "bf16"),
    "table1_ff512": _wl("table1_ff512", 7, 256, 256, (700, 512, 512, 20), (0, 0), 0.95,
                        "superspike", 25.0, "bf16"),
}
CONFIG_ORDER = ["tiny_ff", "shd_ff128", "shd_rec128", "wide_ff1024", "deep_rec2048"]


@dataclass
class Inputs:
    X: np.ndarray                       # uint8 [T, B, N_0], values 0/1
    W: List[np.ndarray]                 # L arrays float32 [N_l, N_{l+1}]
    R: List[Optional[np.ndarray]]       # L-1 entries: float32 [N, N] (from, to) or None
    labels: np.ndarray                  # int32 [B]
    rates: np.ndarray                   # float64 [N_0] per-channel firing probability


def generate(wl: Workload, w_gain: float = 1.0, seed: Optional[int] = None) -> Inputs:
    """Draw one batch for `wl`.

    Draw order (fixed, so a seed names the bytes): channel rates, X, W^1..W^L,
    recurrent matrices in layer order, labels.  Weight standard deviation is
    w_gain / sqrt(fan_in); recurrent matrices use rec_gain * w_gain / sqrt(N).
    """
    rng = np.random.default_rng(wl.seed if seed is None else seed)
    N0 = wl.sizes[0]
    if wl.rate_lo == wl.rate_hi:
        rates = np.full(N0, wl.rate_lo, dtype=np.float64)
    else:
        rates = rng.uniform(wl.rate_lo, wl.rate_hi, size=N0)
    X = np.empty((wl.T, wl.B, N0), dtype=np.uint8)
    r32 = rates.astype(np.float32)
    for t in range(wl.T):  # per time step, to bound the temporary
        X[t] = rng.random((wl.B, N0), dtype=np.float32) < r32
    W = []
    for l in range(wl.n_layers):
        fan_in = wl.sizes[l]
        W.append((rng.standard_normal((wl.sizes[l], wl.sizes[l + 1]))
                  * (w_gain / np.sqrt(fan_in))).astype(np.float32))
    R: List[Optional[np.ndarray]] = []
    for l, rec in enumerate(wl.recurrent):
        n = wl.sizes[l + 1]
        if rec:
            R.append((rng.standard_normal((n, n))
                      * (wl.rec_gain * w_gain / np.sqrt(n))).astype(np.float32))
        else:
            R.append(None)
    labels = rng.integers(0, wl.sizes[-1], size=wl.B).astype(np.int32)
    return Inputs(X=X, W=W, R=R, labels=labels, rates=rates)
