"""Shared test helpers: workload -> oracle Net conversion, tiny random nets."""
import numpy as np

from oracle.snn_oracle import Net


def net_of(wl, gemm_round=None):
    rnd = gemm_round if gemm_round is not None else ("bf16" if wl.precision == "bf16" else "none")
    return Net(sizes=tuple(wl.sizes), recurrent=tuple(wl.recurrent), beta=tuple(wl.beta),
               theta=wl.theta, surrogate=wl.surrogate, slope=wl.slope, gemm_round=rnd,
               loss=getattr(wl, "loss", "max"), adapt_decay=getattr(wl, "adapt_decay", None),
               adapt_step=getattr(wl, "adapt_step", None))


def tiny_net(rng, sizes=(5, 4, 6, 3), recurrent=(False, True), T=7, B=2, surrogate="sigmoid",
             slope=3.0, beta=(0.9, 0.8, 0.85), theta=1.0, p=0.5, gain=1.5, gemm_round="none", loss="max",
             adapt_decay=None, adapt_step=None):
    net = Net(sizes=tuple(sizes), recurrent=tuple(recurrent), beta=tuple(beta), theta=theta,
              surrogate=surrogate, slope=slope, gemm_round=gemm_round, loss=loss,
              adapt_decay=adapt_decay, adapt_step=adapt_step)
    L = len(sizes) - 1
    X = (rng.random((T, B, sizes[0])) < p).astype(np.uint8)
    W = [rng.standard_normal((sizes[l], sizes[l + 1])) * gain / np.sqrt(sizes[l]) for l in range(L)]
    R = [rng.standard_normal((sizes[l + 1], sizes[l + 1])) * 0.5 / np.sqrt(sizes[l + 1])
         if recurrent[l] else None for l in range(L - 1)]
    labels = rng.integers(0, sizes[-1], size=B)
    return net, X, W, R, labels
