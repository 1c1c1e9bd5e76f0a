"""Scalar brute-force version of the oracle (pure Python floats, nested loops).

TEST INFRASTRUCTURE ONLY; for tiny networks.  It restates Eq. 1-2, the LI
readout, the cross-entropy (max over time or summed over time) and the reverse sweep one number at a
time, with explicit indices, so that an indexing or transposition slip in the
vectorised oracle shows up as a mismatch.  Unrounded arithmetic only.
"""
from __future__ import annotations

import math


def _surr(kind, k, x):
    if kind == "superspike":
        return 1.0 / (1.0 + k * abs(x)) ** 2
    if kind == "arctan":
        return (k / 2.0) / (1.0 + (math.pi * k * x / 2.0) ** 2)
    if kind == "sigmoid":
        s = 1.0 / (1.0 + math.exp(-k * x))
        return k * s * (1.0 - s)
    if kind == "triangular":
        return max(0.0, 1.0 - abs(k * x))
    if kind == "boxcar":
        return 0.5 if abs(k * x) <= 1.0 else 0.0
    if kind == "ste":
        return 1.0
    raise ValueError(kind)


def run(sizes, recurrent, beta, theta, surrogate, slope, X, W, R, labels, loss_kind="max",
        adapt_decay=None, adapt_step=None):
    """Forward + backward.  X[t][b][i] in {0,1}; W[l][i][j]; R[l][i][j] or None.

    beta[l] is a number or a list with one decay per neuron of layer l.
    loss_kind: "max" (logit = largest readout value over time, gradient to the first step
    that reaches it) or "integral" (logit = the readout trace summed over time, so every
    step receives the logit's gradient).
    adapt_decay, adapt_step: per spiking layer, the adaptive threshold theta + A with
    A' = adapt_decay * A + adapt_step * spike (None: plain LIF).

    Returns a dict with V, S (per spiking layer, [t][b][n]), Y [t][b][c], loss,
    dW (per layer [i][j]), dR and dbeta (per layer, per neuron).
    """

    def bt(l, n):
        return beta[l][n] if isinstance(beta[l], (list, tuple)) else beta[l]

    T = len(X)
    B = len(X[0])
    L = len(sizes) - 1
    C = sizes[L]
    H = L - 1                                    # number of spiking layers

    gam = list(adapt_decay) if adapt_decay is not None else [0.0] * H
    kap = list(adapt_step) if adapt_step is not None else [0.0] * H
    V = [[[[0.0] * sizes[l + 1] for _ in range(B)] for _ in range(T)] for l in range(H)]
    S = [[[[0.0] * sizes[l + 1] for _ in range(B)] for _ in range(T)] for l in range(H)]
    A = [[[[0.0] * sizes[l + 1] for _ in range(B)] for _ in range(T)] for l in range(H)]
    Y = [[[0.0] * C for _ in range(B)] for _ in range(T)]

    # ---------------- forward, one sample at a time ----------------
    for b in range(B):
        v = [[0.0] * sizes[l + 1] for l in range(H)]
        adp = [[0.0] * sizes[l + 1] for l in range(H)]
        y = [0.0] * C
        for t in range(T):
            below = [float(X[t][b][i]) for i in range(sizes[0])]
            for l in range(H):
                n_out = sizes[l + 1]
                spikes = [1.0 if v[l][n] - (theta + adp[l][n]) > 0.0 else 0.0 for n in range(n_out)]
                new_v = [0.0] * n_out
                for n in range(n_out):
                    cur = 0.0
                    for i in range(sizes[l]):
                        cur += below[i] * W[l][i][n]
                    rec = 0.0
                    if R[l] is not None:
                        for i in range(n_out):
                            rec += spikes[i] * R[l][i][n]
                    new_v[n] = bt(l, n) * v[l][n] + cur + rec - (theta + adp[l][n]) * spikes[n]
                    V[l][t][b][n] = v[l][n]
                    S[l][t][b][n] = spikes[n]
                    A[l][t][b][n] = adp[l][n]
                v[l] = new_v
                adp[l] = [gam[l] * adp[l][n] + kap[l] * spikes[n] for n in range(n_out)]
                below = spikes
            for c in range(C):
                j = 0.0
                for i in range(sizes[L - 1]):
                    j += below[i] * W[L - 1][i][c]
                y[c] = bt(L - 1, c) * y[c] + j
                Y[t][b][c] = y[c]

    # ---------------- loss ----------------
    if loss_kind == "integral":
        z = [[0.0] * C for _ in range(B)]
        for b in range(B):
            for c in range(C):
                for t in range(T):
                    z[b][c] += Y[t][b][c]
        tstar = [[0] * C for _ in range(B)]
    else:
        z = [[max(Y[t][b][c] for t in range(T)) for c in range(C)] for b in range(B)]
        tstar = [[min(t for t in range(T) if Y[t][b][c] == z[b][c]) for c in range(C)]
                 for b in range(B)]
    loss = 0.0
    dz = [[0.0] * C for _ in range(B)]
    for b in range(B):
        m = max(z[b])
        den = sum(math.exp(z[b][c] - m) for c in range(C))
        loss += (m + math.log(den) - z[b][labels[b]]) / B
        for c in range(C):
            dz[b][c] = (math.exp(z[b][c] - m) / den - (1.0 if c == labels[b] else 0.0)) / B

    # ---------------- backward, one sample at a time ----------------
    dW = [[[0.0] * sizes[l + 1] for _ in range(sizes[l])] for l in range(L)]
    dR = [None if R[l] is None else [[0.0] * sizes[l + 1] for _ in range(sizes[l + 1])]
          for l in range(H)]
    dbeta = [[0.0] * sizes[l + 1] for l in range(L)]
    for b in range(B):
        hy = [0.0] * C
        g = [[0.0] * sizes[l + 1] for l in range(H)]          # dL/dV_{t+1}
        ga = [[0.0] * sizes[l + 1] for l in range(H)]         # dL/dA_{t+1}
        for t in range(T - 1, -1, -1):
            for c in range(C):
                into_y = dz[b][c] if (loss_kind == "integral" or tstar[b][c] == t) else 0.0
                hy[c] = bt(L - 1, c) * hy[c] + into_y
                if t >= 1:
                    dbeta[L - 1][c] += hy[c] * Y[t - 1][b][c]
            below = S[H - 1][t][b] if H >= 1 else [float(x) for x in X[t][b]]
            for i in range(sizes[L - 1]):
                for c in range(C):
                    dW[L - 1][i][c] += below[i] * hy[c]
            d_s = [sum(hy[c] * W[L - 1][i][c] for c in range(C)) for i in range(sizes[L - 1])]
            for l in range(H - 1, -1, -1):
                n_out = sizes[l + 1]
                d_i = list(g[l])
                src = S[l - 1][t][b] if l >= 1 else [float(x) for x in X[t][b]]
                for i in range(sizes[l]):
                    for n in range(n_out):
                        dW[l][i][n] += src[i] * d_i[n]
                new_g = [0.0] * n_out
                new_ga = [0.0] * n_out
                for n in range(n_out):
                    thr = theta + A[l][t][b][n]
                    q = d_s[n] - thr * g[l][n] + kap[l] * ga[l][n]
                    if R[l] is not None:
                        for m_ in range(n_out):
                            q += g[l][m_] * R[l][n][m_]
                            # and the recurrent weight gradient, entry (n -> m_)
                        for m_ in range(n_out):
                            dR[l][n][m_] += S[l][t][b][n] * d_i[m_]
                    dbeta[l][n] += g[l][n] * V[l][t][b][n]
                    sg = _surr(surrogate, slope, V[l][t][b][n] - thr)
                    new_g[n] = bt(l, n) * g[l][n] + sg * q
                    new_ga[n] = gam[l] * ga[l][n] - S[l][t][b][n] * g[l][n] - sg * q
                if l >= 1:
                    d_s = [sum(d_i[n] * W[l][i][n] for n in range(n_out)) for i in range(sizes[l])]
                g[l] = new_g
                ga[l] = new_ga
    return dict(V=V, S=S, A=A, Y=Y, z=z, tstar=tstar, loss=loss, dz=dz, dW=dW, dR=dR, dbeta=dbeta)
