"""CPU oracle for surrogate-gradient BPTT through a layered LIF network.

TEST INFRASTRUCTURE ONLY.  This is a plain, slow, float64 NumPy statement of
what the training step computes.  Only the tests, the smoke check and the
benchmark's `cpu_baseline` leg may import it; the product path never does, and
it shares no code with the HIP kernels.

The network is the stack the paper builds in its Section 2.1.2 network listing:
  Linear(no bias) -> LIF -> ... -> Linear(no bias) -> LI readout
unrolled over time exactly like a deep RNN: at every time step the input passes
through all layers in order.  The backward pass is the reverse sweep that
reverse-mode differentiation of that unrolled loop performs, with the
derivative of the Heaviside step replaced by a surrogate (Section 2.1.1).

Readings of points the paper leaves open (each also listed in the design
notes of this repository):
  * Heaviside at exactly zero: no spike (spike iff V - theta > 0).
  * Spike is taken from the carried-in potential, then the potential is
    updated (Eq. 1 uses V_t, Eq. 2 produces V_{t+1}); initial state zero.
  * Reset is theta * S_t (Eq. 2) and is NOT detached in the backward pass:
    the LIF listing uses the same traced `spikes` value for output and reset.
  * beta: Net.beta holds one scalar per layer; `betas` (one array per layer,
    one entry per neuron / class) overrides it.  The LIF listing holds beta as
    a per-neuron parameter clipped to [0, 1] inside the forward function; here
    the parameter itself is kept in [0, 1]: `sgd_step` clips after the update
    (the forward values are the same; a parameter pushed outside the interval
    comes back instead of staying there with zero gradient).
  * LI readout: y_t = beta_o * y_{t-1} + J_t, y_{-1} = 0, the updated y_t is
    what is emitted; no threshold, no reset.
  * Loss "max": softmax cross-entropy on z[b,c] = max_t y_t[b,c], mean over the
    batch; the sub-gradient of the max goes to the FIRST maximising step.
  * Loss "integral" (Section 2.1.3 names an integral cross-entropy for rate-coded
    objectives and gives no formula): the same cross-entropy on the readout
    trace summed over time, z[b,c] = sum_t y_t[b,c]; no label smoothing.
  * Arctan surrogate: (k/2) / (1 + (pi k x / 2)^2), the derivative of
    (1/pi) arctan(pi k x / 2) + 1/2.  The paper only names it.
  * Boxcar surrogate (only named): 1/2 where |k x| <= 1, else 0 (a box of
    width 2/k and height 1/2).  Straight-through estimator (the default the
    paper states for its activation builder): derivative 1 everywhere.
  * Recurrent LIF: V_{t+1} = beta V_t + I_t + S_t R - theta S_t with S_t the
    spikes just emitted from V_t; R is [from, to].  The paper only mentions
    recurrent models.
  * Neurons with an adaptive firing threshold (Section 2.1.2 names them and gives no
    equations): every neuron carries a second state A_t >= 0, A_0 = 0, that raises its
    threshold, theta_t = theta + A_t.  Eq. 1-2 are applied with the threshold in force:
        S_t = H(V_t - theta_t),   V_{t+1} = beta V_t + X_t - theta_t S_t,
    and each spike raises the threshold by `adapt_step`, which then decays:
        A_{t+1} = adapt_decay A_t + adapt_step S_t.
    adapt_step = 0 is the plain LIF neuron.  The reverse sweep differentiates through both
    states (A_t reaches the loss through the spike decision, the reset magnitude and
    A_{t+1}); neither term is detached.  adapt_decay and adapt_step are fixed per layer.
  * "bf16" GEMM mode: the weight matrices (W and R) are rounded to bfloat16
    (round to nearest even) wherever they enter a product, forward and
    backward; 0/1 spikes are exact; all state, the surrogate, the loss, the
    current gradients and all accumulation stay unrounded.  (The device carries
    the current gradients into its bfloat16 products as a hi+lo pair, which
    loses less than 2^-16 relative; a single rounding of those operands was
    tried first and rejected: values next to a rounding boundary round
    differently in fp32 and fp64, which alone moves weight gradients by more
    than the 1e-4 bound.)

parity unpinned (fixed by this file, nothing in the paper to check against):
the arctan constant, the boxcar's width and height, the loss reduction (mean),
the readout equation, the form of the integral loss and the adaptive-threshold equations.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np


@dataclass(frozen=True)
class Net:
    sizes: Tuple[int, ...]            # N_0 .. N_L
    recurrent: Tuple[bool, ...]       # L-1 flags
    beta: Tuple[float, ...]           # L decays, last = readout
    theta: float
    surrogate: str                    # superspike | arctan | sigmoid | triangular | boxcar | ste
    slope: float
    gemm_round: str = "none"          # "none" | "bf16"
    loss: str = "max"                 # "max" | "integral": how the readout trace is reduced over time
    adapt_decay: Optional[Tuple[float, ...]] = None   # L-1 values in [0, 1]: decay of the threshold adaptation
    adapt_step: Optional[Tuple[float, ...]] = None    # L-1 values >= 0: rise of the threshold per spike (0: plain LIF)

    @property
    def L(self) -> int:
        return len(self.sizes) - 1


# --------------------------------------------------------------------------
# bfloat16 rounding (round to nearest, ties to even), used only in bf16 mode
# --------------------------------------------------------------------------
def rne_bf16(x: np.ndarray) -> np.ndarray:
    """Round to the nearest bfloat16 (8 significant bits), return float64.

    The value is first taken to float32 (the precision the device holds it
    in), then the low 16 bits are rounded away, ties to even.
    """
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


def _q(net: Net, a: np.ndarray) -> np.ndarray:
    return rne_bf16(a) if net.gemm_round == "bf16" else a


# --------------------------------------------------------------------------
# surrogate derivative (Section 2.1.1) and its antiderivative (test switch)
# --------------------------------------------------------------------------
def surrogate_grad(kind: str, k: float, x: np.ndarray) -> np.ndarray:
    """Backward function bwd(x) of the spiking activation, x = V - theta."""
    if kind == "superspike":          # surrogate listing: 1 / (1 + k|x|)^2
        return 1.0 / (1.0 + k * np.abs(x)) ** 2
    if kind == "arctan":              # reading stated in the module header
        return (k / 2.0) / (1.0 + (np.pi * k * x / 2.0) ** 2)
    if kind == "sigmoid":             # derivative of sigmoid(k x)
        s = 1.0 / (1.0 + np.exp(-k * x))
        return k * s * (1.0 - s)
    if kind == "triangular":          # surrogate listing: max(0, 1 - |k x|)
        return np.maximum(0.0, 1.0 - np.abs(k * x))
    if kind == "boxcar":              # named in Section 2.1.1, no formula: 1/2 on |k x| <= 1, else 0
        return np.where(np.abs(k * x) <= 1.0, 0.5, 0.0)
    if kind == "ste":                 # straight-through estimator (the stated default): derivative 1
        return np.ones_like(np.asarray(x, dtype=np.float64))
    raise ValueError(kind)


def smooth_step(kind: str, k: float, x: np.ndarray) -> np.ndarray:
    """A function whose exact derivative is surrogate_grad (smooth stand-in for
    the Heaviside step; only used to check the backward sweep by finite
    differences)."""
    if kind == "superspike":
        return 0.5 + x / (1.0 + k * np.abs(x))
    if kind == "arctan":
        return 0.5 + np.arctan(np.pi * k * x / 2.0) / np.pi
    if kind == "sigmoid":
        return 1.0 / (1.0 + np.exp(-k * x))
    if kind == "triangular":
        xc = np.clip(x, -1.0 / k, 1.0 / k)
        return 0.5 + xc - 0.5 * k * xc * np.abs(xc)
    if kind == "boxcar":
        return 0.5 + 0.5 * np.clip(x, -1.0 / k, 1.0 / k)
    if kind == "ste":
        return 0.5 + x
    raise ValueError(kind)


# --------------------------------------------------------------------------
# forward
# --------------------------------------------------------------------------
@dataclass
class Trace:
    I: List[np.ndarray] = field(default_factory=list)   # per spiking layer [T,B,N]
    V: List[np.ndarray] = field(default_factory=list)   # potential the spike decision used
    S: List[np.ndarray] = field(default_factory=list)   # spikes (0/1, or smooth values)
    A: List[np.ndarray] = field(default_factory=list)   # threshold adaptation in force at each step (zeros: plain LIF)
    J: Optional[np.ndarray] = None                      # readout currents [T,B,C]
    Y: Optional[np.ndarray] = None                      # readout trace    [T,B,C]
    z: Optional[np.ndarray] = None                      # max over time    [B,C]
    tstar: Optional[np.ndarray] = None                  # first argmax     [B,C]
    loss_b: Optional[np.ndarray] = None                 # per-sample CE    [B]
    loss: float = 0.0
    v_final: List[np.ndarray] = field(default_factory=list)


Forced = Dict[Tuple[int, int], List[Tuple[int, int, int]]]
"""(spiking layer index 0-based, t) -> list of (b, n, value): decisions to impose."""


def _betas(net: Net, betas):
    """Per-layer decay, per neuron: the given arrays, else the layer scalars."""
    if betas is None:
        return [np.full(net.sizes[l + 1], net.beta[l], dtype=np.float64) for l in range(net.L)]
    out = [np.asarray(b, np.float64) for b in betas]
    assert [len(b) for b in out] == [net.sizes[l + 1] for l in range(net.L)]
    return out


def _adaptation(net: Net):
    """Per spiking layer (decay, step) of the threshold adaptation; (0, 0) for plain LIF layers."""
    n = net.L - 1
    dec = net.adapt_decay if net.adapt_decay is not None else (0.0,) * n
    stp = net.adapt_step if net.adapt_step is not None else (0.0,) * n
    assert len(dec) == n and len(stp) == n
    return [(float(d), float(k)) for d, k in zip(dec, stp)]


def forward(net: Net, X: np.ndarray, W: Sequence[np.ndarray],
            R: Sequence[Optional[np.ndarray]], labels: np.ndarray,
            forced: Optional[Forced] = None, smooth: bool = False,
            batch_norm: Optional[int] = None,
            betas: Optional[Sequence[np.ndarray]] = None) -> Trace:
    """Unroll the network over time (Eq. 1-2 per spiking layer, LI readout).

    X: [T,B,N_0] 0/1.  W[l]: [N_l, N_{l+1}].  R[l]: [N,N] or None.
    `batch_norm`: divisor of the mean loss (defaults to B; lets a caller run a
    subset of a larger batch and keep the larger batch's scaling).
    """
    T, B, _ = X.shape
    L = net.L
    Wq = [_q(net, np.asarray(w, np.float64)) for w in W]
    Rq = [None if r is None else _q(net, np.asarray(r, np.float64)) for r in R]
    th = net.theta
    be = _betas(net, betas)
    ad = _adaptation(net)
    tr = Trace()
    for l in range(L - 1):
        n = net.sizes[l + 1]
        tr.I.append(np.zeros((T, B, n)))
        tr.V.append(np.zeros((T, B, n)))
        tr.S.append(np.zeros((T, B, n)))
        tr.A.append(np.zeros((T, B, n)))
    C = net.sizes[L]
    tr.J = np.zeros((T, B, C))
    tr.Y = np.zeros((T, B, C))
    v = [np.zeros((B, net.sizes[l + 1])) for l in range(L - 1)]   # V_0 = 0
    a = [np.zeros((B, net.sizes[l + 1])) for l in range(L - 1)]   # A_0 = 0
    y = np.zeros((B, C))                                          # y_{-1} = 0
    Xf = X.astype(np.float64)
    for t in range(T):
        s_in = Xf[t]
        for l in range(L - 1):
            cur = s_in @ Wq[l]                       # Linear, no bias
            th_t = th + a[l]                         # threshold in force (plain LIF: a = 0)
            if smooth:
                s = smooth_step(net.surrogate, net.slope, v[l] - th_t)
            else:
                s = (v[l] - th_t > 0.0).astype(np.float64)        # Eq. 1
            if forced and (l, t) in forced:
                for (b, nn, val) in forced[(l, t)]:
                    s[b, nn] = float(val)
            tr.I[l][t] = cur
            tr.V[l][t] = v[l]
            tr.S[l][t] = s
            tr.A[l][t] = a[l]
            nxt = be[l] * v[l] + cur - th_t * s                   # Eq. 2
            if Rq[l] is not None:
                nxt = nxt + s @ Rq[l]
            v[l] = nxt
            a[l] = ad[l][0] * a[l] + ad[l][1] * s                 # each spike raises the threshold, which then decays
            s_in = s
        jt = s_in @ Wq[L - 1]
        y = be[L - 1] * y + jt
        tr.J[t] = jt
        tr.Y[t] = y
    tr.v_final = v
    if net.loss == "integral":
        tr.z = tr.Y.sum(axis=0)
        tr.tstar = np.zeros((B, C), dtype=np.int64)               # not used
    else:
        tr.z = tr.Y.max(axis=0)
        tr.tstar = tr.Y.argmax(axis=0)                            # first maximiser
    zmax = tr.z.max(axis=1, keepdims=True)
    lse = zmax[:, 0] + np.log(np.exp(tr.z - zmax).sum(axis=1))
    tr.loss_b = lse - tr.z[np.arange(B), labels]
    tr.loss = float(tr.loss_b.sum() / (B if batch_norm is None else batch_norm))
    return tr


# --------------------------------------------------------------------------
# backward
# --------------------------------------------------------------------------
@dataclass
class Grads:
    dz: Optional[np.ndarray] = None
    dJ: Optional[np.ndarray] = None
    dS: List[np.ndarray] = field(default_factory=list)   # dL/dS per spiking layer
    dI: List[np.ndarray] = field(default_factory=list)   # dL/dI per spiking layer
    dW: List[np.ndarray] = field(default_factory=list)   # L entries
    dR: List[Optional[np.ndarray]] = field(default_factory=list)
    dbeta: List[np.ndarray] = field(default_factory=list) # L entries, one value per neuron / class


def backward(net: Net, X: np.ndarray, W: Sequence[np.ndarray],
             R: Sequence[Optional[np.ndarray]], labels: np.ndarray, tr: Trace,
             batch_norm: Optional[int] = None,
             betas: Optional[Sequence[np.ndarray]] = None) -> Grads:
    """Reverse sweep over the unrolled loop.

    g[l] is dL/dV_{t+1} of spiking layer l while step t is processed.  A
    potential V_t reaches the loss through beta*V_t into V_{t+1} and through
    the spike S_t, which feeds the next layer at step t, the reset
    -theta_t*S_t, (if recurrent) S_t R into V_{t+1} and (if the threshold
    adapts) adapt_step*S_t into A_{t+1}.  dS_t/dV_t is the surrogate at
    V_t - theta_t, dS_t/dA_t its negative; A_t also scales the reset
    (-S_t g) and decays into A_{t+1}.  ga[l] is dL/dA_{t+1}.  beta_n multiplies V_t[:, n] on the way to
    V_{t+1}[:, n], so dL/dbeta_n = sum over t and b of g_{t+1} V_t (readout:
    h_t y_{t-1}).
    """
    T, B, _ = X.shape
    L = net.L
    Wq = [_q(net, np.asarray(w, np.float64)) for w in W]
    Rq = [None if r is None else _q(net, np.asarray(r, np.float64)) for r in R]
    th = net.theta
    be = _betas(net, betas)
    ad = _adaptation(net)
    Bn = B if batch_norm is None else batch_norm
    C = net.sizes[L]

    zmax = tr.z.max(axis=1, keepdims=True)
    p = np.exp(tr.z - zmax)
    p /= p.sum(axis=1, keepdims=True)
    onehot = np.zeros((B, C))
    onehot[np.arange(B), labels] = 1.0
    gr = Grads()
    gr.dz = (p - onehot) / Bn

    gr.dJ = np.zeros((T, B, C))
    for l in range(L - 1):
        n = net.sizes[l + 1]
        gr.dS.append(np.zeros((T, B, n)))
        gr.dI.append(np.zeros((T, B, n)))
    gr.dW = [np.zeros_like(w, dtype=np.float64) for w in W]
    gr.dR = [None if r is None else np.zeros_like(r, dtype=np.float64) for r in R]
    gr.dbeta = [np.zeros(net.sizes[l + 1]) for l in range(L)]

    Xf = X.astype(np.float64)
    h = np.zeros((B, C))                                   # dL/dy_{t+1} carried back
    g = [np.zeros((B, net.sizes[l + 1])) for l in range(L - 1)]
    ga = [np.zeros((B, net.sizes[l + 1])) for l in range(L - 1)]
    tgrid = tr.tstar
    for t in range(T - 1, -1, -1):
        # readout: y_t = beta y_{t-1} + J_t; z picks y at tstar, or sums y over all steps
        h = be[L - 1] * h + (gr.dz if net.loss == "integral" else gr.dz * (tgrid == t))
        dJt = h
        if t >= 1:
            gr.dbeta[L - 1] += (h * tr.Y[t - 1]).sum(axis=0)   # y_t = beta y_{t-1} + J_t, y_{-1} = 0
        gr.dJ[t] = dJt
        s_below = tr.S[L - 2][t] if L >= 2 else Xf[t]
        gr.dW[L - 1] += s_below.T @ dJt
        d_s = dJt @ Wq[L - 1].T                            # dL/dS^{L-1}_t
        for l in range(L - 2, -1, -1):
            gr.dS[l][t] = d_s
            dIt = g[l]                                     # dV_{t+1}/dI_t = 1
            gr.dI[l][t] = dIt
            s_in = tr.S[l - 1][t] if l >= 1 else Xf[t]
            gr.dW[l] += s_in.T @ dIt
            if Rq[l] is not None:
                gr.dR[l] += tr.S[l][t].T @ dIt
            A_t = tr.A[l][t] if tr.A else 0.0
            q = d_s - (th + A_t) * g[l] + ad[l][1] * ga[l]     # dL/dS_t
            if Rq[l] is not None:
                q = q + dIt @ Rq[l].T
            sg = surrogate_grad(net.surrogate, net.slope, tr.V[l][t] - th - A_t)
            gr.dbeta[l] += (g[l] * tr.V[l][t]).sum(axis=0)      # V_{t+1} = beta V_t + ..
            ga[l] = ad[l][0] * ga[l] - tr.S[l][t] * g[l] - sg * q
            g[l] = be[l] * g[l] + sg * q
            if l >= 1:
                d_s = dIt @ Wq[l].T
    return gr


def sgd_step(W: Sequence[np.ndarray], R: Sequence[Optional[np.ndarray]], gr: Grads,
             lr: float):
    """Plain SGD on the (unrounded) master parameters."""
    Wn = [np.asarray(w, np.float64) - lr * d for w, d in zip(W, gr.dW)]
    Rn = [None if r is None else np.asarray(r, np.float64) - lr * d
          for r, d in zip(R, gr.dR)]
    return Wn, Rn


def sgd_step_beta(betas: Sequence[np.ndarray], gr: Grads, lr: float):
    """SGD on the decays, kept inside [0, 1] (the clip of the LIF listing)."""
    return [np.clip(np.asarray(b, np.float64) - lr * d, 0.0, 1.0) for b, d in zip(betas, gr.dbeta)]


def train_step(net: Net, X, W, R, labels, lr: float):
    """Forward, backward and one SGD step: the unit of work the benchmark times."""
    tr = forward(net, X, W, R, labels)
    gr = backward(net, X, W, R, labels, tr)
    Wn, Rn = sgd_step(W, R, gr, lr)
    return tr, gr, Wn, Rn
