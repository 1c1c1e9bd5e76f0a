"""Pins for the CPU oracle: closed forms, library routines, finite differences,
brute force and structural invariants.  None of these re-types the oracle's own
recursion; each would fail for a plausible slip (dropped term, wrong sign or
index, transposed operand, detached reset, off-by-one in time)."""
import math
import os

import numpy as np
import pytest
import scipy.signal
import scipy.special
import torch

import workloads
from oracle import snn_oracle as O
from oracle import snn_scalar
from tests.helpers import net_of, tiny_net

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def single_neuron(beta, theta, c, T, surrogate="superspike", slope=25.0):
    """One always-on input with weight c feeding one LIF neuron and a 1-class readout."""
    net = O.Net(sizes=(1, 1, 1), recurrent=(False,), beta=(beta, 0.5), theta=theta,
                surrogate=surrogate, slope=slope)
    X = np.ones((T, 1, 1), np.uint8)
    W = [np.array([[c]]), np.array([[1.0]])]
    return net, X, W, [None], np.array([0])


# ---------------------------------------------------------------- Eq. 1-2
def test_worked_example_constant_current():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "lif_constant_current.txt"))
            if l.strip() and not l.startswith("#")]
    net, X, W, R, lab = single_neuron(0.9, 1.0, 0.3, len(rows))
    tr = O.forward(net, X, W, R, lab)
    for t, v, s in rows:
        assert tr.V[0][int(t), 0, 0] == pytest.approx(float(v), abs=1e-9)
        assert tr.S[0][int(t), 0, 0] == float(s)


@pytest.mark.parametrize("c_num,c_den,theta_num", [(3, 8, 1), (7, 16, 1), (5, 8, 2), (9, 8, 1), (1, 4, 1)])
def test_non_leaky_neuron_exact_rational(c_num, c_den, theta_num):
    """beta = 1 (integrate and fire, Section 2.1.2's non-leaking neuron): under a constant current
    the potential stays a multiple of 1/c_den, so Eq. 1-2 can be iterated in exact rational
    arithmetic; the currents are dyadic, so the float recursion has to agree exactly, ties at the
    threshold (strict inequality: no spike at V = theta, which c = 1/4 reaches) included.  The
    long-run firing rate is c/theta when the reset keeps up (c <= theta); with c > theta the
    neuron fires at every step and the potential grows by c - theta per step."""
    from fractions import Fraction
    T = 120
    c, theta = Fraction(c_num, c_den), Fraction(theta_num)
    net, X, W, R, lab = single_neuron(1.0, float(theta), float(c), T)
    tr = O.forward(net, X, W, R, lab)
    v, spikes = Fraction(0), []
    for t in range(T):
        s = 1 if v > theta else 0
        spikes.append(s)
        assert tr.S[0][t, 0, 0] == s
        assert tr.V[0][t, 0, 0] == float(v)
        v = v + c - theta * s
    if c <= theta:
        assert abs(sum(spikes) / T - float(c / theta)) <= 2.0 / T
    else:
        assert sum(spikes) == T - 1            # S_0 = 0 (V_0 = 0), then every step
        assert tr.V[0][-1, 0, 0] == pytest.approx(float(c + (T - 2) * (c - theta)))


@pytest.mark.parametrize("beta,theta,c", [(0.9, 1.0, 0.3), (0.95, 1.0, 0.08), (0.8, 2.0, 0.5),
                                          (0.9, 1.0, 0.1001), (0.9, 1.0, 0.0999), (0.5, 1.0, 3.0)])
def test_first_spike_time_closed_form(beta, theta, c):
    """Before the first spike V_t = c (1 - beta^t) / (1 - beta); the neuron fires first at
    the smallest t with V_t > theta, i.e. floor(ln(1 - theta (1-beta)/c) / ln beta) + 1,
    and never if c/(1-beta) <= theta."""
    T = 200
    net, X, W, R, lab = single_neuron(beta, theta, c, T)
    tr = O.forward(net, X, W, R, lab)
    spikes = np.flatnonzero(tr.S[0][:, 0, 0])
    if c / (1 - beta) <= theta:
        assert spikes.size == 0
        t = np.arange(T)
        assert np.allclose(tr.V[0][:, 0, 0], c * (1 - beta ** t) / (1 - beta), atol=1e-12)
        return
    t1 = math.floor(math.log(1 - theta * (1 - beta) / c) / math.log(beta)) + 1
    assert spikes[0] == t1
    t = np.arange(t1 + 1)
    assert np.allclose(tr.V[0][:t1 + 1, 0, 0], c * (1 - beta ** t) / (1 - beta), atol=1e-12)
    # after the reset the same geometric law restarts from beta*V - theta + c
    v0 = beta * tr.V[0][t1, 0, 0] + c - theta
    t2 = spikes[1]
    j = np.arange(t2 - t1)
    assert np.allclose(tr.V[0][t1 + 1:t2 + 1, 0, 0],
                       beta ** j * v0 + c * (1 - beta ** j) / (1 - beta), atol=1e-12)


@pytest.mark.parametrize("c", [0.5, 0.375, 0.25])
def test_non_leaky_spike_count(c):
    """beta = 1, theta = 1: total charge t*c minus one unit per spike must stay in (.., 1];
    number of spikes emitted at steps <= t is max(0, ceil(t c) - 1)."""
    T = 40
    net, X, W, R, lab = single_neuron(1.0, 1.0, c, T)
    tr = O.forward(net, X, W, R, lab)
    counts = np.cumsum(tr.S[0][:, 0, 0])
    for t in range(T):
        assert counts[t] == max(0, math.ceil(t * c) - 1)


def test_charge_balance_and_structure():
    """v_T = sum_t beta^(T-1-t) (I_t - theta S_t + S_t R): ties spikes to potentials."""
    rng = np.random.default_rng(5)
    net, X, W, R, lab = tiny_net(rng, sizes=(12, 9, 7, 4), recurrent=(True, False), T=25, B=3,
                                 surrogate="superspike", slope=25.0, gain=2.5)
    tr = O.forward(net, X, W, R, lab)
    T = X.shape[0]
    for l in range(2):
        assert tr.S[l].sum() > 0, "test must actually spike"
        drive = tr.I[l] - net.theta * tr.S[l]
        if R[l] is not None:
            drive = drive + tr.S[l] @ R[l]
        w = net.beta[l] ** (T - 1 - np.arange(T))
        assert np.allclose(np.tensordot(w, drive, axes=(0, 0)), tr.v_final[l], atol=1e-12)
        assert np.all(tr.S[l][0] == 0)                        # V_0 = 0 cannot spike
        assert np.array_equal(tr.S[l], (tr.V[l] > net.theta).astype(float))
    gr = O.backward(net, X, W, R, lab, tr)
    for l in range(2):
        assert np.all(gr.dI[l][T - 1] == 0)                   # last current never reaches the loss
    assert np.allclose(gr.dz.sum(axis=1), 0, atol=1e-15)


def test_silent_network():
    wl = workloads.CONFIGS["tiny_ff"]
    inp = workloads.generate(wl)
    net = net_of(wl)
    W0 = [np.zeros_like(w) for w in inp.W]
    tr = O.forward(net, inp.X, W0, inp.R, inp.labels)
    assert all(s.sum() == 0 for s in tr.S)
    assert np.all(tr.Y == 0)
    assert tr.loss == pytest.approx(math.log(10), abs=1e-15)
    gr = O.backward(net, inp.X, W0, inp.R, inp.labels, tr)
    # hidden spikes are all zero, so dW_out = S^T dJ = 0; dS = dJ * 0 = 0 upstream
    assert all(np.all(d == 0) for d in gr.dW)


# ---------------------------------------------------------------- library routines
def test_readout_is_a_first_order_filter():
    rng = np.random.default_rng(1)
    net, X, W, R, lab = tiny_net(rng, sizes=(8, 6, 5), recurrent=(False,), T=30, B=4,
                                 beta=(0.9, 0.83), gain=3.0, surrogate="superspike")
    tr = O.forward(net, X, W, R, lab)
    assert tr.S[0].sum() > 0
    assert np.allclose(tr.J, tr.S[0] @ W[1], atol=1e-13)
    Y = scipy.signal.lfilter([1.0], [1.0, -net.beta[1]], tr.J, axis=0)
    assert np.allclose(tr.Y, Y, atol=1e-12)


def test_lif_without_threshold_is_a_delayed_filter():
    rng = np.random.default_rng(2)
    net, X, W, R, lab = tiny_net(rng, sizes=(8, 6, 5), recurrent=(False,), T=30, B=4,
                                 beta=(0.9, 0.83), theta=1e9)
    tr = O.forward(net, X, W, R, lab)
    cur = X.astype(float) @ W[0]
    assert np.allclose(tr.I[0], cur, atol=1e-13)
    filt = scipy.signal.lfilter([1.0], [1.0, -net.beta[0]], cur, axis=0)
    assert np.all(tr.V[0][0] == 0)
    assert np.allclose(tr.V[0][1:], filt[:-1], atol=1e-12)    # one-step delay


def test_loss_matches_scipy_and_argmax_is_first():
    rng = np.random.default_rng(3)
    net, X, W, R, lab = tiny_net(rng, sizes=(6, 5, 4), recurrent=(False,), T=12, B=5, gain=3.0,
                                 surrogate="superspike")
    tr = O.forward(net, X, W, R, lab)
    ref = -scipy.special.log_softmax(tr.z, axis=1)[np.arange(5), lab]
    assert np.allclose(tr.loss_b, ref, atol=1e-13)
    assert tr.loss == pytest.approx(ref.mean(), abs=1e-14)
    gr = O.backward(net, X, W, R, lab, tr)
    sm = scipy.special.softmax(tr.z, axis=1)
    sm[np.arange(5), lab] -= 1
    assert np.allclose(gr.dz, sm / 5, atol=1e-14)
    # silent classes: readout identically zero, first maximiser must be step 0
    W0 = [W[0], np.zeros_like(W[1])]
    assert np.all(O.forward(net, X, W0, R, lab).tstar == 0)


def test_bf16_rounding_matches_library():
    rng = np.random.default_rng(4)
    x = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-6, 6, 20000),
                        # exact ties: halfway between two neighbouring bfloat16 values in [1, 2)
                        (256 + 2 * np.arange(0, 64) + 1) / 256.0, [0.0, -0.0, 1.0, -1.0]])
    want = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(O.rne_bf16(x), want)


# ---------------------------------------------------------------- gradients
def fd_grads(net, X, W, R, lab, h=1e-6):
    def loss(Wp, Rp):
        return O.forward(net, X, Wp, Rp, lab, smooth=True).loss
    dW, dR = [], []
    for l, w in enumerate(W):
        d = np.zeros_like(w)
        for idx in np.ndindex(*w.shape):
            Wp = [a.copy() for a in W]; Wp[l][idx] += h
            Wm = [a.copy() for a in W]; Wm[l][idx] -= h
            d[idx] = (loss(Wp, R) - loss(Wm, R)) / (2 * h)
        dW.append(d)
    for l, r in enumerate(R):
        if r is None:
            dR.append(None); continue
        d = np.zeros_like(r)
        for idx in np.ndindex(*r.shape):
            Rp = [None if a is None else a.copy() for a in R]; Rp[l][idx] += h
            Rm = [None if a is None else a.copy() for a in R]; Rm[l][idx] -= h
            d[idx] = (loss(W, Rp) - loss(W, Rm)) / (2 * h)
        dR.append(d)
    return dW, dR


@pytest.mark.parametrize("surrogate,slope", [("sigmoid", 3.0), ("superspike", 4.0),
                                             ("arctan", 2.0), ("triangular", 0.5), ("boxcar", 0.4), ("ste", 1.0)])
@pytest.mark.parametrize("recurrent", [(False, False), (True, True), (False, True)])
def test_backward_is_exact_gradient_of_smoothed_network(surrogate, slope, recurrent):
    """With the step replaced by the surrogate's antiderivative the reverse sweep must be the
    true gradient: checks the reset path (not detached), the recurrent path, the one-step
    delay, every transpose and the readout."""
    rng = np.random.default_rng(11)
    net, X, W, R, lab = tiny_net(rng, recurrent=recurrent, surrogate=surrogate, slope=slope)
    tr = O.forward(net, X, W, R, lab, smooth=True)
    gr = O.backward(net, X, W, R, lab, tr)
    dW, dR = fd_grads(net, X, W, R, lab)
    for l in range(net.L):
        assert np.abs(gr.dW[l]).max() > 1e-4
        assert np.allclose(gr.dW[l], dW[l], rtol=2e-6, atol=2e-9), (l, np.abs(gr.dW[l] - dW[l]).max())
    for l in range(net.L - 1):
        if R[l] is not None:
            assert np.allclose(gr.dR[l], dR[l], rtol=2e-6, atol=2e-9)


@pytest.mark.parametrize("recurrent", [(False, False), (True, True)])
def test_integral_loss_backward_is_exact_gradient_of_smoothed_network(recurrent):
    """Same finite-difference check with the readout trace summed over time."""
    rng = np.random.default_rng(12)
    net, X, W, R, lab = tiny_net(rng, recurrent=recurrent, surrogate="sigmoid", slope=3.0, loss="integral")
    tr = O.forward(net, X, W, R, lab, smooth=True)
    gr = O.backward(net, X, W, R, lab, tr)
    dW, dR = fd_grads(net, X, W, R, lab)
    for l in range(net.L):
        assert np.abs(gr.dW[l]).max() > 1e-4
        assert np.allclose(gr.dW[l], dW[l], rtol=2e-6, atol=2e-9), (l, np.abs(gr.dW[l] - dW[l]).max())
    for l in range(net.L - 1):
        if R[l] is not None:
            assert np.allclose(gr.dR[l], dR[l], rtol=2e-6, atol=2e-9)


def test_integral_loss_closed_forms():
    """z is the sum over time of a first-order filter of J (library filter + library
    log-softmax), and the readout's reverse recursion with dz fed in at every step has the
    closed form dJ_t = dz (1 - beta^(T-t)) / (1 - beta)."""
    from scipy.signal import lfilter
    from scipy.special import log_softmax
    rng = np.random.default_rng(22)
    net, X, W, R, lab = tiny_net(rng, sizes=(10, 8, 4), recurrent=(False,), T=15, B=3, beta=(0.9, 0.8),
                                 surrogate="superspike", slope=25.0, gain=3.0, loss="integral")
    tr = O.forward(net, X, W, R, lab)
    assert tr.S[0].sum() > 5
    Y = lfilter([1.0], [1.0, -net.beta[1]], tr.J, axis=0)
    assert np.allclose(tr.z, Y.sum(axis=0), atol=1e-12)
    want = -log_softmax(Y.sum(axis=0), axis=1)[np.arange(3), lab].mean()
    assert tr.loss == pytest.approx(want, rel=1e-12)
    gr = O.backward(net, X, W, R, lab, tr)
    T = X.shape[0]
    t = np.arange(T)[:, None, None]
    closed = gr.dz[None] * (1.0 - net.beta[1] ** (T - t)) / (1.0 - net.beta[1])
    assert np.allclose(gr.dJ, closed, atol=1e-14)
    # and it differs from the max-over-time loss on the same network
    import dataclasses
    tr_max = O.forward(dataclasses.replace(net, loss="max"), X, W, R, lab)
    assert abs(tr_max.loss - tr.loss) > 1e-3


def test_surrogates_are_derivatives_of_their_smooth_steps():
    x = np.linspace(-3, 3, 601) + 1e-4
    for kind, k in [("sigmoid", 3.0), ("superspike", 25.0), ("arctan", 2.0), ("triangular", 0.5),
                    ("boxcar", 0.7), ("ste", 1.0)]:
        h = 1e-6
        fd = (O.smooth_step(kind, k, x + h) - O.smooth_step(kind, k, x - h)) / (2 * h)
        assert np.allclose(fd, O.surrogate_grad(kind, k, x), atol=1e-6), kind
    # printed formulas of the surrogate listing, at hand-picked points
    assert O.surrogate_grad("superspike", 25.0, np.array([0.0, 0.04, -0.2]))  \
        == pytest.approx([1.0, 0.25, 1 / 36.0])
    assert O.surrogate_grad("triangular", 0.5, np.array([0.0, 1.0, -3.0])) == pytest.approx([1, 0.5, 0])
    assert O.surrogate_grad("arctan", 2.0, np.array([0.0]))[0] == pytest.approx(1.0)
    assert O.surrogate_grad("boxcar", 1.0, np.array([0.0, 0.99, -1.0, 1.01, -3.0])) == pytest.approx([0.5, 0.5, 0.5, 0, 0])
    assert O.surrogate_grad("boxcar", 4.0, np.array([0.2, 0.3])) == pytest.approx([0.5, 0.0])
    assert O.surrogate_grad("ste", 7.0, np.array([-5.0, 0.0, 2.0])) == pytest.approx([1.0, 1.0, 1.0])


def test_readout_weight_gradient_of_the_real_spiking_network():
    """Spikes do not depend on the readout weights, so central differences on W^L of the
    true (Heaviside) network must match dW^L."""
    rng = np.random.default_rng(21)
    net, X, W, R, lab = tiny_net(rng, sizes=(10, 8, 4), recurrent=(True,), T=15, B=3,
                                 beta=(0.9, 0.8), surrogate="superspike", slope=25.0, gain=3.0)
    tr = O.forward(net, X, W, R, lab)
    assert tr.S[0].sum() > 5
    gr = O.backward(net, X, W, R, lab, tr)
    h = 1e-6
    fd = np.zeros_like(W[1])
    for idx in np.ndindex(*W[1].shape):
        Wp = [W[0], W[1].copy()]; Wp[1][idx] += h
        Wm = [W[0], W[1].copy()]; Wm[1][idx] -= h
        fd[idx] = (O.forward(net, X, Wp, R, lab).loss - O.forward(net, X, Wm, R, lab).loss) / (2 * h)
    assert np.allclose(gr.dW[1], fd, rtol=1e-6, atol=1e-9)
    # closed form of the readout's reverse recursion: dJ_t = dz beta^(t*-t) for t <= t*
    T = X.shape[0]
    t = np.arange(T)[:, None, None]
    closed = np.where(t <= tr.tstar[None], gr.dz[None] * net.beta[1] ** (tr.tstar[None] - t), 0.0)
    assert np.allclose(gr.dJ, closed, atol=1e-15)


# ---------------------------------------------------------------- brute force
@pytest.mark.parametrize("recurrent", [(False, False), (True, False), (True, True)])
@pytest.mark.parametrize("surrogate,slope", [("superspike", 25.0), ("arctan", 2.0), ("boxcar", 1.0), ("ste", 1.0)])
def test_vectorised_oracle_equals_scalar_brute_force(recurrent, surrogate, slope):
    rng = np.random.default_rng(31)
    net, X, W, R, lab = tiny_net(rng, sizes=(6, 5, 4, 3), recurrent=recurrent, T=9, B=3,
                                 surrogate=surrogate, slope=slope, gain=2.5)
    tr = O.forward(net, X, W, R, lab)
    gr = O.backward(net, X, W, R, lab, tr)
    assert tr.S[0].sum() > 0 and tr.S[1].sum() > 0
    ref = snn_scalar.run(net.sizes, net.recurrent, net.beta, net.theta, surrogate, slope,
                         X.tolist(), [w.tolist() for w in W],
                         [None if r is None else r.tolist() for r in R], lab.tolist())
    for l in range(2):
        assert np.allclose(tr.V[l], np.array(ref["V"][l]), atol=1e-12)
        assert np.array_equal(tr.S[l], np.array(ref["S"][l]))
    assert np.allclose(tr.Y, np.array(ref["Y"]), atol=1e-12)
    assert np.array_equal(tr.tstar, np.array(ref["tstar"]))
    assert tr.loss == pytest.approx(ref["loss"], abs=1e-12)
    for l in range(3):
        assert np.allclose(gr.dW[l], np.array(ref["dW"][l]), atol=1e-12)
    for l in range(2):
        if R[l] is not None:
            assert np.allclose(gr.dR[l], np.array(ref["dR"][l]), atol=1e-12)


# ---------------------------------------------------------------- per-neuron decay
def _random_betas(rng, net):
    return [rng.uniform(0.6, 0.98, size=net.sizes[l + 1]) for l in range(net.L)]


@pytest.mark.parametrize("recurrent", [(False, False), (True, True)])
def test_per_neuron_beta_equals_scalar_brute_force(recurrent):
    """Per-neuron decays (the LIF listing's beta parameter) and their gradient, against the
    one-number-at-a-time version."""
    rng = np.random.default_rng(41)
    net, X, W, R, lab = tiny_net(rng, sizes=(6, 5, 4, 3), recurrent=recurrent, T=9, B=3,
                                 surrogate="superspike", slope=25.0, gain=2.5)
    betas = _random_betas(rng, net)
    tr = O.forward(net, X, W, R, lab, betas=betas)
    gr = O.backward(net, X, W, R, lab, tr, betas=betas)
    assert tr.S[0].sum() > 0 and tr.S[1].sum() > 0
    ref = snn_scalar.run(net.sizes, net.recurrent, [b.tolist() for b in betas], net.theta, "superspike", 25.0,
                         X.tolist(), [w.tolist() for w in W],
                         [None if r is None else r.tolist() for r in R], lab.tolist())
    for l in range(2):
        assert np.allclose(tr.V[l], np.array(ref["V"][l]), atol=1e-12)
        assert np.array_equal(tr.S[l], np.array(ref["S"][l]))
    assert np.allclose(tr.Y, np.array(ref["Y"]), atol=1e-12)
    assert tr.loss == pytest.approx(ref["loss"], abs=1e-12)
    for l in range(3):
        assert np.allclose(gr.dW[l], np.array(ref["dW"][l]), atol=1e-12)
        assert np.allclose(gr.dbeta[l], np.array(ref["dbeta"][l]), atol=1e-12)
        assert np.abs(gr.dbeta[l]).max() > 0
    # scalars are the special case of equal entries
    tr0 = O.forward(net, X, W, R, lab)
    tr1 = O.forward(net, X, W, R, lab, betas=[np.full(net.sizes[l + 1], net.beta[l]) for l in range(net.L)])
    assert np.array_equal(tr0.Y, tr1.Y)


@pytest.mark.parametrize("loss", ["max", "integral"])
@pytest.mark.parametrize("recurrent", [(False, False), (True, True)])
def test_dbeta_is_exact_gradient_of_smoothed_network(recurrent, loss):
    """Central differences on every decay of the smoothed network (reset, recurrence and
    readout included)."""
    rng = np.random.default_rng(42)
    net, X, W, R, lab = tiny_net(rng, recurrent=recurrent, surrogate="sigmoid", slope=3.0, loss=loss)
    betas = _random_betas(rng, net)
    tr = O.forward(net, X, W, R, lab, smooth=True, betas=betas)
    gr = O.backward(net, X, W, R, lab, tr, betas=betas)
    h = 1e-6
    for l in range(net.L):
        fd = np.zeros_like(betas[l])
        for n in range(len(betas[l])):
            bp = [b.copy() for b in betas]; bp[l][n] += h
            bm = [b.copy() for b in betas]; bm[l][n] -= h
            fd[n] = (O.forward(net, X, W, R, lab, smooth=True, betas=bp).loss
                     - O.forward(net, X, W, R, lab, smooth=True, betas=bm).loss) / (2 * h)
        assert np.abs(fd).max() > 1e-5
        assert np.allclose(gr.dbeta[l], fd, rtol=2e-6, atol=2e-9), (l, np.abs(gr.dbeta[l] - fd).max())


def test_readout_dbeta_of_the_real_spiking_network_and_clip():
    """Spikes do not depend on the readout decay, so central differences on it hold for the
    true (Heaviside) network; the update keeps decays inside [0, 1]."""
    rng = np.random.default_rng(43)
    net, X, W, R, lab = tiny_net(rng, sizes=(10, 8, 4), recurrent=(True,), T=15, B=3,
                                 beta=(0.9, 0.8), surrogate="superspike", slope=25.0, gain=3.0)
    betas = _random_betas(rng, net)
    tr = O.forward(net, X, W, R, lab, betas=betas)
    gr = O.backward(net, X, W, R, lab, tr, betas=betas)
    h = 1e-6
    for c in range(4):
        bp = [b.copy() for b in betas]; bp[1][c] += h
        bm = [b.copy() for b in betas]; bm[1][c] -= h
        fd = (O.forward(net, X, W, R, lab, betas=bp).loss - O.forward(net, X, W, R, lab, betas=bm).loss) / (2 * h)
        # the first maximiser does not move for a perturbation this small
        assert gr.dbeta[1][c] == pytest.approx(fd, rel=1e-5, abs=1e-9)
    new = O.sgd_step_beta(betas, gr, lr=1e6)
    assert all(np.all((b >= 0.0) & (b <= 1.0)) for b in new)
    assert any(np.any(b == 0.0) or np.any(b == 1.0) for b in new)
    same = O.sgd_step_beta(betas, gr, lr=1e-3)
    assert np.allclose(same[0], betas[0] - 1e-3 * gr.dbeta[0], atol=0, rtol=0)


# ---------------------------------------------------------------- adaptive threshold
def adaptive_neuron(beta, theta, c, T, decay, step):
    net = O.Net(sizes=(1, 1, 1), recurrent=(False,), beta=(beta, 0.5), theta=theta, surrogate="superspike",
                slope=25.0, adapt_decay=(decay,), adapt_step=(step,))
    return net, np.ones((T, 1, 1), np.uint8), [np.array([[c]]), np.array([[1.0]])], [None], np.array([0])


@pytest.mark.parametrize("c_num,c_den,k_num,k_den", [(1, 2, 1, 2), (3, 4, 1, 4), (5, 8, 1, 8), (7, 4, 3, 8)])
def test_adaptive_threshold_exact_rational(c_num, c_den, k_num, k_den):
    """No leak, no decay of the adaptation (beta = 1, adapt_decay = 1), constant dyadic current:
    everything is exactly representable, so Eq. 1-2 with the threshold in force can be iterated
    in rational arithmetic and the float recursion must agree exactly.  The k-th spike is taken
    at threshold theta + (k-1) step and removes that much charge, so after n spikes the charge
    balance reads V_T = T c - n theta - step n (n-1) / 2, and the intervals between spikes do
    not shrink (the neuron adapts)."""
    from fractions import Fraction
    T = 160
    c, kappa, theta = Fraction(c_num, c_den), Fraction(k_num, k_den), Fraction(1)
    net, X, W, R, lab = adaptive_neuron(1.0, 1.0, float(c), T, 1.0, float(kappa))
    tr = O.forward(net, X, W, R, lab)
    v, a, times = Fraction(0), Fraction(0), []
    for t in range(T):
        s = 1 if v > theta + a else 0
        assert tr.S[0][t, 0, 0] == s and tr.V[0][t, 0, 0] == float(v) and tr.A[0][t, 0, 0] == float(a)
        if s:
            times.append(t)
        v, a = v + c - (theta + a) * s, a + kappa * s
    n = len(times)
    assert n >= 5
    assert tr.v_final[0][0, 0] == float(T * c - n * theta - kappa * n * (n - 1) / 2)
    gaps = np.diff(times)
    assert np.all(np.diff(gaps) >= -1) and gaps[-1] > gaps[0]      # slows down (up to the grid of whole steps)


def test_adaptation_is_a_filter_of_the_spikes_and_charge_balance():
    """A_t is a first-order filter of the layer's own spike train, one step delayed (library
    filter), the spike decision is V_t > theta + A_t, and the potential at the end balances the
    currents against the resets at the threshold in force."""
    rng = np.random.default_rng(71)
    net, X, W, R, lab = tiny_net(rng, sizes=(12, 9, 7, 4), recurrent=(True, False), T=40, B=3, surrogate="superspike",
                                 slope=25.0, gain=3.0, adapt_decay=(0.9, 0.7), adapt_step=(0.4, 0.25))
    tr = O.forward(net, X, W, R, lab)
    T = X.shape[0]
    for l in range(2):
        assert tr.S[l].sum() > 10
        filt = scipy.signal.lfilter([0.0, net.adapt_step[l]], [1.0, -net.adapt_decay[l]], tr.S[l], axis=0)
        assert np.allclose(tr.A[l], filt, atol=1e-13)
        assert np.array_equal(tr.S[l], (tr.V[l] > net.theta + tr.A[l]).astype(float))
        drive = tr.I[l] - (net.theta + tr.A[l]) * tr.S[l]
        if R[l] is not None:
            drive = drive + tr.S[l] @ R[l]
        w = net.beta[l] ** (T - 1 - np.arange(T))
        assert np.allclose(np.tensordot(w, drive, axes=(0, 0)), tr.v_final[l], atol=1e-12)
    # the adaptation lowers the firing rate of the same network
    import dataclasses
    plain = O.forward(dataclasses.replace(net, adapt_step=(0.0, 0.0)), X, W, R, lab)
    assert plain.S[0].sum() > tr.S[0].sum()


def test_zero_adaptation_step_is_the_plain_neuron():
    rng = np.random.default_rng(72)
    net, X, W, R, lab = tiny_net(rng, sizes=(9, 7, 6, 4), recurrent=(False, True), T=14, B=4, surrogate="arctan",
                                 slope=2.0, gain=2.5)
    import dataclasses
    zero = dataclasses.replace(net, adapt_decay=(0.8, 0.9), adapt_step=(0.0, 0.0))
    a, b = O.forward(net, X, W, R, lab), O.forward(zero, X, W, R, lab)
    assert all(np.array_equal(x, y) for x, y in zip(a.V, b.V)) and a.loss == b.loss
    ga, gb = O.backward(net, X, W, R, lab, a), O.backward(zero, X, W, R, lab, b)
    assert all(np.array_equal(x, y) for x, y in zip(ga.dW, gb.dW))
    assert np.array_equal(ga.dR[1], gb.dR[1])


@pytest.mark.parametrize("surrogate,slope", [("sigmoid", 3.0), ("superspike", 4.0), ("arctan", 2.0)])
@pytest.mark.parametrize("recurrent", [(False, False), (True, True)])
def test_adaptive_backward_is_exact_gradient_of_smoothed_network(surrogate, slope, recurrent):
    """Central differences on every weight of the smoothed network with adapting thresholds: the
    paths through the spike decision (-surrogate), through the reset magnitude (-S g) and through
    the adaptation's own memory must all be in the reverse sweep, with the right signs."""
    rng = np.random.default_rng(73)
    net, X, W, R, lab = tiny_net(rng, recurrent=recurrent, surrogate=surrogate, slope=slope,
                                 adapt_decay=(0.85, 0.6), adapt_step=(0.5, 0.3))
    tr = O.forward(net, X, W, R, lab, smooth=True)
    assert np.abs(tr.A[0]).max() > 0.1
    gr = O.backward(net, X, W, R, lab, tr)
    dW, dR = fd_grads(net, X, W, R, lab)
    for l in range(net.L):
        assert np.abs(gr.dW[l]).max() > 1e-4
        assert np.allclose(gr.dW[l], dW[l], rtol=2e-6, atol=2e-9), (l, np.abs(gr.dW[l] - dW[l]).max())
    for l in range(net.L - 1):
        if R[l] is not None:
            assert np.allclose(gr.dR[l], dR[l], rtol=2e-6, atol=2e-9)
    # the sweep that ignores the adaptation is a different (wrong) gradient here
    import dataclasses
    wrong = O.backward(dataclasses.replace(net, adapt_step=(0.0, 0.0)), X, W, R, lab, tr)
    assert not np.allclose(wrong.dW[0], dW[0], rtol=1e-3, atol=1e-6)


@pytest.mark.parametrize("recurrent", [(False, False), (True, False)])
def test_adaptive_vectorised_oracle_equals_scalar_brute_force(recurrent):
    rng = np.random.default_rng(74)
    net, X, W, R, lab = tiny_net(rng, sizes=(6, 5, 4, 3), recurrent=recurrent, T=12, B=3, surrogate="superspike",
                                 slope=25.0, gain=3.0, adapt_decay=(0.9, 0.5), adapt_step=(0.3, 0.6))
    betas = _random_betas(rng, net)
    tr = O.forward(net, X, W, R, lab, betas=betas)
    gr = O.backward(net, X, W, R, lab, tr, betas=betas)
    assert tr.S[0].sum() > 0 and tr.S[1].sum() > 0
    ref = snn_scalar.run(net.sizes, net.recurrent, [b.tolist() for b in betas], net.theta, "superspike", 25.0,
                         X.tolist(), [w.tolist() for w in W], [None if r is None else r.tolist() for r in R],
                         lab.tolist(), adapt_decay=net.adapt_decay, adapt_step=net.adapt_step)
    for l in range(2):
        assert np.allclose(tr.V[l], np.array(ref["V"][l]), atol=1e-12)
        assert np.allclose(tr.A[l], np.array(ref["A"][l]), atol=1e-12)
        assert np.array_equal(tr.S[l], np.array(ref["S"][l]))
    assert tr.loss == pytest.approx(ref["loss"], abs=1e-12)
    for l in range(3):
        assert np.allclose(gr.dW[l], np.array(ref["dW"][l]), atol=1e-12)
        assert np.allclose(gr.dbeta[l], np.array(ref["dbeta"][l]), atol=1e-12)
    if R[0] is not None:
        assert np.allclose(gr.dR[0], np.array(ref["dR"][0]), atol=1e-12)


# ---------------------------------------------------------------- invariants
def test_batch_permutation_duplication_and_time_shift():
    rng = np.random.default_rng(41)
    net, X, W, R, lab = tiny_net(rng, sizes=(9, 7, 6, 4), recurrent=(False, True), T=14, B=4,
                                 surrogate="superspike", slope=25.0, gain=2.5)
    tr = O.forward(net, X, W, R, lab)
    gr = O.backward(net, X, W, R, lab, tr)
    perm = np.array([2, 0, 3, 1])
    trp = O.forward(net, X[:, perm], W, R, lab[perm])
    grp = O.backward(net, X[:, perm], W, R, lab[perm], trp)
    assert np.array_equal(trp.S[1], tr.S[1][:, perm])
    assert np.allclose(trp.Y, tr.Y[:, perm], atol=1e-13)
    for l in range(3):
        assert np.allclose(grp.dW[l], gr.dW[l], atol=1e-13)
    # duplicating every sample leaves the mean loss and the gradients unchanged
    X2 = np.concatenate([X, X], axis=1); lab2 = np.concatenate([lab, lab])
    tr2 = O.forward(net, X2, W, R, lab2)
    gr2 = O.backward(net, X2, W, R, lab2, tr2)
    assert tr2.loss == pytest.approx(tr.loss, abs=1e-13)
    for l in range(3):
        assert np.allclose(gr2.dW[l], gr.dW[l], atol=1e-13)
    assert np.allclose(gr2.dR[1], gr.dR[1], atol=1e-13)
    # a subset with the full batch's normalisation gives the same per-sample tensors
    sub = np.array([1, 3])
    trs = O.forward(net, X[:, sub], W, R, lab[sub], batch_norm=4)
    grs = O.backward(net, X[:, sub], W, R, lab[sub], trs, batch_norm=4)
    assert np.allclose(grs.dI[0], gr.dI[0][:, sub], atol=1e-15)
    # prepending a silent input step delays everything by one step
    Xs = np.concatenate([np.zeros_like(X[:1]), X], axis=0)
    trs = O.forward(net, Xs, W, R, lab)
    assert np.array_equal(trs.S[1][1:], tr.S[1]) and np.all(trs.S[1][0] == 0)
    assert np.allclose(trs.V[0][1:], tr.V[0], atol=1e-13)
    assert np.allclose(trs.Y[1:], tr.Y, atol=1e-13)


def test_forced_decisions_and_sgd():
    rng = np.random.default_rng(51)
    net, X, W, R, lab = tiny_net(rng, sizes=(9, 7, 4), recurrent=(False,), T=10, B=2,
                                 beta=(0.9, 0.8), surrogate="superspike", slope=25.0, gain=2.5)
    tr = O.forward(net, X, W, R, lab)
    t, b, n = 4, 1, 3
    flipped = 1 - int(tr.S[0][t, b, n])
    trf = O.forward(net, X, W, R, lab, forced={(0, t): [(b, n, flipped)]})
    assert trf.S[0][t, b, n] == flipped
    assert np.array_equal(trf.S[0][:t], tr.S[0][:t])
    # the imposed decision enters the reset: V_{t+1} differs by exactly theta
    assert abs(abs(trf.V[0][t + 1, b, n] - tr.V[0][t + 1, b, n]) - net.theta) < 1e-12
    assert np.array_equal(trf.V[0][:, 1 - b], tr.V[0][:, 1 - b])   # other sample untouched
    gr = O.backward(net, X, W, R, lab, tr)
    Wn, Rn = O.sgd_step(W, R, gr, 0.1)
    assert np.allclose(Wn[0], W[0] - 0.1 * gr.dW[0], atol=0) and Rn == [None]


def test_bf16_mode_close_to_fp32_mode():
    wl = workloads.CONFIGS["tiny_ff"]
    inp = workloads.generate(wl, w_gain=3.0)
    a = O.forward(net_of(wl, "none"), inp.X, inp.W, inp.R, inp.labels)
    b = O.forward(net_of(wl, "bf16"), inp.X, inp.W, inp.R, inp.labels)
    assert abs(a.loss - b.loss) / abs(a.loss) < 2e-2
    # bf16 mode is exactly the unrounded algorithm on rounded weights (spikes are 0/1)
    Wr = [O.rne_bf16(w) for w in inp.W]
    c = O.forward(net_of(wl, "none"), inp.X, Wr, inp.R, inp.labels)
    assert np.array_equal(b.V[0], c.V[0]) and b.loss == c.loss


@pytest.mark.parametrize("recurrent", [(False, False), (True, True)])
def test_bf16_mode_backward_is_the_unrounded_sweep_on_rounded_weights(recurrent):
    """The bf16 product mode rounds W and R wherever they enter a product of the reverse sweep
    too (dS = dI W^T, g R^T), and nothing else: its gradients are bit for bit those of the
    unrounded sweep run on rne_bf16(W), rne_bf16(R), and they differ from the sweep on the
    unrounded weights.  A reverse sweep that forgot the rounding in one of its products fails."""
    rng = np.random.default_rng(61)
    net, X, W, R, lab = tiny_net(rng, sizes=(9, 7, 6, 4), recurrent=recurrent, T=12, B=3,
                                 surrogate="superspike", slope=25.0, gain=2.5, gemm_round="bf16")
    W = [w.astype(np.float32).astype(np.float64) for w in W]          # fp32-valued masters
    R = [None if r is None else r.astype(np.float32).astype(np.float64) for r in R]
    betas = _random_betas(rng, net)
    import dataclasses
    plain = dataclasses.replace(net, gemm_round="none")
    Wr = [O.rne_bf16(w) for w in W]
    Rr = [None if r is None else O.rne_bf16(r) for r in R]
    assert any(np.any(a != b) for a, b in zip(W, Wr))
    tr_b = O.forward(net, X, W, R, lab, betas=betas)
    gr_b = O.backward(net, X, W, R, lab, tr_b, betas=betas)
    tr_r = O.forward(plain, X, Wr, Rr, lab, betas=betas)
    gr_r = O.backward(plain, X, Wr, Rr, lab, tr_r, betas=betas)
    assert tr_b.S[0].sum() > 0 and tr_b.S[1].sum() > 0
    differs = False
    # the same forward trace handed to the sweep on unrounded weights: only the products differ
    gr_u = O.backward(plain, X, W, R, lab, tr_b, betas=betas)
    for l in range(net.L):
        assert np.array_equal(gr_b.dW[l], gr_r.dW[l])
        assert np.array_equal(gr_b.dbeta[l], gr_r.dbeta[l])
        differs |= bool(np.any(gr_b.dW[l] != gr_u.dW[l]))
    for l in range(net.L - 1):
        assert np.array_equal(gr_b.dI[l], gr_r.dI[l])
        assert np.array_equal(gr_b.dS[l], gr_r.dS[l])
        if R[l] is not None:
            assert np.array_equal(gr_b.dR[l], gr_r.dR[l])
            assert np.any(gr_b.dI[l] != gr_u.dI[l])                   # g R^T saw the rounded R
    assert differs
    assert np.any(gr_b.dS[0] != gr_u.dS[0])                           # dS = dI W^T saw the rounded W
    assert np.any(gr_b.dS[1] != gr_u.dS[1])                           # and so did the readout's


@pytest.mark.parametrize("recurrent", [(False, False), (True, True)])
def test_integral_loss_equals_scalar_brute_force(recurrent):
    """The integral cross-entropy, forward and reverse, one number at a time."""
    rng = np.random.default_rng(62)
    net, X, W, R, lab = tiny_net(rng, sizes=(6, 5, 4, 3), recurrent=recurrent, T=9, B=3,
                                 surrogate="superspike", slope=25.0, gain=2.5, loss="integral")
    betas = _random_betas(rng, net)
    tr = O.forward(net, X, W, R, lab, betas=betas)
    gr = O.backward(net, X, W, R, lab, tr, betas=betas)
    assert tr.S[0].sum() > 0 and tr.S[1].sum() > 0
    ref = snn_scalar.run(net.sizes, net.recurrent, [b.tolist() for b in betas], net.theta, "superspike", 25.0,
                         X.tolist(), [w.tolist() for w in W],
                         [None if r is None else r.tolist() for r in R], lab.tolist(), loss_kind="integral")
    assert np.allclose(tr.z, np.array(ref["z"]), atol=1e-12)
    assert tr.loss == pytest.approx(ref["loss"], abs=1e-12)
    assert np.allclose(gr.dz, np.array(ref["dz"]), atol=1e-14)
    for l in range(3):
        assert np.allclose(gr.dW[l], np.array(ref["dW"][l]), atol=1e-12)
        assert np.allclose(gr.dbeta[l], np.array(ref["dbeta"][l]), atol=1e-12)
    for l in range(2):
        if R[l] is not None:
            assert np.allclose(gr.dR[l], np.array(ref["dR"][l]), atol=1e-12)
    # and the scalar version's two losses differ on this network
    ref_max = snn_scalar.run(net.sizes, net.recurrent, [b.tolist() for b in betas], net.theta, "superspike", 25.0,
                             X.tolist(), [w.tolist() for w in W],
                             [None if r is None else r.tolist() for r in R], lab.tolist())
    assert abs(ref_max["loss"] - ref["loss"]) > 1e-3


def test_workload_generator_statistics():
    wl = workloads.CONFIGS["shd_ff128"].scaled(T=64, B=32)
    inp = workloads.generate(wl)
    assert inp.X.dtype == np.uint8 and inp.X.shape == (64, 32, 700) and inp.X.max() == 1
    assert 0.005 <= inp.rates.min() and inp.rates.max() <= 0.04
    assert abs(inp.X.mean() - inp.rates.mean()) < 2e-3
    assert abs(inp.W[0].std() * math.sqrt(700) - 1) < 0.02
    assert inp.labels.min() >= 0 and inp.labels.max() < 20
    again = workloads.generate(wl)
    assert np.array_equal(again.X, inp.X) and np.array_equal(again.W[1], inp.W[1])
