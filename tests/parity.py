"""Parity harness: run the HIP path and the oracle on the same seeded inputs and compare.

Spike decisions where the oracle's potential is within BAND of the threshold may
legitimately go either way (fp32 on the device against fp64 in the oracle).  After
such a flip the sample's later trajectory differs, so the harness imposes the
device's decision on the oracle at the first mismatch of a sample (which must be
inside the band, else the test fails), re-runs the oracle for that sample and
repeats.  The number of imposed decisions is reported.
"""
from __future__ import annotations

import numpy as np

from oracle import snn_oracle as O

BAND = 1e-5          # |V - theta| below which a spike decision may differ
TOL_STATE = 1e-5     # potentials / readout: |a-b| <= TOL_STATE * max(1, |b|)
TOL_LOSS = 1e-5      # relative
TOL_GRAD = 1e-4      # per tensor, max norm and 2-norm, relative


class ParityError(AssertionError):
    pass


def _splice(tr: O.Trace, sub: O.Trace, idx: np.ndarray, B: int):
    for l in range(len(tr.S)):
        tr.I[l][:, idx] = sub.I[l]
        tr.V[l][:, idx] = sub.V[l]
        tr.S[l][:, idx] = sub.S[l]
        tr.A[l][:, idx] = sub.A[l]
        tr.v_final[l][idx] = sub.v_final[l]
    tr.J[:, idx] = sub.J
    tr.Y[:, idx] = sub.Y
    tr.z[idx] = sub.z
    tr.tstar[idx] = sub.tstar
    tr.loss_b[idx] = sub.loss_b
    tr.loss = float(tr.loss_b.sum() / B)


def reconciled_forward(net: O.Net, X, W, R, labels, S_gpu, max_rounds: int = 200, band: float = BAND, betas=None):
    """Oracle forward with the device's near-threshold decisions imposed.

    S_gpu: list of uint8 arrays [T,B,N] per spiking layer.  Returns (trace, n_imposed).
    """
    T, B, _ = X.shape
    tr = O.forward(net, X, W, R, labels, betas=betas)
    forced = {b: {} for b in range(B)}          # per sample: (l,t) -> [(n,val)]
    imposed = 0
    for _ in range(max_rounds):
        todo = []
        for l in range(net.L - 1):
            diff = tr.S[l] != S_gpu[l]
            if not diff.any():
                continue
            for b in np.flatnonzero(diff.any(axis=(0, 2))):
                if any(b == bb for bb, _, _ in todo):
                    continue
                t = int(np.flatnonzero(diff[:, b].any(axis=1))[0])
                todo.append((int(b), l, t))
            # a sample whose first mismatch is in layer l must be fixed before its
            # higher layers are looked at
        if not todo:
            return tr, imposed
        idx = np.array(sorted({b for b, _, _ in todo}))
        for b, l, t in todo:
            ns = np.flatnonzero(tr.S[l][t, b] != S_gpu[l][t, b])
            for n in ns:
                dist = abs(tr.V[l][t, b, n] - net.theta - tr.A[l][t, b, n])      # to the threshold in force
                if dist > band:
                    raise ParityError(f"spike mismatch outside the band: layer {l + 1} t={t} b={b} n={n} "
                                      f"|V-theta|={dist:.3e} oracle V={tr.V[l][t, b, n]!r} "
                                      f"device spike={int(S_gpu[l][t, b, n])}")
                forced[b].setdefault((l, t), []).append((int(n), int(S_gpu[l][t, b, n])))
                imposed += 1
        sub_forced = {}
        for j, b in enumerate(idx):
            for key, lst in forced[int(b)].items():
                sub_forced.setdefault(key, []).extend((j, n, v) for n, v in lst)
        sub = O.forward(net, X[:, idx], W, R, labels[idx], forced=sub_forced, batch_norm=B, betas=betas)
        _splice(tr, sub, idx, B)
    raise ParityError("spike reconciliation did not converge")


def close_state(name, a, b, tol=TOL_STATE, count_above=None):
    """|a - b| <= tol max(1, |b|) element by element; returns the largest scaled error.
    `count_above`: a dict that receives, under `name`, how many elements exceed TOL_STATE (for
    cases that are held to a wider band and report how often the standard one is passed)."""
    a = np.asarray(a, np.float64); b = np.asarray(b, np.float64)
    err = np.abs(a - b) / np.maximum(1.0, np.abs(b))
    if count_above is not None:
        count_above[name] = int((err > TOL_STATE).sum())
        count_above["_elements"] = count_above.get("_elements", 0) + err.size
    if not (err.max() <= tol):
        i = np.unravel_index(np.argmax(err), err.shape)
        raise ParityError(f"{name}: max scaled error {err.max():.3e} > {tol:g} at {i}: device {a[i]!r} oracle {b[i]!r}")
    return float(err.max())


def close_grad(name, a, b, tol=TOL_GRAD):
    a = np.asarray(a, np.float64); b = np.asarray(b, np.float64)
    ninf = np.abs(b).max()
    n2 = np.sqrt((b * b).sum())
    einf = np.abs(a - b).max()
    e2 = np.sqrt(((a - b) ** 2).sum())
    if ninf == 0:
        if einf != 0:
            raise ParityError(f"{name}: oracle gradient is zero, device max {einf:.3e}")
        return 0.0, 0.0
    if not (einf <= tol * ninf and e2 <= tol * n2):
        raise ParityError(f"{name}: rel max-norm error {einf / ninf:.3e}, rel 2-norm error {e2 / n2:.3e} > {tol:g}")
    return float(einf / ninf), float(e2 / n2)


def compare_forward(net: O.Net, inp, snn, loss_gpu, report=None, betas=None):
    """Fetch the device's forward tensors and check them against the reconciled oracle."""
    Lh = net.L - 1
    S_gpu = [snn.get_tensor("spikes", l + 1) for l in range(Lh)]
    tr, imposed = reconciled_forward(net, inp.X, inp.W, inp.R, inp.labels, S_gpu, betas=betas)
    rep = {"imposed_decisions": imposed, "spike_rate": [float(s.mean()) for s in S_gpu]}
    for l in range(Lh):
        assert np.array_equal(S_gpu[l], tr.S[l].astype(np.uint8))
        rep[f"V{l + 1}"] = close_state(f"V^{l + 1}", snn.get_tensor("membrane", l + 1), tr.V[l])
        rep[f"I{l + 1}"] = close_state(f"I^{l + 1}", snn.get_tensor("current", l + 1), tr.I[l])
        if net.adapt_step is not None and net.adapt_step[l] > 0:
            rep[f"A{l + 1}"] = close_state(f"A^{l + 1}", snn.get_tensor("adaptation", l + 1), tr.A[l])
    rep["Y"] = close_state("Y", snn.get_tensor("readout_trace"), tr.Y)
    rep["z"] = close_state("z", snn.get_tensor("logits"), tr.z)
    # first maximiser: must agree unless two steps tie within tolerance; then follow the device
    ts = snn.get_tensor("argmax_t")
    bad = np.argwhere(ts != tr.tstar)
    for b, c in bad:
        if abs(tr.Y[ts[b, c], b, c] - tr.z[b, c]) > TOL_STATE * max(1.0, abs(tr.z[b, c])):
            raise ParityError(f"argmax over time differs at b={b} c={c}: device {ts[b, c]} oracle {tr.tstar[b, c]}")
        tr.tstar[b, c] = ts[b, c]
    rep["argmax_ties"] = int(len(bad))
    rel = abs(loss_gpu - tr.loss) / abs(tr.loss)
    if not rel <= TOL_LOSS:
        raise ParityError(f"loss: device {loss_gpu!r} oracle {tr.loss!r} rel {rel:.3e}")
    rep["loss_rel"] = float(rel)
    # a sample's loss is logsumexp(z) - z[label]: it inherits the absolute error of the logits,
    # which are compared at TOL_STATE * max(1, |z|)
    zscale = np.maximum(1.0, np.abs(tr.z).max(axis=1))
    lb = snn.get_tensor("loss_per_sample")
    if not np.all(np.abs(lb - tr.loss_b) <= 2 * TOL_STATE * zscale):
        raise ParityError(f"per-sample loss: max error {np.abs(lb - tr.loss_b).max():.3e}")
    if report is not None:
        report.update(rep)
    return tr


def compare_backward(net: O.Net, inp, snn, tr, report=None, tol=TOL_GRAD, betas=None, learn_beta=False):
    gr = O.backward(net, inp.X, inp.W, inp.R, inp.labels, tr, betas=betas)
    rep = {}
    close_grad("dz", snn.get_tensor("d_logits"), gr.dz, tol)
    # current gradients
    rep["dJ"] = close_grad("dJ", snn.get_tensor("d_readout_current"), gr.dJ, tol)
    for l in range(net.L - 1):
        dI = snn.get_tensor("d_current", l + 1)
        rep[f"dI{l + 1}"] = close_grad(f"dI^{l + 1}", dI, gr.dI[l], tol)
        assert np.all(dI[-1] == 0)
    for l in range(net.L - 1):
        if l < net.L - 1:
            rep[f"dS{l + 1}"] = close_grad(f"dS^{l + 1}", snn.get_tensor("d_spikes", l + 1), gr.dS[l], tol)
    for l in range(net.L):
        rep[f"dW{l + 1}"] = close_grad(f"dW^{l + 1}", snn.get_tensor("grad_w", l + 1), gr.dW[l], tol)
    for l in range(net.L - 1):
        if inp.R[l] is not None:
            rep[f"dR{l + 1}"] = close_grad(f"dR^{l + 1}", snn.get_tensor("grad_r", l + 1), gr.dR[l], tol)
    if learn_beta:
        for l in range(net.L):
            rep[f"dbeta{l + 1}"] = close_grad(f"dbeta^{l + 1}", snn.get_tensor("grad_beta", l + 1), gr.dbeta[l], tol)
    if report is not None:
        report.update(rep)
    return gr


def sampled_step_parity(net: O.Net, inp, snn, loss_gpu, idx, n_rows=48, seed=0, report=None, tol=TOL_GRAD,
                        tol_state=TOL_STATE, band=BAND):
    """Parity at sizes where the oracle is run on a subset of the batch.

    Samples of a batch only meet in the mean of the loss and in the sums over rows that
    give dW and dR.  So (a) the oracle runs forward and backward on the samples `idx`
    alone; every per-sample tensor of the device (currents, potentials, spikes, readout,
    logits, first maximiser, per-sample loss, and dz, dJ, dI, dS scaled by |idx|/B for the
    1/B of the batch mean) is compared on those samples at the usual tolerances; (b) the
    device's loss must be the mean of its per-sample losses; (c) rows of dW^l and dR^l
    drawn at random must equal the fp64 contraction over all T*B rows of the device's own
    spikes and current gradients, which checks the split products at full size given their
    inputs (the inputs themselves are covered by (a) on the sampled chains).
    snn.backward() must have been called.
    """
    idx = np.asarray(idx)
    B = inp.X.shape[1]
    Lh = net.L - 1
    rep = {}
    Xs, ls = inp.X[:, idx], inp.labels[idx]
    S_full = [snn.get_tensor("spikes", l + 1) for l in range(Lh)]
    tr, imposed = reconciled_forward(net, Xs, inp.W, inp.R, ls, [s[:, idx] for s in S_full], band=band)
    rep["imposed_decisions"] = imposed
    rep["spike_rate"] = [float(s.mean()) for s in S_full]
    above = {}
    for l in range(Lh):
        assert np.array_equal(S_full[l][:, idx], tr.S[l].astype(np.uint8))
        rep[f"V{l + 1}"] = close_state(f"V^{l + 1}", snn.get_tensor("membrane", l + 1)[:, idx], tr.V[l], tol_state, above)
        rep[f"I{l + 1}"] = close_state(f"I^{l + 1}", snn.get_tensor("current", l + 1)[:, idx], tr.I[l], tol_state, above)
    rep["Y"] = close_state("Y", snn.get_tensor("readout_trace")[:, idx], tr.Y, tol_state, above)
    rep["z"] = close_state("z", snn.get_tensor("logits")[idx], tr.z, tol_state, above)
    rep["state_elements"] = above.pop("_elements")
    rep["above_1e-5"] = above
    ts = snn.get_tensor("argmax_t")[idx]
    bad = np.argwhere(ts != tr.tstar)
    for b, c in bad:
        if abs(tr.Y[ts[b, c], b, c] - tr.z[b, c]) > tol_state * max(1.0, abs(tr.z[b, c])):
            raise ParityError(f"argmax over time differs at sample {idx[b]} c={c}")
        tr.tstar[b, c] = ts[b, c]
    rep["argmax_ties"] = int(len(bad))
    lb = snn.get_tensor("loss_per_sample")
    zscale = np.maximum(1.0, np.abs(tr.z).max(axis=1))
    if not np.all(np.abs(lb[idx] - tr.loss_b) <= 2 * tol_state * zscale):
        raise ParityError(f"per-sample loss: max error {np.abs(lb[idx] - tr.loss_b).max():.3e}")
    mean = float(lb.astype(np.float64).mean())
    if not abs(loss_gpu - mean) <= TOL_LOSS * abs(mean):
        raise ParityError(f"loss {loss_gpu!r} is not the mean of the per-sample losses {mean!r}")

    gr = O.backward(net, Xs, inp.W, inp.R, ls, tr)
    k = len(idx) / B
    close_grad("dz", snn.get_tensor("d_logits")[idx], gr.dz * k, tol)
    dJ_full = snn.get_tensor("d_readout_current")
    rep["dJ"] = close_grad("dJ", dJ_full[:, idx], gr.dJ * k, tol)
    dI_full = []
    for l in range(Lh):
        dI = snn.get_tensor("d_current", l + 1)
        dI_full.append(dI)
        rep[f"dI{l + 1}"] = close_grad(f"dI^{l + 1}", dI[:, idx], gr.dI[l] * k, tol)
        rep[f"dS{l + 1}"] = close_grad(f"dS^{l + 1}", snn.get_tensor("d_spikes", l + 1)[:, idx], gr.dS[l] * k, tol)
    dI_full.append(dJ_full)

    rng = np.random.default_rng(seed)

    def rows_of(name, got, src, d):
        # got[rows] against sum over (t, b) of src[t, b, rows]^T d[t, b, :]
        K = src.shape[2]
        rows = np.sort(rng.choice(K, size=min(n_rows, K), replace=False))
        a = src[:, :, rows].reshape(-1, len(rows)).astype(np.float64)
        want = a.T @ d.reshape(-1, d.shape[2]).astype(np.float64)
        return close_grad(name, got[rows], want, tol)

    below = [inp.X] + S_full
    for l in range(net.L):
        rep[f"dW{l + 1}"] = rows_of(f"dW^{l + 1}", snn.get_tensor("grad_w", l + 1), below[l], dI_full[l])
    for l in range(Lh):
        if inp.R[l] is not None:
            # S_t R enters V_{t+1} beside I_t, so dR pairs S_t with the gradient of I_t
            rep[f"dR{l + 1}"] = rows_of(f"dR^{l + 1}", snn.get_tensor("grad_r", l + 1), S_full[l], dI_full[l])
    if report is not None:
        report.update(rep)
    return rep
