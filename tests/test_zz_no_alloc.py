"""snn_weight_grad_static, the entry point that allocates nothing (its split partial sums live in
a static device array), against the weight-gradient step of a context (snn_run_step, partial sums
in the caller's workspace) on the same inputs: two calls in a row, the second on a smaller
product, so that the array still holds the first call's partial sums when the second runs."""
import ctypes as C

import numpy as np
import pytest

from tests import parity

pytestmark = pytest.mark.gpu


def context_weight_grad(T, B, K, N, X, G):
    """dW^1 = X^T G by the existing entry points: a K-N-4 network with fp32 products whose layer-1
    current gradients are imposed through snn_set_tensor."""
    from paper_2402_18994_amd.binding import SNN
    rng = np.random.default_rng(1)
    W = [rng.standard_normal((K, N)).astype(np.float32), rng.standard_normal((N, 4)).astype(np.float32)]
    snn = SNN(T, B, (K, N, 4), (False,), (0.9, 0.9), 1.0, "superspike", 25.0, "fp32", W)
    snn.set_tensor("d_current", 1, G.reshape(T, B, N))
    snn.run_step("weight_grad", 1, x=X.reshape(T, B, K))
    out = snn.get_tensor("grad_w", 1)
    snn.destroy()
    return out


@pytest.mark.parametrize("shapes", [[(64, 128, 700, 128), (31, 7, 44, 20)], [(40, 24, 300, 200), (16, 16, 64, 32)]],
                         ids=["headline-layer-then-ragged", "multi-tile-then-small"])
def test_static_scratch_weight_gradient_matches_the_context_step(shapes):
    import torch
    from paper_2402_18994_amd import binding
    dev = torch.device("cuda:0")
    for i, (T, B, K, N) in enumerate(shapes):
        rng = np.random.default_rng(100 + i)
        M = T * B
        X = (rng.random((M, K)) < 0.08).astype(np.uint8)
        G = (rng.standard_normal((M, N)) * 10.0 ** rng.integers(-4, 1, size=(M, 1))).astype(np.float32)
        print(f"\n[case] static weight gradient M={M} K={K} N={N}", flush=True)
        want = context_weight_grad(T, B, K, N, X, G)
        Xd, Gd = torch.from_numpy(X).to(dev), torch.from_numpy(G).to(dev)
        dW = torch.full((K, N), float("nan"), dtype=torch.float32, device=dev)
        binding.weight_grad_static(Xd, Gd, dW)
        torch.cuda.synchronize()
        got = dW.cpu().numpy()
        assert np.isfinite(got).all()
        parity.close_grad("dW static vs context", got, want)
        # both against the plain definition (fp64 contraction over all rows)
        ref = X.astype(np.float64).T @ G.astype(np.float64)
        parity.close_grad("dW static vs definition", got, ref)
        # bit-repeatable: the summation order is fixed
        dW2 = torch.empty_like(dW)
        binding.weight_grad_static(Xd, Gd, dW2)
        torch.cuda.synchronize()
        assert torch.equal(dW, dW2)


def test_static_scratch_entry_point_refuses_what_it_cannot_hold():
    import torch
    from paper_2402_18994_amd import binding
    lib = binding.load_library()
    dev = torch.device("cuda:0")
    S = torch.zeros((64, 8), dtype=torch.uint8, device=dev)
    G = torch.zeros((64, 8), dtype=torch.float32, device=dev)
    W = torch.zeros((8, 8), dtype=torch.float32, device=dev)
    call = lambda s, g, w, M, K, N: lib.snn_weight_grad_static(s, g, w, C.c_int64(M), K, N, None)
    assert call(None, G.data_ptr(), W.data_ptr(), 64, 8, 8) == 1
    assert call(S.data_ptr(), G.data_ptr(), W.data_ptr(), 0, 8, 8) == 2
    assert call(S.data_ptr(), G.data_ptr(), W.data_ptr(), 64, 6, 8) == 2          # K not a multiple of 4
    assert call(S.data_ptr(), G.data_ptr() + 4, W.data_ptr(), 64, 8, 8) == 2      # misaligned
    assert call(S.data_ptr(), G.data_ptr(), W.data_ptr(), 64, 2048, 2048) == 7    # K * N beyond the scratch
    assert call(S.data_ptr(), G.data_ptr(), W.data_ptr(), 1 << 25, 8, 8) == 7     # M beyond the limit
    assert b"static scratch" in lib.snn_last_error(None)
    assert call(S.data_ptr(), G.data_ptr(), W.data_ptr(), 64, 8, 8) == 0
    torch.cuda.synchronize()
    assert float(W.abs().max()) == 0.0
