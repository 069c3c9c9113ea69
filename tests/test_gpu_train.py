"""GPU parity of a whole training run: forward, loss, backward and the gradient-descent update, repeated.

The oracle's loop (oracle.train) keeps the same arrays in fp32 between steps and sums in fp64.  Per epoch the
loss must agree within 1e-5 * (1 + epoch) relative (errors of earlier epochs feed the later ones; a ReLU whose
input is within rounding of zero may switch differently on the two sides, which moves the loss by far less),
and the final weights within 1e-4 absolute.  The weight update alone is one fused multiply-add:
|gpu - oracle| <= 1e-6 * (|W| + |lr dW|).
"""
import numpy as np
import pytest

import oracle
from util import say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gcn():
    import paper_2212_05009_amd as g
    return g


@pytest.fixture(scope="module")
def dev():
    import torch
    assert torch.cuda.is_available()
    return torch.device("cuda:0")


def test_sgd_update(gcn, dev):
    import torch
    rng = np.random.default_rng(2)
    for n in (1, 255, 128 * 16, 100003):
        W = rng.standard_normal(n).astype(np.float32); dW = rng.standard_normal(n).astype(np.float32)
        Wd = torch.from_numpy(W).to(dev); dWd = torch.from_numpy(dW).to(dev)
        say(f"sgd n={n}")
        gcn.gcn_sgd_update(Wd, dWd, 0.37)
        torch.cuda.synchronize()
        want = oracle.sgd_update(W, dW, np.float32(0.37))
        lim = 1e-6 * (np.abs(W) + np.abs(np.float32(0.37) * dW))
        assert np.all(np.abs(Wd.cpu().numpy().astype(np.float64) - want) <= lim)
    with pytest.raises(TypeError):
        gcn.gcn_sgd_update(torch.zeros(4, device=dev), torch.zeros(5, device=dev), 0.1)


def test_training_run_config1(gcn, dev, c1):
    import torch
    w = c1
    n, dims = w["n"], w["dims"]
    epochs, lr = 12, 0.8
    og = oracle.graph_build(w["src"], w["dst"], n)
    want_losses, want_W = oracle.train(og, w["X"], w["W"], w["y"], lr, epochs)
    A = gcn.gcn_csr_build(torch.from_numpy(w["src"]).to(dev), torch.from_numpy(w["dst"]).to(dev), n)
    X = torch.from_numpy(w["X"]).to(dev)
    Ws = [torch.from_numpy(m.copy()).to(dev) for m in w["W"]]
    y = torch.from_numpy(w["y"]).to(dev)
    H1 = torch.empty(n, dims[1], device=dev); Z2 = torch.empty(n, dims[2], device=dev)
    G2 = torch.empty_like(Z2); G1 = torch.empty_like(H1)
    dWs = [torch.empty_like(W) for W in Ws]
    loss = torch.zeros(1, device=dev)
    got = []
    say(f"training n={n} dims={dims} epochs={epochs}")
    for _ in range(epochs):
        gcn.gcn_layer_fwd(A, X, Ws[0], H1, act=gcn.ACT_RELU)
        gcn.gcn_layer_fwd(A, H1, Ws[1], Z2, act=gcn.ACT_NONE)
        gcn.gcn_softmax_xent(Z2, y, 1.0 / n, loss, G2)
        got.append(float(loss.item()))
        gcn.gcn_layer_bwd(A, H1, Ws[1], G2, dWs[1], dH=G1, Zprev=H1)
        gcn.gcn_layer_bwd(A, X, Ws[0], G1, dWs[0])
        for W, dW in zip(Ws, dWs):
            gcn.gcn_sgd_update(W, dW, lr)
    torch.cuda.synchronize()
    assert all(b < a for a, b in zip(got, got[1:])), got
    for e, (a, b) in enumerate(zip(got, want_losses)):
        assert abs(a - b) <= 1e-5 * (1 + e) * abs(b), (e, a, b)
    for W, Wo in zip(Ws, want_W):
        assert np.max(np.abs(W.cpu().numpy() - Wo)) <= 1e-4
    A.free()
