"""GPU parity of a whole training run: forward, loss, backward and the gradient-descent update, repeated.

Every call (layer forward, loss, layer backward, weight update) of the checked epochs is compared with the oracle
on the GPU's own inputs of that call at the contract's tolerance, 1e-5 * sum|terms| per element; oracle.train, the
oracle's own loop, is pinned on the CPU (finite differences of the dense model for two and three layers).
"""
import numpy as np
import pytest

import oracle
from util import TOL_F32, check_bound, say, to_np

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


def _train_and_check(gcn, dev, w, epochs, lr, checked_epochs):
    """Trains with the benchmark's call sequence (bench.Epoch) plus gcn_sgd_update, and checks EVERY call of the
    epochs in `checked_epochs` against the oracle at the contract's tolerance: the oracle gets the very arrays the
    GPU call had (copied back), so rounding differences of earlier calls and epochs cannot spread into the
    comparison.  The weight update is one fused multiply-add per element: terms W and lr * dW."""
    import torch
    import bench
    n, dims = w["n"], w["dims"]
    L = len(w["W"])
    og = oracle.graph_build(w["src"], w["dst"], n)
    A = gcn.gcn_csr_build(torch.from_numpy(w["src"]).to(dev), torch.from_numpy(w["dst"]).to(dev), n)
    Ws = [torch.from_numpy(m.copy()).to(dev) for m in w["W"]]
    ep = bench.Epoch(gcn, torch, A, torch.from_numpy(w["X"]).to(dev), Ws, torch.from_numpy(w["y"]).to(dev), False)
    losses = []
    for e in range(epochs):
        W_before = [to_np(W).copy() for W in Ws]
        say(f"training n={n} dims={dims} epoch {e}")
        ep.run()
        torch.cuda.synchronize()
        losses.append(float(ep.loss.item()))
        if e in checked_epochs:
            for k in range(L):
                last = k == L - 1
                f = oracle.layer_fwd(og, to_np(ep.H[k]), W_before[k], act="none" if last else "relu")
                check_bound(to_np(ep.Zlast if last else ep.H[k + 1]), f["Z"] if last else f["Hout"], f["Bz"], TOL_F32,
                            f"epoch {e} layer {k} output")
            Z = to_np(ep.Zlast)
            loss, labs, G = oracle.softmax_xent(Z, w["y"], 1.0 / n)
            assert abs(losses[-1] - loss) <= TOL_F32 * max(labs, np.abs(Z).max() * 3)
            onehot = np.zeros_like(G); onehot[np.arange(n), w["y"]] = 1.0 / n
            check_bound(to_np(ep.G[L - 1]), G, G + 2 * onehot, TOL_F32, f"epoch {e} output gradient")
            for k in range(L - 1, -1, -1):
                Hk = to_np(ep.H[k])
                b = oracle.layer_bwd(og, Hk, W_before[k], to_np(ep.G[k]), Zprev=Hk if k > 0 else None, want_dH=k > 0)
                check_bound(to_np(ep.dW[k]), b["dW"], b["BdW"], TOL_F32, f"epoch {e} dW of layer {k}")
                if k > 0:
                    check_bound(to_np(ep.G[k - 1]), b["dH"], b["BdH"], TOL_F32, f"epoch {e} gradient handed to layer {k - 1}")
        dWs = [to_np(dW).copy() for dW in ep.dW]
        for W, dW in zip(Ws, ep.dW):
            gcn.gcn_sgd_update(W, dW, lr)
        torch.cuda.synchronize()
        for k in range(L):
            want = oracle.sgd_update(W_before[k], dWs[k], np.float32(lr))
            bound = np.abs(W_before[k].astype(np.float64)) + np.abs(np.float64(np.float32(lr)) * dWs[k])
            check_bound(to_np(Ws[k]), want, bound, TOL_F32, f"epoch {e} weight update of layer {k}")
    A.free()
    return losses, [to_np(W) for W in Ws], og


def test_training_run_config1(gcn, dev, c1):
    """12 epochs on the smallest configuration, every call of every epoch checked; the loss must fall all the way.
    Against the oracle's own training loop the two loss curves are compared as a plausibility figure only (1e-3
    relative): they are two different roundings of a nonlinear iteration, for which the contract states no bound;
    the per-call checks above are the parity test."""
    w = c1
    epochs, lr = 12, 0.8
    got, Wg, og = _train_and_check(gcn, dev, w, epochs, lr, checked_epochs=set(range(epochs)))
    assert all(b < a for a, b in zip(got, got[1:])), got
    want_losses, want_W = oracle.train(og, w["X"], w["W"], w["y"], lr, epochs)
    for a, b in zip(got, want_losses):
        assert abs(a - b) <= 1e-3 * abs(b)


def test_training_run_config2(gcn, dev):
    """Three epochs on the R-MAT 2^18 configuration at full size (128 -> 128 -> 16), the first and the last checked
    call by call (every element of every result); the loss must fall."""
    from workloads import configs
    say("generating c2_rmat18")
    w = configs.get("c2_rmat18")
    got, _, _ = _train_and_check(gcn, dev, w, epochs=3, lr=0.5, checked_epochs={0, 2})
    assert all(b < a for a, b in zip(got, got[1:])), got
