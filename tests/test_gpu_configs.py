"""GPU parity on the dense-neighbourhood and the sparse-large workloads at a fraction of their size: same
generators, same average degree, same layer widths and layer count (602 -> 128 -> 41 and 100 -> 256 -> 256 -> 47),
the Epoch call sequence bench.py times, fp32 and bf16 features.

Every call is checked on its own: the oracle gets the very inputs the GPU call had (the GPU's own previous
outputs, copied back), so a ReLU that flips between fp32 and fp64 cannot spread.  All rows, all elements:
|gpu - oracle| <= 1e-5 * sum|terms| (2e-2 with bf16 features).
"""
import functools

import numpy as np
import pytest

import oracle
from util import TOL_BF16, TOL_F32, check_bound, say, to_np

pytestmark = pytest.mark.gpu


@functools.lru_cache(maxsize=None)
def _small(name):
    from workloads import configs
    if name == "c3":        # 1/10 of the rows and of the edges: about 490 entries per row as in the full workload
        return configs.dense_neighbourhood(n=23_296, n_directed_edges=11_461_589)
    return configs.sparse_large(n=153_064, scale=18)       # 1/16: the same share of the R-MAT square survives the cut


@pytest.fixture(scope="module", params=[("c3", False), ("c3", True), ("c4", False), ("c4", True)],
                ids=["dense233k/10-f32", "dense233k/10-bf16", "sparse2m4/16-f32", "sparse2m4/16-bf16"])
def run(request):
    import torch
    import bench
    import paper_2212_05009_amd as gcn
    name, bf16 = request.param
    dev = torch.device("cuda:0")
    say(f"generating {name} (scaled), bf16={bf16}")
    w = _small(name)
    n = w["n"]
    og = oracle.graph_build(w["src"], w["dst"], n)
    say(f"gpu build n={n} nnz={og.nnz} dims={w['dims']}")
    A = gcn.gcn_csr_build(torch.from_numpy(w["src"]).to(dev), torch.from_numpy(w["dst"]).to(dev), n)
    X = torch.from_numpy(w["X"]).to(dev)
    if bf16:
        X = X.to(torch.bfloat16)
    Ws = [torch.from_numpy(m).to(dev) for m in w["W"]]
    ep = bench.Epoch(gcn, torch, A, X, Ws, torch.from_numpy(w["y"]).to(dev), bf16)
    ep.run()
    ep.run()
    torch.cuda.synchronize()
    return {"w": w, "og": og, "A": A, "ep": ep, "bf16": bf16, "tol": TOL_BF16 if bf16 else TOL_F32}


def test_arrays_bit_exact(run):
    og, A = run["og"], run["A"]
    assert (A.nr, A.nh, A.nnz) == (og.nr, 0, og.nnz)
    arr = A.arrays()
    for name in ["rowptr", "col", "deg", "colptr", "rowidx"]:
        assert np.array_equal(arr[name].cpu().numpy(), getattr(og, name)), name
    for name in ["val", "val_t"]:
        assert np.array_equal(arr[name].cpu().numpy().view(np.int32), getattr(og, name).view(np.int32)), name


def test_forward_layer_by_layer(run):
    w, og, ep, tol = run["w"], run["og"], run["ep"], run["tol"]
    L = len(w["W"])
    for k in range(L):
        last = k == L - 1
        f = oracle.layer_fwd(og, to_np(ep.H[k]), w["W"][k], act="none" if last else "relu")
        got = ep.Zlast if last else ep.H[k + 1]
        check_bound(to_np(got), f["Z"] if last else f["Hout"], f["Bz"], tol, f"layer {k} output")
        if ep.AH[k] is not None:
            _, bah = oracle.spmm(og.rowptr, og.col, og.val, np.abs(to_np(ep.H[k])))
            check_bound(to_np(ep.AH[k]), f["AH"], bah, tol, f"layer {k} saved A^ H")


def test_loss_and_output_gradient(run):
    w, og, ep, tol = run["w"], run["og"], run["ep"], run["tol"]
    L = len(w["W"])
    Z = to_np(ep.Zlast)
    loss, labs, G = oracle.softmax_xent(Z, w["y"], 1.0 / og.nr)
    assert abs(float(ep.loss.item()) - loss) <= TOL_F32 * max(labs, np.abs(Z).max() * 3)
    onehot = np.zeros_like(G); onehot[np.arange(og.nr), w["y"]] = 1.0 / og.nr
    check_bound(to_np(ep.G[L - 1]), G, G + 2 * onehot, tol, "output gradient")


def test_backward_layer_by_layer(run):
    w, og, ep, tol = run["w"], run["og"], run["ep"], run["tol"]
    L = len(w["W"])
    for k in range(L - 1, -1, -1):
        Hk = to_np(ep.H[k])
        b = oracle.layer_bwd(og, Hk, w["W"][k], to_np(ep.G[k]), Zprev=Hk if k > 0 else None, want_dH=k > 0)
        check_bound(to_np(ep.dW[k]), b["dW"], b["BdW"], tol, f"dW of layer {k}")
        if k > 0:
            check_bound(to_np(ep.G[k - 1]), b["dH"], b["BdH"], tol, f"gradient handed to layer {k - 1}")
