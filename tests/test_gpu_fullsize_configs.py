"""GPU parity at benchmark size on the configurations bench.py times besides the R-MAT 2^18 graph (which
test_gpu_fullsize.py covers): the dense-neighbourhood graph (233 k vertices, 114 M entries, 602 -> 128 -> 41), the
sparse large graph (2.45 M vertices, 126 M entries, 100 -> 256 -> 256 -> 47) with fp32 and with bf16 features, and
one processor's row block (2^22 owned rows, 5.8 M halo rows fetched from a pinned host table, 128 -> 128 -> 32).

Same generators, same sizes, same Epoch call sequence and buffer pitches as the benchmark, so the launch shapes
are the timed ones.  Checked: the graph arrays bit for bit; every call of the epoch on sampled rows / columns
recomputed by the oracle from the GPU's own inputs (util.check_epoch_sampled); for the block the gathered halo
rows bit for bit against the table's defining formula.  1e-5 * sum|terms| (2e-2 with bf16 features).
"""
import gc

import numpy as np
import pytest

import oracle
from util import TOL_BF16, TOL_F32, check_epoch_sampled, sample_rows, say

pytestmark = pytest.mark.gpu

CASES = [("c3_dense233k", "f32"), ("c4_sparse2m4", "f32"), ("c4_sparse2m4", "bf16"), ("c5_block", "f32")]
_held = {}        # one workload and its oracle graph at a time (the sparse large graph serves two cases)


def _workload(name):
    import bench
    from workloads import configs
    if _held.get("name") != name:
        _held.clear()
        gc.collect()
        say(f"generating {name}")
        w = configs.get(name, n_global=bench.pick_block_global_rows()) if name == "c5_block" else configs.get(name)
        say(f"oracle graph build: n={w['n']} raw edges={w['src'].size}")
        og = oracle.graph_build(w["src"], w["dst"], w["n"], w.get("row_lo", 0), w.get("row_hi", w["n"]),
                                deg_global=w.get("deg_global"))
        _held.update(name=name, w=w, og=og)
    return _held["w"], _held["og"]


@pytest.fixture(scope="module", params=CASES, ids=[f"{n}-{d}" for n, d in CASES])
def case(request):
    import torch
    import bench
    import paper_2212_05009_amd as gcn
    name, dtype = request.param
    bf16 = dtype == "bf16"
    dev = torch.device("cuda:0")
    w, og = _workload(name)
    n = w["n"]
    block = "row_lo" in w
    say(f"gpu build {name}: rows={og.nr} halo={og.nh} nnz={og.nnz} dims={w['dims']} {dtype}")
    A = gcn.gcn_csr_build(torch.from_numpy(w["src"]).to(dev), torch.from_numpy(w["dst"]).to(dev), n,
                          w.get("row_lo", 0), w.get("row_hi", n),
                          deg_global=torch.from_numpy(w["deg_global"]).to(dev) if block else None)
    table = None
    if block:
        from workloads import table as wtable
        say(f"pinned host table {n} x {w['dims'][0]}")
        table = torch.empty((n, w["dims"][0]), dtype=torch.float32, pin_memory=True)
        wtable.fill_table_torch(table, w["table_seed"], dev)
        X = table[w["row_lo"]: w["row_hi"]].to(dev)
    else:
        X = torch.from_numpy(w["X"]).to(dev)
        if bf16:
            X = X.to(torch.bfloat16)
    Ws = [torch.from_numpy(m).to(dev) for m in w["W"]]
    ep = bench.Epoch(gcn, torch, A, X, Ws, torch.from_numpy(w["y"]).to(dev), bf16, table=table)
    del X
    say("two epochs as bench.py runs them")
    ep.run()
    ep.run()
    torch.cuda.synchronize()
    yield {"w": w, "og": og, "A": A, "ep": ep, "bf16": bf16, "tol": TOL_BF16 if bf16 else TOL_F32, "table": table,
           "name": name}
    A.free()
    del ep, table
    gc.collect()
    torch.cuda.empty_cache()


def test_graph_arrays_bit_exact(case):
    og, A = case["og"], case["A"]
    assert (A.nr, A.nh, A.nnz) == (og.nr, og.nh, og.nnz)
    arr = A.arrays()
    names = ["rowptr", "col", "deg", "colptr", "rowidx"] + (["halo_gid"] if og.nh else [])
    for name in names:
        assert np.array_equal(arr[name].cpu().numpy(), getattr(og, name)), name
    for name in ["val", "val_t"]:
        assert np.array_equal(arr[name].cpu().numpy().view(np.int32), getattr(og, name).view(np.int32)), name
    del arr


def test_halo_rows_bit_exact(case):
    og, ep, w = case["og"], case["ep"], case["w"]
    if not og.nh:
        pytest.skip("whole graph: no halo rows")
    from workloads import table as wtable
    d = w["dims"][0]
    pick = np.unique(np.concatenate([[0, og.nh - 1], np.random.default_rng(5).integers(0, og.nh, 200_000)]))
    want = wtable.table_rows(og.halo_gid[pick], d, w["table_seed"])          # the table's defining formula, on the CPU
    import torch
    sel = torch.from_numpy(og.nr + pick).to(ep.H[0].device)
    for k in range(len(w["W"])):
        assert np.array_equal(ep.H[k][sel].cpu().numpy(), want), f"halo rows of layer input {k}"


def test_every_call_of_the_epoch(case):
    w, og, ep = case["w"], case["og"], case["ep"]
    rows = sample_rows(og, 1500, seed=7)
    check_epoch_sampled(ep, w, og, rows, case["tol"], log=say)
