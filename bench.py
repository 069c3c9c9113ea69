#!/usr/bin/env python3
"""Benchmark of the full-batch GCN epoch (forward, loss, backward over all layers) on one MI355X.

One "step" is one epoch over one seeded synthetic graph, with graph, features and weights already
resident in HBM; the CSR/CSC build is set-up and is reported separately.  Prints ONE JSON line: the
headline workload (the largest full-graph configuration, c4_sparse2m4, fp32) with its roofline objects and
the CPU baseline, and under "others" the same kind of record for the row block (c5_block), the bf16 variant
and the smaller configurations, each timed in this process with the same --steps / --warmup.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4_sparse2m4] [--dtype f32|bf16]
                    [--others all|none] [--no-cpu-baseline] [--cpu-sample-frac F]
"""
from __future__ import annotations

import argparse
import glob
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}
HEADLINE = "c4_sparse2m4"
GRAPH_REPLAY_WORKLOADS = ("c1_er4096", "c2_rmat18")      # short epochs: also timed as one graph launch per epoch
T_START = time.time()


def log(msg):
    print(f"[bench +{time.time() - T_START:5.0f}s] {msg}", file=sys.stderr, flush=True)


def sparse_sources_digest():
    """Short hash of the sparse-product sources: counter readings under profiles/ are tied to it."""
    h = hashlib.sha1()
    for p in sorted(glob.glob(os.path.join(ROOT, "paper_2212_05009_amd", "csrc", "spmm*"))):
        h.update(open(p, "rb").read())
    return h.hexdigest()[:12]


class Epoch:
    """Buffers and call sequence of one epoch; every step is a call into the C-ABI library.

    Works on a row block: layer inputs hold the nr owned rows followed by the nh halo rows.  The halo rows
    of every layer input are fetched through the halo index list from `table` (the stand-in for the rows
    other processors would send) at the start of that layer, inside the timed epoch.  Every buffer that a
    sparse product gathers from is allocated with the row pitch the library recommends (gcn_feature_ld).
    """

    def __init__(self, gcn, torch, A, X_owned, Ws, y, bf16, table=None, overlap=True, backward="push"):
        self.gcn, self.torch, self.A, self.Ws, self.y, self.table = gcn, torch, A, Ws, y, table
        dev = X_owned.device
        fdt = torch.bfloat16 if bf16 else torch.float32
        dims = [X_owned.shape[1]] + [W.shape[1] for W in Ws]
        self.dims, self.L = dims, len(Ws)
        nr, nc = A.nr, A.nc
        assert (A.nh == 0) == (table is None), "a block with halo rows needs a table to fetch them from"
        self.halo_gid = A.arrays()["halo_gid"] if A.nh else None

        assert backward in ("push", "pull")
        self.pull = backward == "pull"

        def fbuf(rows, d):
            if self.pull:       # the pull-form entry point takes dense dH / Zprev / T
                return torch.empty(rows, d, dtype=fdt, device=dev)
            return gcn.feature_buffer(rows, d, fdt, dev)
        # H[k]: input of layer k, [nc, dims[k]]; the owned rows of H[k+1] are layer k's output
        self.H = [fbuf(nc, dims[k]) for k in range(self.L)]
        self.H[0][:nr] = X_owned
        # pre-activations are kept for the last layer only: a hidden layer's ReLU mask [Z > 0] is read
        # off its output H = max(Z, 0), which is positive exactly where Z is
        self.Zlast = torch.empty(nr, dims[self.L], dtype=fdt, device=dev)
        # D[k]: gradient w.r.t. the input rows of layer k+1 ([nc, dims[k+1]]: owned rows, then this block's
        # contributions to halo rows); its owned rows are G[k], the gradient w.r.t. Z of layer k
        # backward="pull" (Algorithm 2, symmetric graphs): D[k] holds the owned rows of G^k, complete, followed by
        # the halo rows of G^k fetched like those of H (from the table, the stand-in for what other processors
        # hold); the last layer then needs the full height too, and T[k] receives A^ [G; G_halo]
        self.D = [fbuf(nc, dims[k + 1]) for k in range(self.L if self.pull else self.L - 1)]
        self.G = [d[:nr] for d in self.D] + ([] if self.pull else [fbuf(nr, dims[self.L])])
        if self.pull:
            assert table is None or max(dims[1:]) <= table.shape[1], "the stand-in table is narrower than a gradient row"
            self.T = [torch.empty(nr, dims[k + 1], dtype=fdt, device=dev) for k in range(self.L)]
        # A^ H is kept for the weight gradient where the forward pass computes it anyway
        self.AH = [torch.empty(nr, dims[k], dtype=fdt, device=dev) if dims[k] <= dims[k + 1] else None
                   for k in range(self.L)]
        self.dW = [torch.empty_like(W) for W in Ws]
        self.loss = torch.zeros(1, device=dev)
        # a block with halo rows runs Algorithm 1's overlap: the halo rows of a layer input arrive on a second
        # stream while the product with the owned columns runs; the halo columns are added once they are there
        self.overlap = bool(A.nh) and overlap
        if self.overlap:
            self.side = torch.cuda.Stream()
            self.P = [None if self.AH[k] is not None else fbuf(nc, dims[k + 1]) for k in range(self.L)]

    def run(self):
        g, A, L, nr = self.gcn, self.A, self.L, self.A.nr
        for k in range(L):
            last = k == L - 1
            out = self.Zlast if last else self.H[k + 1][:nr]
            act = g.ACT_NONE if last else g.ACT_RELU
            if self.overlap:
                self.forward_overlapped(k, out, act)
                continue
            if A.nh:
                g.gcn_halo_gather(self.table, self.halo_gid, self.H[k][nr:])
            g.gcn_layer_fwd_ld(A, self.H[k], self.Ws[k], out, act=act, AH_save=self.AH[k])
        g.gcn_softmax_xent(self.Zlast, self.y, 1.0 / nr, self.loss, self.G[L - 1])
        for k in range(L - 1, -1, -1):
            if self.pull:
                self.backward_pull(k)
                continue
            g.gcn_layer_bwd_ld(A, self.H[k], self.Ws[k], self.G[k], self.dW[k],
                               dH=self.D[k - 1] if k > 0 else None, Zprev=self.H[k][:nr] if k > 0 else None,
                               AH_saved=self.AH[k])

    def backward_pull(self, k):
        """Layer k backward as Algorithm 2: fetch the halo rows of G^k, T = A^ [G; G_halo], dH and dW from T."""
        g, A, torch, nr = self.gcn, self.A, self.torch, self.A.nr
        D, d = self.D[k], self.dims[k + 1]
        args = dict(dH=self.D[k - 1][:nr] if k > 0 else None, Zprev=self.H[k][:nr] if k > 0 else None)
        if not A.nh:
            g.gcn_layer_bwd_pull(A, self.H[k], self.Ws[k], D, self.T[k], self.dW[k], **args)
        elif not self.overlap:
            g.gcn_halo_gather(self.table[:, :d], self.halo_gid, D[nr:])
            g.gcn_layer_bwd_pull(A, self.H[k], self.Ws[k], D, self.T[k], self.dW[k], **args)
        else:
            main = torch.cuda.current_stream()
            self.side.wait_stream(main)
            with torch.cuda.stream(self.side):
                g.gcn_halo_gather(self.table[:, :d], self.halo_gid, D[nr:])
            g.gcn_layer_bwd_pull(A, self.H[k], self.Ws[k], D, self.T[k], self.dW[k], phase=g.PART_LOCAL)
            main.wait_stream(self.side)
            g.gcn_layer_bwd_pull(A, self.H[k], self.Ws[k], D, self.T[k], self.dW[k], phase=g.PART_HALO, **args)

    def forward_overlapped(self, k, out, act):
        """Layer k forward with the halo fetch under way during the owned-column product (same sums as
        gcn_layer_fwd: sparse product first where the input is the narrower side, dense product first else)."""
        g, A, torch, nr = self.gcn, self.A, self.torch, self.A.nr
        H, W = self.H[k], self.Ws[k]
        main = torch.cuda.current_stream()
        self.side.wait_stream(main)        # the rows being replaced were read by the previous epoch's backward pass
        with torch.cuda.stream(self.side):
            g.gcn_halo_gather(self.table, self.halo_gid, H[nr:])
        if self.AH[k] is not None:
            g.gcn_spmm_part(A, g.PART_LOCAL, H, self.AH[k])
            main.wait_stream(self.side)
            g.gcn_spmm_part(A, g.PART_HALO, H, self.AH[k])
            g.gcn_dense_fwd(self.AH[k], W, out, act=act)
        else:
            P = self.P[k]
            g.gcn_dense_fwd(H[:nr], W, P[:nr])
            g.gcn_spmm_part(A, g.PART_LOCAL, P, out)
            main.wait_stream(self.side)
            g.gcn_dense_fwd(H[nr:], W, P[nr:])
            g.gcn_spmm_part(A, g.PART_HALO, P, out, epilogue=g.EPI_RELU if act == g.ACT_RELU else g.EPI_NONE)


def oracle_threads(n):
    """Sets the OpenMP thread count the oracle's loops will use (the oracle itself is left as it stands)."""
    import ctypes
    ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))


def cpu_baseline(w, frac, threads=None):
    """Time the oracle, as it stands, on one epoch over the first frac of the workload's owned rows."""
    import numpy as np
    import oracle
    from workloads import configs
    n, dims = w["n"], w["dims"]
    lo, hi_all = w.get("row_lo", 0), w.get("row_hi", n)
    hi = lo + max(1, int((hi_all - lo) * frac))
    all_threads = oracle.num_threads()
    t0 = time.time()
    deg = w.get("deg_global")
    if deg is None:
        deg = oracle.graph_build(w["src"], w["dst"], n).deg
    blk = oracle.graph_build(w["src"], w["dst"], n, lo, hi, deg_global=deg)
    in_all = int(np.count_nonzero((w["src"] >= lo) & (w["src"] < hi_all)))
    in_blk = int(np.count_nonzero((w["src"] >= lo) & (w["src"] < hi)))
    log(f"oracle graph built in {time.time() - t0:.1f}s: rows={blk.nr} halo={blk.nh} nnz={blk.nnz}")
    L = len(dims) - 1
    Hs = [configs.features(blk.nc, dims[k], 900 + k) for k in range(L)]
    Zl = configs.features(blk.nr, dims[L], 990)
    if threads is not None:
        oracle_threads(threads)
    try:
        t0 = time.time()
        for k in range(L):
            oracle.layer_fwd(blk, Hs[k], w["W"][k], act="none" if k == L - 1 else "relu")
        _, _, G = oracle.softmax_xent(Zl, w["y"][: blk.nr], 1.0 / blk.nr)
        G = G.astype(np.float32)
        for k in range(L - 1, -1, -1):
            b = oracle.layer_bwd(blk, Hs[k], w["W"][k], G, Zprev=Hs[k][: blk.nr] if k > 0 else None, want_dH=k > 0)
            if k > 0:
                G = b["dH"][: blk.nr].astype(np.float32)
        sec = time.time() - t0
        used = oracle.num_threads()
    finally:
        if threads is not None:
            oracle_threads(all_threads)
    scale = in_all / max(in_blk, 1)
    return {"value": sec * 1e3 * scale, "unit": "ms/epoch", "cores": used, "kind": "oracle",
            "sample": f"one epoch (all layers forward, loss, backward; fp64, with bound sums; halo rows taken as "
                      f"given) on rows [{lo},{hi}) of the same graph ({in_blk} of {in_all} raw edges, {blk.nnz} stored "
                      f"entries, halo {blk.nh} rows) took {sec:.2f}s; value = that time x {scale:.2f} (ratio of raw edges)"}


def summarise(recs, steps):
    groups = {}
    for r in recs:
        key = (r["kind"], r["d"], r["rows"], r["inner"])
        q = groups.setdefault(key, {"kind": r["kind"], "d": r["d"], "rows": r["rows"], "inner": r["inner"],
                                    "launches": 0, "ms": 0.0, "alg_bytes": r["alg_bytes"],
                                    "touched_bytes": r["touched_bytes"], "flops": r["flops"]})
        q["launches"] += 1
        q["ms"] += r["ms"]
    rows = []
    for q in groups.values():
        avg = q["ms"] / q["launches"]
        rows.append({"kind": q["kind"], "d": q["d"], "rows": q["rows"], "inner": q["inner"],
                     "launches_per_step": q["launches"] / steps, "avg_ms": round(avg, 5),
                     "ms_per_step": round(q["ms"] / steps, 5),
                     "alg_GBps": round(q["alg_bytes"] / avg / 1e6, 2) if avg > 0 else None,
                     "touched_GBps": round(q["touched_bytes"] / avg / 1e6, 2) if avg > 0 else None,
                     "TFLOPps": round(q["flops"] / avg / 1e9, 3) if avg > 0 else None})
    rows.sort(key=lambda k: -k["ms_per_step"])
    return rows


def pick_block_global_rows():
    """Rows of the host-resident feature table of the row block: 2^27 (64 GiB) as specified if the runtime
    grants such a pinned allocation, else the largest power of two it does.  Measured on the GPU machine (295 GiB of
    host memory): one pinned allocation of 32 GiB is granted, 40 GiB and 64 GiB are refused with an out-of-memory
    error, so 2^26 rows x 128 fp32 (32 GiB) it is; the block itself (owned rows, halo rows, entries) does not
    depend on it."""
    return 1 << 26


def run_case(gcn, torch, name, dtype, steps, warmup, *, natural_ids=False, backward="push", overlap=True,
             calibrate_copy=False, w=None, keep_workload=False, one_stream=False):
    """Generates (or reuses) a workload, builds the block, times `steps` epochs.  Returns (record, workload)."""
    import numpy as np
    from workloads import configs
    dev = torch.device("cuda:0")
    bf16 = dtype == "bf16"
    t0 = time.time()
    if w is None:
        kw = {}
        if natural_ids:
            kw["permute"] = False
        if name == "c5_block":
            kw["n_global"] = pick_block_global_rows()
        w = configs.get(name, **kw)
        log(f"workload {name}: n={w['n']} raw directed edges={w['src'].size} dims={w['dims']} generated in {time.time() - t0:.1f}s")
    n, dims = w["n"], w["dims"]

    src, dst = torch.from_numpy(w["src"]).to(dev), torch.from_numpy(w["dst"]).to(dev)
    block = "row_lo" in w
    deg_global = torch.from_numpy(w["deg_global"]).to(dev) if block else None
    torch.cuda.synchronize()
    t0 = time.time()
    A = gcn.gcn_csr_build(src, dst, n, w.get("row_lo", 0), w.get("row_hi", n), deg_global=deg_global)
    torch.cuda.synchronize()
    build_ms = (time.time() - t0) * 1e3
    del src, dst, deg_global
    log(f"csr+csc build: {build_ms:.1f} ms, nr={A.nr} nh={A.nh} nnz={A.nnz}")

    table = None
    if block:
        from workloads import table as wtable
        if bf16:
            raise SystemExit("the block workload keeps its host table in fp32")
        t0 = time.time()
        table = torch.empty((n, dims[0]), dtype=torch.float32, pin_memory=True)      # host-resident feature table
        wtable.fill_table_torch(table, w["table_seed"], dev)
        X = table[w["row_lo"]: w["row_hi"]].to(dev)
        log(f"host feature table {n} x {dims[0]} fp32 ({table.numel() * 4 / 2**30:.1f} GiB, pinned) filled in {time.time() - t0:.1f}s")
    else:
        X = torch.from_numpy(w["X"]).to(dev)
        if bf16:
            X = X.to(torch.bfloat16)
    Ws = [torch.from_numpy(m).to(dev) for m in w["W"]]
    y = torch.from_numpy(w["y"]).to(dev)
    ep = Epoch(gcn, torch, A, X, Ws, y, bf16, table=table, overlap=overlap, backward=backward)
    del X

    one_stream = one_stream or calibrate_copy      # a counter run attributes its dispatches by order
    if one_stream:
        gcn.gcn_debug_set_tuning("GCN_OVERLAP", 0)
    for _ in range(warmup):
        ep.run()
    torch.cuda.synchronize()

    # Breakdown pass (not the timed region): every launch bracketed by HIP events, to find the dominant kernel.
    # Timing every launch costs about 10 % of a short epoch, so the timed region below only times that kernel.
    # In this pass the library runs every kernel on the caller's stream, one after the other (GCN_OVERLAP = 0), so
    # that each duration is the kernel's own; the timed region runs the library as it is by default, with dense
    # products beside sparse ones on large inputs.
    bsteps = max(1, min(steps, 5))
    gcn.gcn_debug_set_tuning("GCN_OVERLAP", 0)
    gcn.gcn_profile_filter(None)
    gcn.gcn_profile_enable(True)
    for _ in range(bsteps):
        ep.run()
    torch.cuda.synchronize()
    gcn.gcn_profile_enable(False)
    recs, dropped = gcn.gcn_profile_records()
    kernels = summarise(recs, bsteps)
    dom0 = kernels[0]
    if not one_stream:
        gcn.gcn_debug_set_tuning("GCN_OVERLAP", None)
        ep.run()                  # the side stream and its events exist before the timed region
        torch.cuda.synchronize()

    # Timed region: exactly `steps` epochs; HIP events only around the launches of the dominant kernel (on the
    # launch stream, inside the library) and one event per epoch boundary for the median and the minimum.
    gcn.gcn_profile_filter([dom0["kind"]], dom0["d"])
    gcn.gcn_profile_enable(True)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        marks[i].record()
        ep.run()
    marks[steps].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    gcn.gcn_profile_enable(False)
    gcn.gcn_profile_filter(None)
    ms_per_step = (t1 - t0) * 1e3 / steps
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))
    loss = float(ep.loss.item())
    log(f"{name} {dtype}: {ms_per_step:.3f} ms/epoch (median {per_step[len(per_step) // 2]:.3f}, min {per_step[0]:.3f}), loss={loss:.5f}")
    live, dropped2 = gcn.gcn_profile_records()
    dropped += dropped2
    live_all = summarise(live, steps)
    live = [k for k in live_all if (k["kind"], k["d"], k["rows"], k["inner"]) ==
            (dom0["kind"], dom0["d"], dom0["rows"], dom0["inner"])]
    dom = live[0] if live else dom0
    same = [k for k in live_all if (k["kind"], k["d"]) == (dom0["kind"], dom0["d"])]
    if not live and same:
        # the timed region launched this product on ranges of rows: one product = the launches of one epoch together
        ms = sum(k["ms_per_step"] for k in same)
        dom = dict(dom0)
        dom["avg_ms"] = round(ms, 5); dom["ms_per_step"] = round(ms, 5)
        dom["launches_per_step"] = 1.0
        for f in ("TFLOPps", "alg_GBps", "touched_GBps"):
            dom[f] = round(sum((k[f] or 0.0) * k["ms_per_step"] for k in same) / ms, 3)
        dom["row_range_launches"] = round(sum(k["launches_per_step"] for k in same), 1)

    # A latency-bound epoch replayed as one HIP graph launch: the calls of an epoch only enqueue kernels on the
    # caller's stream, so the whole epoch can be captured once and replayed (reported beside the eager figure, which
    # stays `value`).  Whole graphs only (the row block's epoch drives streams of its own).
    graph_replay = None
    if name in GRAPH_REPLAY_WORKLOADS and A.nh == 0 and not one_stream:
        try:
            cg = torch.cuda.CUDAGraph()
            with torch.cuda.graph(cg):
                ep.run()
            for _ in range(3):
                cg.replay()
            torch.cuda.synchronize()
            g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            g0.record()
            for _ in range(steps):
                cg.replay()
            g1.record()
            torch.cuda.synchronize()
            graph_replay = {"ms_per_step": round(g0.elapsed_time(g1) / steps, 5), "steps": steps,
                            "loss": round(float(ep.loss.item()), 6)}
            del cg
        except Exception as e:      # noqa: BLE001 - the eager figure stands on its own
            graph_replay = {"error": f"{type(e).__name__}: {e}"[:200]}

    if calibrate_copy:
        # identity gather = plain copy: reads 2^19 x 128 fp32 (256 MiB) + 2 MiB of indices, writes 256 MiB;
        # then a permutation gather of 64-byte rows (2^22 x 16 fp32): reads 256 MiB + 16 MiB of indices, writes 256 MiB
        rows = 1 << 19
        T = torch.ones(rows, 128, device=dev)
        R = torch.empty_like(T)
        idx = torch.arange(rows, dtype=torch.int32, device=dev)
        gcn.gcn_halo_gather(T, idx, R)
        rows = 1 << 22
        T = torch.ones(rows, 16, device=dev)
        R = torch.empty_like(T)
        idx = torch.from_numpy(np.random.default_rng(7).permutation(rows).astype(np.int32)).to(dev)
        gcn.gcn_halo_gather(T, idx, R)
        torch.cuda.synchronize()
        del T, R, idx

    is_gemm = dom["kind"].startswith("gemm_") and dom["kind"] != "gemm_tn_sum"
    intensity = (dom["TFLOPps"] or 0) * 1e3 / max(dom["alg_GBps"] or 1e-9, 1e-9)      # flop per byte
    if is_gemm and intensity > MFMA_PEAK_TFLOPS[dtype] * 1e3 / HBM_PEAK_GBS:
        roof = {"bound": "mfma", "achieved": dom["TFLOPps"], "peak": MFMA_PEAK_TFLOPS[dtype], "unit": "TFLOP/s",
                "frac": round(dom["TFLOPps"] / MFMA_PEAK_TFLOPS[dtype], 4), "traffic": None}
    else:
        roof = {"bound": "hbm", "achieved": dom["alg_GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(dom["alg_GBps"] / HBM_PEAK_GBS, 4), "traffic": None}
    # HBM-side bytes per launch of that kernel, from the rocprofv3 counter runs summarised under profiles/
    # (FETCH_SIZE + WRITE_SIZE, each scaled by what the counter reads for a copy of known size): a line
    # "bench-traffic: ..." there, stamped with the digest of the sparse-product sources it was measured on.
    # A reading taken on other sources is not attached.
    traffic_file = os.path.join(ROOT, "profiles", f"epoch_{name}_{dtype}.md")
    if os.path.exists(traffic_file) and not natural_ids and backward == "push":
        want = f"kernel={dom['kind']} d={dom['d']} "
        digest = sparse_sources_digest()
        for line in open(traffic_file):
            if line.startswith("bench-traffic:") and want in line:
                kv = dict(t.split("=") for t in line.split()[1:])
                if kv.get("sources") != digest:
                    roof["traffic_stale"] = f"{os.path.relpath(traffic_file, ROOT)} was measured on sources {kv.get('sources')}, these are {digest}"
                    continue
                roof["traffic"] = float(kv["read_bytes"]) + float(kv["write_bytes"])
                roof["traffic_GBps"] = round(roof["traffic"] / dom["avg_ms"] / 1e6, 2)
                roof["traffic_source"] = os.path.relpath(traffic_file, ROOT)
                roof["traffic_commit"] = kv.get("commit")
    roof["kernel"] = f"{dom['kind']} d={dom['d']} rows={dom['rows']} inner={dom['inner']}"
    roof["avg_launch_ms"] = dom["avg_ms"]
    roof["launches_timed"] = round(dom["launches_per_step"] * steps)
    roof["touched_GBps"] = dom["touched_GBps"]

    # the costliest dense product of the epoch against its own roofline (from the pass that times every launch)
    dense = [k for k in kernels if k["kind"] in ("gemm_nn", "gemm_tn")]
    dense_roof = None
    if dense:
        g = max(dense, key=lambda k: k["ms_per_step"])
        f_mfma = (g["TFLOPps"] or 0.0) / MFMA_PEAK_TFLOPS[dtype]
        f_hbm = (g["alg_GBps"] or 0.0) / HBM_PEAK_GBS
        dense_roof = ({"bound": "mfma", "achieved": g["TFLOPps"], "peak": MFMA_PEAK_TFLOPS[dtype], "unit": "TFLOP/s",
                       "frac": round(f_mfma, 4)} if f_mfma >= f_hbm else
                      {"bound": "hbm", "achieved": g["alg_GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(f_hbm, 4)})
        dense_roof["kernel"] = f"{g['kind']} d={g['d']} rows={g['rows']} inner={g['inner']}"
        dense_roof["avg_launch_ms"] = g["avg_ms"]

    out = {"metric": "GCN full-batch epoch ms (fwd+bwd) on 1 MI355X", "value": round(ms_per_step, 4), "unit": "ms/epoch",
           "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 4),
           "median_ms": round(per_step[len(per_step) // 2], 4), "min_ms": round(per_step[0], 4),
           "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic",
           "config": {"workload": name + ("+natural-ids" if natural_ids else ""), "backward": backward,
                      "halo_overlap": ep.overlap, "n": n, "owned_rows": A.nr, "halo_rows": A.nh, "nnz": A.nnz, "dims": dims,
                      "layers": len(dims) - 1, "feature_pitch": "gcn_feature_ld"},
           "epochs_per_s": round(1e3 / ms_per_step, 2), "loss": round(loss, 6), "csr_csc_build_ms": round(build_ms, 2),
           "launches_per_epoch": round(sum(k["launches_per_step"] for k in kernels), 1),
           "roofline": roof, "dense_roofline": dense_roof, "kernels": kernels,
           "kernels_from": f"a separate pass of {bsteps} epochs with every launch timed, all on one stream",
           "dense_beside_sparse": "off (--one-stream or a counter run)" if one_stream else "library default (on for large inputs)",
           "profile_records_dropped": dropped}
    if graph_replay is not None:
        out["graph_replay"] = graph_replay

    if calibrate_copy:
        # the sparse products of one epoch in launch order: lets a counter run attribute its dispatches
        per_epoch = len(recs) // bsteps
        out["sparse_launch_order"] = [[r["kind"], r["d"]] for r in recs[:per_epoch] if r["kind"] in ("spmm", "spmm_t")]
        out["sparse_sources"] = sparse_sources_digest()

    if block:
        # the host link's own rate: one plain copy of as many bytes as a halo fetch moves, from the same pinned
        # table, next to the rate of the gather kernel that reads the table through the index list
        nb = A.nh
        dst_buf = torch.empty(nb, dims[0], device=dev)
        srcv = table[1024: 1024 + nb]
        best = None
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); dst_buf.copy_(srcv, non_blocking=True); e1.record(); torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            best = ms if best is None else min(best, ms)
        link = nb * dims[0] * 4 / best / 1e6
        gk = [k for k in kernels if k["kind"] == "gather" and k["d"] == dims[0]]
        gath = (nb * dims[0] * 4 / gk[0]["avg_ms"] / 1e6) if gk else None
        out["host_link"] = {"plain_pinned_copy_GBps": round(link, 2), "copy_bytes": nb * dims[0] * 4,
                            "gather_host_GBps": round(gath, 2) if gath else None,
                            "gather_frac_of_link": round(gath / link, 4) if gath else None,
                            "gather_avg_ms": gk[0]["avg_ms"] if gk else None,
                            "note": "bytes delivered over the host link / time; the epoch fetches the halo rows once per layer"}
        del dst_buf
    A.free()
    del ep, table
    torch.cuda.empty_cache()
    return out, (w if keep_workload else None)


def host_mem_gib():
    try:
        for line in open("/proc/meminfo"):
            if line.startswith("MemTotal:"):
                return round(int(line.split()[1]) / 2**20, 1)
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--natural-ids", action="store_true",
                    help="c2_rmat18 only: keep the generator's vertex numbering instead of the seeded random relabelling "
                         "(an extra figure; the workload as specified relabels)")
    ap.add_argument("--others", default=None, choices=["all", "none"],
                    help="also time the other configurations in this process and list them under \"others\" "
                         "(default: all for the headline workload, none otherwise)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--backward", default="push", choices=["push", "pull"],
                    help="push: dH = A^T (G W^T) with contributions to halo rows (the default, any graph); "
                         "pull: Algorithm 2, halo rows of G fetched and T = A [G; G_halo] shared by dH and dW (symmetric graphs)")
    ap.add_argument("--no-overlap", action="store_true",
                    help="block workloads: fetch the halo rows before the layer instead of during its owned-column product")
    ap.add_argument("--cpu-sample-frac", type=float, default=None)
    ap.add_argument("--one-stream", action="store_true",
                    help="keep every kernel on the caller's stream (GCN_OVERLAP=0): no dense product beside a sparse one")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run two row copies of known size (for scaling hardware byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the row block of one processor); "
              "--gpus N with N > 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2212_05009_amd as gcn      # raises if the HIP library is missing: there is no fallback

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.natural_ids and args.workload != "c2_rmat18":
        raise SystemExit("--natural-ids applies to c2_rmat18")
    others_mode = args.others or ("all" if (args.workload == HEADLINE and args.dtype == "f32" and args.backward == "push"
                                           and not args.calibrate_copy) else "none")

    out, w = run_case(gcn, torch, args.workload, args.dtype, args.steps, args.warmup, natural_ids=args.natural_ids,
                      backward=args.backward, overlap=not args.no_overlap, calibrate_copy=args.calibrate_copy, one_stream=args.one_stream,
                      keep_workload=True)
    out["host_mem_total_GiB"] = host_mem_gib()

    if not args.no_cpu_baseline:
        frac = args.cpu_sample_frac
        if frac is None:
            # about 12 M stored entries x the layer widths of the headline workload: 10-30 s of oracle work
            frac = min(1.0, 1.2e7 / max(out["config"]["nnz"], 1))
        out["cpu_baseline"] = cpu_baseline(w, frac)

    others = []
    if others_mode == "all":
        # (name, dtype, extra): every record is produced by the same run_case; a case is skipped, and said so, when the
        # process has already run long (the default run has to stay within a few minutes)
        plan = [(HEADLINE, "bf16", {}), ("c5_block", "f32", {}), ("c2_rmat18", "f32", {}), ("c2_rmat18", "f32", {"natural_ids": True}),
                ("c3_dense233k", "f32", {}), ("c1_er4096", "f32", {})]
        for name, dt, extra in plan:
            if time.time() - T_START > 330:
                others.append({"config": {"workload": name}, "dtype": dt, "skipped": "time budget of the default run"})
                continue
            reuse = w if (name == args.workload and not extra) else None
            rec, _ = run_case(gcn, torch, name, dt, args.steps, args.warmup, w=reuse, **extra)
            if name == "c1_er4096":
                rec["epoch_us"] = round(rec["value"] * 1e3, 1)      # latency-bound: microseconds and launch count, no roofline claim
                rec["roofline_note"] = "latency-bound (0.6 MB of matrix): epoch_us and launches_per_epoch are the figures"
            others.append(rec)
        w = None
        if not args.no_cpu_baseline and time.time() - T_START < 400:
            # single-thread oracle time on the two small configurations
            from workloads import configs
            for name, frac in (("c1_er4096", 1.0), ("c2_rmat18", 1.0 / 16)):
                ws = configs.get(name)
                one = cpu_baseline(ws, frac, threads=1)
                for rec in others:
                    if rec["config"]["workload"] == name and "skipped" not in rec:
                        rec["cpu_baseline_1thread"] = one
    out["others"] = others
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
