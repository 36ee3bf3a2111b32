#!/usr/bin/env python3
"""Benchmark of the aggregation hot path on one MI355X.

A step is one forward pass of the 5-layer GIN of configuration 5 (R-MAT scale 20, hidden 64):
per layer one aggregation (Eq. 3) and one Update GEMM (+ReLU), all through the C-ABI library,
inputs resident in HBM.  One-time preparation (neighbor partitioning, Sec. 4.1) is done before
the timed region and reported separately, as the paper does.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0

# HBM bytes per aggregation launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (see
# profiles/), keyed by (config, ngs); None until measured.
MEASURED_TRAFFIC_BYTES = {}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=5, choices=[3, 5])
    ap.add_argument("--ngs", type=int, default=0)
    ap.add_argument("--dw", type=int, default=0)
    ap.add_argument("--wpb", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy, the known-size kernel against which the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run are scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2006_06608_amd as gnn
    from gnn_synth import BASE_SEED, config_graph, config_spec, features, glorot

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = args.config
    spec = config_spec(cfg)
    t0 = time.time()
    g = config_graph(cfg)
    n, nnz = g.n, g.nnz
    dims = spec["dims"]
    dim = dims[0]
    layers = len(dims) - 1
    X = features(n, dim, BASE_SEED + cfg)
    Ws = [glorot(dims[i], dims[i + 1], BASE_SEED + cfg, stream=20 + i) for i in range(layers)]
    log(f"generated config {cfg}: n={n} nnz={nnz} in {time.time() - t0:.1f}s")

    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    rp, ci = d(g.rowptr), d(g.colidx)
    Xd = d(X)
    Wd = [d(W) for W in Ws]
    gnn.gnn_validate_csr_device(n, nnz, rp, ci)

    ngs, dw, wpb = gnn.gnn_decide(n, nnz, 0, dim)
    ngs = args.ngs or ngs
    dw = args.dw or dw
    wpb = args.wpb or wpb
    ws = gnn.alloc_workspace(n, nnz, max(dims), ngs)
    stream = torch.cuda.current_stream()

    # one-time preparation, timed on its own
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    gnn.gnn_partition_build(n, nnz, rp, ngs, ws)
    e1.record()
    torch.cuda.synchronize()
    prep_ms = e0.elapsed_time(e1)
    _, num_ng, _ = gnn.gnn_workspace_status(ws)

    bufs = [torch.empty(n, dim, device="cuda"), torch.empty(n, dim, device="cuda")]
    nev = layers * args.steps
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(nev)]
    for a, b in evs:  # give every event its handle
        a.record()
        b.record()
    torch.cuda.synchronize()

    def step(k):
        H = Xd
        for l in range(layers):
            out = bufs[l & 1]
            ea, eb = evs[k * layers + l] if k >= 0 else (None, None)
            gnn.gnn_layer_forward_timed(gnn.GNN_GIN, n, nnz, rp, ci, None, 0.0, H, dims[l], Wd[l], None, dims[l + 1],
                                        l != layers - 1, out, ngs, dw, wpb, gnn.GNN_FLAG_REUSE_PARTITION, ws, stream,
                                        ea, eb)
            H = out
        return H

    if args.calibrate_copy:
        ca = torch.empty(1 << 26, dtype=torch.float32, device="cuda")
        cb = torch.empty_like(ca)
        cb.copy_(ca)
        torch.cuda.synchronize()
        del ca, cb

    for _ in range(args.warmup):
        step(-1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(k)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    gnn.gnn_workspace_status(ws)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    agg_ms = float(np.mean([a.elapsed_time(b) for a, b in evs]))

    # algorithmic bytes of one aggregation launch (the kernel also writes the rows without
    # neighbours): per edge one neighbour row + its column index; per node its output row and, for
    # GIN, its own input row, plus its two group-offset words; per neighbor group its 16-byte tuple
    agg_bytes = nnz * (4 * dim + 4) + n * (4 * dim + 4 * dim + 4) + num_ng * 16
    achieved = agg_bytes / (agg_ms * 1e-3) / 1e9
    edges_dim = float(nnz) * dim
    value = layers * edges_dim / (ms_per_step * 1e-3)

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        sample_layers = 2 if cfg == 5 else layers
        H = X
        t0 = time.perf_counter()
        for l in range(sample_layers):
            H = oracle.gin_layer(g.rowptr, g.colidx, 0.0, H, Ws[l], None, relu=True)
        dt = time.perf_counter() - t0
        cpu = {"value": sample_layers * edges_dim / dt, "unit": "edge*dim/s", "cores": 1, "kind": "oracle",
               "sample": f"layers 1-{sample_layers} of {layers} on the full graph ({dt:.1f} s)",
               "ms_per_layer": dt * 1e3 / sample_layers}

    rec = {
        "metric": "aggregation edges*dim/s (5-layer GIN forward, whole step incl. Update GEMMs)",
        "value": value,
        "unit": "edge*dim/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"cfg{cfg}: {spec['desc']}; n={n}, directed edges={nnz}, {layers} layers",
                   "ngs": ngs, "dw": dw, "waves_per_block": wpb, "neighbor_groups": num_ng},
        "roofline": {"bound": "hbm", "kernel": ("k_aggregate_pipe" if ngs <= 8 else "k_aggregate") + "<4,1,8,false,true> (GIN, Dim 64)", "achieved": achieved,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get((cfg, ngs)),
                     "algorithmic_bytes_per_launch": agg_bytes, "avg_kernel_ms": agg_ms},
        "cpu_baseline": cpu,
        "aggregation_only_edges_dim_per_s": edges_dim / (agg_ms * 1e-3),
        "layer_ms": ms_per_step / layers,
        "prep_partition_ms": prep_ms,
    }
    print(json.dumps(rec), flush=True)


if __name__ == "__main__":
    main()
