#!/usr/bin/env python3
"""Benchmark of the aggregation hot path on one MI355X.

Default workload (the headline): configuration 5, one forward pass of the 5-layer GIN (hidden 64)
on the R-MAT scale-20 graph: per layer one aggregation (Eq. 3) and one Update GEMM (+ReLU), all
through the C-ABI library, inputs resident in HBM.  One-time preparation (renumbering, CSR
relabelling, neighbor partitioning: Sec. 4.1 / 5.1) happens before the timed region and is
reported separately, as the paper does.  Prints ONE JSON line on stdout.

Other configurations (--config 1..4) run the remaining workloads; --ngs/--dw/--wpb/--flags give
the parameter sweeps; --no-renumber keeps the generated ids, --renumber renumbers whatever the rule says.
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

# Bytes that crossed the L2 <-> fabric boundary (Infinity Cache + HBM; the counters cannot tell the two
# apart) per aggregation launch, from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs of this command,
# scaled by what the same counters read for a plain 256 MiB copy (FETCH_SIZE x2.0, WRITE_SIZE x1.0 on this
# machine).  Every entry names the summary it comes from and the kernel variant that was profiled; it is
# used only when the library reports that very variant for the launch being timed.
MEASURED_TRAFFIC = [
    {"cfg": 5, "replicate": 1, "renumbered": True, "dim": 64, "bytes_beyond_l2": 2.956e9,
     "variant": "k_aggregate<4,2,4,3,false,true,0> groups/block=32 ngs=32 waves/block=4 flush=ordered tiles=xcd-runs",
     "source": "profiles/aggregate_gin_dim64_cfg5_rmat.md"},
    {"cfg": 5, "replicate": 1, "renumbered": False, "dim": 64, "bytes_beyond_l2": 3.127e9,
     "variant": "k_aggregate<4,2,4,3,false,true,0> groups/block=32 ngs=32 waves/block=4 flush=ordered tiles=xcd-runs",
     "source": "profiles/aggregate_gin_dim64_cfg5_rmat_scrambled_ids.md"},
    {"cfg": 4, "replicate": 1, "renumbered": True, "dim": 16, "bytes_beyond_l2": 0.216e9,
     "variant": "k_aggregate<4,1,8,2,true,false,0> groups/block=64 ngs=32 waves/block=4 flush=ordered tiles=xcd-runs",
     "source": "profiles/aggregate_gcn_cfg4_community_renumbered.md"},
    {"cfg": 4, "replicate": 1, "renumbered": False, "dim": 16, "bytes_beyond_l2": 0.475e9,
     "variant": "k_aggregate<4,1,8,2,true,false,0> groups/block=64 ngs=32 waves/block=4 flush=ordered tiles=xcd-runs",
     "source": "profiles/aggregate_gcn_cfg4_community_shuffled.md"},
    {"cfg": 3, "replicate": 43, "renumbered": False, "dim": 64, "bytes_beyond_l2": 1.058e9,
     "variant": "k_gin_layer_fused_w<4,2,4,3,false,true,0> groups/block=16 ngs=16 waves/block=8 flush=ordered tiles=xcd-runs",
     "source": "profiles/gin_layer_fused_dim64_cfg3_x43_large_batch.md"},
]


def host_cores():
    """Cores this process may use: its affinity mask, capped by the thread count the environment sets."""
    cores = len(os.sched_getaffinity(0))
    for var in ("OMP_NUM_THREADS", "MAX_JOBS"):
        v = os.environ.get(var, "")
        if v.isdigit() and int(v) > 0:
            cores = min(cores, int(v))
    return max(cores, 1)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=5, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--ngs", type=int, default=0)
    ap.add_argument("--dw", type=int, default=0)
    ap.add_argument("--wpb", type=int, default=0)
    ap.add_argument("--flags", type=int, default=0, help="extra GNN_FLAG_* bits for the aggregation")
    ap.add_argument("--renumber", action="store_true",
                    help="apply gnn_reorder whatever its rule says (default: the rule of Sec. 5.1 decides)")
    ap.add_argument("--no-renumber", action="store_true", help="keep the generated ids (no gnn_reorder)")
    ap.add_argument("--renumber-device", action="store_true",
                    help="renumber on the GPU instead: gnn_reorder_device + gnn_apply_perm_csr_device (round-based schedule)")
    ap.add_argument("--hidden", type=int, default=0, help="override the hidden dimension of the model (sweep)")
    ap.add_argument("--replicate", type=int, default=1,
                    help="run on this many disjoint copies of the configuration's graph (e.g. --config 3 "
                         "--replicate 43: a Type II batch of 1.9 M nodes)")
    ap.add_argument("--variant", default="default", choices=["default", "planted", "natural"],
                    help="id order of the generated graph: configuration 4 'planted' (community-contiguous ids), "
                         "configuration 5 'natural' (R-MAT ids not scrambled)")
    ap.add_argument("--graph", action="store_true",
                    help="capture the step in a HIP graph and time replays (launch-bound small configurations)")
    ap.add_argument("--edge-vectors", action="store_true",
                    help="also time gnn_aggregate_edge (a feature vector per stored entry, Sec. 3.1) at the headline width")
    ap.add_argument("--train", action="store_true",
                    help="also time a training step (forward + gnn_layer_backward of every layer, no optimizer)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the measured ceilings (device copy, stream read, bare row gathers) reported beside the peak")
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
    from gnn_synth import BASE_SEED, config_graph, config_spec, features, glorot, replicate

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = args.config
    spec = config_spec(cfg)
    kind = "gin" if spec["kind"] == "gin" else "gcn"
    t0 = time.time()
    g = replicate(config_graph(cfg, variant=args.variant), args.replicate)
    rp_h, ci_h = g.rowptr, g.colidx
    n, nnz = g.n, g.nnz
    dims = list(spec["dims"])
    if args.hidden and len(dims) > 2:
        dims = [dims[0]] + [args.hidden] * (len(dims) - 2) + [dims[-1]]
    layers = len(dims) - 1  # 0 for configuration 1 (a single aggregation)
    X = features(n, dims[0], BASE_SEED + cfg)
    Ws = [glorot(dims[i], dims[i + 1], BASE_SEED + cfg, stream=20 + i) for i in range(layers)]
    log(f"generated config {cfg}: n={n} nnz={nnz} in {time.time() - t0:.1f}s")

    prep = {}
    _, aes0 = gnn.gnn_aes(rp_h, ci_h)
    prep["aes"] = aes0
    ew_h = None
    if kind == "gcn":
        t0 = time.perf_counter()
        ew_h = gnn.gnn_gcn_norm(rp_h, ci_h)
        prep["gcn_norm_host_ms"] = (time.perf_counter() - t0) * 1e3
    perm = None
    # One-time preparation, as in the paper's pipeline: community-aware renumbering when the rule of
    # Sec. 5.1 (sqrt(AES) > floor(sqrt(N)/100)) asks for it.  --renumber forces it, --no-renumber skips it.
    if not args.no_renumber and not args.renumber_device:
        t0 = time.perf_counter()
        perm, iperm, _, did = gnn.gnn_reorder(rp_h, ci_h, force=args.renumber)
        prep["reorder_host_ms"] = (time.perf_counter() - t0) * 1e3
        prep["reorder_rule_says"] = bool(did)
        args.renumber = bool(did)
        if not did:
            perm = None
    if args.renumber and perm is not None:
        t0 = time.perf_counter()
        if ew_h is None:
            rp_h, ci_h = gnn.gnn_apply_perm_csr(rp_h, ci_h, perm)
        else:
            rp_h, ci_h, ew_h = gnn.gnn_apply_perm_csr(rp_h, ci_h, perm, ew_h)
        prep["relabel_host_ms"] = (time.perf_counter() - t0) * 1e3
        prep["aes_after"] = gnn.gnn_aes(rp_h, ci_h)[1]

    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    rp, ci = d(rp_h), d(ci_h)
    ew = None if ew_h is None else d(ew_h)
    if args.renumber_device:
        # the whole preparation on the device; the host copies are refreshed for the oracle's leg
        gnn.gnn_validate_csr_device(n, nnz, rp, ci)
        gnn.gnn_reorder_device(n, nnz, rp, ci)  # first call: module load and allocator warm-up
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        perm_d, _, rounds = gnn.gnn_reorder_device(n, nnz, rp, ci)
        torch.cuda.synchronize()
        prep["reorder_device_ms"] = (time.perf_counter() - t0) * 1e3
        prep["reorder_device_rounds"] = rounds
        t0 = time.perf_counter()
        if ew is None:
            rp, ci = gnn.gnn_apply_perm_csr_device(n, nnz, rp, ci, perm_d)
        else:
            rp, ci, ew = gnn.gnn_apply_perm_csr_device(n, nnz, rp, ci, perm_d, ew)
        torch.cuda.synchronize()
        prep["relabel_device_ms"] = (time.perf_counter() - t0) * 1e3
        perm = perm_d.cpu().numpy()
        rp_h, ci_h = rp.cpu().numpy(), ci.cpu().numpy()
        ew_h = None if ew is None else ew.cpu().numpy()
        prep["aes_after"] = gnn.gnn_aes(rp_h, ci_h)[1]
        args.renumber = True
    Xd = d(X)
    if args.renumber:  # rows of X move with their nodes (device gather, part of the preparation)
        Xp = torch.empty_like(Xd)
        gnn.gnn_permute_rows(n, dims[0], d(perm), Xd, Xp)
        Xd = Xp
    Wd = [d(W) for W in Ws]
    gnn.gnn_validate_csr_device(n, nnz, rp, ci)

    agg_dim = dims[0] if (kind == "gin" or layers == 0) else dims[1]
    ngs, dw, wpb = gnn.gnn_decide(n, nnz, 0, agg_dim)
    ngs = args.ngs or ngs
    ws = gnn.alloc_workspace(n, nnz, max(dims), ngs)
    REUSE = gnn.GNN_FLAG_REUSE_PARTITION | args.flags
    KIND = gnn.GNN_GIN if kind == "gin" else gnn.GNN_GCN

    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    gnn.gnn_partition_build(n, nnz, rp, ngs, ws)
    e1.record()
    torch.cuda.synchronize()
    prep["partition_ms"] = e0.elapsed_time(e1)
    _, num_ng, _ = gnn.gnn_workspace_status(ws)

    if args.calibrate_copy:
        ca = torch.empty(1 << 26, dtype=torch.float32, device="cuda")
        cb = torch.empty_like(ca)
        cb.copy_(ca)
        torch.cuda.synchronize()
        del ca, cb

    # ---- the headline aggregation of the configuration, timed alone over the same number of steps
    # (Dim 64 GIN for configs 3/5, Dim 96 GCN for config 4, Dim 16 GCN for configs 1/2)
    head_dim = dims[0] if (kind == "gin" or cfg in (1, 4)) else dims[1]
    Xh = Xd if head_dim == dims[0] else torch.randn(n, head_dim, device="cuda")
    outh = torch.empty(n, head_dim, device="cuda")

    # arguments marshalled once, as a serving loop would do: the call itself only enqueues kernels
    head = gnn.AggregateCall(n, nnz, rp, ci, ew if kind == "gcn" else None, 0.0 if kind == "gin" else None, Xh, outh,
                             head_dim, ngs, args.dw, args.wpb, REUSE, ws)

    for _ in range(args.warmup):
        head()
    torch.cuda.synchronize()
    ha, hb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ha.record()
    for _ in range(args.steps):
        head()
    hb.record()
    torch.cuda.synchronize()
    head_call_ms = ha.elapsed_time(hb) / args.steps

    # ---- optional: aggregation with a feature vector on every stored entry, at the same width
    edge_vec = None
    if args.edge_vectors:
        Ev = torch.randn(nnz, head_dim, device="cuda")
        oute = torch.empty(n, head_dim, device="cuda")
        wse = gnn.alloc_workspace(n, nnz, head_dim, ngs)
        gnn.gnn_partition_build(n, nnz, rp, ngs, wse)
        for _ in range(args.warmup):
            gnn.gnn_aggregate_edge(n, nnz, rp, ci, Ev, Xh, oute, head_dim, ngs, args.dw, args.wpb, REUSE, wse)
        torch.cuda.synchronize()
        ea, eb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ea.record()
        for _ in range(args.steps):
            gnn.gnn_aggregate_edge(n, nnz, rp, ci, Ev, Xh, oute, head_dim, ngs, args.dw, args.wpb, REUSE, wse)
        eb.record()
        torch.cuda.synchronize()
        gnn.gnn_workspace_status(wse)
        ev_ms = ea.elapsed_time(eb) / args.steps
        ev_bytes = nnz * head_dim * 4 + 2 * n * head_dim * 4 + nnz * 4 + 4 * n  # E once, X once, out once, indices
        edge_vec = {"dim": head_dim, "call_ms": ev_ms, "edge_vector_bytes": nnz * head_dim * 4,
                    "compulsory_bytes": ev_bytes, "compulsory_GBps": ev_bytes / (ev_ms * 1e-3) / 1e9,
                    "kernel": gnn.gnn_bench_last_aggregation()}
        del Ev, oute, wse

    # ---- the step: the configuration's model forward (configuration 1: the single aggregation)
    nlay = max(layers, 1)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for a, b in evs:  # torch creates an event's handle on its first record
        a.record()
        b.record()
    torch.cuda.synchronize()

    # One gnn_model_forward call per step (all layers enqueued by the library); the arguments of each
    # timed step, with its own event taps around every layer's aggregation kernel, are marshalled
    # beforehand, as a serving loop would do.
    if layers:
        mws = torch.empty(gnn.gnn_model_workspace_bytes(n, nnz, dims, ngs), dtype=torch.uint8, device="cuda")
        gnn.gnn_partition_build(n, nnz, rp, ngs, mws)
        out_final = torch.empty(n, dims[-1], device="cuda")

        def model_call(k):
            # step k taps the aggregation kernel of layer k % layers only: two event records per step
            # keep the taps from spacing out the kernels of small graphs
            if k < 0:
                return gnn.ModelCall(KIND, n, nnz, rp, ci, ew, 0.0, Xd, dims, Wd, None, out_final, ngs, args.dw,
                                     args.wpb, REUSE, mws)
            tap = k % layers
            ea, eb = evs[k]
            return gnn.ModelCall(KIND, n, nnz, rp, ci, ew, 0.0, Xd, dims, Wd, None, out_final, ngs, args.dw, args.wpb,
                                 REUSE, mws, None, [ea if l == tap else None for l in range(layers)],
                                 [eb if l == tap else None for l in range(layers)])
        untimed = model_call(-1)
        timed = [model_call(k) for k in range(args.steps)]

    def step(k):
        if layers == 0:
            head()
        elif k < 0:
            untimed()
        else:
            timed[k]()

    for _ in range(args.warmup):
        step(-1)
    torch.cuda.synchronize()
    graph_ms = None
    if args.graph:
        # the library only enqueues kernels (no memset nodes, no synchronisation), so a step can be
        # captured; replays are checked against the eager result
        eager = None
        if layers:
            step(-1)
            torch.cuda.synchronize()
            eager = out_final.clone()
        cg = torch.cuda.CUDAGraph()
        cap_stream = torch.cuda.Stream()
        with torch.cuda.graph(cg, stream=cap_stream):
            step(-1)
        for _ in range(args.warmup):
            cg.replay()
        torch.cuda.synchronize()
        tg = time.perf_counter()
        for _ in range(args.steps):
            cg.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - tg) * 1e3 / args.steps
        if eager is not None:
            # (rows finished by float atomics, GNN_FLAG_ATOMIC_FLUSH, may differ in their last bits)
            err = (out_final - eager).abs().max().item() / max(eager.abs().max().item(), 1e-30)
            assert err <= 1e-5, f"graph replay differs from eager by {err:.3e}"
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(k)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    gnn.gnn_workspace_status(mws if layers else ws)
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # dominant kernel: the aggregation at the model's widest aggregated dimension (layer 1)
    if layers > 0:
        samples = [[] for _ in range(layers)]
        for k in range(args.steps):
            samples[k % layers].append(evs[k][0].elapsed_time(evs[k][1]))
        agg_ms_layers = np.array([np.mean(x) if x else float("nan") for x in samples])
        dom_dim = agg_dim
        dom_ms = float(agg_ms_layers[0]) if kind == "gcn" else float(np.nanmean(agg_ms_layers))
    else:
        agg_ms_layers = np.array([head_call_ms])
        dom_dim, dom_ms = head_dim, head_call_ms

    def algorithmic_bytes(dim):
        # per edge one neighbour row + its column index (+ its weight for GCN); per node its output row
        # (+ its own input row for GIN) and its group-offset word; per neighbor group its 16-byte tuple
        per_edge = 4 * dim + 4 + (4 if kind == "gcn" else 0)
        per_node = 4 * dim + 4 + (4 * dim if kind == "gin" else 0)
        return nnz * per_edge + n * per_node + num_ng * 16

    dom_bytes = algorithmic_bytes(dom_dim)
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9
    if not layers:
        agg_dims = [head_dim]
    elif kind == "gin":
        agg_dims = [dims[0]] * layers
    else:  # GCN aggregates at the narrower of a layer's two widths (at the output width on request)
        narrow = not (args.flags & gnn.GNN_FLAG_GCN_UPDATE_FIRST)
        agg_dims = [dims[l] if narrow and dims[l] < dims[l + 1] else dims[l + 1] for l in range(layers)]
    edges_dim_step = float(nnz) * float(sum(agg_dims))
    value = edges_dim_step / (ms_per_step * 1e-3)

    train_ms = None
    if args.train and layers > 0:
        # every configuration's graph is symmetric (GCN weights too), so it is its own transpose and
        # the forward partition serves the backward aggregation
        bws = torch.empty(max(gnn.gnn_backward_workspace_bytes(n, nnz, dims[l], dims[l + 1], ngs) for l in range(layers)),
                          dtype=torch.uint8, device="cuda")
        gnn.gnn_partition_build(n, nnz, rp, ngs, bws)
        Hs = [Xd] + [torch.empty(n, dims[l + 1], device="cuda") for l in range(layers)]
        As = [torch.empty(n, dims[l], device="cuda") for l in range(layers)] if kind == "gin" else None
        dHs = [torch.empty(n, dims[l], device="cuda") for l in range(layers)] + [torch.randn(n, dims[-1], device="cuda")]
        dWs = [torch.empty(dims[l], dims[l + 1], device="cuda") for l in range(layers)]

        def train_step():
            for l in range(layers):
                relu = l != layers - 1
                if kind == "gin":
                    gnn.gnn_aggregate_gin(n, nnz, rp, ci, 0.0, Hs[l], As[l], dims[l], ngs, args.dw, args.wpb, REUSE, ws)
                    gnn.gnn_update_gemm(n, dims[l], dims[l + 1], As[l], Wd[l], None, relu, Hs[l + 1])
                else:
                    gnn.gnn_layer_forward(KIND, n, nnz, rp, ci, ew, 0.0, Hs[l], dims[l], Wd[l], None, dims[l + 1], relu,
                                          Hs[l + 1], ngs, args.dw, args.wpb, REUSE, ws)
            for l in reversed(range(layers)):
                relu = l != layers - 1
                P = As[l] if kind == "gin" else Hs[l]
                gnn.gnn_layer_backward(KIND, n, nnz, rp, ci, ew, 0.0, P, dims[l], Wd[l], dims[l + 1], relu, Hs[l + 1],
                                       dHs[l + 1], dHs[l] if l > 0 else None, dWs[l], None, ngs, args.dw, args.wpb,
                                       REUSE, bws)

        for _ in range(args.warmup):
            train_step()
        torch.cuda.synchronize()
        tt = time.perf_counter()
        for _ in range(args.steps):
            train_step()
        torch.cuda.synchronize()
        train_ms = (time.perf_counter() - tt) * 1e3 / args.steps
        gnn.gnn_workspace_status(bws)

    # ---- what the memory system delivers on this machine, beside the published peak: a plain device copy,
    # a read-only stream, a bare gather of uniformly random rows of this X and of this graph's own index
    # stream (the aggregation kernel's loads without tuples, reduction and stores)
    ceilings = None
    if not args.no_ceilings:
        def timed_us(fn, reps=5):
            fn()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / reps * 1e3

        sink = torch.zeros(1, device="cuda")
        big = torch.ones(1 << 28, dtype=torch.float32, device="cuda")  # 1 GiB
        half = big[: 1 << 26]
        dst = torch.empty(1 << 26, dtype=torch.float32, device="cuda")
        t_copy = timed_us(lambda: dst.copy_(half))
        t_read = timed_us(lambda: gnn.gnn_bench_stream_read(big, sink))
        ceilings = {"device_copy_256MiB_GBps": 2 * half.numel() * 4 / t_copy / 1e3,
                    "stream_read_1GiB_GBps": big.numel() * 4 / t_read / 1e3}
        del big, half, dst
        # at the width of the kernel the roofline object describes (dom_dim)
        if any(dom_dim == 4 * (1 << t) * c for t in range(7) for c in range(1, 5)) and nnz >= 8:
            Xg = Xh if dom_dim == head_dim else torch.randn(n, dom_dim, device="cuda")
            rnd = torch.randint(0, n, (nnz,), dtype=torch.int32, device="cuda")
            t_rnd = timed_us(lambda: gnn.gnn_bench_gather_rows(n, dom_dim, Xg, rnd, sink))
            t_own = timed_us(lambda: gnn.gnn_bench_gather_rows(n, dom_dim, Xg, ci, sink))
            row_bytes = (nnz // 8) * 8 * dom_dim * 4
            ceilings.update({"gather_dim": dom_dim,
                             "gather_uniform_random_rows_GBps": row_bytes / t_rnd / 1e3,
                             "gather_graph_colidx_GBps": row_bytes / t_own / 1e3,
                             "gather_graph_colidx_us": t_own})
            del rnd

    cpu = None
    if not args.no_cpu_baseline:
        # The oracle as it stands, on the host of this box: first the plain single-thread loops on a bounded
        # sample, then the same loops on disjoint row ranges over all cores this process may use.
        import oracle
        cores = host_cores()
        t0 = time.perf_counter()
        if layers == 0:
            oracle.aggregate_gcn(rp_h, ci_h, ew_h, X)
            done_dims, sample = [head_dim], "the single aggregation"
        else:
            sample_layers = min(layers, 2) if cfg == 5 else layers  # about 7 s of single-thread work
            H = X if perm is None else oracle.permute_rows(X, perm)
            for l in range(sample_layers):
                if kind == "gin":
                    H = oracle.gin_layer(rp_h, ci_h, 0.0, H, Ws[l], None, relu=True)
                else:
                    H = oracle.gcn_layer(rp_h, ci_h, ew_h, H, Ws[l], None, relu=True)
            done_dims = agg_dims[:sample_layers]
            sample = f"layers 1-{sample_layers} of {layers} on the full graph"
        dt1 = time.perf_counter() - t0
        t0 = time.perf_counter()
        if layers == 0:
            oracle.aggregate_gcn_threads(rp_h, ci_h, ew_h, X, cores)
            all_dims = [head_dim]
        else:
            H = X if perm is None else oracle.permute_rows(X, perm)
            for l in range(layers):
                relu = l != layers - 1
                if kind == "gin":
                    H = oracle.gin_layer_threads(rp_h, ci_h, 0.0, H, Ws[l], None, relu, cores)
                else:
                    H = oracle.gcn_layer_threads(rp_h, ci_h, ew_h, H, Ws[l], None, relu, cores)
            all_dims = agg_dims
        dtn = time.perf_counter() - t0
        cpu = {"value": float(nnz) * sum(all_dims) / dtn, "unit": "edge*dim/s", "cores": cores, "kind": "oracle",
               "sample": f"the whole step ({len(all_dims)} layer(s), full graph) as disjoint row ranges of the oracle's "
                         f"loops on {cores} threads ({dtn:.1f} s)",
               "single_core": {"value": float(nnz) * sum(done_dims) / dt1, "cores": 1,
                               "sample": f"{sample} ({dt1:.1f} s)"}}

    # which kernel the library enqueues for the dominant aggregation (asked from the library itself)
    if layers:  # layer 1 holds the dominant aggregation
        gnn.gnn_layer_forward(KIND, n, nnz, rp, ci, ew, 0.0, Xd, dims[0], Wd[0], None, dims[1], True,
                              torch.empty(n, dims[1], device="cuda"), ngs, args.dw, args.wpb, REUSE, mws)
    else:
        head()
    torch.cuda.synchronize()
    variant = gnn.gnn_bench_last_aggregation()
    fused = variant.startswith("k_gin_layer_fused")
    kname = variant.split(" ")[0] + (" (aggregation + Update GEMM in one kernel)" if fused else "")
    traffic, traffic_source = None, None
    if not (args.hidden or args.flags or args.renumber_device or args.variant != "default"):
        for e in MEASURED_TRAFFIC:
            if (e["cfg"], e["replicate"], e["renumbered"], e["dim"]) == (cfg, args.replicate, bool(args.renumber), dom_dim):
                if e["variant"] == variant:
                    traffic, traffic_source = e["bytes_beyond_l2"], e["source"]
                else:
                    traffic_source = f"{e['source']} describes {e['variant']!r}, not the variant timed here: not used"
    # compulsory bytes (perfect reuse): X once, out once, indices (and weights) once, group offsets once
    compulsory = n * 4 * dom_dim * 2 + nnz * (4 + (4 if kind == "gcn" else 0)) + 4 * n
    if fused:  # the fused layer also reads W and writes the layer output instead of the aggregate
        compulsory = n * 4 * (dom_dim + dims[1]) + nnz * 4 + 4 * n + 4 * dom_dim * dims[1]
    if ceilings is not None and traffic is not None:
        # bytes beyond L2 per second against what a bare random gather of rows reaches on this machine
        ceilings["traffic_GBps"] = traffic / (dom_ms * 1e-3) / 1e9
        # (comparable only for rows of whole 128-byte lines: the gather figure counts useful bytes, the
        # counters fetched sectors)
        if "gather_uniform_random_rows_GBps" in ceilings and dom_dim * 4 % 128 == 0:
            ceilings["traffic_frac_of_random_gather"] = ceilings["traffic_GBps"] / ceilings["gather_uniform_random_rows_GBps"]
    # The fraction of the HBM roofline: bytes that really left L2 (measured, an upper bound on HBM bytes since
    # Infinity-Cache hits are among them) when a profile of this very kernel variant exists, else the
    # compulsory bytes (a lower bound on what any schedule must move).  The gather-model rate, which counts
    # every neighbour row as if it came from memory and so can exceed the peak, is reported beside it.
    roof_bytes = traffic if traffic is not None else compulsory
    roof_kind = "bytes_beyond_l2" if traffic is not None else "compulsory_bytes"
    roof_rate = roof_bytes / (dom_ms * 1e-3) / 1e9
    rec = {
        "metric": "aggregation edges*dim/s over one model forward (aggregations + Update GEMMs)",
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
        "config": {"workload": f"cfg{cfg}{'' if args.replicate == 1 else f' x{args.replicate} copies'}: {spec['desc']}; "
                               f"n={n}, directed entries={nnz}, layers={layers}",
                   "ngs": ngs, "dw": args.dw or dw, "waves_per_block": args.wpb or wpb, "neighbor_groups": num_ng,
                   "renumbered": bool(args.renumber), "flags": args.flags, "id_order": args.variant},
        "roofline": {"bound": "hbm", "kernel": f"{kname} ({kind.upper()}, Dim {dom_dim})", "kernel_variant": variant,
                     "achieved": roof_rate, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": roof_rate / HBM_PEAK_GBPS,
                     "frac_kind": roof_kind,
                     "traffic": traffic, "traffic_source": traffic_source,
                     "frac_beyond_l2": None if traffic is None else traffic / (dom_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                     "compulsory_bytes_per_launch": compulsory,
                     "frac_compulsory": compulsory / (dom_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                     "algorithmic_bytes_per_launch": dom_bytes, "algorithmic_GBps": achieved,
                     "avg_kernel_ms": dom_ms,
                     "measured_ceilings": ceilings},
        "cpu_baseline": cpu,
        "aggregation_kernel_ms_per_layer": [float(x) for x in agg_ms_layers],
        "aggregation_only_edges_dim_per_s": float(nnz) * dom_dim / (dom_ms * 1e-3),
        "layer_ms": ms_per_step / nlay,
        "headline_aggregation": {"dim": head_dim, "call_ms": head_call_ms,
                                 "edges_dim_per_s": float(nnz) * head_dim / (head_call_ms * 1e-3),
                                 "algorithmic_GBps": algorithmic_bytes(head_dim) / (head_call_ms * 1e-3) / 1e9},
        "edge_vector_aggregation": edge_vec,
        "prep": prep,
        "dims": dims,
        "step_api": "gnn_model_forward" if layers else "gnn_aggregate_gcn",
        "graph_replay_ms_per_step": graph_ms,
        "train_step_ms": train_ms,
    }
    print(json.dumps(rec), flush=True)


if __name__ == "__main__":
    main()
