#!/usr/bin/env python3
"""Benchmark of the TMA trainer hot path on one MI355X.

One "step" = one pass of the whole path on the configs[1] workload, inputs
already resident in HBM: random K-way node assignment of the 1M-node global
graph, extraction of one partition's induced subgraph, gather of its feature
rows and labels, full-batch forward + backward + SGD step of the 2-layer
mean-aggregation GraphSAGE model on it, and the averaging of K parameter
vectors.  Prints ONE JSON line (metric, roofline of the dominant kernel, CPU
oracle baseline).
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published peaks
PEAK_HBM_GBS = 8000.0
PEAK_MFMA_F32_TFLOPS = 157.3
PEAK_MFMA_BF16_TFLOPS = 2500.0

WORKLOAD = dict(n_nodes=1_000_000, avg_degree=20, gamma=2.1, K=8, part=0, F=128, hidden=256, classes=47,
                seeds=dict(graph=11, feat=12, label=13, part=14, weights=15), lr=1e-3)
# configs[0]: the small case the oracle finishes in a blink (uniform random graph, 100,000 undirected edges)
TINY = dict(n_nodes=20_000, n_edges=100_000, K=4, part=0, F=64, hidden=64, classes=16,
            seeds=dict(graph=1, feat=2, label=3, part=4, weights=5), lr=1e-3)

def cpu_baseline_leg(sample):
    """The oracle, as it stands, timed on this machine's host cores on a bounded sample of the workload: one thread
    (the canonical figure), then the same loops split over rows on all cores."""
    import numpy as np
    import oracle
    from oracle import model as omodel
    p_o = [tuple(np.asarray(t, dtype=np.float64) for t in l) for l in sample["params"]]
    encoder = sample.get("encoder", "sage")

    def run(threads):
        oracle.set_threads(threads)
        try:
            t = time.perf_counter()
            if "full" in sample:
                sample["full"](oracle, omodel, p_o)
            else:
                omodel.train_step(sample["rowptr"], sample["colidx"], sample["X"], sample["y"], p_o, sample["lr"],
                                  encoder=encoder)
            return time.perf_counter() - t
        finally:
            oracle.set_threads(1)

    sec = run(1)
    out = {"value": round(sample["edges"] / sec, 1), "unit": "edges/s", "cores": 1, "kind": "oracle",
           "sample": sample["what"] + f", {sec:.1f} s single-threaded fp64"}
    ncores = min(oracle.hardware_threads(), int(os.environ.get("OMP_NUM_THREADS", "1024")))
    if ncores > 1:
        sec_all = run(ncores)
        out["all_cores"] = {"value": round(sample["edges"] / sec_all, 1), "unit": "edges/s", "cores": ncores,
                            "seconds": round(sec_all, 2),
                            "what": "the same oracle loops with a parallel-for over rows (aggregation and layer "
                                    "loops); timing leg only"}
    return out


def canonical(name, s):
    """Kernel name as the work tables spell it: without the storage / path suffixes, and with a gather's
    16-byte pieces per row counted as for fp32 rows (a bf16 row of the same width has half as many)."""
    name = name.replace("_generic", "")
    m = re.match(r"(spmm_[a-z]+)_(?:f32|bf16)_g(\d+)x1$", name)
    if m:
        return "%s_f32_g%dx1" % (m.group(1), int(m.group(2)) * 4 // s)
    return name.replace("_bf16", "")


def link_kernel_work(name, n, nnz, dims, dec_dims, Bn, s=4):
    """Same for the link-prediction task with the SAGE encoder (both layers aggregate first), mean over the
    launches of a step where a kernel name is launched with different shapes."""
    F0, F1, F2 = dims
    D0, D1, _ = dec_dims
    rows = 2 * Bn
    gather = lambda F: 2.0 * n * F * s + nnz * 4 + n * 8          # rows once + ids + rowptr, 1/deg + output
    table = {
        "gemm_fwd_128x128": ("mfma", (2.0 * n * 2 * F0 * F1 + 2.0 * n * 2 * F1 * F2) / 2),
        "gemm_bwd_weight_128x128": ("mfma", (2.0 * n * 2 * F0 * F1 + 2.0 * n * 2 * F1 * F2) / 2),
        "gemm_bwd_data_128x128": ("mfma", 2.0 * n * F2 * 2 * F1),
        "gemm_dense_fwd": ("mfma", (2.0 * rows * D0 * D1 + 2.0 * rows * D1) / 2),
        "gemm_dense_bwd_weight": ("mfma", (2.0 * rows * D0 * D1 + 2.0 * rows * D1) / 2),
        "gemm_dense_bwd_data": ("mfma", (2.0 * rows * D0 * D1 + 2.0 * rows * D1) / 2),
        "spmm_mean_f32_g32x1": ("hbm", gather(F0)),
        "spmm_mean_f32_g64x1": ("hbm", gather(F1)),
        # dH1 += A^T dM (dM rows once, dH read and written) and dR = sum of each node's terms (4B rows of F2)
        "spmm_sum_f32_g64x1": ("hbm", ((3.0 * n * F1 * s + nnz * 4 + n * 4) + (4.0 * Bn * F2 * s + 4 * Bn * 4 + n * 4 + n * F2 * s)) / 2),
        "pair_product_fwd": ("hbm", 5.0 * Bn * F2 * s + 12.0 * Bn),        # three gathered rows read, two written
        "pair_product_terms": ("hbm", 9.0 * Bn * F2 * s + 12.0 * Bn),      # + two gradient rows read, four written
        "prelu_fwd": ("hbm", 2.0 * rows * D1 * s),
        "prelu_bwd": ("hbm", 3.0 * rows * D1 * s),
    }
    return table.get(canonical(name, s), (None, 0.0))


def gathered_bytes(name, n, nnz, dims, s=4):
    """Bytes a gather kernel of the headline workload requests when every gathered neighbour row is counted (no
    reuse between rows), next to the algorithmic bytes of kernel_work that count each distinct input row once."""
    F0, F1, C = dims
    Cp = (C * s + 15) // 16 * 16 // s
    return {
        "spmm_mean_f32_g32x1": nnz * (F0 * s + 4) + n * (F0 * s + 8),
        "spmm_combine_f32_g12x1": nnz * (Cp * s + 4) + n * (2 * Cp * s + 8),
        "spmm_sum_f32_g12x1": nnz * (Cp * s + 4) + n * (Cp * s + 4),
    }.get(canonical(name, s))


def kernel_work(name, n, nnz, dims, N=0, nnz_glob=0, K=1, n_params=0, encoder="sage", s=4):
    """Algorithmic work of one launch of kernel `name` in this workload: ("mfma", flops) or ("hbm", bytes).

    Bytes count every array the kernel must touch once (distinct input rows once, however often they are
    gathered; outputs once); flops count the products of the layer's definition, not the padding.  A kernel
    name that both layers launch (the GCN / MLP encoders) gets the mean over its launches of a step."""
    F0, F1, C = dims
    Cp = (C * s + 15) // 16 * 16 // s        # padded width of the transform-first blocks (rows of whole 16-byte pieces)
    name = canonical(name, s)
    # the tile shape of a product and the lanes per row of a gather follow from the widths: not part of the key
    name = re.sub(r"^(gemm_(?:fwd|bwd_weight|bwd_data))_\d+x\d+$", r"\1", name)
    name = re.sub(r"^(spmm_(?:mean|combine|sum|weighted))_f32_g\d+x1$", r"\1", name)
    if encoder != "sage":
        both = (2.0 * n * F0 * F1 + 2.0 * n * F1 * C) / 2
        other = {
            "gemm_dense_fwd": ("mfma", both),                      # Y = X W, both layers
            "gemm_dense_bwd_weight": ("mfma", both),               # dW = X^T G, both layers
            "gemm_dense_bwd_data": ("mfma", 2.0 * n * F1 * C),     # dH1 = G W^T, layer 1 only
            # layer 0 aggregates first: M = S (A + I) S H0, rows of H0 once + ids + rowptr, s + output
            "spmm_weighted": ("hbm", 2.0 * n * F0 * s + nnz * 4 + n * 8),
            # layer 1 transforms first: H2 = S (A + I) Y + b forward and G = S (A + I)^T Q backward
            "spmm_combine": ("hbm", 2.0 * n * Cp * s + nnz * 4 + n * 8),
            # Q = S dZ of layer 1: dH2 read, Q written, s read
            "scale_mask_colsum": ("hbm", n * (C + Cp) * s + n * 4.0),
        }
        if name in other:
            return other[name]
    gemm = {
        "gemm_fwd": 2.0 * n * (2 * F0) * F1,          # Z1 = [H0 | M0] [Ws; Wn]
        "gemm_bwd_weight": 2.0 * n * (2 * F0) * F1,   # [dWs; dWn] = [H0 | M0]^T dZ1
        "gemm_tf_fwd": 2.0 * n * F1 * (2 * C),                # [Ys | Yn] = H1 [Ws | Wn]
        "gemm_tf_bwd_weight": 2.0 * n * F1 * (2 * C),         # [dWs | dWn] = H1^T [dZ | dYn]
        "gemm_tf_bwd_data": 2.0 * n * (2 * C) * F1,           # dH1 = [dZ | dYn] [Ws | Wn]^T
    }
    if name in gemm:
        return "mfma", gemm[name]
    rows_glob = nnz_glob / max(K, 1)     # global entries of the local rows
    hbm = {
        # mean aggregation of H0: rows of H0 once + ids + rowptr/inv_deg + output
        "spmm_mean": n * F0 * s + nnz * 4 + n * 8 + n * F0 * s,
        # layer-1 output: gathered Yn rows once + Ys + ids + rowptr/inv_deg + bias + H2
        "spmm_combine": 2 * n * Cp * s + nnz * 4 + n * 8 + n * Cp * s,
        # dYn = A^T (D^-1 dZ): scaled rows once + ids + rowptr + output
        "spmm_sum": n * Cp * s + nnz * 4 + n * 4 + n * Cp * s,
        "scale_mask_rows": n * C * s + n * 4 + n * Cp * s,
        "softmax_ce": 2 * n * C * s + n * 4,
        "ln_prelu_fwd_f32": 2 * n * F1 * s,                   # Z read, H' written
        "ln_prelu_bwd_f32": 3 * n * F1 * s,                   # Z and dH' read, dZ written
        "gather_rows_w16": n * 4 + 2 * n * F0 * s,            # feature rows: ids + rows read + rows written
        "gather_rows_w4": 3 * n * 4,                          # labels
        "partition": N * 4,
        "scan_reduce_flags": N * 4,
        "scan_apply_flags": N * 4 + N * 4 + n * 4,            # part read, g2l written, l2g written
        "row_count": n * (4 + 16 + 4) + rows_glob * 4 + N * 4,   # l2g, row bounds, deg out; entries; membership table
        "row_fill": n * (4 + 16 + 8 + 4) + rows_glob * 4 + N * 4 + nnz * 4,
        "scan_reduce_deg": n * 4,
        "scan_apply_deg": 2 * n * 4,
        "reduce_splits": None, "reduce_splits_halves": None,
        "sgd": 3 * n_params * 4,
        "average": 2 * K * n_params * 4 + n_params * 4,
    }
    if hbm.get(name):
        return "hbm", float(hbm[name])
    return None, 0.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--prefetch", action="store_true",
                    help="run the timed loop with the next step's partition, extraction and row gathers on a second "
                         "stream (kernels then overlap, so per-kernel durations no longer measure a kernel alone)")
    ap.add_argument("--headline-only", action="store_true",
                    help="skip the measurements reported beside the headline: per-layer fwd+bwd times, the two-stream loop")
    ap.add_argument("--dtype", choices=("f32", "bf16"), default="f32",
                    help="storage of features and activations (bf16: bf16 MFMA products, fp32 accumulation and "
                         "parameters); the headline workload is fp32, bf16 is a second measurement")
    ap.add_argument("--norm-act", action="store_true",
                    help="hidden layers with layer normalisation + PReLU (the paper's encoder variant) instead of "
                         "ReLU; a second measurement, not the headline workload")
    ap.add_argument("--encoder", choices=("sage", "gcn", "mlp"), default="sage",
                    help="the paper's other encoders (GCN, graph-agnostic MLP); a second measurement, not the "
                         "headline workload")
    ap.add_argument("--task", choices=("node", "link", "link-sampled"), default="node",
                    help="link: link prediction (edge mini-batch + random-tail negatives, MLP decoder on the pair "
                         "products of 256-d embeddings, BCE) instead of node classification; link-sampled: the same on "
                         "the sampled message-flow graph of each batch instead of the whole local subgraph; second "
                         "measurements")
    ap.add_argument("--batch", type=int, default=None,
                    help="positive edges per step of the link tasks (default 65536; 1024 for link-sampled)")
    ap.add_argument("--level-sizes", choices=("device", "host"), default="device",
                    help="link-sampled: leave the level sizes of a batch on the device while it is sampled and wait "
                         "for them once (default), or fetch each level's size as soon as it exists (one wait per level)")
    ap.add_argument("--inline-sampling", action="store_true",
                    help="link-sampled with --prefetch: the next batch's extraction and sampling calls are made by the "
                         "thread that trains instead of a worker thread")
    ap.add_argument("--fanouts", default="10,25",
                    help="link-sampled: neighbours kept per node, first layer first (the layer next to the batch last)")
    ap.add_argument("--extract", choices=("async", "sync", "fused"), default="async",
                    help="async (default): the step enqueues the extraction over capacity-sized buffers and never waits for "
                         "the GPU (the sizes, known from the set-up pass, are checked on the device values after the timed "
                         "region); sync: the two-pass extraction that returns the sizes to the host in every step; fused: "
                         "as async, with RandomTMA's assignment recomputed inside the extraction instead of a separate "
                         "assignment kernel and part array (tma_random_subgraph_async)")
    ap.add_argument("--graph", action="store_true",
                    help="beside the headline: capture one whole step (assignment, extraction, row gathers, training pass, "
                         "averaging) as a HIP graph and time its replays (node task, SGD)")
    ap.add_argument("--extraction", type=int, default=0, metavar="NODES",
                    help="time the assignment + induced-subgraph extraction alone on a Chung-Lu graph of NODES nodes "
                         "(e.g. 1000000, 100000000) instead of a configured workload")
    ap.add_argument("--avg-degree", type=float, default=20.0, help="with --extraction: average degree of that graph")
    ap.add_argument("--fused-assignment", action="store_true",
                    help="with --extraction: RandomTMA's assignment recomputed inside the extraction "
                         "(tma_random_subgraph_async) instead of tma_partition + tma_induced_subgraph_async")
    ap.add_argument("--library-reference", action="store_true",
                    help="no step of the path: time the layers' dense products as PLAIN products through the vendor "
                         "library behind torch.matmul, at the same shapes, as a yardstick for the hand-written ones")
    ap.add_argument("--config", type=int, choices=(0, 1, 2, 3, 4), default=1,
                    help="which of the configured workloads: 1 = the headline (default); 0 = the tiny case; 2 = SuperTMA at "
                         "full size; 3 = one trainer's share at billion-edge scale; 4 = 8 trainers on 8 streams with "
                         "parameter averaging every 50 local steps")
    ap.add_argument("--ld", type=int, default=0,
                    help="config 2: row pitch of the 100-wide bf16 feature matrix in elements (100 = dense, 128 = padded)")
    ap.add_argument("--scale", type=float, default=1.0,
                    help="configs 3 and 4: fraction of the configured graph size (1.0 = as configured)")
    ap.add_argument("--summarize-traffic", nargs=4, metavar=("KEY", "FETCH_DIR", "WRITE_DIR", "BENCH_JSON"),
                    help="no GPU work: write profiles/hbm_traffic.json and profiles/bench_<KEY>_hbm_traffic.txt from two "
                         "rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE) of this script and the JSON line one of them printed; "
                         "KEY = configs1, configs2_ld100, ...")
    ap.add_argument("--summarize-kernel-stats", nargs=3, metavar=("KEY", "STATS_DIR", "BENCH_JSON"),
                    help="no GPU work: write profiles/bench_<KEY>_kernel_stats.txt from a `rocprofv3 --kernel-trace --stats "
                         "--output-format csv` run of this script and the JSON line it printed")
    ap.add_argument("--summarize-counters", nargs=2, metavar=("KEY", "PMC_DIR"),
                    help="no GPU work: write profiles/bench_<KEY>.txt, the per-kernel means of the counters of one "
                         "rocprofv3 --pmc run of this script (give its command with --profiled-command, a heading with --title)")
    ap.add_argument("--title", default="Hardware counters per kernel launch")
    ap.add_argument("--calibration-dirs", nargs=2, metavar=("COPY_FETCH_DIR", "COPY_WRITE_DIR"), default=None,
                    help="with --summarize-traffic: counter runs of `bench.py --calibrate-copy` to take the scale factors from")
    ap.add_argument("--profiled-command", default=None,
                    help="with --summarize-traffic: the bench.py command line that the counter runs profiled")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device copy (reference for scaling rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.summarize_counters:
        from paper_2305_09887_amd import benchlib
        print(benchlib.summarize_counters(args.summarize_counters[0], args.summarize_counters[1],
                                          args.profiled_command or "bench.py --headline-only --steps 5 --warmup 2 --no-cpu-baseline",
                                          args.title))
        return
    if args.summarize_kernel_stats:
        from paper_2305_09887_amd import benchlib
        key, sd, bj = args.summarize_kernel_stats
        print(benchlib.summarize_kernel_stats(key, sd, bj, args.profiled_command or "bench.py --headline-only --steps 10 --warmup 3 --no-cpu-baseline"))
        return
    if args.summarize_traffic:
        from paper_2305_09887_amd import benchlib
        key, fd, wd, bj = args.summarize_traffic
        cal = args.calibration_dirs or (None, None)
        got = benchlib.summarize_traffic(key, fd, wd, bj, args.profiled_command or "bench.py --headline-only --steps 5 --warmup 2 --no-cpu-baseline",
                                         cal[0], cal[1])
        print(json.dumps({k: v["bytes"] for k, v in got["kernels"].items()}))
        return
    if args.batch is None:
        args.batch = 1024 if args.task == "link-sampled" else 65536
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (trainers are independent; nothing is sharded "
                 "across GPUs). Use --gpus 1.")

    import numpy as np
    import torch
    from paper_2305_09887_amd import benchlib, binding as B, synth
    from paper_2305_09887_amd.trainer import LocalTrainer, SampledLinkTrainer, SubgraphPrefetcher

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    B.lib()
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")       # 1 GiB read + 1 GiB written per copy
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": src.numel() * 4, "calibrate_copy_bytes_written": src.numel() * 4,
                          "copies": 5}))
        return
    if args.library_reference:
        print(json.dumps(benchlib.run_library_reference(args)), flush=True)
        return
    if args.extraction:
        out, _ = benchlib.run_extraction(args)
        print(json.dumps(out), flush=True)
        return
    if args.config >= 2:
        if args.task != "node" or args.encoder != "sage" or args.norm_act or args.prefetch or args.dtype != "f32":
            sys.exit("bench.py: --config 2, 3 and 4 run the SAGE node task in the configuration's own dtype")
        if args.config == 4 and args.steps == 50:
            args.steps = 200                      # 4 rounds of 50 local steps
        out, sample = {2: benchlib.run_supertma, 3: benchlib.run_share, 4: benchlib.run_aggregation}[args.config](args)
        if not args.no_cpu_baseline:
            out["cpu_baseline"] = cpu_baseline_leg(sample)
        print(json.dumps(out), flush=True)
        return
    w = TINY if args.config == 0 else WORKLOAD
    N, K, p = w["n_nodes"], w["K"], w["part"]
    dims = [w["F"], w["hidden"], w["classes"]]
    dec_dims = None
    if args.task != "node":      # hidden size 256 for encoder and decoder (the paper's setting for its mid-size graphs)
        dims = [w["F"], w["hidden"], w["hidden"]]
        dec_dims = [w["hidden"], w["hidden"], 1]
    L = len(dims) - 1
    sd = w["seeds"]

    t0 = time.time()
    if args.config == 0:
        rowptr, colidx = synth.uniform_graph(N, w["n_edges"], seed=sd["graph"])
    else:
        rowptr, colidx = synth.chung_lu_graph(N, w["avg_degree"], w["gamma"], seed=sd["graph"])
    X = synth.features(N, dims[0], seed=sd["feat"])
    y = synth.labels(N, dims[-1], seed=sd["label"])
    params = synth.sage_params(dims, seed=sd["weights"])
    print(f"[bench] inputs generated in {time.time() - t0:.1f}s: nnz={int(rowptr[-1])}", file=sys.stderr, flush=True)

    dev = torch.device("cuda:0")
    d_rowptr, d_colidx = torch.as_tensor(rowptr).to(dev), torch.as_tensor(colidx).to(dev)
    feat_dtype = torch.bfloat16 if args.dtype == "bf16" else torch.float32
    sb = 2 if args.dtype == "bf16" else 4          # bytes per stored feature / activation element
    peak_mfma = PEAK_MFMA_BF16_TFLOPS if args.dtype == "bf16" else PEAK_MFMA_F32_TFLOPS
    d_X, d_y = torch.as_tensor(X).to(dev).to(feat_dtype), torch.as_tensor(y).to(dev)
    part = torch.empty(N, dtype=torch.int32, device=dev)

    # set-up pass: learn the local sizes, allocate every persistent buffer
    B.tma_partition(N, K, sd["part"], out=part)
    sub = B.tma_induced_subgraph(d_rowptr, d_colidx, part, p)
    n_loc, nnz_loc = sub["n_loc"], sub["nnz_loc"]
    Xl = torch.empty((n_loc, dims[0]), dtype=feat_dtype, device=dev)
    yl = torch.empty(n_loc, dtype=torch.int32, device=dev)
    if args.encoder != "sage":   # one weight matrix per layer
        params = [(Ws, b) for Ws, _, b in params]
    if args.norm_act:   # gamma = 1, beta = 0, slope = 0.25 on the hidden layers
        params = [tuple(l) + ((np.ones(dims[i + 1], np.float32), np.zeros(dims[i + 1], np.float32),
                               np.full(1, 0.25, np.float32)) if i < L - 1 else ()) for i, l in enumerate(params)]
    link = {}
    if dec_dims is not None:
        link = dict(decoder_dims=dec_dims, batch_size=args.batch, batch_seed=sd["part"] + 1, nnz=nnz_loc)
    sampled = args.task == "link-sampled"
    fanouts = [int(f) for f in args.fanouts.split(",")] if sampled else None
    if sampled:
        if args.encoder == "mlp" or args.norm_act or len(fanouts) != L:
            sys.exit("bench.py: link-sampled runs the SAGE or GCN encoder with ReLU and needs one fan-out per layer")
        tr = SampledLinkTrainer(sub["rowptr"], sub["colidx"], nnz_loc, Xl, dims, dec_dims, fanouts, args.batch,
                                batch_seed=sd["part"] + 1, params=params, nnz_cap=nnz_loc + nnz_loc // 4 + 4096,
                                encoder=args.encoder, device_counts=args.level_sizes == "device")
    else:
        tr = LocalTrainer(sub["rowptr"], sub["colidx"], sub["inv_deg"], Xl, yl, dims, params=params,
                          norm_act=args.norm_act, encoder=args.encoder, **link)
    if dec_dims is not None:
        rng = np.random.default_rng(sd["weights"] + 1)
        K_dec = len(dec_dims) - 1
        tr.load_params(params, [(synth.glorot(a, b, rng),) + ((np.full(1, 0.25, np.float32),) if k < K_dec - 1 else ())
                                for k, (a, b) in enumerate(zip(dec_dims[:-1], dec_dims[1:]))])
    peers = [tr.W.clone() for _ in range(K - 1)]      # the other K-1 trainers' parameter vectors
    W_all = [tr.W] + peers
    ptrs = torch.tensor([t.data_ptr() for t in W_all], dtype=torch.int64, device=dev)
    W_global = torch.empty_like(tr.W)
    cap = n_loc + n_loc // 8 + 1024              # capacities a caller would choose from the expected sizes
    cap_nnz = nnz_loc + nnz_loc // 4 + 4096

    # Two loops over the same work.  The headline loop runs everything on one stream, so that the timed region,
    # the per-kernel events and the profiler's durations describe kernels running alone.  The two-stream loop runs
    # the next step's partition, extraction and row gathers (they depend on the assignment seed only) on a second
    # stream while this step trains: the host's wait for the subgraph sizes never idles the training stream.
    # Every step still does all of its own work: K steps = K extractions + K training passes.
    two_stream = SubgraphPrefetcher(d_rowptr, d_colidx, N, K, p, cap, cap_nnz, tables=(d_X,) if sampled else (d_X, d_y))
    state = {"next": None, "trained": None}

    held = None
    if args.extract == "async":
        held = B.tma_induced_subgraph_async(d_rowptr, d_colidx, part, p, cap, cap_nnz)
    elif args.extract == "fused":
        held = B.tma_random_subgraph_async(d_rowptr, d_colidx, K, sd["part"], p, cap, cap_nnz)

    def prepare_sampled(prefetch, after):
        """Sampled task: the next step's assignment, extraction, row gather AND batch sampling on the extraction
        stream (the batch depends on the subgraph, the feature rows and the seeds only), driven by the trainer's
        worker thread while this thread enqueues the training pass."""
        if tr._side is not prefetch.stream:
            tr.enable_prefetch(stream=prefetch.stream, auto=False, background=not args.inline_sampling)

        def prepare():
            s, rows, ready = prefetch.start(sd["part"], after=after)
            tr.set_graph(s["rowptr"], s["colidx"], s["nnz_loc"], ready=ready)
            tr.set_data(rows[0])

        tr.prefetch_sample(prepare)

    def step(prefetch=two_stream if args.prefetch else None):
        if prefetch is None:
            if args.extract != "fused":
                B.tma_partition(N, K, sd["part"], out=part)
            if held is not None:      # same buffers every step; views at the sizes the set-up pass reported
                if args.extract == "fused":
                    B.tma_random_subgraph_async(d_rowptr, d_colidx, K, sd["part"], p, cap, cap_nnz, out=held)
                else:
                    B.tma_induced_subgraph_async(d_rowptr, d_colidx, part, p, cap, cap_nnz, out=held)
                s = dict(l2g=held["l2g"][:n_loc], rowptr=held["rowptr"][:n_loc + 1], colidx=held["colidx"][:nnz_loc],
                         inv_deg=held["inv_deg"][:n_loc], nnz_loc=nnz_loc)
            else:
                s = B.tma_induced_subgraph(d_rowptr, d_colidx, part, p, cap_n_loc=cap, cap_nnz_loc=cap_nnz)
        elif sampled:
            if tr._pending is None or tr._side is not prefetch.stream:
                prepare_sampled(prefetch, None)
        else:
            if state["next"] is None:
                state["next"] = prefetch.start(sd["part"])
            s, rows, ready = state["next"]
            torch.cuda.current_stream().wait_event(ready)
            tr.set_data(*rows)
        if prefetch is None:
            B.tma_gather_rows(s["l2g"], d_X, out=Xl)
            B.tma_gather_rows(s["l2g"], d_y, out=yl)
        if sampled and prefetch is None:
            tr.set_graph(s["rowptr"], s["colidx"], s["nnz_loc"])
        elif not sampled:
            tr.set_graph(s["rowptr"], s["colidx"], s["inv_deg"], nnz=s["nnz_loc"])
        tr.step(w["lr"])
        B.tma_average(W_all, W_global_out=W_global, ptr_table=ptrs)
        if prefetch is not None:
            trained = torch.cuda.Event()
            trained.record()
            # the allocator may hand the next extraction the buffers that the step before this one read
            if sampled:
                prepare_sampled(prefetch, state["trained"])
            else:
                state["next"] = prefetch.start(sd["part"], after=state["trained"])
            state["trained"] = trained

    def settle():
        """Everything enqueued has run, including what a sampler's worker thread is still enqueueing."""
        if sampled:
            tr._drain()
        torch.cuda.synchronize()

    for _ in range(args.warmup):
        step()
    settle()

    # which kernel dominates: every kernel timed with events over three untimed steps
    B.tma_profile_begin(None)
    for _ in range(3):
        step()
    settle()
    prof = B.tma_profile_end()
    per_step = {k: v[1] / 3.0 for k, v in prof.items()}
    dominant = max(per_step, key=per_step.get)

    B.tma_profile_begin(None)       # the launch order of one step (matched against a profiler's dispatch list)
    step()
    settle()
    B.tma_profile_end()
    kernel_sequence = B.tma_profile_sequence()

    # timed region; the dominant kernel alone carries events
    B.tma_profile_begin(dominant)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for _ in range(args.steps):
        step()
    settle()
    elapsed = time.perf_counter() - t_start
    dom = B.tma_profile_end().get(dominant, (0, 0.0))
    ms_per_step = elapsed * 1e3 / args.steps
    loss = float(tr.loss.item())
    if held is not None and held["sizes"].cpu().tolist() != [n_loc, nnz_loc]:
        sys.exit(f"bench.py: the extraction reported sizes {held['sizes'].cpu().tolist()}, expected {[n_loc, nnz_loc]}")

    # beside the headline: the same step captured once as a HIP graph and replayed (no launch gaps, no host work)
    graph_leg = None
    if args.graph:
        if args.task != "node" or held is None or args.prefetch:
            sys.exit("bench.py: --graph captures the node task's step with --extract async and without --prefetch")
        gs = torch.cuda.Stream()
        gs.wait_stream(torch.cuda.current_stream())
        tr.stream = gs
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=gs):
            step()
        for _ in range(max(args.warmup, 2)):
            graph.replay()
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t_start) * 1e3 / args.steps
        tr.stream = torch.cuda.current_stream()
        graph_leg = {"ms_per_step": round(graph_ms, 4), "eager_ms_per_step": round(ms_per_step, 4),
                     "saved_ms_per_step": round(ms_per_step - graph_ms, 4), "steps": args.steps,
                     "loss_after": float(tr.loss.item())}

    # beside the headline: every encoder layer's forward and backward bracketed by events, median over 20 more steps
    per_layer = None
    if not sampled and not args.headline_only:
        tr.time_layers(True)
        for _ in range(20):
            step()
        t_layers = tr.layer_times_ms()
        tr.time_layers(False)
        per_layer = []
        for l in range(L):
            f, b = float(np.median(t_layers["fwd"][l])), float(np.median(t_layers["bwd"][l]))
            per_layer.append({"layer": l, "F_in": dims[l], "F_out": dims[l + 1], "fwd_ms": round(f, 4), "bwd_ms": round(b, 4),
                              "edges_per_s": round(nnz_loc / ((f + b) * 1e-3), 1)})

    # second measurement, reported beside the headline: the same K steps with the two-stream loop
    # Whether the two streams really overlap is the runtime's choice (streams share a few hardware queues, and two
    # streams on one queue run one after the other, which is slower than one stream): up to four attempts, each with
    # a new side stream, until one beats the one-stream loop; every attempt is reported.
    two_stream_ms, two_stream_tries = None, []
    if not args.prefetch and not args.headline_only:
        for attempt in range(4):
            if attempt:
                two_stream = SubgraphPrefetcher(d_rowptr, d_colidx, N, K, p, cap, cap_nnz,
                                                tables=(d_X,) if sampled else (d_X, d_y))
                state["next"], state["trained"] = None, None
            for _ in range(max(args.warmup, 2)):
                step(two_stream)
            settle()
            t_start = time.perf_counter()
            for _ in range(args.steps):
                step(two_stream)
            settle()
            two_stream_tries.append(round((time.perf_counter() - t_start) * 1e3 / args.steps, 4))
            if two_stream_tries[-1] < ms_per_step:
                break
        two_stream_ms = min(two_stream_tries)
        if sampled:
            tr.disable_prefetch()
        tr.set_data(Xl, yl) if not sampled else tr.set_data(Xl)

    kw = dict(N=N, nnz_glob=int(rowptr[-1]), K=K, n_params=int(tr.W.numel()), encoder=args.encoder)
    def work_of(k):
        if args.task == "link" and args.encoder == "sage":
            hit = link_kernel_work(k, n_loc, nnz_loc, dims, dec_dims, args.batch, s=sb)
            if hit[0]:
                return hit
        if args.task != "node" and k.startswith(("gemm", "spmm", "scale_mask", "softmax", "ln_prelu", "pair_", "prelu")):
            return None, 0.0     # shapes of the link task that the tables do not cover
        return kernel_work(k, n_loc, nnz_loc, dims, s=sb, **kw)

    # HBM bytes per launch as rocprofv3's counters measured them for this workload (profiles/hbm_traffic.json,
    # written by `bench.py --summarize-traffic` from the counter runs named there)
    traffic_table = benchlib.load_traffic("configs1") if (args.config == 1 and args.task == "node" and args.encoder == "sage"
                                                           and args.dtype == "f32" and not args.norm_act) else {}
    bound, work = work_of(dominant)
    avg_ms = dom[1] / max(dom[0], 1)
    if bound == "mfma":
        achieved, peak, unit = work / (avg_ms * 1e-3) / 1e12, peak_mfma, "TFLOP/s"
    else:
        bound = "hbm"
        achieved, peak, unit = work / (avg_ms * 1e-3) / 1e9, PEAK_HBM_GBS, "GB/s"
    roofline = dict(bound=bound, kernel=dominant, achieved=round(achieved, 3), peak=peak, unit=unit,
                    frac=round(achieved / peak, 4), traffic=traffic_table.get(dominant.replace("_generic", "")),
                    avg_launch_ms=round(avg_ms, 5), launches=dom[0],
                    algorithmic_work_per_launch=work)

    # every kernel against its own roofline, from the event-timed profile pass (an event pair adds a few
    # microseconds to a launch, so the short kernels read low; profiles/ holds the rocprofv3 durations)
    kernel_rooflines = {}
    for k, ms in per_step.items():
        b, wk = work_of(k)
        launches = prof[k][0] / 3.0
        if b is None or ms <= 0:
            continue
        per_launch_s = ms * 1e-3 / launches
        traffic = traffic_table.get(k.replace("_generic", ""))
        if b == "mfma":
            kernel_rooflines[k] = {"bound": b, "achieved": round(wk / per_launch_s / 1e12, 2), "peak": peak_mfma,
                                   "unit": "TFLOP/s", "frac": round(wk / per_launch_s / 1e12 / peak_mfma, 4), "traffic": traffic,
                                   "traffic_GBs": round(traffic / per_launch_s / 1e9, 1) if traffic else None}
        else:
            kernel_rooflines[k] = {"bound": b, "achieved": round(wk / per_launch_s / 1e9, 1), "peak": PEAK_HBM_GBS,
                                   "unit": "GB/s", "frac": round(wk / per_launch_s / 1e9 / PEAK_HBM_GBS, 4), "traffic": traffic,
                                   "traffic_GBs": round(traffic / per_launch_s / 1e9, 1) if traffic else None}
            gb = gathered_bytes(k, n_loc, nnz_loc, dims, s=sb) if args.task == "node" and args.encoder == "sage" else None
            if gb:    # every gathered row counted: the rate at which the kernel pulls rows through the memory system
                kernel_rooflines[k]["gathered_GBs"] = round(gb / per_launch_s / 1e9, 1)
                kernel_rooflines[k]["gathered_frac"] = round(gb / per_launch_s / 1e9 / PEAK_HBM_GBS, 4)

    value = L * nnz_loc / (ms_per_step * 1e-3)
    sampled_info = None
    if sampled:      # the step aggregates over the sampled blocks only: count their entries (of the last step)
        entries = [int(tr.blk_rowptr[l][tr.count[l + 1]].item()) for l in range(L)]
        value = sum(entries) / (ms_per_step * 1e-3)
        sampled_info = {"fanouts": fanouts, "level_nodes": list(tr.count), "block_entries": entries,
                        "positives_per_s": round(args.batch / (ms_per_step * 1e-3), 1),
                        "value_definition": "entries of the sampled blocks (all layers) / step time"}
    train_ms = sum(v for k, v in per_step.items()
                   if k.startswith(("spmm", "gemm", "reduce", "softmax", "finish", "sgd", "ln_prelu", "scale_mask", "sum_partials", "edge_batch",
                                    "pair_product", "incidence", "exclusive_scan", "prelu", "bce", "sample_", "mfg_",
                                    "block_", "transpose_")))
    out = {
        "metric": "trainer edges/sec per SAGE layer fwd+bwd; achieved HBM GB/s vs peak",
        "value": round(value, 1), "unit": "edges/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": ("configs[0] Tiny: uniform random graph, 20,000 nodes, 100,000 undirected edges, 64-d fp32 features, "
                                "16 labels; K=4 random node partitions; whole path per step = partition + induced-subgraph "
                                "extraction of part 0 + row gather + 2-layer mean-SAGE (hidden 64) full-batch fwd+bwd+SGD + "
                                "4-way parameter averaging") if args.config == 0 else
                               "configs[1]: Chung-Lu power-law graph (gamma 2.1), 1M nodes, avg degree 20, 128-d " + ("fp32 " if args.dtype == "f32" else "bf16 (second measurement; the configuration names fp32) ") +
                               "features, 47 classes; K=8 random node partitions; whole path per step = partition + "
                               "induced-subgraph extraction of part 0 + row gather + 2-layer mean-SAGE (hidden 256) "
                               "full-batch fwd+bwd+SGD + 8-way parameter averaging",
                   "n_nodes": N, "nnz_global": int(rowptr[-1]), "K": K, "n_loc": n_loc, "nnz_loc": nnz_loc,
                   "layers": L, "dims": dims, "task": args.task, "sampled": sampled_info, "decoder_dims": dec_dims, "batch_positive_edges": args.batch if dec_dims else None,
                   "encoder": args.encoder, "hidden_activation": "layernorm+prelu" if args.norm_act else "relu", "edge_definition": "directed local CSR entry; value = layers*nnz_loc/step time"},
        "roofline": roofline,
        "kernel_rooflines": kernel_rooflines,
        "kernel_ms_per_step": {k: round(v, 5) for k, v in sorted(per_step.items(), key=lambda kv: -kv[1])},
        "train_only_edges_per_s": round(L * nnz_loc / (train_ms * 1e-3), 1) if train_ms > 0 else None,
        "final_loss": loss,
        "streams": 2 if args.prefetch else 1,
        "kernel_sequence": kernel_sequence,
    }
    if per_layer is not None:
        out["per_layer_fwd_bwd"] = per_layer      # edges_per_s = nnz_loc / (fwd + bwd) of that layer alone
    out["config"]["extract"] = args.extract
    if graph_leg is not None:
        out["hip_graph"] = graph_leg
    if two_stream_ms is not None:
        out["two_stream"] = {"ms_per_step": round(two_stream_ms, 4), "value": round(value * ms_per_step / two_stream_ms, 1),
                             "unit": "edges/s", "steps": args.steps, "attempts_ms": two_stream_tries,
                             "what": "the same steps with the next step's partition, extraction and row gathers on a "
                                     "second stream (bench.py --prefetch times that loop as the headline)"}

    if not args.no_cpu_baseline and args.task == "node" and args.dtype == "f32":
        def full(oracle, omodel, p_o):       # one full step of the same workload at full size
            part_o = oracle.partition(N, K, seed=sd["part"])
            sub_o = oracle.induced_subgraph(rowptr, colidx, part_o, p)
            Xo, yo = X[sub_o["l2g"]], y[sub_o["l2g"]]
            _, p_new = omodel.train_step(sub_o["rowptr"], sub_o["colidx"], Xo, yo, p_o, w["lr"], encoder=args.encoder)
            omodel.aggregate([p_new] + [p_o] * (K - 1))
        out["cpu_baseline"] = cpu_baseline_leg(dict(
            params=params, full=full, edges=L * nnz_loc,
            what=f"one full step of the same workload at full size (n_loc={n_loc}, nnz_loc={nnz_loc})"))
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
