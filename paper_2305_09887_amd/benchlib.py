"""Measurement helpers of bench.py: the algorithmic work of every kernel of an L-layer mean-aggregation GraphSAGE
step (Thm. 1's Abar X W per layer, forward and backward), per-layer event windows that tell which launch of a kernel
name belongs to which layer, stored HBM-traffic figures, and the benchmark loops of the configurations other than the
headline one.  Measurement only: no step of the method is computed here; every numerical step is a call into the
C ABI through ``binding`` / ``trainer``."""
from __future__ import annotations

import json
import os
import sys
import time

import torch

from . import binding as B

PEAK_HBM_GBS = 8000.0
PEAK_MFMA_F32_TFLOPS = 157.3
PEAK_MFMA_BF16_TFLOPS = 2500.0

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")

# kernel families, longest prefix first
FAMILIES = ("gemm_tf_bwd_weight", "gemm_tf_bwd_data", "gemm_tf_fwd", "gemm_bwd_weight", "gemm_bwd_data", "gemm_fwd",
            "spmm_mean", "spmm_combine", "spmm_sum", "scale_mask_rows")


def family(name: str):
    for f in FAMILIES:
        if name.startswith(f):
            return f
    return None


def padded_width(F: int, s: int) -> int:
    return (F * s + 15) // 16 * 16 // s


def sage_layer_work(n: int, nnz: int, dims, s: int, dt: int):
    """{(phase, layer, family): (bound, algorithmic work of that launch[, bytes of a product])} for an L-layer
    model on one graph.

    Bytes count every array the kernel must touch once (each distinct input row once however often it is gathered,
    outputs once: the B_min of a gather); flops count the products of the layer's definition, no padding.  A
    product also carries the bytes of its streamed operands and results (weights left out), because with bf16
    storage its honest ceiling is the smaller of the matrix peak and intensity x HBM bandwidth."""
    out = {}
    L = len(dims) - 1
    for l, (Fi, Fo) in enumerate(zip(dims[:-1], dims[1:])):
        Fp = padded_width(Fo, s)
        g = (2.0 if l < L - 1 else 1.0) * n * Fo * s     # the upstream gradient, and the layer output as ReLU mask
        if B.tma_sage_layer_aggregates_first(Fi, Fo, dt):
            out[("fwd", l, "spmm_mean")] = ("hbm", 2.0 * n * Fi * s + nnz * 4 + n * 8)
            out[("fwd", l, "gemm_fwd")] = ("mfma", 2.0 * n * 2 * Fi * Fo, n * 2.0 * Fi * s + n * Fo * s)
            out[("bwd", l, "gemm_bwd_weight")] = ("mfma", 2.0 * n * 2 * Fi * Fo, n * 2.0 * Fi * s + g)
            if l > 0:
                out[("bwd", l, "gemm_bwd_data")] = ("mfma", 2.0 * n * Fo * 2 * Fi, g + n * 2.0 * Fi * s)
                out[("bwd", l, "spmm_sum")] = ("hbm", 3.0 * n * Fi * s + nnz * 4 + n * 4)    # dM rows once; dH read + written
        else:
            out[("fwd", l, "gemm_tf_fwd")] = ("mfma", 2.0 * n * Fi * 2 * Fo, n * Fi * s + n * 2.0 * Fp * s)
            out[("fwd", l, "spmm_combine")] = ("hbm", 3.0 * n * Fp * s + nnz * 4 + n * 8)    # Yn rows once, Ys, output
            out[("bwd", l, "scale_mask_rows")] = ("hbm", float(n * Fo * s + n * 4 + n * Fp * s))
            out[("bwd", l, "spmm_sum")] = ("hbm", 2.0 * n * Fp * s + nnz * 4 + n * 4)
            out[("bwd", l, "gemm_tf_bwd_weight")] = ("mfma", 2.0 * n * Fi * 2 * Fo, n * Fi * s + g + n * Fp * s)
            if l > 0:
                out[("bwd", l, "gemm_tf_bwd_data")] = ("mfma", 2.0 * n * 2 * Fo * Fi, g + n * Fp * s + n * Fi * s)
    return out


def other_kernel_work(name, n, nnz, F0, C, s, N=0, rows_glob=0, K=1, n_params=0):
    """Kernels outside the layers (loss, optimizer, averaging, partition, extraction, row gather): ("hbm", bytes)."""
    table = {
        "softmax_ce": 2 * n * C * s + n * 4,
        "gather_rows_w16": n * 4 + 2 * n * F0 * s,
        "gather_rows_w4": 3 * n * 4,
        "partition": N * 4,
        "scan_reduce_flags": N * 4,
        "scan_apply_flags": N * 4 + N * 4 + n * 4,
        "row_count": n * (4 + 16 + 4) + rows_glob * 4 + N * 4,
        "row_fill": n * (4 + 16 + 8 + 4) + rows_glob * 4 + N * 4 + nnz * 4,
        "scan_reduce_deg": n * 4,
        "scan_apply_deg": 2 * n * 4,
        "sgd": 3 * n_params * 4,
        "average": 2 * K * n_params * 4 + n_params * 4,
    }
    w = table.get(name.replace("_bf16", ""))
    return ("hbm", float(w)) if w else (None, 0.0)


class LayerWindows:
    """Event-profiler windows around every layer's forward and backward of a LocalTrainer: which kernel names run
    in which (phase, layer), how often and for how long.  Uses the trainer's own layer marks."""

    def __init__(self, tr):
        self.tr, self.open, self.seen = tr, set(), {}

    def _mark(self, which, l):
        key = (which, l)
        if key not in self.open:
            B.tma_profile_begin(None)
            self.open.add(key)
        else:
            self.open.discard(key)
            for name, (cnt, ms) in B.tma_profile_end().items():
                c, t = self.seen.get(key + (name,), (0, 0.0))
                self.seen[key + (name,)] = (c + cnt, t + ms)
        return None

    def run(self, step_fn, repeats=2):
        self.tr._mark = self._mark
        try:
            for _ in range(repeats):
                step_fn()
            torch.cuda.synchronize()
        finally:
            del self.tr._mark
        return {k: (c / repeats, t / repeats) for k, (c, t) in self.seen.items()}


def work_by_name(windows, layer_work):
    """Mean algorithmic work per launch of every kernel NAME that the layers launch: a name that several layers
    use with different shapes gets the mean over its launches of a step."""
    tot, cnt, bound, byt = {}, {}, {}, {}
    for (phase, l, name), (launches, _) in windows.items():
        fam = family(name)
        hit = layer_work.get((phase, l, fam))
        if not hit:
            continue
        tot[name] = tot.get(name, 0.0) + hit[1]
        cnt[name] = cnt.get(name, 0.0) + launches
        bound[name] = hit[0]
        if len(hit) > 2:
            byt[name] = byt.get(name, 0.0) + hit[2]
    return {k: (bound[k], tot[k] / max(cnt[k], 1.0)) + ((byt[k] / max(cnt[k], 1.0),) if k in byt else ())
            for k in tot}


def load_traffic(config_key: str):
    """{kernel name: HBM bytes per launch} measured with rocprofv3 counters for this configuration, or {}."""
    try:
        with open(TRAFFIC_FILE) as f:
            return {k: v["bytes"] for k, v in json.load(f).get(config_key, {}).get("kernels", {}).items()}
    except (OSError, ValueError):
        return {}


def rooflines(per_step, prof, repeats, work_of, peak_mfma, traffic):
    out = {}
    for k, ms in per_step.items():
        b, wk, *streamed = work_of(k)
        launches = prof[k][0] / float(repeats)
        if b is None or ms <= 0 or launches <= 0:
            continue
        sec = ms * 1e-3 / launches
        tr = traffic.get(k)
        if b == "mfma":
            a, peak, unit = wk / sec / 1e12, peak_mfma, "TFLOP/s"
        else:
            a, peak, unit = wk / sec / 1e9, PEAK_HBM_GBS, "GB/s"
        out[k] = {"bound": b, "achieved": round(a, 2), "peak": peak, "unit": unit, "frac": round(a / peak, 4),
                  "us_per_launch": round(sec * 1e6, 2), "traffic": tr,
                  "traffic_GBs": round(tr / sec / 1e9, 1) if tr else None}
        if streamed:      # a product against its other ceiling: streamed operands and results per time
            out[k]["streamed_GBs"] = round(streamed[0] / sec / 1e9, 1)
            out[k]["hbm_frac"] = round(streamed[0] / sec / 1e9 / PEAK_HBM_GBS, 4)
    return out


def dominant_roofline(name, dom, work_of, peak_mfma, traffic):
    bound, work, *streamed = work_of(name)
    avg_ms = dom[1] / max(dom[0], 1)
    if bound == "mfma":
        achieved, peak, unit = work / (avg_ms * 1e-3) / 1e12, peak_mfma, "TFLOP/s"
    else:
        bound = "hbm"
        achieved, peak, unit = work / (avg_ms * 1e-3) / 1e9, PEAK_HBM_GBS, "GB/s"
    out = dict(bound=bound, kernel=name, achieved=round(achieved, 3), peak=peak, unit=unit,
               frac=round(achieved / peak, 4), traffic=traffic.get(name), avg_launch_ms=round(avg_ms, 5),
               launches=dom[0], algorithmic_work_per_launch=work)
    if streamed:
        out["streamed_bytes_per_launch"] = streamed[0]
        out["streamed_GBs"] = round(streamed[0] / (avg_ms * 1e-3) / 1e9, 1)
        out["hbm_frac"] = round(streamed[0] / (avg_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)
    return out


def _log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def _timed_loop(step, steps, warmup, peak_mfma, work_of_factory, traffic):
    """Warm-up, all-kernel event pass, per-layer windows, timed region with events on the dominant kernel."""
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    B.tma_profile_begin(None)
    for _ in range(3):
        step()
    torch.cuda.synchronize()
    prof = B.tma_profile_end()
    per_step = {k: v[1] / 3.0 for k, v in prof.items()}
    dominant = max(per_step, key=per_step.get)
    work_of = work_of_factory()
    B.tma_profile_begin(None)
    step()
    torch.cuda.synchronize()
    B.tma_profile_end()
    sequence = B.tma_profile_sequence()
    B.tma_profile_begin(dominant)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    dom = B.tma_profile_end().get(dominant, (0, 0.0))
    return dict(ms_per_step=elapsed * 1e3 / steps, per_step=per_step, prof=prof, dominant=dominant, dom=dom,
                sequence=sequence,
                roofline=dominant_roofline(dominant, dom, work_of, peak_mfma, traffic),
                kernel_rooflines=rooflines(per_step, prof, 3, work_of, peak_mfma, traffic))


def oracle_sample(rowptr, colidx, X, y, params, lr, m, edges_equiv, what):
    """Inputs of a bounded oracle timing run (bench.py's cpu_baseline leg): the first m local rows with the entries
    among them, as host arrays.  Nothing here calls the oracle."""
    import numpy as np
    rp = rowptr[: m + 1].cpu().numpy().astype(np.int64)
    ci_all = colidx[: int(rp[-1])].cpu().numpy()
    rows = np.repeat(np.arange(m), np.diff(rp))
    keep = ci_all < m
    rps = np.zeros(m + 1, dtype=np.int32)
    rps[1:] = np.cumsum(np.bincount(rows[keep], minlength=m))
    return dict(rowptr=rps, colidx=ci_all[keep].astype(np.int32), X=X[:m].float().cpu().numpy(), y=y[:m].cpu().numpy(),
                params=params, lr=lr, edges=edges_equiv, what=what)


# ----------------------------------------------------------------------------------------------- configs[2]
def run_supertma(args):
    """configs[2]: stochastic-block graph, 2.4 M nodes in 2,400 planted communities, about 60 M edges (90 % inside a
    community), 100-d bf16 features with community-dependent means, super-nodes = communities assigned at random to
    K = 16 partitions (Sec. 3.2.2), 3-layer mean-SAGE (hidden 256).  Step = SuperTMA assignment + extraction of one
    part + row gather + full-batch forward, backward, SGD + 16-way averaging."""
    from . import synth, synth_torch as st
    from .trainer import LocalTrainer
    dev = torch.device("cuda:0")
    nb, bs, K, p = 2400, 1000, 16, 0
    dims, C, lr = [100, 256, 256, 47], 47, 1e-3
    N, s, dt = nb * bs, 2, B.TMA_BF16
    t0 = time.time()
    rowptr, colidx, block = st.sbm_graph(nb, bs, 54_000_000, 6_000_000, seed=21, device=dev)
    ld = int(args.ld) if args.ld else dims[0]
    if ld < dims[0] or (ld * s) % 4:
        sys.exit("bench.py: --ld must be at least the feature width and give rows of whole 4-byte words")
    Xfull = torch.zeros((N, ld), dtype=torch.bfloat16, device=dev)
    Xfull[:, :dims[0]] = st.community_features(block, nb, dims[0], seed=22, dtype=torch.bfloat16)
    X = Xfull[:, :dims[0]]
    y = (block % C).to(torch.int32)
    params = synth.sage_params(dims, seed=25)
    torch.cuda.synchronize()
    nnz_glob = int(rowptr[-1])
    _log(f"inputs generated on the GPU in {time.time() - t0:.1f}s: N={N} nnz={nnz_glob} ld={ld}")
    part = torch.empty(N, dtype=torch.int32, device=dev)
    B.tma_partition(N, K, 24, cluster=block, n_clusters=nb, out=part)
    sub = B.tma_induced_subgraph(rowptr, colidx, part, p)
    n_loc, nnz_loc = sub["n_loc"], sub["nnz_loc"]
    Xl_full = torch.zeros((n_loc, ld), dtype=torch.bfloat16, device=dev)
    Xl = Xl_full[:, :dims[0]]
    yl = torch.empty(n_loc, dtype=torch.int32, device=dev)
    tr = LocalTrainer(sub["rowptr"], sub["colidx"], sub["inv_deg"], Xl, yl, dims, params=params)
    W_all = [tr.W] + [tr.W.clone() for _ in range(K - 1)]
    ptrs = torch.tensor([t.data_ptr() for t in W_all], dtype=torch.int64, device=dev)
    W_global = torch.empty_like(tr.W)
    cap, cap_nnz = n_loc + n_loc // 8 + 1024, nnz_loc + nnz_loc // 4 + 4096

    held = B.tma_induced_subgraph_async(rowptr, colidx, part, p, cap, cap_nnz)

    def step():     # nothing in it waits for the GPU: the extraction leaves its sizes on the device (checked below)
        B.tma_partition(N, K, 24, cluster=block, n_clusters=nb, out=part)
        B.tma_induced_subgraph_async(rowptr, colidx, part, p, cap, cap_nnz, out=held)
        B.tma_gather_rows(held["l2g"][:n_loc], X, out=Xl)
        B.tma_gather_rows(held["l2g"][:n_loc], y, out=yl)
        tr.set_graph(held["rowptr"][:n_loc + 1], held["colidx"][:nnz_loc], held["inv_deg"][:n_loc], nnz=nnz_loc)
        tr.step(lr)
        B.tma_average(W_all, W_global_out=W_global, ptr_table=ptrs)

    L = len(dims) - 1
    lw = sage_layer_work(n_loc, nnz_loc, dims, s, dt)
    traffic = load_traffic(f"configs2_ld{ld}")

    def factory():
        wbn = work_by_name(LayerWindows(tr).run(step), lw)
        return lambda k: wbn.get(k) or other_kernel_work(k, n_loc, nnz_loc, dims[0], C, s, N=N, rows_glob=nnz_glob / K,
                                                         K=K, n_params=int(tr.W.numel()))

    r = _timed_loop(step, args.steps, args.warmup, PEAK_MFMA_BF16_TFLOPS, factory, traffic)
    if held["sizes"].cpu().tolist() != [n_loc, nnz_loc]:
        sys.exit(f"bench.py: the extraction reported sizes {held['sizes'].cpu().tolist()}, expected {[n_loc, nnz_loc]}")
    deg = (sub["rowptr"][1:] - sub["rowptr"][:-1]).float()
    out = _result(args, r, L * nnz_loc, "bf16", {
        "workload": f"configs[2] SuperTMA: stochastic-block graph, 2.4M nodes in 2,400 planted communities of 1,000, "
                    f"{nnz_glob // 2} undirected edges (54M drawn inside communities, 6M across), 100-d bf16 features with "
                    f"community-dependent means stored with row pitch {ld}, 47 classes; super-nodes = communities, K=16; "
                    "whole path per step = SuperTMA assignment + extraction of part 0 + row gather + 3-layer mean-SAGE "
                    "(hidden 256) full-batch fwd+bwd+SGD + 16-way parameter averaging",
        "n_nodes": N, "nnz_global": nnz_glob, "K": K, "n_loc": n_loc, "nnz_loc": nnz_loc, "layers": L, "dims": dims,
        "feature_row_pitch": ld, "mean_local_degree": round(float(deg.mean()), 2), "max_local_degree": int(deg.max()),
        "edge_definition": "directed local CSR entry; value = layers*nnz_loc/step time"}, tr)
    m = min(60_000, n_loc)            # about 10 s of single-threaded oracle work
    sample = oracle_sample(sub["rowptr"], sub["colidx"], Xl, yl, params, lr, m, None,
                           f"one full 3-layer step on the first {m} local nodes and the entries among them "
                           f"(of n_loc={n_loc}, nnz_loc={nnz_loc})")
    sample["edges"] = L * len(sample["colidx"])
    return out, sample


def _result(args, r, edges_per_step, dtype, config, tr):
    return {
        "metric": "trainer edges/sec per SAGE layer fwd+bwd; achieved HBM GB/s vs peak",
        "value": round(edges_per_step / (r["ms_per_step"] * 1e-3), 1), "unit": "edges/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(r["ms_per_step"], 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic", "config": config,
        "roofline": r["roofline"], "kernel_rooflines": r["kernel_rooflines"],
        "kernel_ms_per_step": {k: round(v, 5) for k, v in sorted(r["per_step"].items(), key=lambda kv: -kv[1])},
        "final_loss": float(tr.loss.item()) if tr is not None else None, "streams": 1,
        "kernel_sequence": r["sequence"],
    }


# ------------------------------------------------------------------------------- the extraction on its own
def run_extraction(args):
    """Assignment + node-induced subgraph extraction alone (Sec. 3.2.2; Preliminaries), at a global graph size of the
    caller's choice: a Chung-Lu power-law graph (gamma 2.1) of --extraction nodes with --avg-degree, drawn on the
    GPU; K = 8, part 0; the extraction that leaves its sizes on the device.  Step = tma_partition +
    tma_induced_subgraph_async.  Reports microseconds per step and every kernel against its algorithmic bytes."""
    from . import synth_torch as st
    dev = torch.device("cuda:0")
    N, K, p = int(args.extraction), 8, 0
    t0 = time.time()
    rowptr, colidx = st.chung_lu_graph(N, args.avg_degree, 2.1, seed=41, device=dev)
    torch.cuda.synchronize()
    nnz_glob = int(rowptr[-1])
    _log(f"graph drawn on the GPU in {time.time() - t0:.1f}s: N={N} nnz={nnz_glob}")
    part = torch.empty(N, dtype=torch.int32, device=dev)
    B.tma_partition(N, K, 44, out=part)
    first = B.tma_induced_subgraph(rowptr, colidx, part, p)
    n_loc, nnz_loc = first["n_loc"], first["nnz_loc"]
    rows_glob = int((rowptr[1:] - rowptr[:-1])[first["l2g"].long()].sum())     # global entries of the part's rows
    max_row = int((rowptr[1:] - rowptr[:-1]).max())
    cap, cap_nnz = n_loc + n_loc // 8 + 1024, nnz_loc + nnz_loc // 4 + 4096
    fused = bool(args.fused_assignment)
    if fused:    # the assignment recomputed inside the extraction: no part array, no assignment kernel
        held = B.tma_random_subgraph_async(rowptr, colidx, K, 44, p, cap, cap_nnz)
    else:
        held = B.tma_induced_subgraph_async(rowptr, colidx, part, p, cap, cap_nnz)
    same = all(torch.equal(held[k][:m], first[k][:m]) for k, m in
               (("g2l", N), ("l2g", n_loc), ("rowptr", n_loc + 1), ("colidx", nnz_loc), ("inv_deg", n_loc)))
    if not same or held["sizes"].cpu().tolist() != [n_loc, nnz_loc]:
        sys.exit("bench.py: the two forms of the extraction disagree")
    del first

    def step():
        if fused:
            B.tma_random_subgraph_async(rowptr, colidx, K, 44, p, cap, cap_nnz, out=held)
        else:
            B.tma_partition(N, K, 44, out=part)
            B.tma_induced_subgraph_async(rowptr, colidx, part, p, cap, cap_nnz, out=held)

    def factory():
        return lambda k: other_kernel_work(k, n_loc, nnz_loc, 0, 0, 0, N=N, rows_glob=rows_glob, K=K)

    r = _timed_loop(step, args.steps, args.warmup, PEAK_MFMA_BF16_TFLOPS, factory, {})
    out = _result(args, r, N, "int32", {
        "workload": f"extraction alone: Chung-Lu power-law graph (gamma 2.1), {N} nodes, {nnz_glob} CSR entries "
                    f"(longest row {max_row}), K=8 random node assignment, part 0; step = "
                    + ("node-induced subgraph extraction with the assignment recomputed inside it (no part array)"
                       if fused else "assignment of all ids + node-induced subgraph extraction")
                    + ", sizes left on the device (no host wait)",
        "n_nodes": N, "nnz_global": nnz_glob, "K": K, "n_loc": n_loc, "nnz_loc": nnz_loc,
        "entries_of_the_parts_rows": rows_glob, "fused_assignment": fused}, None)
    out["metric"], out["unit"] = "global nodes assigned and extracted per second", "nodes/s"
    algorithmic = sum(other_kernel_work(k, n_loc, nnz_loc, 0, 0, 0, N=N, rows_glob=rows_glob, K=K)[1] * c
                      for k, c in (("partition", 0 if fused else 1), ("scan_reduce_flags", 1), ("scan_apply_flags", 1), ("row_count", 1),
                                   ("scan_apply_deg", 1), ("row_fill", 1)))
    out["extraction"] = {"us_per_step": round(r["ms_per_step"] * 1e3, 1), "algorithmic_bytes_per_step": algorithmic,
                         "algorithmic_GBs": round(algorithmic / (r["ms_per_step"] * 1e-3) / 1e9, 1),
                         "frac_of_hbm_peak": round(algorithmic / (r["ms_per_step"] * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
    return out, None


# --------------------------------------------------------------- the vendor library's plain products, for scale
def run_library_reference(args):
    """NOT part of the path: the dense products of the configured layers as PLAIN matrix products through the
    vendor library that torch.matmul calls (no concatenated operands, no bias / ReLU / mask / scale epilogues, no
    split reduction), timed with events at the same shapes, so that the hand-written products can be read against
    what the chip's own library reaches at these shapes.  Returns one JSON-able dict."""
    dev = torch.device("cuda:0")
    torch.backends.cuda.matmul.allow_tf32 = False

    def timed(fn, reps):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e-3

    rows = []

    def product(what, n, k, m, dt, reduce_rows=False, reps=20):
        if reduce_rows:      # weight-gradient shape: [k, n] x [n, m], the long dimension reduced
            a = torch.randn(n, k, device=dev, dtype=dt)
            b = torch.randn(n, m, device=dev, dtype=dt)
            sec = timed(lambda: torch.matmul(a.t(), b), reps)
        else:
            a = torch.randn(n, k, device=dev, dtype=dt)
            b = torch.randn(k, m, device=dev, dtype=dt)
            c = torch.empty(n, m, device=dev, dtype=dt)
            sec = timed(lambda: torch.matmul(a, b, out=c), reps)
        streamed = (n * k + n * m) * a.element_size()
        rows.append({"what": what, "dtype": str(dt).replace("torch.", ""), "n": n, "k": k, "m": m,
                     "us": round(sec * 1e6, 1), "TFLOPs": round(2.0 * n * k * m / sec / 1e12, 1),
                     "streamed_GBs": round(streamed / sec / 1e9, 1)})
        del a, b

    n1 = 125_237
    product("configs[1] layer 0 forward, [H|M] x [Ws;Wn]", n1, 256, 256, torch.float32)
    product("configs[1] layer 0 weight gradient, [H|M]^T x dZ", n1, 256, 256, torch.float32, reduce_rows=True)
    product("configs[1] layer 1 forward (transform first), H x [Ws|Wn]", n1, 256, 96, torch.float32)
    product("configs[1] layer 1 weight gradient, H^T x [dZ|dYn]", n1, 256, 96, torch.float32, reduce_rows=True)
    product("configs[1] layer 1 data gradient, [dZ|dYn] x [Ws|Wn]^T", n1, 96, 256, torch.float32)
    product("fp32, large reduction (the library's ceiling)", 16_384, 8192, 8192, torch.float32, reps=3)
    n3 = int(12_496_872 * args.scale)
    product("configs[3] 256-wide layer forward", n3, 512, 256, torch.bfloat16, reps=5)
    product("configs[3] 256-wide layer data gradient", n3, 256, 512, torch.bfloat16, reps=5)
    product("configs[3] 256-wide layer weight gradient", n3, 512, 256, torch.bfloat16, reduce_rows=True, reps=5)
    return {"library_reference": rows, "note": "plain products through torch.matmul (the vendor library), event-timed; "
            "a yardstick for the hand-written fused products, not a step of the path"}


# ----------------------------------------------------------------------------------------------- configs[3]
def run_share(args):
    """configs[3]: one trainer's share at billion-edge scale.  The Chung-Lu graph of 100 M nodes / 1.3 B edges is not
    materialised: the part's node count comes from the K = 8 assignment of the 100 M ids (the library's call), and
    the part's own entries are drawn directly (synth_torch.chung_lu_share).  128-d bf16 features, 3-layer mean-SAGE
    (hidden 256).  Step = assignment of the 100 M ids + full-batch forward, backward, SGD + 8-way averaging."""
    from . import synth, synth_torch as st
    from .trainer import LocalTrainer
    dev = torch.device("cuda:0")
    scale = args.scale
    N, K, p = int(100_000_000 * scale), 8, 0
    total = 2.6e9 * scale
    dims, C, lr, s, dt = [128, 256, 256, 47], 47, 1e-3, 2, B.TMA_BF16
    t0 = time.time()
    part = torch.empty(N, dtype=torch.int32, device=dev)
    B.tma_partition(N, K, 34, out=part)
    n_loc = int((part == p).sum())
    rp64, colidx = st.chung_lu_share(N, total, 2.1, n_loc, seed=31, device=dev)
    nnz_loc = int(rp64[-1])
    rowptr = rp64.to(torch.int32)
    deg = rp64[1:] - rp64[:-1]
    inv_deg = torch.where(deg > 0, 1.0 / deg.clamp(min=1).float(), torch.zeros((), device=dev))
    max_deg, iso = int(deg.max()), float((deg == 0).float().mean())
    del rp64, deg
    g = torch.Generator(device=dev)
    g.manual_seed(32)
    X = torch.empty((n_loc, dims[0]), dtype=torch.bfloat16, device=dev)
    for a in range(0, n_loc, 1 << 21):
        X[a:a + (1 << 21)] = torch.randn((min(1 << 21, n_loc - a), dims[0]), generator=g, device=dev).to(torch.bfloat16)
    g.manual_seed(33)
    y = torch.randint(0, C, (n_loc,), generator=g, device=dev, dtype=torch.int32)
    params = synth.sage_params(dims, seed=35)
    torch.cuda.synchronize()
    _log(f"share generated on the GPU in {time.time() - t0:.1f}s: n_loc={n_loc} nnz_loc={nnz_loc} max degree {max_deg}")
    tr = LocalTrainer(rowptr, colidx, inv_deg, X, y, dims, params=params)
    W_all = [tr.W] + [tr.W.clone() for _ in range(K - 1)]
    ptrs = torch.tensor([t.data_ptr() for t in W_all], dtype=torch.int64, device=dev)
    W_global = torch.empty_like(tr.W)

    def step():
        B.tma_partition(N, K, 34, out=part)
        tr.step(lr)
        B.tma_average(W_all, W_global_out=W_global, ptr_table=ptrs)

    L = len(dims) - 1
    lw = sage_layer_work(n_loc, nnz_loc, dims, s, dt)
    traffic = load_traffic("configs3")

    def factory():
        wbn = work_by_name(LayerWindows(tr).run(step), lw)
        return lambda k: wbn.get(k) or other_kernel_work(k, n_loc, nnz_loc, dims[0], C, s, N=N, K=K,
                                                         n_params=int(tr.W.numel()))

    r = _timed_loop(step, args.steps, args.warmup, PEAK_MFMA_BF16_TFLOPS, factory, traffic)
    out = _result(args, r, L * nnz_loc, "bf16", {
        "workload": f"configs[3]: one trainer's share of a Chung-Lu power-law graph (gamma 2.1) of {N} nodes and "
                    f"{total / 2:.3g} undirected edges, K=8 random node assignment, part 0; the share's entries are drawn "
                    "directly (the global graph is not materialised), 128-d bf16 features, 47 classes; step = assignment "
                    "of all global ids + 3-layer mean-SAGE (hidden 256) full-batch fwd+bwd+SGD + 8-way parameter averaging"
                    + ("" if scale == 1.0 else f" [scaled to {scale:g} of the configured size]"),
        "n_nodes": N, "K": K, "n_loc": n_loc, "nnz_loc": nnz_loc, "layers": L, "dims": dims,
        "max_local_degree": max_deg, "isolated_share": round(iso, 3),
        "edge_definition": "directed local CSR entry; value = layers*nnz_loc/step time"}, tr)
    m = min(100_000, n_loc)           # about 12 s of single-threaded oracle work
    # the step's cost is dominated by the rows (dense products), so the oracle's rate is extrapolated per row
    sample = oracle_sample(rowptr, colidx, X, y, params, lr, m, L * nnz_loc * (m / n_loc),
                           f"extrapolated: one full 3-layer step on the first {m} of {n_loc} local rows, counted as "
                           "that share of the part's entries")
    return out, sample


# ----------------------------------------------------------------------------------------------- configs[4]
def run_aggregation(args):
    """configs[4]: model aggregation on one GPU (Alg. 1 and 2): Chung-Lu graph of 10 M nodes / 200 M edges, K = 8
    random partitions, 8 trainers time-sliced on 8 HIP streams, each full-batch 2-layer mean-SAGE (128-256-47, fp32),
    on-device parameter averaging every 50 local steps.  A "step" here is one local step of every trainer."""
    from . import synth, synth_torch as st
    from .aggregation import ModelAggregation
    from .trainer import LocalTrainer
    dev = torch.device("cuda:0")
    scale = args.scale
    N, K, every = int(10_000_000 * scale), 8, 50
    dims, C, lr, s, dt = [128, 256, 47], 47, 1e-3, 4, B.TMA_F32
    t0 = time.time()
    rowptr, colidx = st.chung_lu_graph(N, 40, 2.1, seed=41, device=dev)
    nnz_glob = int(rowptr[-1])
    g = torch.Generator(device=dev)
    g.manual_seed(42)
    X = torch.randn((N, dims[0]), generator=g, device=dev)
    g.manual_seed(43)
    y = torch.randint(0, C, (N,), generator=g, device=dev, dtype=torch.int32)
    params = synth.sage_params(dims, seed=45)
    part = B.tma_partition(N, K, 44)
    trainers, sizes = [], []
    t_ext = time.perf_counter()
    for p in range(K):
        sub = B.tma_induced_subgraph(rowptr, colidx, part, p)
        Xl, yl = B.tma_gather_rows(sub["l2g"], X), B.tma_gather_rows(sub["l2g"], y)
        trainers.append(LocalTrainer(sub["rowptr"], sub["colidx"], sub["inv_deg"], Xl, yl, dims, params=params,
                                     stream=torch.cuda.Stream()))
        sizes.append((sub["n_loc"], sub["nnz_loc"]))
    torch.cuda.synchronize()
    t_ext = time.perf_counter() - t_ext
    del X, rowptr, colidx
    _log(f"graph generated and 8 parts extracted in {time.time() - t0:.1f}s: nnz={nnz_glob}, parts {sizes}")
    L = len(dims) - 1
    edges_per_step = L * sum(z for _, z in sizes)
    agg = ModelAggregation(trainers)
    rounds = max(args.steps // every, 1)
    # warm-up
    agg.run_rounds(1, max(args.warmup, 1), lr)
    agg.synchronize()
    # kernel profile of one trainer alone (kernels of different streams overlap in the timed loop)
    tr0 = trainers[0]
    with torch.cuda.stream(tr0.stream):
        def solo():
            tr0.step(lr)
        lw = sage_layer_work(sizes[0][0], sizes[0][1], dims, s, dt)
        wbn = work_by_name(LayerWindows(tr0).run(solo), lw)
        B.tma_profile_begin(None)
        for _ in range(3):
            solo()
        tr0.stream.synchronize()
        prof = B.tma_profile_end()
    per_step = {k: v[1] / 3.0 for k, v in prof.items()}
    dominant = max(per_step, key=per_step.get)
    work_of = lambda k: wbn.get(k) or other_kernel_work(k, sizes[0][0], sizes[0][1], dims[0], C, s, K=K,
                                                        n_params=int(tr0.W.numel()))
    solo_ms = sum(per_step.values())
    # timed region: rounds x 50 local steps of all 8 trainers, phi after each round
    for t in trainers:
        t.steps_done = 0
    agg.history.clear()
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    agg.run_rounds(rounds, every, lr)
    agg.synchronize()
    elapsed = time.perf_counter() - t_start
    steps = rounds * every
    ms_per_step = elapsed * 1e3 / steps
    # the averaging call alone, event-timed on the aggregation stream
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(agg.agg_stream):
        e0.record()
        for _ in range(50):
            B.tma_average([t.W for t in trainers], W_global_out=agg.W_global, ptr_table=agg.ptr_table, stream=agg.agg_stream)
        e1.record()
    e1.synchronize()
    avg_us = e0.elapsed_time(e1) * 1e3 / 50
    # the dominant kernel alone, events on its launches, one trainer
    B.tma_profile_begin(dominant)
    with torch.cuda.stream(tr0.stream):
        for _ in range(10):
            tr0.step(lr)
        tr0.stream.synchronize()
    dom = B.tma_profile_end().get(dominant, (0, 0.0))
    traffic = load_traffic("configs4")
    # wall-clock mode: interval = 50 median steps, four intervals
    for t in trainers:
        t.steps_done = 0
    agg.history.clear()
    hist = agg.run_timed(dt_int=every * ms_per_step * 1e-3, dt_train=4.2 * every * ms_per_step * 1e-3, lr=lr)
    agg.synchronize()
    out = {
        "metric": "trainer edges/sec per SAGE layer fwd+bwd; achieved HBM GB/s vs peak",
        "value": round(edges_per_step / (ms_per_step * 1e-3), 1), "unit": "edges/s", "n_gpus": 1, "steps": steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"configs[4]: model aggregation on one GPU: Chung-Lu power-law graph (gamma 2.1), {N} nodes, "
                               f"{nnz_glob // 2} undirected edges, 128-d fp32 features, 47 classes; K=8 random node partitions, "
                               "8 trainers on 8 HIP streams, each full-batch 2-layer mean-SAGE (hidden 256); on-device parameter "
                               f"averaging every {every} local steps; a step = one local step of all 8 trainers "
                               "(extraction is done once, before the loop)"
                               + ("" if scale == 1.0 else f" [scaled to {scale:g} of the configured size]"),
                   "n_nodes": N, "nnz_global": nnz_glob, "K": K, "parts": [{"n_loc": a, "nnz_loc": b} for a, b in sizes],
                   "layers": L, "dims": dims, "rounds": rounds, "steps_per_round": every,
                   "edge_definition": "directed local CSR entry; value = layers * sum of nnz_loc over the 8 trainers / step time"},
        "roofline": dominant_roofline(dominant, dom, work_of, PEAK_MFMA_F32_TFLOPS, traffic),
        "kernel_rooflines": rooflines(per_step, prof, 3, work_of, PEAK_MFMA_F32_TFLOPS, traffic),
        "kernel_ms_per_step": {k: round(v, 5) for k, v in sorted(per_step.items(), key=lambda kv: -kv[1])},
        "aggregation": {"steps_per_trainer": [t_.steps_done for t_ in trainers], "history_step_count_trigger": [[every * (r + 1)] * K for r in range(rounds)],
                        "average_call_us": round(avg_us, 2), "n_params": int(tr0.W.numel()),
                        "one_trainer_alone_ms_per_step": round(solo_ms, 4),
                        "time_slicing_speedup_vs_serial": round(K * solo_ms / ms_per_step, 3),
                        "extraction_of_8_parts_with_row_gathers_s": round(t_ext, 3),
                        "timed_mode": {"dt_int_ms": round(every * ms_per_step, 2), "rounds": len(hist),
                                       "steps_at_each_round": hist}},
        "final_loss": float(trainers[0].loss.item()), "streams": K,
    }
    m = min(300_000, sizes[0][0])       # about 11 s of single-threaded oracle work
    sample = oracle_sample(tr0.rowptr, tr0.colidx, tr0.X, tr0.labels, params, lr, m, L * sizes[0][1] * (m / sizes[0][0]),
                           f"extrapolated: one trainer's full step on the first {m} of its {sizes[0][0]} local rows, "
                           "counted as that share of its entries")
    return out, sample


# ------------------------------------------------------------------------- HBM traffic from rocprofv3 counter runs
def _counter_rows(directory, counter):
    """[(dispatch id, kernel symbol, value)] of one counter from a rocprofv3 --pmc run's CSV, in dispatch order."""
    import csv
    import glob
    files = glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise SystemExit(f"no *counter_collection.csv under {directory}")
    rows = []
    with open(files[0]) as f:
        for r in csv.DictReader(f):
            if r["Counter_Name"] == counter:
                rows.append((int(r["Dispatch_Id"]), r["Kernel_Name"], float(r["Counter_Value"])))
    rows.sort()
    return rows


def _per_timer_name(rows, sequence, first_symbol="partition_kernel"):
    """Matches the library's launches of the profiled run against the step's launch sequence (the library's timer
    names in launch order): the dispatches of library kernels between two launches of the step's first kernel are
    one step.  Returns {timer name: (mean counter value, kernel symbol, launches averaged)}."""
    lib_rows = [r for r in rows if "tma::" in r[1]]
    starts = [i for i, r in enumerate(lib_rows) if first_symbol in r[1]]
    acc = {}
    used = 0
    for a, b in zip(starts, starts[1:] + [len(lib_rows)]):
        step = lib_rows[a:b]
        if len(step) != len(sequence):
            continue
        used += 1
        for name, (_, symbol, value) in zip(sequence, step):
            s, c, sym = acc.get(name, (0.0, 0, symbol))
            if sym != symbol:
                raise SystemExit(f"timer {name} maps to two kernels: {sym[:80]} / {symbol[:80]}")
            acc[name] = (s + value, c + 1, sym)
    if not used:
        raise SystemExit(f"no step of {len(sequence)} library launches found in the counter run "
                         f"({len(starts)} candidate steps of lengths {sorted({b - a for a, b in zip(starts, starts[1:])})})")
    return {k: (s / c, sym, c) for k, (s, c, sym) in acc.items()}


def summarize_traffic(config_key, fetch_dir, write_dir, bench_json, command, calib_fetch_dir=None, calib_write_dir=None):
    """Writes profiles/hbm_traffic.json (read back by bench.py for `roofline.traffic`) and the text summary
    profiles/<config_key>_hbm_traffic.txt from two rocprofv3 --pmc runs of bench.py (FETCH_SIZE, then WRITE_SIZE)."""
    with open(bench_json) as f:
        bench = json.loads([l for l in f.read().splitlines() if l.startswith("{")][-1])
    sequence = bench["kernel_sequence"]
    try:
        with open(TRAFFIC_FILE) as f:
            table = json.load(f)
    except (OSError, ValueError):
        table = {}
    cal = table.get("calibration", {"fetch_factor": 2.0, "write_factor": 1.0,
                                    "what": "FETCH_SIZE / WRITE_SIZE of a plain 1 GiB device copy (bench.py --calibrate-copy)"})
    if calib_fetch_dir and calib_write_dir:
        cf = max(v for _, k, v in _counter_rows(calib_fetch_dir, "FETCH_SIZE") if "copyBuffer" in k)
        cw = max(v for _, k, v in _counter_rows(calib_write_dir, "WRITE_SIZE") if "copyBuffer" in k)
        cal = {"fetch_factor": round(1048576.0 / cf, 2), "write_factor": round(1048576.0 / cw, 2),
               "fetch_kib_per_gib_copy": cf, "write_kib_per_gib_copy": cw,
               "what": "FETCH_SIZE / WRITE_SIZE of a plain 1 GiB device copy (bench.py --calibrate-copy): 1,048,576 KiB read and written"}
    table["calibration"] = cal
    fe = _per_timer_name(_counter_rows(fetch_dir, "FETCH_SIZE"), sequence)
    wr = _per_timer_name(_counter_rows(write_dir, "WRITE_SIZE"), sequence)
    kernels = {}
    for name in fe:
        f_kib, sym, cnt = fe[name]
        w_kib = wr.get(name, (0.0, sym, 0))[0]
        kernels[name] = {"fetch_kib": round(f_kib, 1), "write_kib": round(w_kib, 1),
                         "bytes": round((f_kib * cal["fetch_factor"] + w_kib * cal["write_factor"]) * 1024), "symbol": sym[:160],
                         "launches_averaged": cnt}
    table[config_key] = {"command": command, "workload": bench["config"]["workload"][:200], "kernels": kernels}
    os.makedirs(os.path.dirname(TRAFFIC_FILE), exist_ok=True)
    with open(TRAFFIC_FILE, "w") as f:
        json.dump(table, f, indent=1, sort_keys=True)
    rl = bench.get("kernel_rooflines", {})
    with open(os.path.join(ROOT, "profiles", f"bench_{config_key}_hbm_traffic.txt"), "w") as f:
        f.write(f"HBM traffic per kernel launch, {bench['config']['workload'][:160]}...\n\n")
        f.write("commands (MI355X box, repo root, after `cd /tmp && export TMPDIR=/tmp`), one counter per run:\n")
        f.write(f"  rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d <fetch_dir> -o b -- python3 {command}\n")
        f.write(f"  rocprofv3 --pmc WRITE_SIZE --kernel-trace --output-format csv -d <write_dir> -o b -- python3 {command}\n")
        f.write(f"  python3 bench.py --summarize-traffic {config_key} <fetch_dir> <write_dir> <json line of that command>\n")
        f.write(f"calibration: {cal['what']}: FETCH_SIZE factor {cal['fetch_factor']}, WRITE_SIZE factor {cal['write_factor']}\n")
        f.write("scaled_MB = (FETCH_KiB * fetch factor + WRITE_KiB * write factor) * 1024 / 1e6; algorithmic_MB = bench.py's work model "
                "(each distinct input row once); launches are matched to the library's kernel names through the launch order of a step\n\n")
        f.write("%-28s %-11s %-11s %-10s %-14s %-7s kernel symbol\n" % ("name", "FETCH_KiB", "WRITE_KiB", "scaled_MB", "algorithmic_MB", "ratio"))
        for name, k in sorted(kernels.items(), key=lambda kv: -kv[1]["bytes"]):
            r = rl.get(name)
            alg = None
            if r and r["bound"] == "hbm":
                alg = r["achieved"] * 1e9 * r.get("us_per_launch", 0) * 1e-6 if "us_per_launch" in r else None
            if r and r["bound"] == "hbm" and alg is None and bench.get("kernel_ms_per_step", {}).get(name):
                alg = r["achieved"] * 1e9 * bench["kernel_ms_per_step"][name] * 1e-3
            f.write("%-28s %-11.0f %-11.0f %-10.1f %-14s %-7s %s\n" % (
                name, k["fetch_kib"], k["write_kib"], k["bytes"] / 1e6, ("%.1f" % (alg / 1e6)) if alg else "-",
                ("%.2f" % (k["bytes"] / alg)) if alg else "-", k["symbol"][:110]))
    return table[config_key]


def summarize_kernel_stats(config_key, stats_dir, bench_json, command):
    """Writes profiles/bench_<config_key>_kernel_stats.txt from a `rocprofv3 --kernel-trace --stats --output-format csv`
    run of bench.py and the JSON line that run printed."""
    import csv
    import glob
    files = glob.glob(os.path.join(stats_dir, "**", "*kernel_stats.csv"), recursive=True)
    if not files:
        raise SystemExit(f"no *kernel_stats.csv under {stats_dir}")
    with open(bench_json) as f:
        bench = json.loads([l for l in f.read().splitlines() if l.startswith("{")][-1])
    rows = []
    with open(files[0]) as f:
        for r in csv.DictReader(f):
            rows.append((r["Name"], int(r["Calls"]), float(r["TotalDurationNs"]) / 1e3, float(r["AverageNs"]) / 1e3,
                         float(r["Percentage"])))
    rows.sort(key=lambda r: -r[2])
    dom = bench["roofline"]
    out = os.path.join(ROOT, "profiles", f"bench_{config_key}_kernel_stats.txt")
    with open(out, "w") as f:
        f.write(f"Kernel time per launch, {bench['config']['workload'][:220]}...\n\n")
        f.write("command (MI355X box, repo root, after `cd /tmp && export TMPDIR=/tmp`):\n")
        f.write(f"  rocprofv3 --kernel-trace --stats --output-format csv -d <dir> -o b -- python3 {command}\n")
        f.write(f"  python3 bench.py --summarize-kernel-stats {config_key} <dir> <json line of that command>\n")
        f.write(f"(the run: {bench['warmup']} warm-up steps, 3 + 2 + 1 steps of the event-profile passes, {bench['steps']} timed steps)\n\n")
        f.write("%-8s %-12s %-10s %-7s kernel\n" % ("calls", "total_us", "avg_us", "pct"))
        others = [0, 0.0, 0.0]
        for name, calls, total, avg, pct in rows:
            if "tma::" not in name:        # the input generators' and the framework's own kernels: one line below
                others = [others[0] + calls, others[1] + total, others[2] + pct]
                continue
            if pct < 0.05 and len(rows) > 60:
                continue
            f.write("%-8d %-12.1f %-10.2f %-7.2f %s\n" % (calls, total, avg, pct, name.replace("void ", "")[:150]))
        if others[0]:
            f.write("%-8d %-12.1f %-10s %-7.2f (kernels outside the library: drawing the synthetic inputs, copies, fills)\n"
                    % (others[0], others[1], "-", others[2]))
        f.write(f"\nbench.py (the same run, under the profiler): {bench['ms_per_step'] * 1e3:.1f} us per step, value {bench['value']:.4g} {bench['unit']}\n")
        f.write(f"dominant kernel {dom['kernel']}: bench.py's HIP events give {dom['avg_launch_ms'] * 1e3:.1f} us per launch -> "
                f"{dom['achieved']} {dom['unit']} = {dom['frac'] * 100:.1f} % of {dom['peak']} ({dom['bound']} bound)\n\n")
        f.write("per-kernel rates from the event-timed pass of the same run (algorithmic work / time):\n")
        for k, v in bench["kernel_ms_per_step"].items():
            r = bench["kernel_rooflines"].get(k)
            if r:
                also = ("; operands + results %.0f GB/s = %.1f %% of the HBM peak" % (r["streamed_GBs"], r["hbm_frac"] * 100)
                        if "hbm_frac" in r else "")
                f.write("  %-34s %9.1f us/step  %9.1f %s  (%.1f %% of %s%s)\n" % (k, v * 1e3, r["achieved"], r["unit"], r["frac"] * 100, r["peak"], also))
            else:
                f.write("  %-34s %9.1f us/step\n" % (k, v * 1e3))
        for extra in ("aggregation", "cpu_baseline", "per_layer_fwd_bwd", "two_stream"):
            if bench.get(extra):
                f.write(f"\n{extra}: {json.dumps(bench[extra])}\n")
    return out


def summarize_counters(key, directory, command, title):
    """Writes profiles/bench_<key>.txt: the mean over the launches of every library kernel of each counter that a
    `rocprofv3 --pmc ... --kernel-trace --output-format csv` run of bench.py collected, with a few derived ratios
    where their counters are there."""
    import csv
    import glob
    files = glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise SystemExit(f"no *counter_collection.csv under {directory}")
    acc, counters = {}, []
    with open(files[0]) as f:
        for r in csv.DictReader(f):
            if "tma::" not in r["Kernel_Name"]:
                continue
            c = r["Counter_Name"]
            if c not in counters:
                counters.append(c)
            a = acc.setdefault(r["Kernel_Name"], {}).setdefault(c, [0.0, 0])
            a[0] += float(r["Counter_Value"])
            a[1] += 1
    mean = {k: {c: v[0] / v[1] for c, v in d.items()} for k, d in acc.items()}
    launches = {k: max(v[1] for v in d.values()) for k, d in acc.items()}
    derived = []
    if {"SQ_INSTS_VALU", "SQ_INSTS_MFMA"} <= set(counters):
        derived.append(("valu/mfma", lambda m: (m["SQ_INSTS_VALU"] - m["SQ_INSTS_MFMA"]) / m["SQ_INSTS_MFMA"] if m.get("SQ_INSTS_MFMA") else None))
    if {"SQ_INSTS_LDS", "SQ_INSTS_MFMA"} <= set(counters):
        derived.append(("lds/mfma", lambda m: m["SQ_INSTS_LDS"] / m["SQ_INSTS_MFMA"] if m.get("SQ_INSTS_MFMA") else None))
    if {"TCP_TCC_READ_REQ_LATENCY_sum", "TCP_TCC_READ_REQ_sum"} <= set(counters):
        derived.append(("read_latency_cycles", lambda m: m["TCP_TCC_READ_REQ_LATENCY_sum"] / m["TCP_TCC_READ_REQ_sum"] if m.get("TCP_TCC_READ_REQ_sum") else None))
    if {"TCC_HIT_sum", "TCC_MISS_sum"} <= set(counters):
        derived.append(("L2_hit_share", lambda m: m["TCC_HIT_sum"] / (m["TCC_HIT_sum"] + m["TCC_MISS_sum"]) if m.get("TCC_HIT_sum", 0) + m.get("TCC_MISS_sum", 0) else None))
    order = sorted(mean, key=lambda k: -mean[k].get(counters[0], 0.0))
    out = os.path.join(ROOT, "profiles", f"bench_{key}.txt")
    with open(out, "w") as f:
        f.write(title + "\n\ncommand (MI355X box, repo root, after `cd /tmp && export TMPDIR=/tmp`):\n")
        f.write(f"  rocprofv3 --pmc {' '.join(counters)} --kernel-trace --output-format csv -d <dir> -o b -- python3 {command}\n")
        f.write(f"  python3 bench.py --summarize-counters {key} <dir>\n")
        f.write("Means over the launches of each library kernel (a name launched with several shapes is averaged over them).\n\n")
        cols = counters + [d[0] for d in derived]
        f.write("launches " + " ".join("%-14s" % c[:14] for c in cols) + " kernel\n")
        for k in order:
            m = mean[k]
            vals = [m.get(c) for c in counters] + [fn(m) for _, fn in derived]
            f.write("%-8d " % launches[k] + " ".join("%-14s" % ("-" if v is None else ("%.4g" % v)) for v in vals)
                    + " " + k.replace("void ", "")[:140] + "\n")
    return out
