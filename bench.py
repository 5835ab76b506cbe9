#!/usr/bin/env python3
"""Benchmark of the GNN-layer hot path (aggregation + Update) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5] [--verify]

A step is one forward pass of every layer of a workload with all inputs already resident in HBM.
The timed region holds exactly K steps between two device synchronisations.  With no --config the
workload is config 4 (the dense power-law graph at dim 602: the largest work of the five on one GPU),
and configs 5, 2 and 3 are timed after it and reported under "other_configs" of the same line.

One JSON line is printed: whole-step throughput in GEdges/s, the roofline figures of the dominant
kernel (the aggregation kernel) from HIP events recorded on the launch stream inside the timed
region, and the CPU oracle timed on the host cores as a baseline.  The roofline object carries three
byte counts side by side: bytes measured with rocprofv3 counters where the L2 hands requests to the
memory fabric (`achieved`, `frac`: the fraction of the 8 TB/s HBM peak; read from
profiles/measured_traffic.json, which records the commit it was measured at), the gather-model
bytes (every neighbour row counted once per edge; above the HBM peak where caches serve repeats, and
then labelled as a cache-bandwidth figure), and the compulsory bytes of a perfect cache.

One GPU only: collectives and sharding are not part of this build.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak

HEADLINE_CONFIG = 4            # timed when no --config is given; the others follow under "other_configs"
OTHER_CONFIGS = (5, 2, 3)
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "measured_traffic.json")


BUILD_KNOBS = {}          # --build-knob KEY=VALUE: knobs of mgg_build_partition for the timed run
NON_DEFAULT_RUN = False   # set by --option / --build-knob: the record of measured traffic does not describe such a run


def measured_traffic(workload: str, layer: int):
    """Bytes per aggregation launch that crossed from L2 to the memory fabric, from rocprofv3 --pmc runs
    (read and write requests destined for DRAM, 32-byte units, scaled by what the same counters read for
    a 1 GiB copy), as recorded in profiles/measured_traffic.json together with the commit the kernels
    were at.  None when that workload and layer were not measured, or when the run changes the library's
    defaults (the record was taken with them)."""
    if NON_DEFAULT_RUN:
        return None
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f)
        e = rec["workloads"][workload][f"layer{layer}"]
        return {"bytes": int(e["bytes"]), "commit": rec.get("commit"), "profile": e.get("profile")}
    except (OSError, KeyError, ValueError, TypeError):
        return None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def to_dev(a, dev, pad_rows_to_bytes=0):
    """Host array -> device tensor.  With pad_rows_to_bytes the rows are laid out with a leading
    dimension rounded up so that every row starts on that byte boundary (the API takes ld_x)."""
    import torch
    if a.dtype == np.uint16:
        t = torch.from_numpy(a.view(np.int16).copy()).to(dev).view(torch.bfloat16)
    else:
        t = torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    if pad_rows_to_bytes and t.dim() == 2:
        per = pad_rows_to_bytes // t.element_size()
        ld = (t.shape[1] + per - 1) // per * per
        if ld != t.shape[1]:
            buf = torch.zeros((t.shape[0], ld), dtype=t.dtype, device=dev)
            buf[:, :t.shape[1]].copy_(t)
            return buf[:, :t.shape[1]]
    return t


def gather_model_bytes(nnz, n_own, dim, elem_bytes, gcn, out_bytes=4):
    """Algorithmic bytes of one aggregation launch: per neighbour one embedding row, its 4-byte
    id and (GCN) the 4-byte normalisation factor of the neighbour; per owned row its own
    embedding, the output row (fp32, or bf16 ahead of a bf16 MFMA), two row-pointer entries and its
    normalisation factor."""
    per_edge = dim * elem_bytes + 4 + (4 if gcn else 0)
    per_row = dim * elem_bytes + dim * out_bytes + 12
    return nnz * per_edge + n_own * per_row


def compulsory_bytes(nnz, n_own, num_halo, dim, elem_bytes, gcn, out_bytes=4):
    """Bytes a perfect cache would still have to move: every table row once (the owned rows are read
    at least for their own term), the ids (and GCN factors) once, the output rows once."""
    return (n_own + num_halo) * dim * elem_bytes + nnz * (4 + (4 if gcn else 0)) + n_own * (dim * out_bytes + 12)


def cpu_baseline_leg(w, layer, x_local_np, x_halo_np, halo_gid, n_own, cpu_budget_s):
    """The oracle as it stands (never tuned for this), timed on the host cores on a bounded
    sample of the same workload: layer 0, aggregate + update, on a random subset of owned rows."""
    import oracle
    deg_share = (np.diff(w.row_ptr)[w.lb:w.ub]).astype(np.int64)
    work = deg_share * w.dim
    # about 1.2e9 multiply-adds per second and thread (measured on the box's EPYC cores)
    budget = cpu_budget_s * 1.2e9 * max(1, oracle.num_threads())
    rows = np.arange(n_own)
    if work.sum() > budget:
        rng = np.random.default_rng(1)
        perm = rng.permutation(n_own)
        take = int(np.searchsorted(np.cumsum(work[perm]), budget)) + 1
        rows = np.sort(perm[:take])
    sample_edges = int(deg_share[rows].sum())
    t0 = time.perf_counter()
    h = oracle.aggregate(w.row_ptr, w.col, layer.mode, x_local_np, lb=w.lb, ub=w.ub, x_halo=x_halo_np,
                         halo_gid=halo_gid, eps=layer.eps, rows=rows)
    for i, m in enumerate(layer.weights):
        h = oracle.update(h, m, None, layer.acts[i])
    cpu_s = time.perf_counter() - t0
    cpu_model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            cpu_model = next((ln.split(":", 1)[1].strip() for ln in f if ln.startswith("model name")), cpu_model)
    except OSError:
        pass
    return {"value": round(sample_edges / cpu_s / 1e9, 5), "unit": "GEdges/s", "cores": oracle.num_threads(),
            "kind": "oracle", "cpu": cpu_model,
            "sample": f"layer 0 (aggregate + update) on {rows.size} of {n_own} owned rows, "
                      f"{sample_edges} edges, {cpu_s:.1f}s"}


ABLATIONS = [
    # name, build options, run-time options -- one-GPU counterparts of the paper's kernel ablations
    ("default", {}, {}),
    ("no neighbour partitioning (a whole row per wavefront, section 7.2 'NP')", {"ps": 64, "dist": 1024, "xcd_min_deg": -1}, {}),
    ("no interleaving (local and remote lists in two launches, section 7.2 'WI')", {}, {"split_phases": 1}),
    ("no XCD-aware schedule", {"xcd_min_deg": -1}, {}),
    ("source classes by hash (8 classes, one per XCD)", {"hot_phases": -1}, {}),
    ("no short-row bin", {"short_max": -1}, {}),
    ("halo rows staged through LDS, two stages per wavefront (section 5.2)", {}, {"lds_halo": 1}),
    ("one work item per wavefront (no pipelining across items)", {}, {"items_per_wave": 1}),
    ("no column slabs", {}, {"col_slab_bytes": 1}),
    ("source classes by popularity, 4 hot phases per XCD", {"hot_phases": 4}, {}),
]


def run_ablations(cfg: int, iters: int = 20):
    """Aggregation time of layer 0 under each variant; returns a list of dicts."""
    import torch
    from paper_2209_06800_amd import binding, inputs
    dev = "cuda:0"
    w = inputs.config(cfg)
    layer = w.layers[0]
    esz = 2 if w.dtype == "bf16" else 4
    pad = 128 if (w.dim * esz) % 16 else 0
    rows = []
    base_ms = None
    for name, build, opts in ABLATIONS:
        part = binding.mgg_build_partition(w.row_ptr, w.col, w.parts, w.part_id, w.bounds, **build)
        hg = part.export()["halo_gid"]
        xl = to_dev(w.x[w.lb:w.ub], dev, pad)
        xh = to_dev(w.x[hg], dev, pad) if hg.size else None
        out = torch.empty((int(part.info.n_own), w.dim), dtype=torch.float32, device=dev)
        for k, v in opts.items():
            part.set_option(k, v)
        ms = min(binding.mgg_time_aggregate(part, layer.mode, xl, xh, out, eps=layer.eps, iters=iters) for _ in range(3))
        nnz = int(part.info.nnz_local + part.info.nnz_remote)
        base_ms = ms if base_ms is None else base_ms
        rows.append({"variant": name, "agg_ms": round(ms, 4), "gedges_per_s": round(nnz / ms / 1e6, 3),
                     "slowdown_vs_default": round(ms / base_ms, 3)})
        log(f"[ablation] {name}: {ms:.4f} ms  {nnz / ms / 1e6:.2f} GEdges/s  x{ms / base_ms:.3f}")
        part.destroy()
        del xl, xh, out
    return rows


def run_tuner(cfg: int, exhaustive: bool, iters: int = 10):
    """The greedy search of section 6 (ps, dist, wpb) on layer 0's aggregation, driven with
    measured latencies; with `exhaustive` the whole 6 x 5 x 5 grid is measured as well."""
    import itertools
    import torch
    from paper_2209_06800_amd import binding, inputs
    dev = "cuda:0"
    w = inputs.config(cfg)
    layer = w.layers[0]
    esz = 2 if w.dtype == "bf16" else 4
    pad = 128 if (w.dim * esz) % 16 else 0
    part = binding.mgg_build_partition(w.row_ptr, w.col, w.parts, w.part_id, w.bounds)
    info = part.info
    hg = part.export()["halo_gid"]
    xl = to_dev(w.x[w.lb:w.ub], dev, pad)
    xh = to_dev(w.x[hg], dev, pad) if hg.size else None
    out = torch.empty((int(info.n_own), w.dim), dtype=torch.float32, device=dev)
    default_ms = binding.mgg_time_aggregate(part, layer.mode, xl, xh, out, eps=layer.eps, iters=iters)
    default = (int(info.ps), int(info.dist), int(info.wpb))
    part.destroy()
    # the paper's ranges, with ps up to the 64 lanes of a wavefront instead of the 32 of a warp
    tuner = binding.Tuner(64, 16, 16)
    t0 = time.time()
    best, best_ms = binding.mgg_tune_aggregate(w.row_ptr, w.col, w.parts, w.part_id, w.bounds, layer.mode, xl, xh, out,
                                               tuner, eps=layer.eps, iters=iters)
    table = tuner.table()
    res = {"workload": w.name, "default_knobs": default, "default_ms": round(default_ms, 4),
           "search": {"trials": len(table), "best_knobs": best, "best_ms": round(best_ms, 4),
                      "first_trial_ms": round(table[0][1], 4), "seconds": round(time.time() - t0, 1),
                      "table": [[list(k), round(ms, 4)] for k, ms in table]}}
    for k, ms in table:
        log(f"[tune] trial ps={k[0]:2d} dist={k[1]:2d} wpb={k[2]:2d}: {ms:.4f} ms")
    log(f"[tune] best {best}: {best_ms:.4f} ms after {len(table)} trials (default {default}: {default_ms:.4f} ms)")
    if exhaustive:
        grid = {}
        for ps, dist, wpb in itertools.product([1, 2, 4, 8, 16, 32, 64], [1, 2, 4, 8, 16], [1, 2, 4, 8, 16]):
            try:
                p2 = binding.mgg_build_partition(w.row_ptr, w.col, w.parts, w.part_id, w.bounds, ps=ps, dist=dist, wpb=wpb)
                grid[(ps, dist, wpb)] = binding.mgg_time_aggregate(p2, layer.mode, xl, xh, out, eps=layer.eps, iters=iters)
                p2.destroy()
            except binding.MggError as e:
                if e.status != binding.ERR_ALLOC:
                    raise
                grid[(ps, dist, wpb)] = float("inf")
            log(f"[tune] grid ps={ps:2d} dist={dist:2d} wpb={wpb:2d}: {grid[(ps, dist, wpb)]:.4f} ms")
        gbest = min(grid, key=grid.get)
        res["exhaustive"] = {"configs": len(grid), "best_knobs": gbest, "best_ms": round(grid[gbest], 4),
                             "search_best_over_grid_best": round(best_ms / grid[gbest], 4),
                             "table": [[list(k), round(v, 4)] for k, v in grid.items()]}
        log(f"[tune] grid best {gbest}: {grid[gbest]:.4f} ms; greedy / grid = {best_ms / grid[gbest]:.3f}")
    return res


def calibrate_gather(dims=(64, 100, 256), n_halo: int = 1 << 22, per_row: int = 32, launches: int = 2):
    """Launches the aggregation kernel on two graphs whose cache behaviour is known by construction.

    cold: part 0 of 2 owns n_halo / per_row rows, each with per_row neighbours that together form
    one random permutation of the n_halo rows of part 1.  Every halo row (>= 1 GiB in total, far
    beyond L2 and the Infinity Cache) is gathered exactly once per launch: all gathers miss, the
    L2-miss bytes are known, and a counter run (rocprofv3 --pmc FETCH_SIZE) can be scaled for
    gather traffic, not only for streaming.

    hot: the same number of gathers, but drawn from 4096 halo rows only (at most 4 MB, resident in
    every XCD's L2): all gathers hit.  The two rates bracket what any schedule can reach."""
    import torch
    from paper_2209_06800_amd import binding
    dev = "cuda:0"
    n_dst = n_halo // per_row
    rng = np.random.default_rng(5)
    out_lines = []
    for kind in ("cold", "hot"):
        n_src = n_halo if kind == "cold" else 4096
        row_ptr = np.zeros(n_dst + n_src + 1, dtype=np.int64)
        row_ptr[1:n_dst + 1] = per_row * np.arange(1, n_dst + 1)
        row_ptr[n_dst + 1:] = row_ptr[n_dst]
        if kind == "cold":
            src = rng.permutation(n_halo).reshape(n_dst, per_row)
        else:
            src = rng.integers(0, n_src, size=(n_dst, per_row))
        col = (n_dst + np.sort(src, axis=1).ravel()).astype(np.int32)
        part = binding.mgg_build_partition(row_ptr, col, 2, 0, [0, n_dst, n_dst + n_src], xcd_min_deg=-1)
        for dim in dims:
            xl = torch.empty((n_dst, dim), dtype=torch.float32, device=dev).normal_()
            xh = torch.empty((n_src, dim), dtype=torch.float32, device=dev).normal_()
            out = torch.empty((n_dst, dim), dtype=torch.float32, device=dev)
            ms = binding.mgg_time_aggregate(part, "gin", xl, xh, out, iters=launches)
            gathered = n_halo * dim * 4
            expect = (n_halo if kind == "cold" else n_src) * dim * 4 + n_halo * 4 + n_dst * (dim * 4 + 12)
            out_lines.append({"kind": kind, "dim": dim, "row_bytes": dim * 4, "gathers": n_halo, "table_rows": n_src,
                              "expected_fetch_bytes": expect, "ms": round(ms, 4),
                              "gathered_gbs": round(gathered / ms / 1e6, 1)})
            log(f"[calibrate-gather] {kind} dim {dim}: {n_halo} gathers of {dim * 4} B from {n_src} table rows; "
                f"expected L2-miss reads {expect} B per launch; {ms:.4f} ms = {gathered / ms / 1e6:.0f} GB/s gathered")
            del xl, xh, out
        part.destroy()
    return out_lines


def probe_gather():
    """The rate at which the memory hierarchy delivers gathered rows to the CUs, by where the rows live:
    random rows of 256 bytes and of 1 KB from tables between 1 MB (inside one XCD's L2) and 2 GB (HBM)."""
    from paper_2209_06800_amd import binding
    rows = []
    for row_bytes in (256, 1024):
        for mb in (1, 2, 3, 4, 5, 6, 7, 8, 12, 16, 32, 64, 256, 2048):
            gbs = binding.mgg_probe_gather(mb << 20, row_bytes)
            rows.append({"row_bytes": row_bytes, "table_mb": mb, "gathered_gbs": round(gbs, 1)})
            log(f"[probe-gather] rows of {row_bytes} B from a {mb} MB table: {gbs / 1e3:.2f} TB/s")
    return rows


def run_orders(cfg: int, iters: int = 20):
    """Whole-layer time (mgg_layer_forward, HIP events on the launch stream) with the aggregation
    first -- the paper's formulation -- and with the first matrix product first, which gathers
    rows of the output width instead of the input width."""
    import torch
    from paper_2209_06800_amd import binding, inputs
    dev = "cuda:0"
    w = inputs.config(cfg)
    part = binding.mgg_build_partition(w.row_ptr, w.col, w.parts, w.part_id, w.bounds)
    info = part.info
    hg = part.export()["halo_gid"]
    nnz = int(info.nnz_local + info.nnz_remote)
    esz = 2 if w.dtype == "bf16" else 4
    rows = []
    xl = xh = None
    for li, layer in enumerate(w.layers):
        d_in = layer.dims[0]
        if li == 0:
            pad = 128 if (d_in * esz) % 16 else 0
            xl, xh = to_dev(w.x[w.lb:w.ub], dev, pad), (to_dev(w.x[hg], dev, pad) if hg.size else None)
        else:
            xl = out_prev
            xh = to_dev(inputs.layer2_halo_table(w.notes["layer2_halo_seed"], int(info.num_halo), d_in), dev)
        ws = [to_dev(m, dev) for m in layer.weights]
        res = {"layer": li, "dims": layer.dims}
        for order in ("agg_first", "update_first"):
            need = binding.mgg_layer_workspace_bytes(part, layer.mode, ws, layer.acts, eps=layer.eps, order=order)
            wsp = torch.empty(need, dtype=torch.uint8, device=dev)
            out = torch.empty((int(info.n_own), layer.dims[-1]), dtype=torch.float32, device=dev)
            for _ in range(3):
                binding.mgg_layer_forward(part, layer.mode, xl, xh, ws, layer.acts, eps=layer.eps, workspace=wsp, out=out, order=order)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(iters):
                binding.mgg_layer_forward(part, layer.mode, xl, xh, ws, layer.acts, eps=layer.eps, workspace=wsp, out=out, order=order)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / iters
            res[order + "_ms"] = round(ms, 4)
            res[order + "_gedges_per_s"] = round(nnz / ms / 1e6, 3)
            if order == "agg_first":
                out_prev = out
            del wsp
        res["speedup"] = round(res["agg_first_ms"] / res["update_first_ms"], 3)
        log(f"[orders] layer {li} {layer.dims}: aggregate first {res['agg_first_ms']} ms, update first {res['update_first_ms']} ms "
            f"(x{res['speedup']}; includes transforming the {int(info.num_halo)} halo rows on this GPU)")
        rows.append(res)
    part.destroy()
    return {"workload": w.name, "edges": nnz, "n_own": int(info.n_own), "num_halo": int(info.num_halo), "layers": rows}


UPDATE_SHAPES = [
    # name, rows, d_in, d_out, dtype of A, dtype of W, dtype of out -- the Update calls of the five configs
    ("cfg2 64->64", 262144, 64, 64, "f32", "f32", "f32"),
    ("cfg3 128->128 (linear 1)", 524288, 128, 128, "f32", "bf16", "bf16"),
    ("cfg3 128->128 (linear 2)", 524288, 128, 128, "bf16", "bf16", "f32"),
    ("cfg4 602->256", 232965, 602, 256, "f32", "f32", "f32"),
    ("cfg5 100->256", 306128, 100, 256, "f32", "f32", "f32"),
    ("cfg5 256->47", 306128, 256, 47, "f32", "f32", "f32"),
    ("cfg5 256->47, halo rows", 1771062, 256, 47, "f32", "f32", "f32"),
]


def run_update_shapes(iters: int = 20, vendor: bool = True):
    """mgg_update alone on the Update shapes of the configs (ReLU fused), HIP events on the launch
    stream; torch.matmul -- the vendor GEMM, no epilogue, one dtype for input and output -- beside it."""
    import torch
    from paper_2209_06800_amd import binding
    dev = "cuda:0"
    tdt = {"f32": torch.float32, "bf16": torch.bfloat16}
    rows = []
    for name, n, k, m, adt, wdt, odt in UPDATE_SHAPES:
        a = torch.randn(n, (k + 7) // 8 * 8, device=dev).to(tdt[adt])[:, :k]     # rows start on 16-byte boundaries
        w = (torch.randn(k, m, device=dev) * 0.1).to(tdt[wdt])
        out = torch.empty(n, m, device=dev, dtype=tdt[odt])

        def timed(fn):
            for _ in range(3):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(iters):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / iters

        ms = timed(lambda: binding.mgg_update(a, w, None, "relu", out=out))
        byts = n * k * a.element_size() + n * m * out.element_size() + k * m * w.element_size()
        r = {"shape": name, "rows": n, "d_in": k, "d_out": m, "dtypes": f"{adt}/{wdt}/{odt}", "us": round(ms * 1e3, 1),
             "tflops": round(2.0 * n * k * m / ms / 1e9, 1), "gbs": round(byts / ms / 1e6)}
        if vendor:
            av, wv = a.to(tdt[wdt]).contiguous(), w
            ov = torch.empty(n, m, device=dev, dtype=tdt[wdt])
            r["vendor_us"] = round(timed(lambda: torch.matmul(av, wv, out=ov)) * 1e3, 1)
        rows.append(r)
        log(f"[update] {name}: {r['us']} us, {r['tflops']} TFLOP/s, {r['gbs']} GB/s" + (f" (vendor GEMM {r['vendor_us']} us)" if vendor else ""))
        del a, w, out
    # config 3's MLP as one call: both products in one kernel, hidden activations kept on chip
    n, k = 524288, 128
    a = torch.randn(n, k, device=dev)
    w1, w2 = [(torch.randn(k, k, device=dev) * 0.1).bfloat16() for _ in range(2)]
    out = torch.empty(n, k, device=dev)
    for _ in range(3):
        binding.mgg_update_mlp(a, w1, w2, ("relu", "none"), out=out)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        binding.mgg_update_mlp(a, w1, w2, ("relu", "none"), out=out)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / iters
    r = {"shape": "cfg3 MLP 128->128->128, one kernel", "rows": n, "d_in": k, "d_out": k, "dtypes": "f32/bf16/f32", "us": round(ms * 1e3, 1),
         "tflops": round(4.0 * n * k * k / ms / 1e9, 1), "gbs": round((n * k * 8 + 4 * k * k) / ms / 1e6), "vendor_us": None}
    rows.append(r)
    log(f"[update] {r['shape']}: {r['us']} us, {r['tflops']} TFLOP/s, {r['gbs']} GB/s")
    return rows


def run_embedding_bags(iters: int = 20, cpu_budget_s: float = 10.0):
    """Embedding lookup + element-wise addition of a recommendation model (section 8.3) through the
    aggregation path.  Synthetic stand-in for a click-log batch (the paper uses Criteo Kaggle, which is
    not available here): 26 tables of 2^18 rows each, concatenated; a sample looks up one row in every
    table, rows drawn from a Zipf-like law (exponent 1.05) per table; 2^20 samples; dim 64 fp32.  The
    table is cut by rows over 4 GPUs, this GPU holds the first quarter and serves the rest from a halo
    table of the distinct rows its samples need."""
    import torch
    import oracle
    from paper_2209_06800_amd import binding
    dev = "cuda:0"
    n_tables, rows_per_table, n_bags, dim = 26, 1 << 18, 1 << 20, 64
    table_rows = n_tables * rows_per_table
    rng = np.random.default_rng(220906800 + 83)
    # Zipf-like ranks by inverse transform on a truncated power law, then a fixed shuffle of ranks per table
    u = rng.random((n_bags, n_tables))
    a = 1.05
    ranks = np.floor(((rows_per_table ** (1 - a) - 1) * u + 1) ** (1 / (1 - a))).astype(np.int64) - 1
    ranks = np.clip(ranks, 0, rows_per_table - 1)
    perm = np.stack([rng.permutation(rows_per_table) for _ in range(n_tables)])
    idx = (perm[np.arange(n_tables)[None, :], ranks] + np.arange(n_tables)[None, :] * rows_per_table).astype(np.int32)
    idx = np.sort(idx, axis=1).ravel()
    ptr = np.arange(0, (n_bags + 1) * n_tables, n_tables, dtype=np.int64)
    lo, hi = 0, table_rows // 4
    t0 = time.time()
    part = binding.mgg_build_bags(ptr, idx, table_rows, lo, hi)
    info = part.info
    hg = part.export()["halo_gid"]
    log(f"[bags] {n_bags} bags x {n_tables} lookups over {table_rows} rows x {dim}: local lookups {info.nnz_local}, remote "
        f"{info.nnz_remote}, distinct remote rows {info.num_halo}, built in {time.time() - t0:.1f}s")
    table = rng.standard_normal((table_rows, dim), dtype=np.float32)
    t_local, t_halo = to_dev(table[lo:hi], dev), to_dev(table[hg], dev)
    out = torch.empty((n_bags, dim), dtype=torch.float32, device=dev)
    for _ in range(3):
        binding.mgg_bag_sum(part, t_local, t_halo, out=out)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        binding.mgg_bag_sum(part, t_local, t_halo, out=out)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / iters
    lookups = int(info.nnz_local + info.nnz_remote)
    model_bytes = lookups * (dim * 4 + 4) + n_bags * (dim * 4 + 8)
    # check a sample of bags against the oracle and time the oracle on a bounded sample
    sel = np.sort(rng.choice(n_bags, size=4096, replace=False))
    sub_ptr = np.arange(0, (sel.size + 1) * n_tables, n_tables, dtype=np.int64)
    sub_idx = idx.reshape(n_bags, n_tables)[sel].ravel()
    ref = oracle.bag_sum(sub_ptr, sub_idx, table)
    got = out[torch.from_numpy(sel).to(dev)].cpu().numpy().astype(np.float64)
    err = np.abs(got - ref).max()
    n_cpu = min(n_bags, 1 << 18)
    t0 = time.perf_counter()
    oracle.bag_sum(ptr[:n_cpu + 1], idx[:n_cpu * n_tables], table)
    cpu_s = time.perf_counter() - t0
    res = {"workload": "embedding_bags_26x2^18_rows_dim64_2^20_samples", "lookups": lookups, "bags": n_bags,
           "local_share": round(info.nnz_local / lookups, 3), "num_halo": int(info.num_halo), "ms": round(ms, 4),
           "glookups_per_s": round(lookups / ms / 1e6, 2), "gather_model_gbs": round(model_bytes / ms / 1e6, 1),
           "frac_of_hbm_peak": round(model_bytes / ms / 1e6 / HBM_PEAK_GBS, 3), "max_abs_err_vs_oracle_on_4096_bags": float(err),
           "cpu_oracle_glookups_per_s": round(n_cpu * n_tables / cpu_s / 1e9, 4), "cpu_cores": oracle.num_threads()}
    log(f"[bags] {ms:.4f} ms per batch, {res['glookups_per_s']} GLookups/s, gather-model {res['gather_model_gbs']} GB/s "
        f"({res['frac_of_hbm_peak']} of 8 TB/s); max error on 4096 sampled bags {err:.2e}; oracle {res['cpu_oracle_glookups_per_s']} GLookups/s")
    part.destroy()
    return res


def run(cfg: int, steps: int, warmup: int, verify: bool, cpu_budget_s: float = 20.0, calibrate_copy: bool = False,
        cold_iters: int = 5, part_id=None, split: str = "nodes", order_iters: int = 10):
    import torch
    from paper_2209_06800_amd import binding, inputs

    dev = "cuda:0"
    torch.cuda.set_device(0)
    t0 = time.time()
    w = inputs.config(cfg)
    if split == "edges" and w.parts > 1:
        # Algorithm 1 (section 4.1 Step-1): contiguous ranges with about E / P edges each instead of N / P nodes
        from paper_2209_06800_amd import binding as _b
        w.bounds = _b.mgg_split_edge_balanced(w.row_ptr, w.parts)
        w.name += "_edge_balanced"
    if part_id is not None and part_id != w.part_id:
        # another share of the same graph (share 0, the heaviest under the equal-node split, is the default)
        if not 0 <= part_id < w.parts:
            raise SystemExit(f"--part-id must be in [0, {w.parts})")
        w.part_id = part_id
        w.name += f"_share{part_id}"
    log(f"[bench] generated {w.name}: {inputs.graph_stats(w.row_ptr)} in {time.time() - t0:.1f}s")
    t0 = time.time()
    part = binding.mgg_build_partition(w.row_ptr, w.col, w.parts, w.part_id, w.bounds, **BUILD_KNOBS)
    info = part.info
    halo_gid = part.export()["halo_gid"]
    nnz = int(info.nnz_local + info.nnz_remote)
    log(f"[bench] partition {w.part_id}/{w.parts}: n_own={info.n_own} nnz_local={info.nnz_local} "
        f"nnz_remote={info.nnz_remote} halo={info.num_halo} items={info.n_items} split_rows={info.n_split_rows} "
        f"short_rows={info.n_short_rows} in {time.time() - t0:.1f}s")

    bf16 = w.dtype == "bf16"
    esz = 2 if bf16 else 4
    x_local_np, x_halo_np = w.x[w.lb:w.ub], w.x[halo_gid]
    # per layer: device inputs, weights, buffers
    layers = []
    for li, layer in enumerate(w.layers):
        d_in = layer.dims[0]
        if li == 0:
            # rows that are not a multiple of 16 bytes are laid out on 128-byte lines so that the
            # kernel can use 16-byte loads (config 4: 602 floats -> leading dimension 608)
            pad = 128 if (d_in * esz) % 16 else 0
            xl, xh = to_dev(x_local_np, dev, pad), (to_dev(x_halo_np, dev, pad) if halo_gid.size else None)
            lesz = esz
        else:
            # layer 2 reads layer 1's output for owned rows; halo rows are a seeded stand-in for
            # what the other partitions would have produced
            xl = layers[li - 1]["out"]
            xh = to_dev(inputs.layer2_halo_table(w.notes["layer2_halo_seed"], int(info.num_halo), d_in), dev)
            lesz = 4
        ws = [to_dev(m, dev) for m in layer.weights]
        # the aggregation result is laid out as mgg_layer_forward lays it out: rows start on 32-byte boundaries,
        # fp32 -- or bf16 when the weights are bf16 (the bf16 MFMA rounds its input the same way)
        agg_dt = torch.bfloat16 if bf16 else torch.float32
        agg = torch.empty((int(info.n_own), (d_in + 7) // 8 * 8), dtype=agg_dt, device=dev)[:, :d_in]
        hid = None
        if len(ws) == 2:
            hid = torch.empty((int(info.n_own), layer.dims[1]), dtype=torch.bfloat16 if bf16 else torch.float32, device=dev)
        out = torch.empty((int(info.n_own), layer.dims[-1]), dtype=torch.float32, device=dev)
        layers.append(dict(layer=layer, xl=xl, xh=xh, ws=ws, agg=agg, hid=hid, out=out, esz=lesz,
                           bytes=gather_model_bytes(nnz, int(info.n_own), d_in, lesz, layer.mode == "gcn", 2 if bf16 else 4),
                           bytes_c=compulsory_bytes(nnz, int(info.n_own), int(info.num_halo), d_in, lesz, layer.mode == "gcn", 2 if bf16 else 4),
                           flops=sum(2.0 * info.n_own * layer.dims[i] * layer.dims[i + 1] for i in range(len(ws)))))

    def step(events=None):
        for li, L in enumerate(layers):
            layer = L["layer"]
            if events is not None:
                events[li][0].record()
            binding.mgg_aggregate(part, layer.mode, L["xl"], L["xh"], eps=layer.eps, out=L["agg"])
            if events is not None:
                events[li][1].record()
            if len(L["ws"]) == 1:
                binding.mgg_update(L["agg"], L["ws"][0], None, layer.acts[0], out=L["out"])
            else:
                binding.mgg_update_mlp(L["agg"], L["ws"][0], L["ws"][1], layer.acts, hidden=L["hid"], out=L["out"])
            if events is not None:
                events[li][2].record()

    if calibrate_copy:
        # a plain device-to-device copy of known size, so that a counter run (rocprofv3 --pmc
        # FETCH_SIZE / WRITE_SIZE) can be scaled: each launch reads 1 GiB and writes 1 GiB
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)       # an elementwise kernel, not a DMA copy
        torch.cuda.synchronize()
        del src, dst

    for _ in range(max(warmup, 1)):
        step()
    torch.cuda.synchronize()

    ev = [[[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in layers] for _ in range(steps)]
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for k in range(steps):
        step(ev[k])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    ms_per_step = elapsed * 1e3 / steps

    agg_all = [[ev[k][li][0].elapsed_time(ev[k][li][1]) for k in range(steps)] for li in range(len(layers))]
    upd_all = [[ev[k][li][1].elapsed_time(ev[k][li][2]) for k in range(steps)] for li in range(len(layers))]
    agg_ms = [float(np.mean(v)) for v in agg_all]
    upd_ms = [float(np.mean(v)) for v in upd_all]

    # Outside the timed region: the same aggregations with cold caches.  Between two launches a 1 GiB
    # scratch buffer is overwritten, which pushes the tables out of L2 and of the Infinity Cache.
    cold_ms = [None] * len(layers)
    if cold_iters > 0:
        scratch = torch.empty(1 << 28, dtype=torch.float32, device=dev)
        cold = [[] for _ in layers]
        for _ in range(cold_iters):
            for li, L in enumerate(layers):
                scratch.fill_(1.0)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                binding.mgg_aggregate(part, L["layer"].mode, L["xl"], L["xh"], eps=L["layer"].eps, out=L["agg"])
                e1.record()
                torch.cuda.synchronize()
                cold[li].append(e0.elapsed_time(e1))
        cold_ms = [float(np.median(v)) for v in cold]
        del scratch
    dom = int(np.argmax([L["bytes"] for L in layers]))

    def rates(nbytes, ms):
        gbs = nbytes / (ms * 1e-3) / 1e9
        return {"bytes": int(nbytes), "gbs": round(gbs, 1), "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}

    per_layer = []
    for li, L in enumerate(layers):
        med = float(np.median(agg_all[li]))
        mt = measured_traffic(w.name, li)
        rec = {
            "layer": li, "agg_dim": L["layer"].dims[0], "agg_ms": round(agg_ms[li], 4),
            "agg_gedges_per_s": round(nnz / (agg_ms[li] * 1e-3) / 1e9, 3),
            "agg_ms_median": round(med, 4), "agg_ms_min": round(float(np.min(agg_all[li])), 4),
            "agg_ms_cold_cache": None if cold_ms[li] is None else round(cold_ms[li], 4),
            "agg_model": rates(L["bytes"], agg_ms[li]),              # every neighbour row once per edge: what reaches the CUs
            "agg_compulsory": rates(L["bytes_c"], agg_ms[li]),       # a perfect cache
            "agg_measured": None if mt is None else rates(mt["bytes"], agg_ms[li]),   # left L2 for the memory fabric (counters)
            "update_ms": round(upd_ms[li], 4),
            "update_tflops": round(L["flops"] / (upd_ms[li] * 1e-3) / 1e12, 2),
        }
        per_layer.append(rec)

    mt = measured_traffic(w.name, dom)
    model, comp = per_layer[dom]["agg_model"], per_layer[dom]["agg_compulsory"]
    if mt is not None:
        basis, nbytes = "measured", mt["bytes"]
    else:               # no counter run of this workload on record: the perfect-cache bytes are a lower bound on the traffic
        basis, nbytes = "compulsory", layers[dom]["bytes_c"]
    achieved = nbytes / (agg_ms[dom] * 1e-3) / 1e9
    roofline = {
        "bound": "hbm", "kernel": f"aggregate (layer {dom}, dim {layers[dom]['layer'].dims[0]})",
        "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
        "basis": basis,                       # which byte count `achieved` and `frac` use
        "traffic": None if mt is None else mt["bytes"],
        "traffic_commit": None if mt is None else mt["commit"],
        "traffic_profile": None if mt is None else mt["profile"],
        "kernel_ms": round(agg_ms[dom], 4), "kernel_ms_median": per_layer[dom]["agg_ms_median"],
        # the same launch against the two model byte counts; the gather-model figure exceeds the HBM peak where
        # L2 serves repeated rows and is then a statement about cache bandwidth, not about HBM
        "gather_model": dict(model, bound="l2" if model["frac_of_hbm_peak"] > 1.0 else "hbm"),
        "compulsory": comp,
    }

    # Outside the timed region too: the same layers through mgg_layer_forward, in the paper's order and with
    # MGG_ORDER_AUTO, which applies the first weight matrix before the aggregation when that narrows the rows
    # (same values within rounding; both forms are parity-tested at full size).
    order_ms = {}
    if order_iters > 0:
        for order in ("agg_first", "auto"):
            tot = 0.0
            xl_prev = None
            for li, L in enumerate(layers):
                layer = L["layer"]
                xl = L["xl"] if li == 0 else xl_prev
                need = binding.mgg_layer_workspace_bytes(part, layer.mode, L["ws"], layer.acts, eps=layer.eps, order=order)
                wsp = torch.empty(need, dtype=torch.uint8, device=dev)
                o = torch.empty_like(L["out"])
                for _ in range(2):
                    binding.mgg_layer_forward(part, layer.mode, xl, L["xh"], L["ws"], layer.acts, eps=layer.eps, workspace=wsp, out=o, order=order)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(order_iters):
                    binding.mgg_layer_forward(part, layer.mode, xl, L["xh"], L["ws"], layer.acts, eps=layer.eps, workspace=wsp, out=o, order=order)
                e1.record()
                torch.cuda.synchronize()
                tot += e0.elapsed_time(e1) / order_iters
                xl_prev = o
                del wsp
            order_ms[order] = round(tot, 4)

    if verify:
        import oracle
        rng = np.random.default_rng(0)
        deg = np.diff(w.row_ptr)[w.lb:w.ub]
        rows = np.unique(np.concatenate([np.argsort(deg)[-4:], rng.integers(0, int(info.n_own), 200)]))
        L0 = layers[0]
        ref = oracle.aggregate(w.row_ptr, w.col, L0["layer"].mode, x_local_np, lb=w.lb, ub=w.ub, x_halo=x_halo_np,
                               halo_gid=halo_gid, eps=L0["layer"].eps, rows=rows)
        got = L0["agg"][torch.from_numpy(rows).to(dev)].float().cpu().numpy().astype(np.float64)
        err = np.abs(got - ref)
        if L0["agg"].dtype == torch.bfloat16:      # rounded to bf16 on the way out: half a unit in the 8th bit
            bound, what = 2.0 ** -8 * np.abs(ref) + 1e-30, "2^-8 |ref|"
        else:
            bound, what = 1e-6 + 1e-4 * np.abs(ref), "(1e-6 + 1e-4|ref|)"
        log(f"[bench] verify layer-0 aggregation on {rows.size} sampled rows: max abs err {err.max():.3e}, "
            f"max err / {what} = {(err / bound).max():.3f}")

    cpu_baseline = None
    if cpu_budget_s > 0:
        cpu_baseline = cpu_baseline_leg(w, layers[0]["layer"], x_local_np, x_halo_np, halo_gid, int(info.n_own),
                                        cpu_budget_s)
    n_own = int(info.n_own)
    result = {
        "metric": "aggregation GEdges/s and achieved HBM GB/s (% of peak) per layer, 1 MI355X",
        "value": round(nnz * len(layers) / (ms_per_step * 1e-3) / 1e9, 4),
        "unit": "GEdges/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 in, f32 accumulate" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": w.name, "share": f"{w.part_id}/{w.parts}", "n_own": n_own, "nnz_local": int(info.nnz_local),
                   "nnz_remote": int(info.nnz_remote), "num_halo": int(info.num_halo),
                   "layers": [L["layer"].dims for L in layers], "ps": int(info.ps), "dist": int(info.dist),
                   "short_max": int(info.short_max)},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "per_layer": per_layer,
        # every layer through mgg_layer_forward: the paper's order, and the order MGG_ORDER_AUTO picks
        "layer_forward_ms": order_ms or None,
        "layer_forward_auto_gedges_per_s": round(nnz * len(layers) / (order_ms["auto"] * 1e-3) / 1e9, 4) if order_ms else None,
    }
    part.destroy()
    return result


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=None, choices=[1, 2, 3, 4, 5],
                    help="time this config only (default: config 4, then 5, 2 and 3 under other_configs)")
    ap.add_argument("--time-budget", type=float, default=420.0,
                    help="seconds after which no further config of other_configs is started")
    ap.add_argument("--verify", action="store_true", help="compare sampled rows with the CPU oracle")
    ap.add_argument("--cpu-seconds", type=float, default=20.0, help="budget of the cpu_baseline leg (0 = skip it)")
    ap.add_argument("--ablations", action="store_true",
                    help="time the aggregation of layer 0 with neighbour partitioning, interleaving, the XCD-aware "
                         "schedule, the short-row bin, LDS staging and column slabs switched one at a time, and exit")
    ap.add_argument("--tune", action="store_true",
                    help="run the greedy search over ps / dist / wpb (section 6) on layer 0's aggregation and exit")
    ap.add_argument("--tune-exhaustive", action="store_true",
                    help="like --tune, and measure the whole 150-point grid beside it")
    ap.add_argument("--order-iters", type=int, default=10,
                    help="calls of mgg_layer_forward per layer and order timed after the timed region (0 = skip)")
    ap.add_argument("--cold-iters", type=int, default=5,
                    help="aggregation launches per layer timed with cold caches after the timed region (0 = skip)")
    ap.add_argument("--split", choices=["nodes", "edges"], default="nodes",
                    help="node ranges of the shares: equal node counts (default) or the edge-balanced split of Algorithm 1")
    ap.add_argument("--part-id", type=int, default=None, help="time another share of the graph than share 0")
    ap.add_argument("--embedding-bags", action="store_true",
                    help="time the embedding-bag sum of a synthetic recommendation-model batch (section 8.3) and exit")
    ap.add_argument("--update-shapes", action="store_true",
                    help="time mgg_update alone on the Update shapes of the five configs and exit")
    ap.add_argument("--no-vendor", action="store_true", help="with --update-shapes: skip the torch.matmul comparison")
    ap.add_argument("--compare-orders", action="store_true",
                    help="time every layer as Update(Aggregate(X)) and as Aggregate(X W) (+ bias, activation) and exit")
    ap.add_argument("--calibrate-gather", action="store_true",
                    help="launch the aggregation kernel on a graph that gathers each of 4 Mi table rows exactly once "
                         "(known L2-miss bytes; reference for rocprofv3 --pmc runs) and exit")
    ap.add_argument("--option", action="append", default=[], metavar="KEY=VALUE",
                    help="a run-time switch of the library (mgg_set_option) for the whole run, e.g. col_slab_bytes=128")
    ap.add_argument("--build-knob", action="append", default=[], metavar="KEY=VALUE",
                    help="a knob of mgg_build_partition for the timed run, e.g. hot_phases=-2 or xcd_min_deg=128")
    ap.add_argument("--probe-gather", action="store_true",
                    help="time a bare gather kernel on tables from 1 MB to 2 GB (the ceilings of the gather path) and exit")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch a 1 GiB device copy three times (reference for rocprofv3 --pmc runs)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures one GPU's share on one MI355X; multi-GPU runs are not part of this build "
              "(no collectives, no second GPU). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    global NON_DEFAULT_RUN
    for kv in args.option:
        from paper_2209_06800_amd import binding
        key, _, val = kv.partition("=")
        binding.mgg_set_option(key, int(val))
        NON_DEFAULT_RUN = True
    for kv in args.build_knob:
        key, _, val = kv.partition("=")
        BUILD_KNOBS[key] = int(val)
        NON_DEFAULT_RUN = True
    if args.embedding_bags:
        print(json.dumps(run_embedding_bags()), flush=True)
        return
    if args.update_shapes:
        print(json.dumps({"update_shapes": run_update_shapes(vendor=not args.no_vendor)}), flush=True)
        return
    if args.compare_orders:
        print(json.dumps(run_orders(args.config or HEADLINE_CONFIG)), flush=True)
        return
    if args.probe_gather:
        print(json.dumps({"probe_gather": probe_gather()}), flush=True)
        return
    if args.calibrate_gather:
        print(json.dumps({"calibrate_gather": calibrate_gather()}), flush=True)
        return
    if args.tune or args.tune_exhaustive:
        print(json.dumps(run_tuner(args.config or 2, args.tune_exhaustive)), flush=True)
        return
    if args.ablations:
        cfg = args.config or HEADLINE_CONFIG
        print(json.dumps({"workload_config": cfg, "ablations": run_ablations(cfg)}), flush=True)
        return
    t_begin = time.time()
    res = run(args.config or HEADLINE_CONFIG, args.steps, args.warmup, args.verify, args.cpu_seconds, args.calibrate_copy,
              args.cold_iters, args.part_id, args.split, args.order_iters)
    if args.config is None:
        # the other configs, same protocol, without the CPU leg; each adds its per-layer and roofline figures
        others = []
        for cfg in OTHER_CONFIGS:
            if time.time() - t_begin > args.time_budget:
                log(f"[bench] time budget reached: config {cfg} not run")
                continue
            r = run(cfg, args.steps, args.warmup, args.verify, 0.0, False, args.cold_iters, None, "nodes", args.order_iters)
            others.append({k: r[k] for k in ("value", "unit", "ms_per_step", "steps", "dtype", "config", "roofline", "per_layer",
                                             "layer_forward_ms", "layer_forward_auto_gedges_per_s")})
        res["other_configs"] = others
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
