#!/usr/bin/env python3
"""Benchmark of the sparse graph attention hot path (forward + backward) on one MI355X.

A step is one pass of the whole path — gta_attn_fwd then gta_attn_bwd — over one seeded
synthetic workload whose inputs are already resident in HBM.  Prints ONE JSON line with the
whole-job throughput in edges/s, a roofline object for the dominant kernel (algorithmic bytes
over its HIP-event time) and the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth

PROFILE_DIR = os.path.join(ROOT, "profiles")


def profile_counters(workload: str) -> dict:
    """Counter readings per kernel from the committed rocprofv3 --pmc summary of this workload
    (profiles/all_kernels_<workload>.txt, lines `counters kernel=<pass> key=value ...`): FETCH_SIZE and
    WRITE_SIZE in KiB per dispatch, the factors a plain copy of known size gave for them on the same
    box, and the L2 hit rate.  Empty when the workload has no summary."""
    path = os.path.join(PROFILE_DIR, f"all_kernels_{workload}.txt")
    table: dict = {}
    if not os.path.exists(path):
        return table
    for line in open(path):
        if not line.startswith("counters "):
            continue
        fields = dict(kv.split("=", 1) for kv in line.split()[1:])
        name = fields.pop("kernel")
        table[name] = {k: float(v) for k, v in fields.items()}
        table[name]["source"] = os.path.relpath(path, ROOT)
    return table


def scope_table_bytes(pass_name: str, rows: int, entries: int, row_bytes: int, heads: int):
    """Algorithmic bytes of a pass by the scope table's per-unit figures (every entry gathers its rows,
    streams touched once, nothing kept per entry), or None for kernels that table has no row for:
      forward                      E (2R + 4)      + N_dst (2R + 4H + 8)
      backward, destination-major  E (2R + 4)      + N_dst (4R + 8H + 8)
      backward, source-major       E (2R + 8H + 4) + N_src (4R + 8)"""
    R, H = row_bytes, heads
    if pass_name == "fwd":
        return entries * (2 * R + 4) + rows * (2 * R + 4 * H + 8)
    if pass_name == "bwd_dst":
        return entries * (2 * R + 4) + rows * (4 * R + 8 * H + 8)
    if pass_name == "bwd_src":
        return entries * (2 * R + 8 * H + 4) + rows * (4 * R + 8)
    return None


def algorithmic_bytes(pass_name: str, rows: int, entries: int, row_bytes: int, heads: int, lean: bool) -> int:
    """Bytes the method must move for `rows` rows holding `entries` stored entries: every entry
    gathers its rows (no reuse assumed), streams are touched once.  `lean` = the backward form that
    keeps nothing per stored entry."""
    R, H = row_bytes, heads
    if pass_name == "fwd":          # K,V gathers + index | Q read, out write, lse write, row pointer
        return entries * (2 * R + 4) + rows * (2 * R + 4 * H + 8)
    if pass_name == "bwd_rowstat":  # Y, dY read, lse read, (lse, delta) write
        return rows * (2 * R + 12 * H)
    if pass_name == "bwd_src" and not lean:
        # Q,dY gathers + (lse, delta) + destination id + stored position + dZ write | K,V read, dK,dV write
        return entries * (2 * R + 8 * H + 8 + 4 * H) + rows * (4 * R + 8)
    if pass_name == "bwd_dq":       # K gather + index + dZ read | dQ write, row pointer
        return entries * (R + 4 + 4 * H) + rows * (R + 8)
    if pass_name == "bwd_dst":      # K,V gathers + index | Q,dY,Y read, dQ write, lse read, stats write
        return entries * (2 * R + 4) + rows * (4 * R + 12 * H + 8)
    if pass_name == "bwd_src":      # Q,dY gathers + (lse, delta) + destination id | K,V read, dK,dV write
        return entries * (2 * R + 8 * H + 4) + rows * (4 * R + 8)
    raise KeyError(pass_name)


def cpu_baseline(w, sample_edges: int) -> dict:
    """Times the oracle (as it stands) on the host cores: on the whole workload by default, or with
    sample_edges > 0 on its first destination rows holding about that many entries (K and V keep all
    their rows, so the gathers are spread as in the whole workload)."""
    import gen
    import oracle
    whole = sample_edges <= 0 or sample_edges >= w.nnz
    n_rows = w.n_dst if whole else int(np.searchsorted(w.indptr, sample_edges, side="left"))
    n_rows = max(1, min(n_rows, w.n_dst))
    nnz = int(w.indptr[n_rows])
    indptr, indices = w.indptr[: n_rows + 1], w.indices[:nnz]
    f64 = lambda x: gen.as_f32(x).astype(np.float64)
    Q, dO = f64(w.tensor("Q")[:n_rows]), f64(w.tensor("dO")[:n_rows])
    K, V = f64(w.tensor("K")), f64(w.tensor("V"))
    t0 = time.perf_counter()
    oracle.forward(indptr, indices, Q, K, V)
    t1 = time.perf_counter()
    oracle.backward(indptr, indices, Q, K, V, dO)
    t2 = time.perf_counter()
    cores = int(os.environ.get("OMP_NUM_THREADS", 0)) or (os.cpu_count() or 1)
    what = (f"the whole workload '{w.name}' ({w.n_dst} destination rows, {nnz} entries)" if whole else
            f"first {n_rows} destination rows ({nnz} entries, sources over all {w.n_src} rows of K / V) of "
            f"workload '{w.name}'")
    return {"value": nnz / (t2 - t0), "unit": "edges/s", "cores": cores, "kind": "oracle",
            "sample": f"{what}, fp64 forward {t1 - t0:.2f}s + backward {t2 - t1:.2f}s"}


def stream_ceilings(gta, torch, dev, mib: int, reps: int, log) -> dict:
    """GB/s of plain streaming kernels (read; copy; add) over buffers of `mib` MiB, HIP-event timed."""
    n = mib * (1 << 18)
    a = torch.ones(n, dtype=torch.float32, device=dev)
    b = torch.ones(n, dtype=torch.float32, device=dev)
    dst = torch.empty(n, dtype=torch.float32, device=dev)
    moved = {0: 1, 1: 2, 2: 3}     # buffers touched per launch
    out = {}
    for mode, label in ((0, "read"), (1, "copy"), (2, "add")):
        for _ in range(2):
            gta.gta_stream_probe(mode, dst, a, b)
        torch.cuda.synchronize()
        gta.gta_profile_enable(1)
        for _ in range(reps):
            gta.gta_stream_probe(mode, dst, a, b)
        torch.cuda.synchronize()
        recs = gta.gta_profile_read(reset=True)
        gta.gta_profile_enable(0)
        ms = sorted(r["ms"] for r in recs)[len(recs) // 2]
        out[label] = moved[mode] * n * 4 / (ms * 1e-3) / 1e9
        log(f"  stream probe {label}: {ms:.3f} ms for {moved[mode]} x {mib} MiB -> {out[label]:.0f} GB/s")
    del a, b, dst
    return out


def time_unfused(gta, torch, plan, Q, K, V, dO, w, steps, log) -> dict:
    """The paper's decomposition (Section 2.2): forward SDDMM + softmax + SpMM, backward 3 SpMM +
    1 SDDMM + softmax backward, with Z, U, dU, dZ stored as float [nnz, heads]."""
    scale = 1.0 / float(np.sqrt(w.head_dim))
    E, H = w.nnz, w.heads
    Z = torch.empty((E, H), dtype=torch.float32, device=Q.device)
    U, dU, dZ = torch.empty_like(Z), torch.empty_like(Z), torch.empty_like(Z)
    lse = torch.empty((w.n_dst, H), dtype=torch.float32, device=Q.device)
    Y, dQ = torch.empty_like(Q), torch.empty_like(Q)
    dK, dV = torch.empty_like(K), torch.empty_like(V)

    def step():
        gta.gta_sddmm(plan, Q, K, Z)
        gta.gta_edge_softmax(plan, Z, scale, U, lse)
        gta.gta_spmm(plan, U, V, False, Y)
        gta.gta_spmm(plan, U, dO, True, dV)
        gta.gta_sddmm(plan, dO, V, dU)
        gta.gta_edge_softmax_bwd(plan, U, dU, scale, dZ)
        gta.gta_spmm(plan, dZ, K, False, dQ)
        gta.gta_spmm(plan, dZ, Q, True, dK)

    step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    gta.gta_profile_enable(1)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    recs = gta.gta_profile_read(reset=True)
    gta.gta_profile_enable(0)
    # algorithmic bytes per call: one row gather per entry plus the per-entry arrays, streams once
    R = w.heads * w.head_dim * (4 if w.dtype == "f32" else 2)
    op_bytes = {
        "sddmm": E * (R + 4 + 4 * H) + w.n_dst * (R + 8),                 # gather + index + Z write | X row
        "spmm": E * (R + 4 + 4 * H) + w.n_dst * (R + 8),                  # gather + index + W read | Y row
        "spmm_t": E * (R + 8 + 4 * H) + w.n_src * (R + 8),                # + stored position of the entry
        "edge_softmax": E * 12 * H + w.n_dst * (4 * H + 8),               # Z read twice, U write | lse
        "edge_softmax_bwd": E * 20 * H + w.n_dst * 8,                     # U, dU read twice, dZ write
    }
    per_op: dict = {}
    for r in recs:
        k = per_op.setdefault(r["name"], {"ms": 0.0, "calls": 0})
        k["ms"] += r["ms"]
        k["calls"] += 1
    ops = {}
    for name, k in per_op.items():
        avg = k["ms"] / k["calls"]
        gbs = op_bytes[name] / (avg * 1e-3) / 1e9 if name in op_bytes else 0.0
        ops[name] = {"avg_ms": round(avg, 4), "calls_per_step": k["calls"] // steps, "gbs": round(gbs, 1)}
        log(f"  unfused {name:20s} {avg:9.3f} ms per call x{k['calls'] // steps}  {gbs:8.1f} GB/s")
    return {"ms_per_step": ms, "edges_per_s": E / (ms * 1e-3), "ops": ops,
            "edge_array_bytes": 4 * E * H * 4}


def time_layer(gta, torch, plan, w, steps, log) -> dict:
    """One Sparse Graph Attention layer (Eq. 3-5), forward + backward: X' = X W_o + attention(X W_Q, X W_K, X W_V)."""
    import gen
    if w.n_src != w.n_dst:
        return {"skipped": "the layer form needs a workload with n_src == n_dst"}
    n, d = w.n_dst, w.heads * w.head_dim
    dev = plan.indptr.device
    if w.dtype == "bf16":
        mk = lambda shape, stream: torch.from_numpy(gen.normal(shape, "bf16", w.seed, stream).view(np.int16)).to(dev).view(torch.bfloat16)
        tdtype, el = torch.bfloat16, 2
    else:
        mk = lambda shape, stream: torch.from_numpy(gen.normal(shape, "f32", w.seed, stream)).to(dev)
        tdtype, el = torch.float32, 4
    X, dXout = mk((n, d), STREAM_X), mk((n, d), STREAM_DX)
    Ws = [(mk((d, d), 10 + k).float() * (1.0 / float(np.sqrt(d)))).to(tdtype) for k in range(4)]

    def step():
        _, saved = gta.gta_sga_layer_fwd(plan, X, *Ws, w.heads)
        gta.gta_sga_layer_bwd(plan, X, *Ws, saved, dXout, w.heads)

    step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    gta.gta_profile_enable(1)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    recs = gta.gta_profile_read(reset=True)
    gta.gta_profile_enable(0)
    agg: dict = {}
    for r in recs:
        k = agg.setdefault(r["name"], {"ms": 0.0, "calls": 0})
        k["ms"] += r["ms"]
        k["calls"] += 1
    flops = 2.0 * n * d * d     # one n x d x d product
    tensor = n * d * el         # bytes of one [n, d] tensor
    # (products, tensors moved) per launch: every operand read once, every result written once
    # (linear_dw_group: the four weight gradients of the layer share X: X once and four dY)
    dense = {"linear_nn": (1, 2), "linear_nt": (1, 2), "linear_dw": (1, 2), "linear_dw_group": (4, 5),
             "proj_1to3": (3, 4), "proj_1to1+C": (1, 3), "proj_1to1": (1, 2), "proj_4to1": (4, 5)}
    ops = {}
    dense_ms = 0.0
    for name, k in agg.items():
        avg = k["ms"] / k["calls"]
        entry = {"avg_ms": round(avg, 4), "calls_per_step": k["calls"] // steps}
        if name in dense:
            products, tensors = dense[name]
            entry["tflops"] = round(products * flops / (avg * 1e-3) / 1e12, 1)
            entry["gbs"] = round(tensors * tensor / (avg * 1e-3) / 1e9, 1)
        if name.startswith("linear") or name.startswith("proj"):
            dense_ms += k["ms"] / steps
        ops[name] = entry
        log(f"  layer {name:20s} {avg:9.3f} ms per call x{entry['calls_per_step']}  {entry.get('tflops', '')} TFLOP/s {entry.get('gbs', '')} GB/s")
    return {"ms_per_step": ms, "edges_per_s": w.nnz / (ms * 1e-3), "hidden": d, "dense_ms_per_step": round(dense_ms, 3),
            "ops": ops}


STREAM_X, STREAM_DX = 8, 9


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="large", choices=["tiny", "mid", "large", "partition", "skew"])
    ap.add_argument("--shrink", type=int, default=1, help="divide the workload size (debugging)")
    ap.add_argument("--heads", type=int, default=0,
                    help="run the workload's graph with this many heads instead of its own (experiments)")
    ap.add_argument("--head-dim", type=int, default=0, help="likewise for the head dimension")
    ap.add_argument("--cpu-sample-edges", type=int, default=0,
                    help="time the oracle on the first rows holding about this many entries instead of on "
                         "the whole workload (0 = whole workload)")
    ap.add_argument("--probe-mib", type=int, default=1024,
                    help="buffer size of the streaming probes that measure the achievable bandwidth (0 = skip)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pack-max-deg", type=int, default=0)
    ap.add_argument("--wave-max-deg", type=int, default=0)
    ap.add_argument("--hub-chunk", type=int, default=0)
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also run one plain elementwise copy kernel (reads and writes this many MiB) "
                         "so that profiler byte counters can be scaled against a known size")
    ap.add_argument("--lean-scratch", action="store_true",
                    help="give the backward only the minimum scratch (nothing kept per stored entry)")
    ap.add_argument("--unfused", action="store_true",
                    help="also time the paper's operator-by-operator decomposition (SDDMM, softmax, SpMM ...)")
    ap.add_argument("--layer", action="store_true",
                    help="also time one full layer (QKV / output projections on the matrix cores + attention), "
                         "forward and backward; bf16 workloads with n_src == n_dst only")
    ap.add_argument("--hip-graph", action="store_true",
                    help="record one step into a HIP graph and time its replays (small, launch-bound workloads)")
    ap.add_argument("--verbose", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no cross-GPU sharding or collectives); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import torch
    import gen
    import paper_2604_16715_amd as gta

    def log(*a):
        if args.verbose:
            print(*a, file=sys.stderr, flush=True)

    t0 = time.perf_counter()
    w = gen.workload(args.workload, args.shrink)
    if args.heads > 0 or args.head_dim > 0:   # same graph, other tensor shape: no longer the named workload
        w.heads, w.head_dim = args.heads or w.heads, args.head_dim or w.head_dim
        w.name = f"{w.name}[{w.heads}x{w.head_dim}]"
    host = {k: w.tensor(k) for k in ("Q", "K", "V", "dO")}
    log(f"generated {w.name}: n_dst={w.n_dst} n_src={w.n_src} nnz={w.nnz} in {time.perf_counter() - t0:.1f}s")

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    def up(x):
        if x.dtype == np.uint16:
            return torch.from_numpy(x.view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(x).to(dev)

    indptr, indices = torch.from_numpy(w.indptr).to(dev), torch.from_numpy(w.indices).to(dev)
    Q, K, V, dO = (up(host[k]) for k in ("Q", "K", "V", "dO"))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    plan = gta.gta_plan_create(indptr, indices, w.n_src, pack_max_deg=args.pack_max_deg,
                               wave_max_deg=args.wave_max_deg, hub_chunk=args.hub_chunk)
    torch.cuda.synchronize()
    plan_ms = (time.perf_counter() - t0) * 1e3
    out = torch.empty_like(Q)
    lse = torch.empty((w.n_dst, w.heads), dtype=torch.float32, device=dev)
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)

    def step():
        gta.gta_attn_fwd(plan, Q, K, V, 0.0, out, lse)
        gta.gta_attn_bwd(plan, Q, K, V, out, lse, dO, 0.0, dQ, dK, dV, lean_scratch=args.lean_scratch)

    if args.copy_probe_mib > 0:   # calibration kernel for rocprofv3 --pmc runs (outside the timed region)
        src = torch.ones(args.copy_probe_mib * (1 << 18), dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        gta.gta_stream_probe(1, dst, src)
        torch.cuda.synchronize()
        del src, dst

    timed_step = step
    if args.hip_graph:   # the calls only enqueue kernels, so a step can be recorded once and replayed
        step()           # allocates the scratch buffers before the capture
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.current_stream().wait_stream(side)
        timed_step = graph.replay
    for _ in range(args.warmup):
        timed_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        timed_step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    edges_per_s = w.nnz * args.steps / elapsed

    # per-launch HIP-event timing (events on the launch stream) over the same number of steps
    row_bytes = w.heads * w.head_dim * (4 if w.dtype == "f32" else 2)

    def timed_launches(mode):
        gta.gta_profile_enable(mode)
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        records = gta.gta_profile_read(reset=True)
        gta.gta_profile_enable(0)
        table: dict = {}
        lean = any(r["name"].startswith("bwd_dst") for r in records)   # the form the library actually ran
        for r in records:
            k = table.setdefault(r["name"], {"ms": 0.0, "launches": 0, "rows": r["rows"], "entries": r["entries"]})
            k["ms"] += r["ms"]
            k["launches"] += 1
        for name, k in table.items():
            k["avg_ms"] = k["ms"] / k["launches"]
            parts = name.split(".")
            k["bytes"] = 0 if parts[-1] == "merge" else algorithmic_bytes(parts[0], k["rows"], k["entries"],
                                                                          row_bytes, w.heads, lean)
            k["gbs"] = k["bytes"] / (k["avg_ms"] * 1e-3) / 1e9 if k["avg_ms"] > 0 else 0.0
            log(f"  {name:16s} {k['avg_ms']:9.3f} ms  rows={k['rows']:9d} entries={k['entries']:10d}  "
                f"{k['bytes'] / 1e9:8.3f} GB  {k['gbs']:8.1f} GB/s")
        return table

    kernels = timed_launches(1)
    total_bytes = sum(k["bytes"] for k in kernels.values())
    if args.verbose:
        log("  per-schedule launches (separate grids):")
        timed_launches(2)
    dom_name, dom = max(kernels.items(), key=lambda kv: kv[1]["ms"])
    ceilings = stream_ceilings(gta, torch, dev, args.probe_mib, 5, log) if args.probe_mib > 0 else {}
    counters = profile_counters(w.name)

    def counter_fields(name):
        c = counters.get(name)
        if not c:
            return None, None, None
        traffic = int((c["fetch_kib"] * c["fetch_scale"] + c["write_kib"] * c["write_scale"]) * 1024)
        return traffic, c.get("l2_hit_pct"), c
    traffic, l2_hit, craw = counter_fields(dom_name)
    # the dominant kernel by the scope table's formula (when it has a row for it) and by the bytes this
    # implementation moves (`lean` form: the two coincide; default form: + the dZ store and its index)
    dom_scope = scope_table_bytes(dom_name, dom["rows"], dom["entries"], row_bytes, w.heads)
    dom_scope = dom["bytes"] if dom_scope is None else dom_scope
    gbs = lambda nbytes: nbytes / (dom["avg_ms"] * 1e-3) / 1e9
    step_gbs = total_bytes / (ms_per_step * 1e-3) / 1e9
    result = {
        "metric": "edges/sec, sparse graph attention fwd+bwd, 1 MI355X; achieved HBM GB/s",
        "value": edges_per_s, "unit": "edges/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": w.name, "recipe": w.recipe, "n_dst": w.n_dst, "n_src": w.n_src, "nnz": w.nnz,
                   "heads": w.heads, "head_dim": w.head_dim, "accumulate": "f32",
                   "backward": "recompute-per-entry" if "bwd_dst" in kernels else "dZ-kept-per-entry",
                   "launch": "hip-graph replay" if args.hip_graph else "eager",
                   "plan_ms": plan_ms, "wave_max_deg": int(plan.info().wave_max_deg),
                   "hub_chunk": int(plan.info().hub_chunk),
                   "plan_workspace_bytes": int(plan.workspace.numel()),
                   "scratch_bytes": int(plan.scratch(w.heads, w.head_dim, 1 if w.dtype == "bf16" else 0,
                                                     args.lean_scratch).numel())},
        "hbm": {"algorithmic_bytes_per_step": total_bytes, "achieved_gbs": step_gbs,
                "spec_peak_gbs": HBM_PEAK_GBS, "frac_of_peak": step_gbs / HBM_PEAK_GBS,
                "read_ceiling_gbs": ceilings.get("read"), "copy_ceiling_gbs": ceilings.get("copy"),
                "add_ceiling_gbs": ceilings.get("add"),
                "note": "achieved = algorithmic bytes (every entry gathers its rows, no reuse assumed) over "
                        "time; gathers repeated within the 256 MB Infinity Cache or L2 never reach DRAM, so "
                        "this can exceed what a streaming kernel reaches (the *_ceiling_gbs probes, "
                        "measured in this run)"},
        "kernels": {n: {"avg_ms": round(k["avg_ms"], 4), "gbs": round(k["gbs"], 1)} for n, k in kernels.items()},
        "roofline": {"bound": "hbm", "kernel": dom_name, "achieved": gbs(dom_scope), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": gbs(dom_scope) / HBM_PEAK_GBS, "traffic": traffic,
                     "bytes_per_launch": dom_scope, "avg_launch_ms": dom["avg_ms"],
                     "achieved_impl_model": gbs(dom["bytes"]), "frac_impl_model": gbs(dom["bytes"]) / HBM_PEAK_GBS,
                     "bytes_per_launch_impl_model": dom["bytes"],
                     "frac_of_read_ceiling": gbs(dom_scope) / ceilings["read"] if ceilings else None,
                     "l2_hit_pct": l2_hit,
                     "traffic_note": None if craw is None else
                     f"L2<->fabric bytes per launch (Infinity-Cache hits included; no gfx950 counter separates "
                     f"them from DRAM): (FETCH_SIZE {craw['fetch_kib']:.0f} KiB x {craw['fetch_scale']} + WRITE_SIZE "
                     f"{craw['write_kib']:.0f} KiB x {craw['write_scale']}) x 1024, factors from a copy of known "
                     f"size; from {craw['source']}"},
    }
    if args.unfused:
        result["unfused"] = time_unfused(gta, torch, plan, Q, K, V, dO, w, args.steps, log)
    if args.layer:
        result["layer"] = time_layer(gta, torch, plan, w, args.steps, log)
    if not args.no_cpu_baseline:
        del Q, K, V, dO, out, dQ, dK, dV
        result["cpu_baseline"] = cpu_baseline(w, args.cpu_sample_edges)
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
