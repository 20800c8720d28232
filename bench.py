#!/usr/bin/env python3
"""Benchmark of the GSR-GNN training step (forward + inverse recomputation + backward) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2|cfg1|cfg0|cfg2-bf16|cfg4|dense]
                    [--layers L] [--k K] [--c C] [--index-mode near-ties|all|none] [--no-extras]

A "step" is one gsr_step call: L grouped reversible layers forward, head + loss, and the backward
sweep that rebuilds every layer input instead of storing it.  Inputs are synthetic (seeded circuit
DAG, N(0,1) features, Glorot weights) and resident in HBM before the timed region.  Prints ONE JSON
line: node-layers/s, the roofline of the dominant kernel (HIP events recorded by the library on the
stream it launches on, inside the timed region), the step-level roofline, how faithfully the step
rebuilds its input and its gradients, a sweep over the depth L (peak HBM against L), the other storage /
index modes, and the CPU oracle timed on the host cores.
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

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak
INDEX_MODES = {"none": 0, "all": 1, "near-ties": 2}
COUNTERS_JSON = os.path.join(ROOT, "profiles", "gsr_step_counters.json")


def measured_counters(workload_name, kernel):
    """HBM bytes per launch and pipe occupancy of one kernel class as the rocprofv3 --pmc passes recorded them
    (written by `python -m paper_2603_27156_amd.profile_summary`; the file names the commit and the commands).
    None when no pass was taken on this workload."""
    try:
        with open(COUNTERS_JSON) as f:
            rec = json.load(f)
    except (OSError, ValueError):
        return None, None
    w = rec.get("workloads", {}).get(workload_name)
    if not w or kernel not in w.get("kernels", {}):
        return None, None
    k = w["kernels"][kernel]
    return k, {"commit": w.get("commit", rec.get("commit")), "file": "profiles/gsr_step_counters.json", "summary": w.get("summary")}


def algorithmic_bytes(n, nnz, dg, k, c, b, rms):
    """Bytes each kernel class must move per launch, every array touched once (neighbour gathers
    counted once per source row: the compulsory traffic), averaged over the C launches of a layer.
    n rows, nnz stored adjacency entries, b bytes per stored element, mask = dg/8 bytes per row."""
    mask = dg // 8
    rec = k * b + mask                       # compressed record of one row
    csr = nnz * 8 + n * 4                    # column indices + edge values + row pointers
    emit_fwd = (c - 1) / c if c > 2 else 1.0  # launches that also write the record of their output
    emit_bwd = (c - 1) / c if c > 2 else 1.0
    row = dg * b
    fwd = n * (rec + 2 * row + emit_fwd * rec) + csr
    bwd = n * (rec + 3 * row + emit_bwd * rec) + csr
    ndst = ((c - 1) + (c - 1)) / c           # block 1 updates C-1 planes, blocks 2..C one plane each
    grad = n * (row + mask + (row if rms else 0) + 2 * row * ndst) + csr
    # float32 runs the backward's inverse and the weight gradient as two kernels with H (float32) passed through memory.
    # That H row written and read again is this implementation's doing, not the method's: it is left out, so the two
    # figures add up to block_backward, the method's own
    inv = n * (rec + 2 * row + emit_bwd * rec) + csr
    dwk = n * row
    return {"block_forward": fwd, "block_backward": bwd, "grad": grad, "block_inverse": inv, "weight_gradient": dwk}


def step_bytes(n, nnz, dg, k, c, b, rms, l):
    """Compulsory bytes of one whole step: per layer C forward, C inverse + dW and C gradient launches, plus the
    group sums of a layer when C > 2 (C-1 planes read and a record written, forward and backward; the backward also
    keeps the Y_0 plane)."""
    ab = algorithmic_bytes(n, nnz, dg, k, c, b, rms)
    per_layer = c * (ab["block_forward"] + ab["block_backward"] + ab["grad"])
    if c > 2:
        rec = k * b + dg // 8
        per_layer += n * ((c - 1) * dg * b + rec) + n * ((c - 1) * dg * b + dg * b + rec)
    return per_layer * l


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--layers", type=int, default=0, help="override L")
    ap.add_argument("--k", type=int, default=0, help="override k (sweep over the paper's K = 4 ... 64)")
    ap.add_argument("--c", type=int, default=0, help="override the number of groups C (dense workload: 2 is the paper's split, D/C = 192)")
    ap.add_argument("--max-workgroups", type=int, default=0, help="override the persistent grid (multiple of 8)")
    ap.add_argument("--index-mode", choices=sorted(INDEX_MODES), default=None,
                    help="what the forward sweep keeps for the inverse: the column sets of near-tie rows (default with "
                         "float32 storage; memory flat in L up to that list), all column sets (default with bf16 storage, "
                         "where near-ties are the rule; memory grows with L), or nothing")
    ap.add_argument("--save-indices", action="store_true", help="same as --index-mode all")
    ap.add_argument("--tie-tol", type=float, default=2.0 ** -12)
    ap.add_argument("--hub-threshold", type=int, default=0, help="rows longer than this are reduced in two passes")
    ap.add_argument("--hub-values", type=int, default=0, choices=[0, 1, 2],
                    help="first pass over float32 records: 1 a lane per value, 2 a lane per column group, 0 chosen per graph")
    ap.add_argument("--graph", action="store_true", help="capture the step into a HIP graph and time replays")
    ap.add_argument("--hub-chunk", type=int, default=0, help="neighbours per first-pass partial sum of such rows")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true", help="no per-kernel events in the timed region")
    ap.add_argument("--no-extras", action="store_true", help="skip the fidelity block, the depth sweep, the variants and the operators")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_2603_27156_amd as gsr
    from paper_2603_27156_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 3
    gsr.lib()
    dev = torch.device("cuda:0")

    idx = {"cfg0": 0, "cfg1": 1, "cfg2": 2, "cfg2-bf16": 2, "cfg4": 4, "dense": 5}[args.workload]
    w = synth.workload(idx)
    if args.workload == "cfg2-bf16":
        w = synth.workload(2, dtype="bf16", name="cfg2-1M-bf16")
    if args.layers > 0:
        w = synth.workload(idx, l=args.layers, dtype=w.dtype, name=w.name)
    if args.k > 0:
        w = synth.workload(idx, l=w.l, dtype=w.dtype, name=f"{w.name}-k{args.k}", k=args.k)
    if args.c > 0:
        w = synth.workload(idx, l=w.l, dtype=w.dtype, name=f"{w.name}-c{args.c}", k=w.k, c=args.c)
    if args.max_workgroups:
        gsr.gsr_set_option("max_workgroups", args.max_workgroups)
    if args.hub_threshold:
        gsr.gsr_set_option("hub_threshold", args.hub_threshold)
    if args.hub_values:
        gsr.gsr_set_option("hub_values", args.hub_values)
    if args.hub_chunk:
        gsr.gsr_set_option("hub_chunk", args.hub_chunk)
    t_gen = time.time()
    inp = synth.make_inputs(w, 0)
    g = gsr.gsr_graph_create(inp.rowptr, inp.colidx)
    info = gsr.gsr_graph_info(g)
    t_gen = time.time() - t_gen

    bf16 = w.dtype == "bf16"
    mode_name = "all" if args.save_indices else args.index_mode
    wide = w.dg > 64                    # groups of more than 64 columns run as column blocks; they take "all" or "none"
    if mode_name is None:
        mode_name = "all" if (bf16 or wide) else "near-ties"
    f32 = dict(dtype=torch.float32, device=dev)
    w_out = torch.from_numpy(inp.w_out).to(dev)
    b_out = torch.zeros(1, **f32)
    target = torch.from_numpy(inp.target).to(dev)
    x0_f32 = torch.from_numpy(inp.x0).to(dev).view(w.n, w.c, w.dg).permute(1, 0, 2).contiguous()

    class Run:
        """One configuration of the step with its buffers: everything gsr_step touches is allocated here, once."""

        def __init__(self, l, weights, mode, use_bf16=bf16):
            self.l, self.mode = l, mode
            self.cfg = gsr.Config(n=w.n, d=w.d, c=w.c, k=w.k, l=l, dtype=gsr.GSR_BF16 if use_bf16 else gsr.GSR_F32,
                                  norm=gsr.GSR_NORM_RMS if w.norm == "rms" else gsr.GSR_NORM_NONE, eps=1e-5,
                                  layout=gsr.GSR_LAYOUT_GROUP_PLANAR, save_indices=INDEX_MODES[mode], tie_tol=args.tie_tol)
            self.x0 = x0_f32.to(torch.bfloat16) if use_bf16 else x0_f32
            self.W = weights
            self.loss, self.db = torch.zeros(1, **f32), torch.zeros(1, **f32)
            self.dW, self.dw = torch.empty_like(weights), torch.empty(w.d, **f32)
            self.dx0, self.x0r = torch.empty_like(self.x0), torch.empty_like(self.x0)
            self.ws_bytes = gsr.gsr_workspace_size(g, self.cfg)[1]
            self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=dev)

        def step(self):
            gsr.gsr_step(g, self.cfg, self.x0, self.W, w_out, b_out, target, self.loss, self.dW, self.dw, self.db,
                         dx0_out=self.dx0, x0_rebuilt_out=self.x0r, workspace=self.ws)

        def timed(self, steps, warmup):
            for _ in range(warmup):
                self.step()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                self.step()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / steps

        def rebuild_error(self):
            e = (self.x0r.float() - self.x0.float()).abs().amax(dim=(0, 2))          # per row
            return float(e.max().item()), float((e > 1e-3).float().mean().item())

        def tie_stats(self):
            if self.mode != "near-ties":
                return None
            st = gsr.gsr_step_tie_stats(g, self.cfg, self.ws)
            st["listed_fraction_of_rows"] = st["listed"] / float(w.n * w.c * self.l)
            return st

    def rel(a, b):
        return float((a.double() - b.double()).norm() / b.double().norm().clamp_min(1e-300))

    W = torch.from_numpy(inp.weights).to(dev)
    main_run = Run(w.l, W, mode_name)
    step = main_run.step

    # Timed region: K steps, nothing but the library's launches on the stream.  With --graph the step is captured
    # once into a HIP graph (it only launches kernels) and the K steps are replays.
    gsr.gsr_set_option("profile", 0)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    run = step
    if args.graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        run = graph.replay
        run()
        torch.cuda.synchronize()
    torch.cuda.reset_peak_memory_stats()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    peak_hbm = int(torch.cuda.max_memory_allocated())
    # The same K steps once more with a pair of HIP events around every launch (on the launch stream) for the
    # per-kernel durations: the events themselves cost about 3 % of a step, which is why they are not in `value`.
    mask = 0 if args.no_profile else (1 << gsr.KERNEL_CLASSES) - 1
    ms_per_step_profiled = None
    if mask:
        gsr.gsr_set_option("profile", mask)
        gsr.gsr_profile_reset()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        ms_per_step_profiled = (time.perf_counter() - t1) * 1e3 / args.steps
        gsr.gsr_set_option("profile", 0)
    value = w.n * w.l * args.steps / dt
    rebuilt_err, rebuilt_rows = main_run.rebuild_error()

    kernels = {}
    for kc in range(gsr.KERNEL_CLASSES):
        ms, cnt = gsr.gsr_profile_read(kc)
        if cnt:
            kernels[gsr.gsr_profile_class_name(kc)] = {"launches_per_step": cnt // args.steps,
                                                       "avg_us": 1e3 * ms / cnt, "ms_per_step": ms / args.steps}
    bpe = 2 if bf16 else 4
    roofline = None
    if kernels:
        # (groups wider than 64 columns: a launch handles one 64-column block pair)
        ab = algorithmic_bytes(w.n, info["nnz"], min(w.dg, 64), w.k, w.c, bpe, w.norm == "rms")
        cand = {k: v for k, v in kernels.items() if k in ab}
        dom = max(cand, key=lambda k: cand[k]["ms_per_step"])
        achieved = ab[dom] / (cand[dom]["avg_us"] * 1e-6) / 1e9
        counted, source = measured_counters(w.name, dom)
        roofline = {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK_GBS,
                    "traffic": counted.get("hbm_bytes_per_launch") if counted else None,
                    "algorithmic_bytes_per_launch": ab[dom], "avg_launch_us": cand[dom]["avg_us"],
                    "pipes": counted.get("pipes") if counted else None, "counters_from": source}
        for k in cand:
            kernels[k]["algorithmic_GBps"] = ab[k] / (cand[k]["avg_us"] * 1e-6) / 1e9
            kernels[k]["frac_of_hbm_peak"] = kernels[k]["algorithmic_GBps"] / HBM_PEAK_GBS
    sb = step_bytes(w.n, info["nnz"], w.dg, w.k, w.c, bpe, w.norm == "rms", w.l)
    step_roofline = {"bound": "hbm", "compulsory_bytes_per_step": sb, "achieved": sb / (ms_per_step * 1e-3) / 1e9,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": sb / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS}

    extras = not args.no_extras
    # How faithfully the step rebuilds its input and its gradients: the same step with all column sets of the
    # forward sweep kept (whose inverse is continuous in its input and whose gradients are those of plain
    # back-propagation to rounding: pinned against stored activations in the tests) and with nothing kept.
    fidelity = {"index_mode": mode_name, "x0_rebuild_max_abs_err": rebuilt_err, "rows_rebuilt_off_by_more_than_1e-3": rebuilt_rows,
                "near_tie_rows": main_run.tie_stats()}
    variants = {}
    if extras and w.l * w.n <= 120_000_000:
        others = {}
        for m in ("all", "none", "near-ties"):
            if m == mode_name or (wide and m == "near-ties"):
                continue
            r = Run(w.l, W, m)
            ms = r.timed(1, 1)
            err, rows = r.rebuild_error()
            others[m] = r
            variants[f"index_mode={m}"] = {"ms_per_step": ms, "value": w.n * w.l / (ms * 1e-3), "workspace_bytes": r.ws_bytes,
                                           "x0_rebuild_max_abs_err": err, "rows_rebuilt_off_by_more_than_1e-3": rows,
                                           "near_tie_rows": r.tie_stats()}
        ref = main_run if mode_name == "all" else others["all"]
        for name, r in [(mode_name, main_run)] + [(m, o) for m, o in others.items()]:
            if r is ref:
                continue
            per_layer = [rel(r.dW[l], ref.dW[l]) for l in range(w.l)]
            fidelity[f"{name}_vs_all_indices_kept"] = {"dW_rel_err_max_over_layers": max(per_layer), "dW_rel_err_layer0": per_layer[0],
                                                       "dW_rel_err_all": rel(r.dW, ref.dW), "dX0_rel_err": rel(r.dx0, ref.dx0),
                                                       "dw_out_rel_err": rel(r.dw, ref.dw)}
        del others, ref
        torch.cuda.empty_cache()

    main_run.ws = None            # (its counts have been read; the sweeps below allocate their own)
    torch.cuda.empty_cache()
    # Depth sweep (the graph and X0 of this workload at L = 8 .. 448; weights of one 448-layer draw, prefixes used):
    # peak HBM against L, one timed step each.
    depth_sweep = None
    if extras and idx == 2 and not args.layers and not args.k and not args.c:
        depth_sweep = []
        deep = torch.from_numpy(synth.glorot_uniform(np.random.Generator(np.random.PCG64(1)), w.dg, w.dg,
                                                     (448, w.c, w.dg, w.dg))).to(dev)
        base_alloc = None
        for L in (8, 56, 224, 448):
            torch.cuda.synchronize()
            torch.cuda.empty_cache()
            torch.cuda.reset_peak_memory_stats()
            before = torch.cuda.memory_allocated()
            r = Run(L, deep[:L].contiguous(), mode_name)
            ms = r.timed(1, 1)
            peak = int(torch.cuda.max_memory_allocated())      # before anything else allocates
            err, rows = r.rebuild_error()
            st = r.tie_stats()
            weights_bytes = 2 * L * w.c * w.dg * w.dg * 4
            depth_sweep.append({"l": L, "ms_per_step": ms, "value": w.n * L / (ms * 1e-3),
                                "peak_hbm_bytes": peak, "bytes_allocated_for_the_step": peak - before,
                                "workspace_bytes": r.ws_bytes, "weights_and_weight_gradients_bytes": weights_bytes,
                                "x0_rebuild_max_abs_err": err, "rows_rebuilt_off_by_more_than_1e-3": rows,
                                "near_tie_rows_fraction": st["listed_fraction_of_rows"] if st else None,
                                "near_tie_rows_dropped": st["dropped"] if st else None})
            del r
        del deep
        torch.cuda.empty_cache()
    if extras and idx == 2 and not bf16 and not args.layers and not args.k and not args.c:
        r = Run(w.l, W, "all", use_bf16=True)
        ms = r.timed(1, 1)
        err, rows = r.rebuild_error()
        variants["bf16 storage, index_mode=all"] = {"ms_per_step": ms, "value": w.n * w.l / (ms * 1e-3), "workspace_bytes": r.ws_bytes,
                                                    "x0_rebuild_max_abs_err": err, "rows_rebuilt_off_by_more_than_1e-3": rows,
                                                    "loss": float(r.loss.item())}
        del r
        torch.cuda.empty_cache()

    # the operators exposed on their own, on one group plane of the same workload (outside the timed step)
    operators = None
    if extras and w.dg in (32, 64) and not args.no_profile:
        def avg_us(f, reps=5):
            f()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                f()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps * 1e3
        plane = x0_f32[0].contiguous()                             # [n, dg]
        row, nnz = w.dg * 4, info["nnz"]
        csr = nnz * 8 + w.n * 4
        norm = main_run.cfg.norm
        t_spmm = avg_us(lambda: gsr.gsr_spmm(g, plane))
        t_gs = avg_us(lambda: gsr.gsr_group_sparse(plane, w.k, norm))
        vv, ii = gsr.gsr_group_sparse(plane, w.k, norm)
        t_agg = avg_us(lambda: gsr.gsr_spmm_compressed(g, vv, ii, w.dg))
        def entry(us, nbytes):
            return {"avg_us": us, "algorithmic_GBps": nbytes / (us * 1e-6) / 1e9, "frac_of_hbm_peak": nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS}
        # the two-group pipeline of the Section 4.3 / 4.4 walk-throughs on two such planes
        pa, pb = plane.clone(), x0_f32[1].contiguous()
        t_slot = avg_us(lambda: gsr.gsr_slot_block(g, vv.float(), ii, w.dg))
        t_alg1 = avg_us(lambda: gsr.gsr_alg1_layer_forward(g, pa, pb, w.k), reps=3)
        pa.mul_(1e-3 / max(float(pa.abs().max()), 1e-30)); pb.mul_(1e-3 / max(float(pb.abs().max()), 1e-30))
        t_alg2 = avg_us(lambda: gsr.gsr_alg2_layer_backward(g, pa, pb, w.k), reps=3)
        del pa, pb
        operators = {
            "gsr_slot_block": entry(t_slot, w.n * (w.k * 8 + row) + csr),
            "gsr_alg1_layer_forward": entry(t_alg1, w.n * 4 * row + 2 * csr),
            "gsr_alg2_layer_backward": entry(t_alg2, w.n * 4 * row + 4 * csr),
            "gsr_spmm": entry(t_spmm, w.n * 2 * row + csr),
            "gsr_group_sparse": entry(t_gs, w.n * (row + w.k * 8)),
            "gsr_spmm_compressed": entry(t_agg, w.n * (w.k * 8 + row) + csr),
            "note": "float32, one group plane [n, dg]; compulsory bytes; gsr_spmm_compressed includes the conversion of "
                    "(V, I int32) into records, its index check and one host synchronisation; gsr_slot_block / gsr_alg1 / "
                    "gsr_alg2: the pipeline as the walk-throughs of Sections 4.3 / 4.4 print it (two planes, no weights), "
                    "bytes = both planes read and written once plus the edge lists of its 2 / 4 products",
        }
        del plane, vv, ii

    cpu_baseline = None
    parity = None
    if not args.no_cpu_baseline:
        import oracle
        # bounded sample: the first layers of the same recipe, at most 1M nodes (10-30 s of CPU work)
        ws_n, ws_l = min(w.n, 1_000_000), min(w.l, 4 if w.c <= 4 else 2)
        sw = synth.scaled(w, ws_n, l=ws_l) if ws_n < w.n else synth.workload(idx, l=ws_l, dtype=w.dtype)
        sinp = synth.make_inputs(sw, 0)
        og = oracle.graph_build(sinp.rowptr, sinp.colidx)
        ocfg = oracle.Cfg(sw.d, sw.c, sw.k, oracle.NORM_RMS if sw.norm == "rms" else oracle.NORM_NONE, 1e-5,
                          oracle.STORE_BF16 if bf16 else oracle.STORE_F32)
        variant = {"none": 0, "all": 2, "near-ties": 3}[mode_name]
        same_graph = sw.n == w.n and not wide      # then the library's graph serves the sample as well
        tc = time.perf_counter()
        ref = oracle.step(og, ocfg, sw.l, sinp.x0, sinp.weights, sinp.w_out, 0.0, sinp.target, variant=variant,
                          want=("X0rec", "dW", "dwout", "dX0") if same_graph else (), tie_tol=args.tie_tol)
        tc = time.perf_counter() - tc
        if same_graph:
            # the same sample through the library, compared with the oracle just timed (element-wise bar of the
            # parity tests: |a - b| <= atol + rtol |b|; rows a near-tie decides differently are not taken out here)
            scfg = gsr.Config(n=sw.n, d=sw.d, c=sw.c, k=sw.k, l=sw.l, dtype=gsr.GSR_BF16 if bf16 else gsr.GSR_F32,
                              norm=gsr.GSR_NORM_RMS if sw.norm == "rms" else gsr.GSR_NORM_NONE, eps=1e-5,
                              layout=gsr.GSR_LAYOUT_GROUP_PLANAR, save_indices=INDEX_MODES[mode_name], tie_tol=args.tie_tol)
            sx0 = torch.from_numpy(sinp.x0).to(dev).view(sw.n, sw.c, sw.dg).permute(1, 0, 2).contiguous()
            sx0 = sx0.to(torch.bfloat16) if bf16 else sx0
            sW = torch.from_numpy(sinp.weights).to(dev)
            sloss, sdb = torch.zeros(1, **f32), torch.zeros(1, **f32)
            sdW, sdw = torch.empty_like(sW), torch.empty(sw.d, **f32)
            sdx0, sx0r = torch.empty_like(sx0), torch.empty_like(sx0)
            sws = torch.empty(gsr.gsr_workspace_size(g, scfg)[1], dtype=torch.uint8, device=dev)
            gsr.gsr_step(g, scfg, sx0, sW, torch.from_numpy(sinp.w_out).to(dev), torch.zeros(1, **f32),
                         torch.from_numpy(sinp.target).to(dev), sloss, sdW, sdw, sdb, dx0_out=sdx0, x0_rebuilt_out=sx0r,
                         workspace=sws)
            torch.cuda.synchronize()
            rtol, atol = (1e-2, 1e-2) if bf16 else (1e-4, 1e-5)

            def cmp(got, want):
                got, want = np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64)
                diff = np.abs(got - want)
                return {"max_abs_err": float(diff.max()), "rel_norm_err": float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300)),
                        "fraction_outside_bar": float(np.mean(diff > atol + rtol * np.abs(want)))}

            rows = lambda t: t.float().permute(1, 0, 2).reshape(sw.n, sw.d).cpu().numpy()
            parity = {"rtol": rtol, "atol": atol, "loss_rel_err": abs(float(sloss.item()) - ref["loss"]) / abs(ref["loss"]),
                      "dW": cmp(sdW.cpu().numpy(), ref["dW"]), "dw_out": cmp(sdw.cpu().numpy(), ref["dwout"]),
                      "dX0": cmp(rows(sdx0), ref["dX0"]), "X0_rebuilt": cmp(rows(sx0r), ref["X0rec"]),
                      "near_tie_rows_listed": {"library": gsr.gsr_step_tie_stats(g, scfg, sws)["listed"] if mode_name == "near-ties" else None,
                                               "oracle": int(ref["n_listed"]) if mode_name == "near-ties" else None}}
            del sws, sx0, sdx0, sx0r, ref
        cpu_baseline = {"value": sw.n * sw.l / tc, "unit": "node-layers/s", "cores": oracle.num_threads(),
                        "kind": "oracle", "seconds": tc,
                        "sample": f"same recipe at N={sw.n} nodes, L={sw.l} layers (D={sw.d}, C={sw.c}, k={sw.k}), one full step, "
                                  f"index mode {mode_name}"}

    out = {
        "metric": "node-layers/sec (fwd+inverse+bwd)", "value": value, "unit": "node-layers/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16-storage/f32-accumulate" if bf16 else "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "n": w.n, "nnz": info["nnz"], "max_degree": info["max_degree"], "d": w.d,
                   "c": w.c, "k": w.k, "l": w.l, "norm": w.norm, "hub_rows": info["n_hub_rows"],
                   "index_mode": mode_name, "tie_tol": args.tie_tol if mode_name == "near-ties" else None},
        "ms_per_step_with_kernel_events": ms_per_step_profiled, "hip_graph": bool(args.graph),
        "roofline": roofline, "step_roofline": step_roofline, "cpu_baseline": cpu_baseline, "kernels": kernels,
        "parity_vs_oracle": parity, "fidelity": fidelity, "depth_sweep": depth_sweep, "variants": variants or None, "operators": operators,
        "peak_hbm_bytes": peak_hbm, "workspace_bytes": int(main_run.ws_bytes),
        "loss": float(main_run.loss.item()), "x0_rebuild_max_abs_err": rebuilt_err, "setup_seconds": t_gen,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
