#!/usr/bin/env python3
"""Benchmark of the level sweep (dg4_layer_fwd) on one MI355X.

One step = one pass of the whole hot path over the 1M-gate "large" synthetic AIG: projections, per-edge
scores, segmented softmax, aggregation, output projection + LayerNorm, swept over the whole circuit.
Inputs are resident in HBM before the timed region; graph analysis and uploads are reported separately
and excluded; the weights are brought into matrix-core operand order once, before the timed region
(DG4_WEIGHTS_PACKED; the step with the packing launches inside is reported beside it). Prints ONE JSON
line. The default run also carries: `configs` (the other four configurations of the workload list, each
through the path the library picks for it, plus a 12-layer stack), `level_order_tiles` (the same step
forced through the graph's own 1001 levels), kernel points, the layer with its feed-forward sub-block,
and a point under the paper's general partition and updating strategy (`partition`).
`--ffn` times the layer with its feed-forward sub-block instead (not the headline configuration);
`--partition K,STRIDE,BATCH` times the layer under the general partition.

Roofline accounting: algorithmic bytes are counted on the levelling the timed schedule is free to
follow. The default schedule of a whole-graph sweep is driven by the dependencies, i.e. by the circuit's
Eq. 1 levels, so its compulsory K|V reads are one per DISTINCT (Eq. 1 level, source) pair; the
`level_order_tiles` run follows the graph's own (assigned) levels and is priced on those.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def measured_traffic(profile: str, kernel: str):
    """HBM bytes per launch of `kernel` from a committed rocprofv3 summary (FETCH_SIZE + WRITE_SIZE,
    calibrated against a plain copy there), or None."""
    try:
        text = open(os.path.join(ROOT, "profiles", profile)).read()
    except OSError:
        return None
    m = re.search(r"^.*" + re.escape(kernel) + r".*total\s+([0-9.]+) GB\s*$", text, flags=re.M)
    return float(m.group(1)) * 1e9 if m else None


def algorithmic_bytes(g, cfg, level):
    """Bytes the method has to move for one sweep scheduled by `level` (per-gate figures of the design notes).

    Per gate and layer: read the state row R, write the new state row R, write the gate's K and V
    rows 2R, read its packed neighbour row. Per level and layer: read the K and V rows of the
    DISTINCT sources of the level once (compulsory traffic), 2R each. `gathered` counts every
    neighbour entry instead (what a cache-less gather moves).
    """
    es = 4 if cfg.dtype == "f32" else 2
    R = cfg.hidden * es
    ptr, idx = g.array("nbr_ptr"), g.array("nbr_idx")
    n = g.n
    dst = np.repeat(np.arange(n, dtype=np.int64), np.diff(ptr))
    keep = idx != dst                                   # sources other than the gate itself
    dl, src = level[dst[keep]].astype(np.int64), idx[keep].astype(np.int64)
    distinct = len(np.unique(dl * n + src))
    # neighbour rows: fixed width up to three hops, else the entries themselves
    ell_bytes = n * 4 * (1 << (g.hops + 1)) if g.hops <= 3 else 4 * (len(src) + n)
    per_gate = (R + R + 2 * R) * cfg.n_layers
    compulsory = n * per_gate + ell_bytes * cfg.n_layers + distinct * 2 * R * cfg.n_layers
    gathered = n * per_gate + ell_bytes * cfg.n_layers + len(src) * 2 * R * cfg.n_layers
    return compulsory, gathered


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="large", help="large (default) | medium | small | tiny | stress")
    ap.add_argument("--n-and", type=int, default=None, help="override the number of AND gates (debug)")
    ap.add_argument("--layers", type=int, default=None, help="override the number of stacked layers")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-points", action="store_true",
                    help="skip the stand-alone timings of dg4_qkv_proj and dg4_sparse_attn_fwd over all rows")
    ap.add_argument("--no-level-order", action="store_true",
                    help="skip the extra run with level-ordered tiles (for profiles of the default path only)")
    ap.add_argument("--no-configs", action="store_true", help="skip the timings of the other configurations")
    ap.add_argument("--ffn", action="store_true",
                    help="time the layer WITH its feed-forward sub-block (not the headline configuration; "
                         "the roofline object then prices the step's matrix products against the MFMA peak)")
    ap.add_argument("--partition", default=None, metavar="K,STRIDE,BATCH",
                    help="time the layer under the general partition and updating strategy (cones of depth K "
                         "collected every STRIDE levels, mini-batches of BATCH cones) instead of the headline sweep")
    ap.add_argument("--no-partition-point", action="store_true",
                    help="skip the extra measurement of the partitioned layer (medium graph, k=8, stride 6, 128 cones)")
    ap.add_argument("--level-order", action="store_true",
                    help="the timed sweep follows the graph's own (assigned) levels (DG4_LEVEL_ORDER) and is priced on them")
    ap.add_argument("--per-level", action="store_true", help="force level-by-level launches (DG4_PER_LEVEL)")
    ap.add_argument("--bounded-kv", action="store_true", help="no K|V store (DG4_BOUNDED_KV)")
    ap.add_argument("--cpu-gates", type=int, default=800_000, help="gates in the oracle's timed sample")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device copy (reference point for rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch

    import dg4_synth as synth
    import paper_2502_01681_amd as dg4

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        # a copy kernel of known size: reads 1 GiB, writes 1 GiB per launch
        a = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_(0, 255)
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": 1 << 30, "copy_bytes_written": 1 << 30, "launches": 3}))
        return

    def tensors(w, c, ffn=False):
        td = torch.float32 if c.dtype == "f32" else torch.bfloat16
        X = torch.from_numpy(w.x).cuda().to(td).contiguous()
        W = [(torch.from_numpy(w.wqkv[l]).cuda().to(td).contiguous(), torch.from_numpy(w.wo[l]).cuda().to(td).contiguous(),
              torch.from_numpy(w.rel_bias[l]).cuda().contiguous()) for l in range(c.n_layers)]
        if ffn:
            fw1, fw2 = synth.ffn_weights(c)
            W = [W[l] + (torch.from_numpy(fw1[l]).cuda().to(td).contiguous(), torch.from_numpy(fw2[l]).cuda().to(td).contiguous())
                 for l in range(c.n_layers)]
        return X, W

    def eq1_levels(w, c, g):
        """The circuit's logic levels by Eq. 1 (the graph's own levels may be a deeper, assigned levelling)."""
        if w.level_hint is None:
            return g.array("level")
        g1 = dg4.dg4_build_levels(c.n_nodes, w.edge_src, w.edge_dst, w.edge_inv, c.hops)
        lev = g1.array("level")
        g1.close()
        return lev

    def time_layer(c, g, X, W, steps, warmup, **flags):
        """Device time of `steps` calls of dg4_layer_fwd (events on the stream), the persistent kernel's own
        time where there is one, and the step with the weight packing inside."""
        kw = dict(hidden=c.hidden, heads=c.heads, hops=g.hops, n_layers=c.n_layers, dtype=c.dtype)
        kw.update(flags)
        cold = dg4.LayerConfig(**kw)
        hot = dg4.LayerConfig(**{**kw, "weights_packed": True, "time_sweep": True})
        H = torch.empty_like(X)
        ws = torch.empty(dg4.dg4_layer_workspace_bytes(cold, g), dtype=torch.uint8, device="cuda")
        for _ in range(max(warmup, 1)):
            dg4.dg4_layer_fwd(cold, g, X, W, H, workspace=ws)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        dg4.dg4_layer_fwd(cold, g, X, W, H, workspace=ws)
        b.record()
        torch.cuda.synchronize()
        ms_cold = a.elapsed_time(b)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        sweep_ms = []
        t0 = time.perf_counter()
        for a, b in ev:
            a.record()
            dg4.dg4_layer_fwd(hot, g, X, W, H, workspace=ws)
            b.record()
            try:
                sweep_ms.append(dg4.dg4_sweep_elapsed_ms())     # waits for this step's persistent kernel
            except dg4.DG4Error:
                pass                                            # a path without one
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        dg4.dg4_layer_status(hot, g, ws)                        # raises if a persistent sweep gave up
        ms_dev = float(np.mean([a.elapsed_time(b) for a, b in ev]))
        return {"ms_wall": wall * 1e3 / steps, "ms_dev": ms_dev, "ms_with_packing": ms_cold,
                "ms_kernel": float(np.mean(sweep_ms)) if len(sweep_ms) == steps else None, "H": H, "ws": ws, "cfg": hot}

    def path_of(c, g, flags):
        if flags.get("per_level") or flags.get("bounded_kv"):
            return "level-by-level launches"
        if c.dtype == "bf16" and c.hidden == 256 and c.n_layers == 1 and g.hops <= 2:
            return "sweep_kernel (persistent, weights resident in registers)"
        if flags.get("ffn") and g.hops > 3:
            return "level-by-level launches"
        return "flow_kernel (persistent, weights streamed" + (", several lane groups per neighbour row)" if g.hops > 3 else ")")

    t0 = time.perf_counter()
    over = {}
    if args.n_and is not None:
        over["n_and"] = args.n_and
    if args.layers is not None:
        over["n_layers"] = args.layers
    base = synth.CONFIGS[args.workload]
    w = synth.make(synth.Config(**{**base.__dict__, **over}))
    c = w.cfg
    t_gen = time.perf_counter() - t0
    part = [int(t) for t in args.partition.split(",")] if args.partition else None
    if part:
        c = synth.Config(**{**c.__dict__, "hops": part[0]})
    t0 = time.perf_counter()
    if part:
        g = dg4.dg4_build_partitioned(c.n_nodes, w.edge_src, w.edge_dst, w.edge_inv, part[0], part[1], part[2], w.level_hint)
    else:
        g = dg4.dg4_build_levels(c.n_nodes, w.edge_src, w.edge_dst, w.edge_inv, c.hops, w.level_hint)
    t_build = time.perf_counter() - t0
    # the same analysis on the GPU, edge list resident in device memory (second call timed: the first pays
    # for module loading)
    e_dev = [torch.from_numpy(a).cuda() for a in (w.edge_src, w.edge_dst, w.edge_inv)]
    h_dev = torch.from_numpy(w.level_hint).cuda() if w.level_hint is not None else None
    t_build_dev = None
    for _ in range(2):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        if part:
            g_dev = dg4.dg4_build_partitioned_device(c.n_nodes, *e_dev, part[0], part[1], part[2], h_dev)
        else:
            g_dev = dg4.dg4_build_levels_device(c.n_nodes, *e_dev, c.hops, h_dev)
        t_build_dev = time.perf_counter() - t0
        del g_dev
    del e_dev, h_dev
    t0 = time.perf_counter()
    X, W = tensors(w, c, ffn=args.ffn)
    g.upload()
    torch.cuda.synchronize()
    t_upload = time.perf_counter() - t0

    flags = dict(ffn=args.ffn, per_level=args.per_level, bounded_kv=args.bounded_kv, level_order=args.level_order)
    r = time_layer(c, g, X, W, args.steps, args.warmup, **flags)
    ms_step, ms_dev = r["ms_wall"], r["ms_dev"]
    ms_kernel = r["ms_kernel"] if r["ms_kernel"] is not None else ms_dev
    cfg = r["cfg"]

    n_gates, nnz = g.n, g.nnz
    layers = c.n_layers
    lev_eq1 = eq1_levels(w, c, g)
    depth_eq1 = int(lev_eq1.max()) + 1 if n_gates else 0
    sched_level = g.array("level") if args.bounded_kv or args.level_order else lev_eq1       # (bounded sweeps go through the graph's own levels)
    compulsory, gathered = algorithmic_bytes(g, cfg, sched_level)
    comp_hint, _ = algorithmic_bytes(g, cfg, g.array("level"))
    # The persistent kernel performs every algorithmic transfer of the step itself (residual row in, H
    # and K|V rows out, neighbour rows, one K|V read per distinct source and level); the Q|K|V rows of x
    # that the bulk projection hands it are an implementation detail and are NOT counted.
    achieved = compulsory / (ms_kernel * 1e-3) / 1e9
    persistent = r["ms_kernel"] is not None
    kernel_name = path_of(c, g, flags).split(" ")[0] if persistent else "dg4_layer_fwd"
    out = {
        "metric": "edges/sec per sparse-attn layer fwd (level sweep)",
        "value": nnz * layers / (ms_step * 1e-3),
        "unit": "edges/s",
        "gates_per_s": n_gates * layers / (ms_step * 1e-3),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "ms_per_layer": ms_step / layers,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": c.dtype, "data": "synthetic",
        "config": {"workload": f"{c.name}: {c.n_pi} PIs + {c.n_and} ANDs, {g.n_levels} assigned levels "
                               f"(Eq. 1 depth {depth_eq1}), {c.hops}-hop cones, hidden {c.hidden}, {c.heads} heads, "
                               f"{layers} layer(s); weights packed once before the timed region",
                   "gates": n_gates, "neighbour_edges": nnz, "aig_edges": int(len(w.edge_src)),
                   "levels": g.n_levels, "eq1_depth": depth_eq1, "path": path_of(c, g, flags)},
        "roofline": {"bound": "hbm",
                     "kernel": f"{kernel_name} (persistent level sweep, " + ("tiles by assigned level)" if args.level_order else "dependency-driven tile order)") if persistent
                               else "dg4_layer_fwd (all launches of one step)",
                     "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": measured_traffic("large_sweep_rocprofv3.txt", "sweep_kernel") if c.name == "large" and persistent
                                and not part and not args.ffn and args.n_and is None else None,
                     "accounting": "one K|V read per distinct (Eq. 1 level, source) pair: the levels the timed schedule "
                                   "is free to follow" if sched_level is lev_eq1 else "one K|V read per distinct (assigned level, source) pair",
                     "algorithmic_bytes": compulsory, "algorithmic_bytes_on_assigned_levels": comp_hint,
                     "gathered_bytes": gathered,
                     "kernel_ms": ms_kernel, "step_ms_device": ms_dev, "step_ms_device_with_weight_packing": r["ms_with_packing"],
                     "step_achieved": compulsory / (ms_dev * 1e-3) / 1e9,
                     "step_frac": compulsory / (ms_dev * 1e-3) / 1e9 / HBM_PEAK_GBPS},
        "setup_s": {"generate": t_gen, "dg4_build_partitioned" if part else "dg4_build_levels": t_build,
                    "dg4_build_partitioned_device" if part else "dg4_build_levels_device": t_build_dev, "upload": t_upload},
    }
    if part:
        out["config"]["workload"] += f", partition: stride {part[1]}, mini-batches of {part[2]} cones, marks"
        out["config"]["cones"] = int(len(g.array("cone_root")))
        out["config"]["mini_batches"] = int(g.array("stage").max()) + 1 if g.n else 0
    if args.ffn:
        # With the feed-forward sub-block the step is bound by its matrix products and by the weight
        # stream that feeds them, not by HBM: per gate and layer 2*d*3d (Q|K|V of x) + 2*d*d (Wo) +
        # 2*d*2d (K|V of H) + 16*d*d (feed-forward) flop.
        d = c.hidden
        flop = float(n_gates) * layers * (6 * d * d + 2 * d * d + 4 * d * d + 16 * d * d)
        peak = 2500.0 if c.dtype == "bf16" else 157.3
        out["config"]["workload"] += " + feed-forward sub-block (4x hidden)"
        hbm = out["roofline"]
        out["roofline"] = {"bound": "mfma", "kernel": hbm["kernel"], "achieved": flop / (ms_dev * 1e-3) / 1e12,
                           "peak": peak, "unit": "TFLOP/s", "frac": flop / (ms_dev * 1e-3) / 1e12 / peak,
                           "traffic": None, "flop": flop, "kernel_ms": ms_kernel, "step_ms_device": ms_dev,
                           "hbm_algorithmic_bytes": compulsory, "hbm_frac": hbm["frac"]}
    H = r["H"]
    del r

    headline = args.workload == "large" and args.n_and is None and args.layers is None and not part and not args.ffn \
        and not args.per_level and not args.bounded_kv and not args.level_order

    # For information: the same step with the tiles dealt strictly level by level (the graph's own,
    # assigned levels) instead of the library's dependency-driven order. Same results, bit for bit.
    # Priced on the assigned levels: that schedule cannot share a source between two of them.
    if persistent and not args.no_level_order and not args.level_order and not args.ffn and not part:
        lo = time_layer(c, g, X, W, args.steps, args.warmup, level_order=True)
        k = lo["ms_kernel"] if lo["ms_kernel"] is not None else lo["ms_dev"]
        out["level_order_tiles"] = {"step_ms_device": lo["ms_dev"], "kernel_ms": k,
                                    "algorithmic_bytes": comp_hint,
                                    "roofline_frac": comp_hint / (k * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                                    "step_frac": comp_hint / (lo["ms_dev"] * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                                    "edges_per_s": nnz * layers / (lo["ms_dev"] * 1e-3)}
        del lo

    # The two non-recurrent calls over all rows at once, as pure-kernel roofline points
    # (bf16 MFMA peak 2.5 PFLOP/s dense; both are HBM-bound at this size).
    if not args.no_kernel_points and not args.ffn and not part:
        def timed(fn, reps=5):
            for _ in range(2):
                fn()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / reps
        td = torch.float32 if c.dtype == "f32" else torch.bfloat16
        kcfg = dg4.LayerConfig(c.hidden, c.heads, c.hops, c.n_layers, c.dtype)
        es = 4 if c.dtype == "f32" else 2
        R = c.hidden * es
        Q, K, V, A = (torch.empty_like(X) for _ in range(4))
        pws = torch.empty(dg4.dg4_proj_workspace_bytes(kcfg), dtype=torch.uint8, device="cuda")
        ms_p = timed(lambda: dg4.dg4_qkv_proj(kcfg, X, W[0][0], Q, K, V, workspace=pws))
        flop_p = 2.0 * n_gates * c.hidden * 3 * c.hidden
        ms_a = timed(lambda: dg4.dg4_sparse_attn_fwd(kcfg, g, Q, K, V, W[0][2], A))
        bytes_a = n_gates * 2 * R + (nnz - n_gates) * 2 * R + n_gates * 4 * (1 << (c.hops + 1))
        peak_flops = 2.5e15 if c.dtype == "bf16" else 157.3e12
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        ms_c = timed(lambda: dst.copy_(src))
        out["roofline"]["measured_copy_GBps"] = 2 * (1 << 30) / (ms_c * 1e-3) / 1e9     # 1 GiB read + 1 GiB written
        del src, dst
        out["kernel_points"] = {
            "dg4_qkv_proj": {"ms": ms_p, "GB/s": n_gates * 4 * R / (ms_p * 1e-3) / 1e9,
                             "TFLOP/s": flop_p / (ms_p * 1e-3) / 1e12,
                             "mfma_frac": flop_p / (ms_p * 1e-3) / peak_flops, "hbm_frac": n_gates * 4 * R / (ms_p * 1e-3) / 1e9 / HBM_PEAK_GBPS},
            # compulsory: every Q, K, V row read once, every A row written once, the neighbour rows
            "dg4_sparse_attn_fwd": {"ms": ms_a, "GB/s_gathered": bytes_a / (ms_a * 1e-3) / 1e9,
                                    "GB/s_compulsory": n_gates * (4 * R + 4 * (1 << (c.hops + 1))) / (ms_a * 1e-3) / 1e9,
                                    "hbm_frac_compulsory": n_gates * (4 * R + 4 * (1 << (c.hops + 1))) / (ms_a * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                                    "edges_per_s": nnz / (ms_a * 1e-3)}}
        emb = torch.from_numpy(synth.normal(c.seed + 7, 9, (6, c.hidden), 0.25, False)).cuda()
        ms_s = timed(lambda: dg4.dg4_struct_encode(kcfg, g, X, emb, A))
        bytes_s = n_gates * (2 * R + 12)                       # a row in, a row out, three integers
        out["kernel_points"]["dg4_struct_encode"] = {"ms": ms_s, "GB/s": bytes_s / (ms_s * 1e-3) / 1e9,
                                                     "hbm_frac": bytes_s / (ms_s * 1e-3) / 1e9 / HBM_PEAK_GBPS}
        # the feed-forward sub-block over all rows: 16 d^2 flop per row against 2 rows of traffic, MFMA-bound
        fws = torch.empty(dg4.dg4_ffn_workspace_bytes(kcfg), dtype=torch.uint8, device="cuda")
        W1, W2 = (torch.from_numpy(t[0]).cuda().to(td).contiguous() for t in synth.ffn_weights(c))
        ms_f = timed(lambda: dg4.dg4_ffn_fwd(kcfg, X, W1, W2, A, workspace=fws))
        flop_f = 16.0 * n_gates * c.hidden * c.hidden
        out["kernel_points"]["dg4_ffn_fwd"] = {"ms": ms_f, "TFLOP/s": flop_f / (ms_f * 1e-3) / 1e12,
                                               "mfma_frac": flop_f / (ms_f * 1e-3) / peak_flops,
                                               "GB/s": n_gates * 2 * R / (ms_f * 1e-3) / 1e9}
        # the layer with the feed-forward sub-block after the attention sub-block
        FX, FW = tensors(w, c, ffn=True)
        fl = time_layer(c, g, FX, FW, 3, 2, ffn=True)
        out["ffn_layer"] = {"step_ms_device": fl["ms_dev"], "edges_per_s": nnz * layers / (fl["ms_dev"] * 1e-3),
                            "gates_per_s": n_gates * layers / (fl["ms_dev"] * 1e-3)}
        del Q, K, V, A, fl, FX, FW

    # The other configurations of the workload list, each through the path the library picks for it.
    if headline and not args.no_configs:
        def one(name, steps, warmup, over=None, **fl):
            t0 = time.perf_counter()
            cw = synth.make(synth.Config(**{**synth.CONFIGS[name].__dict__, **(over or {})}))
            cc = cw.cfg
            cg = dg4.dg4_build_levels(cc.n_nodes, cw.edge_src, cw.edge_dst, cw.edge_inv, cc.hops, cw.level_hint)
            CX, CW = tensors(cw, cc)
            FW = tensors(cw, cc, ffn=True)[1] if any(f.get("ffn") for f in fl.values()) else None
            cg.upload()
            setup = time.perf_counter() - t0
            lev = eq1_levels(cw, cc, cg)
            res = {}
            for label, f in fl.items():
                rr = time_layer(cc, cg, CX, FW if f.get("ffn") else CW, steps, warmup, **f)
                comp, gath = algorithmic_bytes(cg, rr["cfg"], cg.array("level") if f.get("bounded_kv") else lev)
                res[label] = {"path": path_of(cc, cg, f), "step_ms_device": rr["ms_dev"], "kernel_ms": rr["ms_kernel"],
                              "step_ms_device_with_weight_packing": rr["ms_with_packing"],
                              "edges_per_s": cg.nnz * cc.n_layers / (rr["ms_dev"] * 1e-3),
                              "gates_per_s": cg.n * cc.n_layers / (rr["ms_dev"] * 1e-3),
                              "algorithmic_bytes": comp, "gathered_bytes": gath,
                              "hbm_frac": comp / (rr["ms_dev"] * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                              "workspace_bytes": int(rr["ws"].numel())}
                del rr
            first = next(iter(res.values()))
            entry = {"workload": f"{cc.name}: {cc.n_pi} PIs + {cc.n_and} ANDs, {cg.n_levels} levels (Eq. 1 depth {int(lev.max()) + 1}), "
                                 f"{cc.hops}-hop cones, hidden {cc.hidden}, {cc.dtype}, {cc.n_layers} layer(s)",
                     "gates": cg.n, "neighbour_edges": cg.nnz, "setup_s": setup}
            entry.update(first)
            for label, v in list(res.items())[1:]:
                entry[label] = v
            del CX, CW, cg
            torch.cuda.empty_cache()
            return entry
        out["configs"] = {
            "tiny": one("tiny", 20, 3, default={}, level_by_level=dict(per_level=True)),
            "small": one("small", 10, 3, default={}, level_by_level=dict(per_level=True)),
            "medium": one("medium", 10, 3, default={}),
            # Section 4.1's depth; with_feed_forward: the complete transformer block per layer
            "medium_12_layers": one("medium", 2, 1, over=dict(n_layers=12), default={}, with_feed_forward=dict(ffn=True)),
            # stress as stored (K|V of finished gates kept for all four layers) and as the workload list
            # defines it: memory bounded to one level's frontier of K|V (level-by-level launches through
            # the 1001 assigned levels, the frontier's K|V projected again for every level that reads it)
            "stress": one("stress", 2, 1, default={}, bounded_kv=dict(bounded_kv=True), level_by_level=dict(per_level=True)),
        }

    # The layer under the paper's general partition and updating strategy (Algorithms 1 and 2 with the
    # paper's k = 8, stride 6, mini-batches of 128 cones, marks) on the 200K-gate graph: every gate is
    # computed once, over the part of its 8-hop cone that its first mini-batch shows.
    if not args.no_partition_point and headline:
        pw = synth.make("medium")
        pc = pw.cfg
        t0 = time.perf_counter()
        pg = dg4.dg4_build_partitioned(pc.n_nodes, pw.edge_src, pw.edge_dst, pw.edge_inv, 8, 6, 128, pw.level_hint)
        t_part = time.perf_counter() - t0
        # the same analysis on the GPU (edge list resident in device memory; second call timed)
        pe_dev = [torch.from_numpy(a).cuda() for a in (pw.edge_src, pw.edge_dst, pw.edge_inv)]
        ph_dev = torch.from_numpy(pw.level_hint).cuda() if pw.level_hint is not None else None
        for _ in range(2):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            pg_dev = dg4.dg4_build_partitioned_device(pc.n_nodes, *pe_dev, 8, 6, 128, ph_dev)
            t_part_dev = time.perf_counter() - t0
            del pg_dev
        del pe_dev, ph_dev
        PX, PW = tensors(pw, pc)
        pr = time_layer(pc, pg, PX, PW, 3, 2)
        ms_part = pr["ms_dev"]
        pcomp, pgath = algorithmic_bytes(pg, pr["cfg"], pg.array("level"))
        out["partition"] = {"workload": f"medium: {pc.n_pi} PIs + {pc.n_and} ANDs, {pg.n_levels} levels, 8-hop cones, "
                                        "stride 6, mini-batches of 128 cones, marks",
                            "path": path_of(pc, pg, {}),
                            "step_ms_device": ms_part, "edges_per_s": pg.nnz / (ms_part * 1e-3),
                            "gates_per_s": pg.n / (ms_part * 1e-3), "gates": pg.n, "neighbour_edges": pg.nnz,
                            "cones": int(len(pg.array("cone_root"))), "mini_batches": int(pg.array("stage").max()) + 1,
                            "dg4_build_partitioned_s": t_part, "dg4_build_partitioned_device_s": t_part_dev,
                            "gathered_GBps": pgath / (ms_part * 1e-3) / 1e9,
                            "compulsory_GBps": pcomp / (ms_part * 1e-3) / 1e9,
                            "traffic": measured_traffic("medium_partition_k8_rocprofv3.txt", "flow_kernel")}
        del pr
        # ... and under the paper's transformer depth as well (Section 4.1: twelve layers): its own configuration
        pc12 = synth.Config(**{**pc.__dict__, "n_layers": 12})
        pw12 = synth.make(pc12)                      # (same seed: the same circuit, weights for twelve layers)
        PX12, PW12 = tensors(pw12, pc12)
        pr12 = time_layer(pc12, pg, PX12, PW12, 2, 1)
        out["partition"]["with_12_layers"] = {"step_ms_device": pr12["ms_dev"], "path": path_of(pc12, pg, {}),
                                              "edges_per_s": pg.nnz * 12 / (pr12["ms_dev"] * 1e-3)}
        del pw12, PX12, PW12, pr12
        # The ablation without marks (every mini-batch recomputes its gates; one copy per mini-batch
        # and gate), against the same partition with marks. At k = 8 this graph would have 66 copies
        # per gate, so the pair is timed at k = 3, stride 2, mini-batches of 128 cones.
        ac = synth.Config(**{**pc.__dict__, "hops": 3})
        mg = dg4.dg4_build_partitioned(pc.n_nodes, pw.edge_src, pw.edge_dst, pw.edge_inv, 3, 2, 128, pw.level_hint)
        ug = dg4.dg4_build_partitioned(pc.n_nodes, pw.edge_src, pw.edge_dst, pw.edge_inv, 3, 2, 128, pw.level_hint, marks=False)
        UX = PX[torch.from_numpy(ug.array("copy_of").astype(np.int64)).cuda()].contiguous()
        rm, ru = time_layer(ac, mg, PX, PW, 3, 2), time_layer(ac, ug, UX, PW, 3, 2)
        ms_m, ms_u = rm["ms_dev"], ru["ms_dev"]
        out["partition"]["marks_ablation"] = {"workload": "medium, 3-hop cones, stride 2, mini-batches of 128 cones",
                                              "path": path_of(ac, mg, {}),
                                              "with_marks": {"step_ms_device": ms_m, "gate_computations": mg.n, "neighbour_edges": mg.nnz},
                                              "without_marks": {"step_ms_device": ms_u, "gate_computations": ug.n, "neighbour_edges": ug.nnz},
                                              "work_ratio": ug.n / mg.n, "time_ratio": ms_u / ms_m}
        del PX, pg, UX, ug, mg, rm, ru
        # The same ablation at the paper's own k = 8, stride 6, mini-batches of 128 cones, on a circuit of the same
        # shape with a tenth of the gates (on the full one the copies' tables alone would take tens of GB).
        kc = synth.Config(**{**pc.__dict__, "n_and": 20_000, "hops": 8})
        kw = synth.make(kc)
        KX, KW = tensors(kw, kc)
        mg = dg4.dg4_build_partitioned(kc.n_nodes, kw.edge_src, kw.edge_dst, kw.edge_inv, 8, 6, 128, kw.level_hint)
        ug = dg4.dg4_build_partitioned(kc.n_nodes, kw.edge_src, kw.edge_dst, kw.edge_inv, 8, 6, 128, kw.level_hint, marks=False)
        UX = KX[torch.from_numpy(ug.array("copy_of").astype(np.int64)).cuda()].contiguous()
        rm, ru = time_layer(kc, mg, KX, KW, 3, 2), time_layer(kc, ug, UX, KW, 3, 2)
        out["partition"]["marks_ablation_k8"] = {
            "workload": f"medium-shaped, {kc.n_pi} PIs + {kc.n_and} ANDs, 8-hop cones, stride 6, mini-batches of 128 cones",
            "path": path_of(kc, mg, {}),
            "with_marks": {"step_ms_device": rm["ms_dev"], "gate_computations": mg.n, "neighbour_edges": mg.nnz},
            "without_marks": {"step_ms_device": ru["ms_dev"], "gate_computations": ug.n, "neighbour_edges": ug.nnz},
            "work_ratio": ug.n / mg.n, "time_ratio": ru["ms_dev"] / rm["ms_dev"]}
        del KX, UX, ug, mg, rm, ru

    if not args.no_cpu_baseline and not part:
        import oracle
        # bounded sample: the same sweep over the lowest levels holding about --cpu-gates gates
        lp = g.array("level_ptr")
        lev_end = int(np.searchsorted(lp, min(args.cpu_gates, n_gates), side="left"))
        lev_end = max(1, min(lev_end, g.n_levels))
        og = oracle.build_levels(c.n_nodes, w.edge_src, w.edge_dst, w.edge_inv, c.hops, w.level_hint)
        t0 = time.perf_counter()
        ffn_kw = dict(zip(("w1", "w2"), synth.ffn_weights(c))) if args.ffn else {}
        oracle.layer_fwd(og, w.x, w.wqkv, w.wo, w.rel_bias, c.heads, store=c.dtype, level_end=lev_end, **ffn_kw)
        dt = time.perf_counter() - t0
        rows = int(lp[lev_end])
        sample_nnz = int(og.nbr_ptr[og.order[:rows] + 1].sum() - og.nbr_ptr[og.order[:rows]].sum())
        out["cpu_baseline"] = {"value": sample_nnz * layers / dt, "unit": "edges/s",
                               "gates_per_s": rows * layers / dt,
                               "cores": oracle.threads(),
                               "kind": "oracle", "seconds": dt,
                               "sample": f"levels [0,{lev_end}) of the same graph: {rows} gates, "
                                         f"{sample_nnz} neighbour edges, fp64, K/V of finished gates cached"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
