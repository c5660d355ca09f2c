#!/usr/bin/env python3
"""Benchmark of the level sweep (dg4_layer_fwd) on one MI355X.

One step = one pass of the whole hot path over the 1M-gate "large" synthetic
AIG: projections, per-edge scores, segmented softmax, aggregation, output
projection + LayerNorm, swept over all of its about 1000 levels. Inputs are
resident in HBM before the timed region; graph analysis (host) and uploads are
reported separately and excluded. Prints ONE JSON line. `--ffn` times the layer with its
feed-forward sub-block instead (not the headline configuration); `--partition K,STRIDE,BATCH`
times the layer under the paper's general graph partition and updating strategy. The default
run also carries kernel points, the feed-forward layer and a partition point (`partition`:
200K-gate graph, k = 8, stride 6, mini-batches of 128 cones; marks against no marks at k = 3).
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

HBM_PEAK_GBPS = 8000.0
# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE,
# calibrated against a plain copy (see profiles/); None until measured for a workload.
TRAFFIC_BYTES = {"large": 8.60e9}     # sweep_kernel: 7.05 GB fetched + 1.55 GB written (profiles/large_sweep_rocprofv3.txt)


def algorithmic_bytes(g, cfg, levels=None):
    """Bytes the method has to move for one sweep (per-gate figures of the design notes).

    Per gate and layer: read the state row R, write the new state row R, write the gate's K and V
    rows 2R, read its packed neighbour row. Per level and layer: read the K and V rows of the
    DISTINCT sources of the level once (compulsory traffic), 2R each. `gathered` counts every
    neighbour entry instead (what a cache-less gather moves).
    """
    es = 4 if cfg.dtype == "f32" else 2
    R = cfg.hidden * es
    level = g.array("level")
    ptr, idx = g.array("nbr_ptr"), g.array("nbr_idx")
    n = g.n
    dst = np.repeat(np.arange(n, dtype=np.int64), np.diff(ptr))
    keep = idx != dst                                   # sources other than the gate itself
    dl, src = level[dst[keep]].astype(np.int64), idx[keep].astype(np.int64)
    if levels is not None:
        sel = dl < levels
        dl, src = dl[sel], src[sel]
        n_rows = int((level < levels).sum())
    else:
        n_rows = n
    distinct = len(np.unique(dl * n + src))
    # neighbour rows: fixed width up to three hops, else the entries themselves
    ell_bytes = n_rows * 4 * (1 << (g.hops + 1)) if g.hops <= 3 else 4 * (len(src) + n_rows)
    per_gate = (R + R + 2 * R) * cfg.n_layers
    compulsory = n_rows * per_gate + ell_bytes * cfg.n_layers + distinct * 2 * R * cfg.n_layers
    gathered = n_rows * per_gate + ell_bytes * cfg.n_layers + len(src) * 2 * R * cfg.n_layers
    return compulsory, gathered


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="large", help="large (default) | medium | small | tiny | stress")
    ap.add_argument("--n-and", type=int, default=None, help="override the number of AND gates (debug)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-points", action="store_true",
                    help="skip the stand-alone timings of dg4_qkv_proj and dg4_sparse_attn_fwd over all rows")
    ap.add_argument("--no-level-order", action="store_true",
                    help="skip the extra run with level-ordered tiles (for profiles of the default path only)")
    ap.add_argument("--ffn", action="store_true",
                    help="time the layer WITH its feed-forward sub-block (not the headline configuration; "
                         "the roofline object then prices the step's matrix products against the MFMA peak)")
    ap.add_argument("--partition", default=None, metavar="K,STRIDE,BATCH",
                    help="time the layer under the general partition and updating strategy (cones of depth K "
                         "collected every STRIDE levels, mini-batches of BATCH cones) instead of the headline sweep")
    ap.add_argument("--no-partition-point", action="store_true",
                    help="skip the extra measurement of the partitioned layer (medium graph, k=8, stride 6, 128 cones)")
    ap.add_argument("--cpu-gates", type=int, default=400_000, help="gates in the oracle's timed sample")
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
    os.environ["DG4_SWEEP_EVENTS"] = "1"      # the library brackets its sweep kernel with two events
    t0 = time.perf_counter()
    w = synth.make(args.workload, n_and=args.n_and)
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
    for _ in range(2 if c.hops <= 3 else 0):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        g_dev = dg4.dg4_build_levels_device(c.n_nodes, *e_dev, c.hops, h_dev)
        t_build_dev = time.perf_counter() - t0
        del g_dev
    del e_dev, h_dev
    cfg = dg4.LayerConfig(c.hidden, c.heads, c.hops, c.n_layers, c.dtype, ffn=args.ffn)
    td = torch.float32 if c.dtype == "f32" else torch.bfloat16
    t0 = time.perf_counter()
    X = torch.from_numpy(w.x).cuda().to(td).contiguous()
    W = [(torch.from_numpy(w.wqkv[l]).cuda().to(td).contiguous(), torch.from_numpy(w.wo[l]).cuda().to(td).contiguous(),
          torch.from_numpy(w.rel_bias[l]).cuda().contiguous()) for l in range(c.n_layers)]
    if args.ffn:
        fw1, fw2 = synth.ffn_weights(c)
        W = [W[l] + (torch.from_numpy(fw1[l]).cuda().to(td).contiguous(), torch.from_numpy(fw2[l]).cuda().to(td).contiguous())
             for l in range(c.n_layers)]
    g.upload()
    torch.cuda.synchronize()
    t_upload = time.perf_counter() - t0
    H = torch.empty_like(X)
    ws = torch.empty(dg4.dg4_layer_workspace_bytes(cfg, g), dtype=torch.uint8, device="cuda")

    for _ in range(args.warmup):
        dg4.dg4_layer_fwd(cfg, g, X, W, H, workspace=ws)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    sweep_ms = []
    for a, b in ev:
        a.record()
        dg4.dg4_layer_fwd(cfg, g, X, W, H, workspace=ws)
        b.record()
        try:
            sweep_ms.append(dg4.dg4_sweep_elapsed_ms())     # waits for this step's sweep kernel
        except dg4.DG4Error:
            pass                                            # configuration without the persistent kernel
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_step = wall * 1e3 / args.steps
    ms_dev = float(np.mean([a.elapsed_time(b) for a, b in ev]))
    ms_kernel = float(np.mean(sweep_ms)) if len(sweep_ms) == args.steps else ms_dev

    n_gates, nnz = g.n, g.nnz
    layers = c.n_layers
    compulsory, gathered = algorithmic_bytes(g, cfg)
    # The sweep kernel performs every algorithmic transfer of the step itself (residual row in, H and
    # K|V rows out, neighbour rows, one K|V read per distinct source and level); the Q|K|V rows of x
    # that the bulk projection hands it are an implementation detail and are NOT counted.
    achieved = compulsory / (ms_kernel * 1e-3) / 1e9
    out = {
        "metric": "edges/sec per sparse-attn layer fwd (level sweep)",
        "value": nnz * layers / (ms_step * 1e-3),
        "unit": "edges/s",
        "gates_per_s": n_gates * layers / (ms_step * 1e-3),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "ms_per_layer": ms_step / layers,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": c.dtype, "data": "synthetic",
        "config": {"workload": f"{c.name}: {c.n_pi} PIs + {c.n_and} ANDs, {g.n_levels} levels, "
                               f"{c.hops}-hop cones, hidden {c.hidden}, {c.heads} heads, {layers} layer(s)",
                   "gates": n_gates, "neighbour_edges": nnz, "aig_edges": int(len(w.edge_src)),
                   "levels": g.n_levels},
        "roofline": {"bound": "hbm",
                     "kernel": "sweep_kernel (persistent level sweep)" if len(sweep_ms) == args.steps
                               else "dg4_layer_fwd (all launches of one step)",
                     "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": None if part else TRAFFIC_BYTES.get(c.name),
                     "algorithmic_bytes": compulsory, "gathered_bytes": gathered,
                     "kernel_ms": ms_kernel, "step_ms_device": ms_dev,
                     "step_achieved": compulsory / (ms_dev * 1e-3) / 1e9},
        "setup_s": {"generate": t_gen, "dg4_build_partitioned" if part else "dg4_build_levels": t_build,
                    "dg4_build_levels_device": t_build_dev, "upload": t_upload},
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

    # For information: the same step with the tiles dealt strictly level by level (the order of the
    # level hint) instead of the library's default dependency-driven order. Same results, bit for bit.
    if len(sweep_ms) == args.steps and not args.no_level_order and not args.ffn and not part:
        os.environ["DG4_SWEEP_LEVEL_ORDER"] = "1"
        for _ in range(args.warmup):
            dg4.dg4_layer_fwd(cfg, g, X, W, H, workspace=ws)
        torch.cuda.synchronize()
        lo_ms, lo_kernel = [], []
        for _ in range(args.steps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            dg4.dg4_layer_fwd(cfg, g, X, W, H, workspace=ws)
            b.record()
            lo_kernel.append(dg4.dg4_sweep_elapsed_ms())
            torch.cuda.synchronize()
            lo_ms.append(a.elapsed_time(b))
        del os.environ["DG4_SWEEP_LEVEL_ORDER"]
        k = float(np.mean(lo_kernel))
        out["level_order_tiles"] = {"step_ms_device": float(np.mean(lo_ms)), "kernel_ms": k,
                                    "roofline_frac": compulsory / (k * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                                    "edges_per_s": nnz * layers / (float(np.mean(lo_ms)) * 1e-3)}

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
        es = 4 if c.dtype == "f32" else 2
        R = c.hidden * es
        Q, K, V, A = (torch.empty_like(X) for _ in range(4))
        pws = torch.empty(dg4.dg4_proj_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
        ms_p = timed(lambda: dg4.dg4_qkv_proj(cfg, X, W[0][0], Q, K, V, workspace=pws))
        flop_p = 2.0 * n_gates * c.hidden * 3 * c.hidden
        ms_a = timed(lambda: dg4.dg4_sparse_attn_fwd(cfg, g, Q, K, V, W[0][2], A))
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
        ms_s = timed(lambda: dg4.dg4_struct_encode(cfg, g, X, emb, A))
        bytes_s = n_gates * (2 * R + 12)                       # a row in, a row out, three integers
        out["kernel_points"]["dg4_struct_encode"] = {"ms": ms_s, "GB/s": bytes_s / (ms_s * 1e-3) / 1e9,
                                                     "hbm_frac": bytes_s / (ms_s * 1e-3) / 1e9 / HBM_PEAK_GBPS}
        # the feed-forward sub-block over all rows: 16 d^2 flop per row against 2 rows of traffic, MFMA-bound
        fws = torch.empty(dg4.dg4_ffn_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
        W1, W2 = (torch.from_numpy(t[0]).cuda().to(td).contiguous() for t in synth.ffn_weights(c))
        ms_f = timed(lambda: dg4.dg4_ffn_fwd(cfg, X, W1, W2, A, workspace=fws))
        flop_f = 16.0 * n_gates * c.hidden * c.hidden
        out["kernel_points"]["dg4_ffn_fwd"] = {"ms": ms_f, "TFLOP/s": flop_f / (ms_f * 1e-3) / 1e12,
                                               "mfma_frac": flop_f / (ms_f * 1e-3) / peak_flops,
                                               "GB/s": n_gates * 2 * R / (ms_f * 1e-3) / 1e9}
        # the layer with the feed-forward sub-block after the attention sub-block (level-by-level launches)
        fcfg = dg4.LayerConfig(c.hidden, c.heads, c.hops, c.n_layers, c.dtype, ffn=True)
        fw1, fw2 = synth.ffn_weights(c)
        FW = [W[l] + (torch.from_numpy(fw1[l]).cuda().to(td).contiguous(), torch.from_numpy(fw2[l]).cuda().to(td).contiguous())
              for l in range(c.n_layers)]
        fwsl = torch.empty(dg4.dg4_layer_workspace_bytes(fcfg, g), dtype=torch.uint8, device="cuda")
        ms_l = timed(lambda: dg4.dg4_layer_fwd(fcfg, g, X, FW, A, workspace=fwsl), reps=3)
        out["ffn_layer"] = {"step_ms_device": ms_l, "edges_per_s": nnz * layers / (ms_l * 1e-3),
                            "gates_per_s": n_gates * layers / (ms_l * 1e-3)}
        del Q, K, V, A, fwsl

    # The layer under the paper's general partition and updating strategy (Algorithms 1 and 2 with the
    # paper's k = 8, stride 6, mini-batches of 128 cones, marks) on the 200K-gate graph: every gate is
    # computed once, over the part of its 8-hop cone that its first mini-batch shows.
    if not args.no_partition_point and not args.ffn and not part and args.workload == "large" and args.n_and is None:
        pw = synth.make("medium")
        pc = pw.cfg
        t0 = time.perf_counter()
        pg = dg4.dg4_build_partitioned(pc.n_nodes, pw.edge_src, pw.edge_dst, pw.edge_inv, 8, 6, 128, pw.level_hint)
        t_part = time.perf_counter() - t0
        pcfg = dg4.LayerConfig(pc.hidden, pc.heads, 8, 1, pc.dtype)
        PX = torch.from_numpy(pw.x).cuda().to(td).contiguous()
        PW = [(torch.from_numpy(pw.wqkv[0]).cuda().to(td).contiguous(), torch.from_numpy(pw.wo[0]).cuda().to(td).contiguous(),
               torch.from_numpy(pw.rel_bias[0]).cuda().contiguous())]
        PH = torch.empty_like(PX)
        pws = torch.empty(dg4.dg4_layer_workspace_bytes(pcfg, pg), dtype=torch.uint8, device="cuda")
        for _ in range(2):
            dg4.dg4_layer_fwd(pcfg, pg, PX, PW, PH, workspace=pws)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(3):
            dg4.dg4_layer_fwd(pcfg, pg, PX, PW, PH, workspace=pws)
        b.record()
        torch.cuda.synchronize()
        ms_part = a.elapsed_time(b) / 3
        pcomp, pgath = algorithmic_bytes(pg, pcfg)
        out["partition"] = {"workload": f"medium: {pc.n_pi} PIs + {pc.n_and} ANDs, {pg.n_levels} levels, 8-hop cones, "
                                        "stride 6, mini-batches of 128 cones, marks",
                            "step_ms_device": ms_part, "edges_per_s": pg.nnz / (ms_part * 1e-3),
                            "gates_per_s": pg.n / (ms_part * 1e-3), "gates": pg.n, "neighbour_edges": pg.nnz,
                            "cones": int(len(pg.array("cone_root"))), "mini_batches": int(pg.array("stage").max()) + 1,
                            "dg4_build_partitioned_s": t_part,
                            "gathered_GBps": pgath / (ms_part * 1e-3) / 1e9,
                            "compulsory_GBps": pcomp / (ms_part * 1e-3) / 1e9}
        # The ablation without marks (every mini-batch recomputes its gates; one copy per mini-batch
        # and gate), against the same partition with marks. At k = 8 this graph would have 66 copies
        # per gate, so the pair is timed at k = 3, stride 2, mini-batches of 128 cones.
        def layer_ms(graph, cfg_, X_, reps):
            H_ = torch.empty_like(X_)
            ws_ = torch.empty(dg4.dg4_layer_workspace_bytes(cfg_, graph), dtype=torch.uint8, device="cuda")
            dg4.dg4_layer_fwd(cfg_, graph, X_, PW, H_, workspace=ws_)
            torch.cuda.synchronize()
            a.record()
            for _ in range(reps):
                dg4.dg4_layer_fwd(cfg_, graph, X_, PW, H_, workspace=ws_)
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / reps
        acfg = dg4.LayerConfig(pc.hidden, pc.heads, 3, 1, pc.dtype)
        mg = dg4.dg4_build_partitioned(pc.n_nodes, pw.edge_src, pw.edge_dst, pw.edge_inv, 3, 2, 128, pw.level_hint)
        ug = dg4.dg4_build_partitioned(pc.n_nodes, pw.edge_src, pw.edge_dst, pw.edge_inv, 3, 2, 128, pw.level_hint, marks=False)
        UX = PX[torch.from_numpy(ug.array("copy_of").astype(np.int64)).cuda()].contiguous()
        ms_m, ms_u = layer_ms(mg, acfg, PX, 3), layer_ms(ug, acfg, UX, 3)
        out["partition"]["marks_ablation"] = {"workload": "medium, 3-hop cones, stride 2, mini-batches of 128 cones",
                                              "with_marks": {"step_ms_device": ms_m, "gate_computations": mg.n, "neighbour_edges": mg.nnz},
                                              "without_marks": {"step_ms_device": ms_u, "gate_computations": ug.n, "neighbour_edges": ug.nnz},
                                              "work_ratio": ug.n / mg.n, "time_ratio": ms_u / ms_m}
        del PX, PH, pws, pg, UX, ug, mg

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
