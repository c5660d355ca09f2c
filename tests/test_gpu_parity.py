"""GPU parity: every C-ABI device call against the CPU oracle, element by element.

Tolerances (max over rows of the relative L2 error): 1e-5 in fp32, 2e-2 in bf16.
"""
import numpy as np
import pytest
import torch

import dg4_synth as synth
import oracle
import paper_2502_01681_amd as dg4
from gpu_utils import TOL, cfg_of, device_weights, row_rel_err, tdtype, to_dev, to_np

pytestmark = pytest.mark.gpu


def graphs(w, hops=None, hint=True):
    c = w.cfg
    hops = c.hops if hops is None else hops
    h = w.level_hint if hint else None
    g = dg4.dg4_build_levels(c.n_nodes, w.edge_src, w.edge_dst, w.edge_inv, hops, h)
    og = oracle.build_levels(c.n_nodes, w.edge_src, w.edge_dst, w.edge_inv, hops, h)
    return g, og


@pytest.mark.parametrize("dtype,d,rows,lo,hi", [
    ("f32", 128, 1000, 0, 1000), ("f32", 128, 333, 7, 301), ("f32", 256, 130, 0, 130),
    ("bf16", 256, 1000, 0, 1000), ("bf16", 256, 257, 1, 256), ("bf16", 128, 95, 0, 95),
    ("bf16", 256, 31, 0, 31), ("bf16", 256, 40, 10, 10),
])
def test_qkv_proj(dtype, d, rows, lo, hi):
    print(f"qkv_proj {dtype} d={d} rows={rows} [{lo},{hi})", flush=True)
    bf = dtype == "bf16"
    S = synth.normal(21, 4, (rows, d), 1.0, bf)
    W = synth.normal(21, 100, (d, 3 * d), d ** -0.5, bf)
    cfg = dg4.LayerConfig(d, d // 32, 2, 1, dtype)
    Sd, Wd = to_dev(S, dtype), to_dev(W, dtype)
    out = [torch.full((rows, d), 7.0, dtype=tdtype(dtype), device="cuda") for _ in range(3)]
    dg4.dg4_qkv_proj(cfg, Sd, Wd, *out, row_begin=lo, row_end=hi)
    torch.cuda.synchronize()
    ref = oracle.qkv_proj(S, W)
    for got, r in zip(out, ref):
        got = to_np(got)
        assert (got[:lo] == 7.0).all() and (got[hi:] == 7.0).all()      # rows outside the range untouched
        if hi > lo:
            assert row_rel_err(got[lo:hi], r[lo:hi]).max() <= TOL[dtype]


@pytest.mark.parametrize("name,n_and,hops,dtype,d", [
    ("tiny", None, 2, "f32", 128), ("tiny", None, 1, "f32", 128), ("tiny", None, 3, "f32", 128),
    ("small", None, 2, "f32", 128), ("tiny", None, 2, "f32", 256), ("tiny", None, 2, "bf16", 128),
    ("medium", 30_000, 2, "bf16", 256), ("stress", 20_000, 3, "bf16", 256),
])
def test_sparse_attn(name, n_and, hops, dtype, d):
    print(f"sparse_attn {name} n_and={n_and} hops={hops} {dtype} d={d}", flush=True)
    w = synth.make(name, n_and=n_and, features=False)
    n, heads, bf = w.cfg.n_nodes, d // 32, dtype == "bf16"
    g, og = graphs(w, hops)
    Q, K, V = (synth.normal(31, s, (n, d), 1.5, bf) for s in (4, 5, 6))
    bias = synth.normal(31, 102, (heads, 4))
    cfg = dg4.LayerConfig(d, heads, hops, 1, dtype)
    A = torch.full((n, d), 3.0, dtype=tdtype(dtype), device="cuda")
    lo, hi = 5, n - 3
    dg4.dg4_sparse_attn_fwd(cfg, g, to_dev(Q, dtype), to_dev(K, dtype), to_dev(V, dtype), to_dev(bias, "f32"),
                            A, row_begin=lo, row_end=hi)
    torch.cuda.synchronize()
    got = to_np(A)
    ref = oracle.sparse_attn(og, heads, Q, K, V, bias, lo, hi)
    assert (got[:lo] == 3.0).all() and (got[hi:] == 3.0).all()
    err = row_rel_err(got[lo:hi], ref[lo:hi])
    assert err.max() <= (TOL[dtype] if bf else 2e-6), err.max()
    # rows with a single source copy that source's V exactly (alpha = 1, Section 3.7)
    single = np.nonzero(np.diff(og.nbr_ptr) == 1)[0]
    single = single[(single >= lo) & (single < hi)]
    assert len(single) > 0 and (got[single] == V[single]).all()


def run_layer(w, cfg, g, level_begin=0, level_end=None, H0=None):
    dtype = cfg.dtype
    X = to_dev(w.x, dtype)
    W = device_weights(w, dtype)
    H = torch.full((w.cfg.n_nodes, cfg.hidden), float("nan"), dtype=tdtype(dtype), device="cuda") if H0 is None else H0
    ws = dg4.dg4_layer_fwd(cfg, g, X, W, H, level_begin, level_end)
    torch.cuda.synchronize()
    dg4.dg4_layer_status(cfg, g, ws)                    # raises if a persistent sweep gave up
    return H


@pytest.mark.parametrize("name,n_and,kw", [
    ("tiny", None, {}), ("small", None, {}), ("tiny", None, dict(hops=3)), ("tiny", None, dict(hops=1)),
    ("tiny", None, dict(n_layers=3)), ("tiny", None, dict(epilogue=False)),
    ("medium", 40_000, {}), ("large", 50_000, {}), ("stress", 30_000, {}),
    ("medium", 40_000, dict(per_level=True)), ("large", 50_000, dict(per_level=True)),
    ("stress", 30_000, dict(n_layers=1)), ("large", 20_000, dict(hops=1)), ("large", 20_000, dict(epilogue=False)),
    ("stress", 3_000, dict(dtype="f32", hidden=128, heads=4)),
])
def test_layer_fwd_end_to_end(name, n_and, kw):
    print(f"layer_fwd e2e {name} n_and={n_and} {kw}", flush=True)
    base = synth.CONFIGS[name]
    over = {k: v for k, v in kw.items() if k in ("hops", "n_layers", "dtype", "hidden", "heads")}
    c = synth.Config(**{**base.__dict__, **over, **({"n_and": n_and} if n_and else {})})
    w = synth.make(c)
    cfg = cfg_of(c, epilogue=kw.get("epilogue", True), per_level=kw.get("per_level", False))
    g, og = graphs(w)
    H = to_np(run_layer(w, cfg, g))
    assert not np.isnan(H).any()                       # every gate written
    ref = oracle.layer_fwd(og, w.x, w.wqkv, w.wo, w.rel_bias, c.heads, store=c.dtype,
                           epilogue=cfg.epilogue)
    err = row_rel_err(H, ref)
    print(f"  max rel err {err.max():.3e}  p99.9 {np.quantile(err, 0.999):.3e}", flush=True)
    assert err.max() <= TOL[c.dtype], err.max()
    # teacher forced: each gate recomputed by the oracle from the GPU's own source rows
    rng = np.random.default_rng(0)
    nodes = rng.choice(c.n_nodes, size=min(c.n_nodes, 2000), replace=False)
    step = oracle.layer_nodes(og, w.x, w.wqkv, w.wo, w.rel_bias, c.heads, H, nodes, store=c.dtype,
                              epilogue=cfg.epilogue)
    assert row_rel_err(H[nodes], step).max() <= TOL[c.dtype]


def test_layer_fwd_schedule_split_and_determinism():
    print("layer_fwd schedule/split/determinism", flush=True)
    w = synth.make("large", n_and=30_000)
    c = w.cfg
    cfg = cfg_of(c)
    g_hint, _ = graphs(w, hint=True)
    g_asap, _ = graphs(w, hint=False)
    Hh = run_layer(w, cfg, g_hint)
    Ha = run_layer(w, cfg, g_asap)
    assert g_hint.n_levels > 3 * g_asap.n_levels
    assert torch.equal(Hh, Ha)                          # the schedule does not change a bit
    assert torch.equal(Hh, run_layer(w, cfg, g_hint))   # nor does a second run
    mid = g_hint.n_levels // 2
    H1 = run_layer(w, cfg, g_hint, 0, mid)
    lev = torch.from_numpy(g_hint.array("level")).cuda()
    assert torch.isnan(H1[lev >= mid].float()).all() and not torch.isnan(H1[lev < mid].float()).any()
    H2 = run_layer(w, cfg, g_hint, mid, None, H0=H1)
    assert torch.equal(H2, Hh)                          # resumed sweep = whole sweep


def test_dataflow_and_level_ordered_tiles_agree():
    # a whole-graph sweep runs in the dependency-driven tile order; the same sweep with the tiles
    # dealt level by level must not change a bit (nor does the per-level launch path change more
    # than rounding)
    print("layer_fwd dataflow order vs level order", flush=True)
    w = synth.make("large", n_and=60_000)
    cfg = cfg_of(w.cfg)
    g, _ = graphs(w, hint=True)
    H_flow = run_layer(w, cfg, g)
    H_level = run_layer(w, cfg_of(w.cfg, level_order=True), g)
    assert torch.equal(H_flow, H_level)
    assert not torch.isnan(H_flow.float()).any()


@pytest.mark.parametrize("name,n_and", [("stress", 30_000), ("large", 30_000)])
def test_level_by_level_sweeps_through_eq1_levels_or_the_hint_agree(name, n_and):
    # level-by-level launches over ALL levels of a graph with a deeper levelling than Eq. 1 go
    # through the Eq. 1 levels (far fewer rounds of launches); forced through the caller's levels
    # they must give the same bits
    print(f"layer_fwd per level: Eq. 1 levels vs hint {name}", flush=True)
    w = synth.make(name, n_and=n_and)
    cfg = cfg_of(w.cfg, per_level=True)
    g, og = graphs(w, hint=True)
    assert g.n_levels > 3 * (int(oracle.levels(w.cfg.n_nodes, w.edge_src, w.edge_dst).max()) + 1)
    H_eq1 = run_layer(w, cfg, g)
    H_hint = run_layer(w, cfg_of(w.cfg, per_level=True, level_order=True), g)
    assert not torch.isnan(H_eq1.float()).any()
    assert torch.equal(H_eq1, H_hint)


@pytest.mark.parametrize("name,n_and,kw", [("stress", 30_000, {}), ("large", 30_000, {}),
                                           ("tiny", None, dict(n_layers=2)), ("small", None, {})])
def test_bounded_kv_sweep(name, n_and, kw):
    # no K|V store: the K|V rows of a level's frontier are projected when the level is processed.
    # Same bits as the sweep with the store, a much smaller workspace, and a resumed sweep works.
    print(f"layer_fwd bounded K|V {name} {kw}", flush=True)
    base = synth.CONFIGS[name]
    c = synth.Config(**{**base.__dict__, **kw, **({"n_and": n_and} if n_and else {})})
    w = synth.make(c)
    g, og = graphs(w)
    cfg_store = cfg_of(c, per_level=True)
    cfg_bound = cfg_of(c, bounded_kv=True)
    H_store = run_layer(w, cfg_store, g)
    H_bound = run_layer(w, cfg_bound, g)
    assert not torch.isnan(H_bound.float()).any()
    assert torch.equal(H_store, H_bound)
    ref = oracle.layer_fwd(og, w.x, w.wqkv, w.wo, w.rel_bias, c.heads, store=c.dtype)
    assert row_rel_err(to_np(H_bound), ref).max() <= TOL[c.dtype]
    big, small = dg4.dg4_layer_workspace_bytes(cfg_store, g), dg4.dg4_layer_workspace_bytes(cfg_bound, g)
    print(f"  workspace {big / 1e6:.1f} MB with the store, {small / 1e6:.1f} MB bounded", flush=True)
    assert small < big
    mid = g.n_levels // 2
    H1 = run_layer(w, cfg_bound, g, 0, mid)
    H2 = run_layer(w, cfg_bound, g, mid, None, H0=H1)
    assert torch.equal(H2, H_bound)


@pytest.mark.parametrize("name,n_and,dtype,hidden", [("tiny", None, "f32", 128), ("small", None, "f32", 256),
                                                     ("large", 70_001, "bf16", 256), ("medium", 30_000, "bf16", 128)])
def test_struct_encode(name, n_and, dtype, hidden):
    # Eq. 2 of Section 3.5 against the oracle, element by element; in place as well
    print(f"struct_encode {name} {dtype} d={hidden}", flush=True)
    base = synth.CONFIGS[name]
    c = synth.Config(**{**base.__dict__, "dtype": dtype, "hidden": hidden, "heads": hidden // 32,
                        **({"n_and": n_and} if n_and else {})})
    w = synth.make(c)
    g, og = graphs(w)
    emb = synth.normal(c.seed + 7, 9, (6, hidden), 0.25, False)
    oa, on = oracle.out_degrees(c.n_nodes, w.edge_src, w.edge_dst, w.edge_inv)
    ref = oracle.struct_encode(w.x, og.level, oa, on, emb, store=dtype)
    cfg = cfg_of(c)
    X = to_dev(w.x, dtype)
    E = to_dev(emb, "f32")
    out = torch.full_like(X, float("nan"))
    dg4.dg4_struct_encode(cfg, g, X, E, out)
    torch.cuda.synchronize()
    got = to_np(out)
    assert not np.isnan(got).any()
    # fp32 arithmetic against fp64: a few fp32 roundings of the terms' magnitudes, plus the one
    # rounding to the stored format
    F = np.stack([og.level, np.ones(c.n_nodes), oa, np.ones(c.n_nodes), on, np.ones(c.n_nodes)], axis=1)
    mag = np.abs(w.x).astype(np.float64) + np.abs(F) @ np.abs(emb).astype(np.float64)
    store_ulp = 2.0 ** -23 if dtype == "f32" else 2.0 ** -7     # a different rounding decision next to a tie
    assert (np.abs(got - ref) <= 8 * 2.0 ** -24 * mag + store_ulp * np.abs(ref)).all()
    assert row_rel_err(got, ref).max() <= TOL[dtype]
    if dtype == "bf16":
        assert (got == ref).mean() > 0.999            # bf16: the same rounding decision almost everywhere
    dg4.dg4_struct_encode(cfg, g, X, E, X)             # in place
    torch.cuda.synchronize()
    assert torch.equal(X, out)


@pytest.mark.parametrize("dtype,d,rows,lo,hi", [
    ("f32", 128, 500, 0, 500), ("f32", 128, 77, 3, 70), ("f32", 256, 65, 0, 65),
    ("bf16", 256, 1000, 0, 1000), ("bf16", 256, 257, 1, 256), ("bf16", 128, 95, 0, 95),
    ("bf16", 256, 31, 0, 31), ("bf16", 256, 40, 10, 10),
])
def test_ffn_fwd(dtype, d, rows, lo, hi):
    print(f"ffn_fwd {dtype} d={d} rows={rows} [{lo},{hi})", flush=True)
    bf = dtype == "bf16"
    S = synth.normal(23, 4, (rows, d), 1.0, bf)
    W1 = synth.normal(23, 200, (d, 4 * d), d ** -0.5, bf)
    W2 = synth.normal(23, 201, (4 * d, d), (4 * d) ** -0.5, bf)
    cfg = dg4.LayerConfig(d, d // 32, 2, 1, dtype)
    out = torch.full((rows, d), 7.0, dtype=tdtype(dtype), device="cuda")
    dg4.dg4_ffn_fwd(cfg, to_dev(S, dtype), to_dev(W1, dtype), to_dev(W2, dtype), out, row_begin=lo, row_end=hi)
    torch.cuda.synchronize()
    got = to_np(out)
    assert (got[:lo] == 7.0).all() and (got[hi:] == 7.0).all()          # rows outside the range untouched
    if hi > lo:
        ref = oracle.ffn(S, W1, W2, store=dtype)
        err = row_rel_err(got[lo:hi], ref[lo:hi])
        print(f"  max rel err {err.max():.3e}", flush=True)
        assert err.max() <= TOL[dtype], err.max()


@pytest.mark.parametrize("name,n_and,kw", [
    ("tiny", None, {}), ("small", None, {}), ("tiny", None, dict(n_layers=3, hops=3)),
    ("large", 30_000, {}), ("large", 30_000, dict(per_level=True)), ("medium", 20_000, {}),
    ("large", 20_000, dict(hops=1)), ("stress", 8_000, {}), ("stress", 8_000, dict(bounded_kv=True)),
    ("medium", 20_000, dict(dtype="f32")),
])
def test_layer_fwd_with_feed_forward(name, n_and, kw):
    """The whole transformer block per layer: attention sub-block, then LN(h + relu(h W1) W2)."""
    print(f"layer_fwd ffn {name} n_and={n_and} {kw}", flush=True)
    base = synth.CONFIGS[name]
    over = {k: v for k, v in kw.items() if k in ("hops", "n_layers", "dtype")}
    c = synth.Config(**{**base.__dict__, **over, **({"n_and": n_and} if n_and else {})})
    w = synth.make(c)
    w1, w2 = synth.ffn_weights(c)
    cfg = cfg_of(c, ffn=True, bounded_kv=kw.get("bounded_kv", False), per_level=kw.get("per_level", False))
    g, og = graphs(w)
    X = to_dev(w.x, c.dtype)
    W = [lw + (to_dev(w1[l], c.dtype), to_dev(w2[l], c.dtype)) for l, lw in enumerate(device_weights(w, c.dtype))]
    Hd = torch.full((c.n_nodes, c.hidden), float("nan"), dtype=tdtype(c.dtype), device="cuda")
    dg4.dg4_layer_fwd(cfg, g, X, W, Hd)
    torch.cuda.synchronize()
    H = to_np(Hd)
    assert not np.isnan(H).any()
    ref = oracle.layer_fwd(og, w.x, w.wqkv, w.wo, w.rel_bias, c.heads, store=c.dtype, w1=w1, w2=w2)
    err = row_rel_err(H, ref)
    print(f"  max rel err {err.max():.3e}  p99.9 {np.quantile(err, 0.999):.3e}", flush=True)
    assert err.max() <= TOL[c.dtype], err.max()
    rng = np.random.default_rng(0)
    nodes = rng.choice(c.n_nodes, size=min(c.n_nodes, 2000), replace=False)
    step = oracle.layer_nodes(og, w.x, w.wqkv, w.wo, w.rel_bias, c.heads, H, nodes, store=c.dtype, w1=w1, w2=w2)
    assert row_rel_err(H[nodes], step).max() <= TOL[c.dtype]
    # and it is not the layer without the sub-block
    plain = oracle.layer_nodes(og, w.x, w.wqkv, w.wo, w.rel_bias, c.heads, H, nodes[:50], store=c.dtype)
    assert row_rel_err(H[nodes[:50]], plain).min() > 10 * TOL[c.dtype]


@pytest.mark.parametrize("ffn", [False, True])
def test_sweep_reads_no_row_before_it_is_written(ffn):
    """Workspace filled with NaN patterns before every run: a K|V row fetched before its gate has
    written it (or a stale cached copy of it) would surface as NaN or as a wrong embedding."""
    print(f"poisoned workspace ffn={ffn}", flush=True)
    w = synth.make("large", n_and=30_000)
    c = w.cfg
    cfg = cfg_of(c, ffn=ffn)
    g, og = graphs(w)
    X = to_dev(w.x, c.dtype)
    W = device_weights(w, c.dtype)
    w1 = w2 = None
    if ffn:
        w1, w2 = synth.ffn_weights(c)
        W = [lw + (to_dev(w1[l], c.dtype), to_dev(w2[l], c.dtype)) for l, lw in enumerate(W)]
    ws = torch.empty(dg4.dg4_layer_workspace_bytes(cfg, g), dtype=torch.uint8, device="cuda")
    nodes = np.arange(c.n_nodes)
    for _ in range(3):
        ws.fill_(0xFF)
        Hd = torch.full((c.n_nodes, c.hidden), float("nan"), dtype=tdtype(c.dtype), device="cuda")
        dg4.dg4_layer_fwd(cfg, g, X, W, Hd, workspace=ws)
        torch.cuda.synchronize()
        H = to_np(Hd)
        assert not np.isnan(H).any()
        step = oracle.layer_nodes(og, w.x, w.wqkv, w.wo, w.rel_bias, c.heads, H, nodes, store=c.dtype, w1=w1, w2=w2)
        assert row_rel_err(H, step).max() <= TOL[c.dtype]


@pytest.mark.parametrize("ffn", [False, True])
@pytest.mark.parametrize("n_pi,n_and", [(3, 0), (2, 1), (32, 5), (7, 17), (32, 40), (16, 500)])
def test_small_graphs_through_the_persistent_kernel(n_pi, n_and, ffn):
    """Ragged and empty tiles, fewer tiles than compute units, primary inputs only: bf16, hidden 256,
    two hops, the configuration the persistent kernel serves."""
    print(f"small graph n_pi={n_pi} n_and={n_and} ffn={ffn}", flush=True)
    c = synth.Config("t", 9, n_pi, n_and, 8, 1.0, 0, 256, 8, 2, 1, "bf16")
    n = c.n_nodes
    if n_and:
        src, dst, inv, _ = synth.aig(c.seed, n_pi, n_and, c.window)
    else:
        src = dst = np.zeros(0, dtype=np.int32); inv = np.zeros(0, dtype=np.uint8)
    x = synth.normal(c.seed, synth.STREAM_X, (n, c.hidden), 1.0, True)
    wqkv, wo, rb = synth.weights(c)
    w1 = w2 = None
    g = dg4.dg4_build_levels(n, src, dst, inv, 2)
    og = oracle.build_levels(n, src, dst, inv, 2)
    W = [(to_dev(wqkv[0], "bf16"), to_dev(wo[0], "bf16"), to_dev(rb[0], "f32"))]
    if ffn:
        w1, w2 = synth.ffn_weights(c)
        W = [W[0] + (to_dev(w1[0], "bf16"), to_dev(w2[0], "bf16"))]
    cfg = cfg_of(c, ffn=ffn)
    ws = torch.empty(dg4.dg4_layer_workspace_bytes(cfg, g), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)
    Hd = torch.full((n, c.hidden), float("nan"), dtype=torch.bfloat16, device="cuda")
    dg4.dg4_layer_fwd(cfg, g, to_dev(x, "bf16"), W, Hd, workspace=ws)
    torch.cuda.synchronize()
    dg4.dg4_layer_status(cfg, g, ws)
    H = to_np(Hd)
    assert not np.isnan(H).any()
    ref = oracle.layer_fwd(og, x, wqkv, wo, rb, c.heads, store="bf16", w1=w1, w2=w2)
    assert row_rel_err(H, ref).max() <= TOL["bf16"]


def test_workspace_reuse_with_new_inputs():
    # the same workspace and output buffer, different features: nothing stale may be read
    print("layer_fwd workspace reuse", flush=True)
    w = synth.make("large", n_and=30_000)
    c = w.cfg
    cfg = cfg_of(c)
    g, og = graphs(w)
    X1 = to_dev(w.x, c.dtype)
    x2 = synth.normal(c.seed + 99, 4, w.x.shape, 1.0, True)
    X2 = to_dev(x2, c.dtype)
    W = device_weights(w, c.dtype)
    H = torch.empty_like(X1)
    ws = torch.empty(dg4.dg4_layer_workspace_bytes(cfg, g), dtype=torch.uint8, device="cuda")
    for X, x in ((X1, w.x), (X2, x2), (X1, w.x)):
        dg4.dg4_layer_fwd(cfg, g, X, W, H, workspace=ws)
        torch.cuda.synchronize()
        ref = oracle.layer_fwd(og, x, w.wqkv, w.wo, w.rel_bias, c.heads, store=c.dtype)
        assert row_rel_err(to_np(H), ref).max() <= TOL[c.dtype]


def test_device_call_errors():
    w = synth.make("tiny")
    c = w.cfg
    g, _ = graphs(w)
    cfg = cfg_of(c)
    X, W = to_dev(w.x, c.dtype), device_weights(w, c.dtype)
    H = torch.zeros_like(X)
    small = torch.empty(1024, dtype=torch.uint8, device="cuda")
    with pytest.raises(dg4.DG4Error) as e:
        dg4.dg4_layer_fwd(cfg, g, X, W, H, workspace=small)
    assert e.value.name == "EWORKSPACE"
    with pytest.raises(dg4.DG4Error) as e:
        dg4.dg4_layer_fwd(cfg, g, X, W, H, level_begin=5, level_end=2)
    assert e.value.name == "EINVAL"
    with pytest.raises(dg4.DG4Error) as e:
        dg4.dg4_layer_fwd(cfg_of(c, hops=3), g, X, W, H)
    assert e.value.name == "EINVAL"
    with pytest.raises(dg4.DG4Error) as e:
        dg4.dg4_sparse_attn_fwd(cfg, g, X, X, X, W[0][2], H, row_begin=0, row_end=c.n_nodes + 1)
    assert e.value.name == "EINVAL"
    assert (H == 0).all()
