"""The persistent dataflow kernel for every shape (fp32 / hidden 128, bf16 / hidden 256, cones of up to
three hops, any number of layers) against the oracle, against level-by-level launches (other kernels,
another summation order: equal up to rounding) and, bit for bit, against itself under other schedules.
"""
import numpy as np
import pytest
import torch

import dg4_synth as synth
import oracle
import paper_2502_01681_amd as dg4
from gpu_utils import TOL, cfg_of, device_weights, elem_err, row_rel_err, tdtype, to_dev, to_np

pytestmark = pytest.mark.gpu


def make(name, n_and=None, **over):
    base = synth.CONFIGS[name]
    c = synth.Config(**{**base.__dict__, **over, **({"n_and": n_and} if n_and else {})})
    return synth.make(c)


def graphs(w, hint=True):
    c = w.cfg
    h = w.level_hint if hint else None
    g = dg4.dg4_build_levels(c.n_nodes, w.edge_src, w.edge_dst, w.edge_inv, c.hops, h)
    og = oracle.build_levels(c.n_nodes, w.edge_src, w.edge_dst, w.edge_inv, c.hops, h)
    return g, og


def run(w, cfg, g, level_begin=0, level_end=None, H0=None, poison=False):
    X, W = to_dev(w.x, cfg.dtype), device_weights(w, cfg.dtype)
    H = torch.full((w.cfg.n_nodes, cfg.hidden), float("nan"), dtype=tdtype(cfg.dtype), device="cuda") if H0 is None else H0
    ws = torch.empty(dg4.dg4_layer_workspace_bytes(cfg, g), dtype=torch.uint8, device="cuda")
    if poison:
        ws.fill_(0xFF)                  # NaN patterns: nothing may be read before it is written
    dg4.dg4_layer_fwd(cfg, g, X, W, H, level_begin, level_end, workspace=ws)
    torch.cuda.synchronize()
    dg4.dg4_layer_status(cfg, g, ws)
    return H


@pytest.mark.parametrize("name,n_and,over", [
    ("tiny", None, {}), ("small", None, {}), ("tiny", None, dict(hops=3)), ("tiny", None, dict(hops=1)),
    ("tiny", None, dict(n_layers=3)), ("small", 3000, dict(n_layers=12)),
    ("stress", 30_000, {}), ("stress", 20_000, dict(n_layers=1)), ("medium", 20_000, dict(n_layers=2)),
    ("medium", 10_000, dict(hops=3)), ("stress", 3_000, dict(dtype="f32", hidden=128, heads=4)),
    # wide, shallow circuits (Eq. 1 depth 4: more than 4096 gates per level): tiles of 32 gates, two of the table's at a time
    ("stress", 20_000, dict(level_cap=3)), ("stress", 20_000, dict(level_cap=3, hops=2, n_layers=2)),
    ("stress", 20_000, dict(level_cap=3, dtype="f32", hidden=128, heads=4, n_layers=2)), ("stress", 17_001, dict(level_cap=2, n_layers=1)),
])
def test_flow_kernel_against_oracle_and_level_by_level(name, n_and, over):
    print(f"flow kernel {name} n_and={n_and} {over}", flush=True)
    w = make(name, n_and, **over)
    c = w.cfg
    g, og = graphs(w)
    H = run(w, cfg_of(c), g, poison=True)
    assert not torch.isnan(H.float()).any()                      # every gate written
    H_pl = to_np(run(w, cfg_of(c, per_level=True), g))
    # other kernels, another summation order: each within TOL of the oracle, so within 2 TOL of each other
    assert row_rel_err(to_np(H), H_pl.astype(np.float64)).max() <= 2 * TOL[c.dtype]
    ref = oracle.layer_fwd(og, w.x, w.wqkv, w.wo, w.rel_bias, c.heads, store=c.dtype)
    Hn = to_np(H)
    err = row_rel_err(Hn, ref)
    print(f"  max rel err {err.max():.3e}, max element err {elem_err(Hn, ref).max():.3e}", flush=True)
    assert err.max() <= TOL[c.dtype]
    assert elem_err(Hn, ref).max() <= 4 * TOL[c.dtype]
    assert torch.equal(H, run(w, cfg_of(c), g))                  # a second run: the same bits


def test_flow_kernel_without_epilogue():
    w = make("tiny")
    g, og = graphs(w)
    cfg = cfg_of(w.cfg, epilogue=False)
    H = run(w, cfg, g)
    ref = oracle.layer_fwd(og, w.x, w.wqkv, w.wo, w.rel_bias, w.cfg.heads, store="f32", epilogue=False)
    assert row_rel_err(to_np(H), ref).max() <= TOL["f32"]
    H_pl = to_np(run(w, cfg_of(w.cfg, epilogue=False, per_level=True), g))
    assert row_rel_err(to_np(H), H_pl.astype(np.float64)).max() <= 2 * TOL["f32"]


@pytest.mark.parametrize("name,n_and,over", [("small", None, {}), ("stress", 20_000, {}), ("medium", 12_000, dict(n_layers=2)),
                                                ("small", 4_000, dict(n_layers=4)), ("stress", 20_000, dict(level_cap=3))])
def test_flow_kernel_schedules_and_resume(name, n_and, over):
    # dependency-driven tiles (on narrow circuits with several layers: flags that go up layer by layer), the
    # graph's own levels, Eq. 1 levels or a caller's deeper levelling, a sweep cut in two: never a different bit
    print(f"flow kernel schedules {name}", flush=True)
    w = make(name, n_and, **over)
    c = w.cfg
    g, _ = graphs(w, hint=True)
    g_asap, _ = graphs(w, hint=False)
    cfg = cfg_of(c)
    H = run(w, cfg, g)
    assert torch.equal(H, run(w, cfg_of(c, level_order=True), g))
    assert torch.equal(H, run(w, cfg, g_asap))
    mid = g.n_levels // 2
    H1 = run(w, cfg, g, 0, mid)
    lev = torch.from_numpy(g.array("level")).cuda()
    assert torch.isnan(H1[lev >= mid].float()).all() and not torch.isnan(H1[lev < mid].float()).any()
    H2 = run(w, cfg, g, mid, None, H0=H1)
    assert torch.equal(H2, H)


@pytest.mark.parametrize("n_layers", [1, 3])
def test_flow_kernel_bounded_wait_and_packed_weights(n_layers):
    # A spin limit of one makes a tile give up on the first unpublished source (with several layers on this
    # narrow circuit: also on a source whose later layers are not in the store yet): the sweep must return,
    # report it, publish nothing more of the abandoned tile, and a normal run afterwards is correct. Then
    # the packed weights of that run serve a third one.
    w = make("small", n_layers=n_layers)
    c = w.cfg
    g, og = graphs(w)
    X, W = to_dev(w.x, c.dtype), device_weights(w, c.dtype)
    H = torch.full((c.n_nodes, c.hidden), float("nan"), dtype=tdtype(c.dtype), device="cuda")
    cfg = cfg_of(c)
    ws = torch.empty(dg4.dg4_layer_workspace_bytes(cfg, g), dtype=torch.uint8, device="cuda")
    print("flow kernel: spin limit 1", flush=True)
    dg4.dg4_layer_fwd(cfg_of(c, spin_limit=1), g, X, W, H, workspace=ws)
    torch.cuda.synchronize()                                    # returns: no hang
    status = dg4.dg4_layer_status(cfg, g, ws, check=False)
    print(f"  status={status}", flush=True)
    assert status in (0, -10)
    if status:
        assert torch.isnan(H.float()).any()                      # an aborted sweep is incomplete, never wrong
    ref = oracle.layer_fwd(og, w.x, w.wqkv, w.wo, w.rel_bias, c.heads, store=c.dtype)
    dg4.dg4_layer_fwd(cfg, g, X, W, H, workspace=ws)
    torch.cuda.synchronize()
    dg4.dg4_layer_status(cfg, g, ws)
    assert row_rel_err(to_np(H), ref).max() <= TOL[c.dtype]
    H3 = torch.full_like(H, float("nan"))
    dg4.dg4_layer_fwd(cfg_of(c, weights_packed=True), g, X, W, H3, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(H, H3)


@pytest.mark.parametrize("name,n_and,k,over", [("medium", 12_000, 8, {}), ("small", 6_000, 5, {}), ("medium", 6_000, 6, dict(n_layers=2))])
def test_flow_kernel_on_wide_rows(name, n_and, k, over):
    # cones deeper than three hops (rows of up to 2^(k+1)-1 sources, several lane groups per gate):
    # against the oracle, against level-by-level launches, and bit for bit against a sweep cut in two
    print(f"flow kernel, wide rows {name} n_and={n_and} k={k} {over}", flush=True)
    w = make(name, n_and, hops=k, **over)
    c = w.cfg
    g, og = graphs(w)
    assert int(np.diff(og.nbr_ptr).max()) > 16
    cfg = cfg_of(c)
    H = run(w, cfg, g, poison=True)
    assert not torch.isnan(H.float()).any()
    ref = oracle.layer_fwd(og, w.x, w.wqkv, w.wo, w.rel_bias, c.heads, store=c.dtype)
    Hn = to_np(H)
    err = row_rel_err(Hn, ref)
    print(f"  max rel err {err.max():.3e}, max element err {elem_err(Hn, ref).max():.3e}", flush=True)
    assert err.max() <= TOL[c.dtype]
    H_pl = to_np(run(w, cfg_of(c, per_level=True), g))
    assert row_rel_err(Hn, H_pl.astype(np.float64)).max() <= 2 * TOL[c.dtype]
    assert torch.equal(H, run(w, cfg, g))
    mid = g.n_levels // 2
    H1 = run(w, cfg, g, 0, mid)
    H2 = run(w, cfg, g, mid, None, H0=H1)
    assert torch.equal(H2, H)


@pytest.mark.parametrize("name,n_and,over", [("tiny", None, {}), ("small", 3000, dict(n_layers=12)), ("stress", 8000, {}),
                                             ("medium", 8000, dict(n_layers=2))])
def test_flow_kernel_with_feed_forward(name, n_and, over):
    # the whole transformer block per layer (attention sub-block, then LN(h + relu(h W1) W2)), up to the
    # paper's twelve layers, in one persistent launch
    print(f"flow kernel + feed-forward {name} n_and={n_and} {over}", flush=True)
    w = make(name, n_and, **over)
    c = w.cfg
    w1, w2 = synth.ffn_weights(c)
    g, og = graphs(w)

    def go(cfg, level_begin=0, level_end=None, H0=None):
        X = to_dev(w.x, c.dtype)
        W = [lw + (to_dev(w1[l], c.dtype), to_dev(w2[l], c.dtype)) for l, lw in enumerate(device_weights(w, c.dtype))]
        H = torch.full((c.n_nodes, c.hidden), float("nan"), dtype=tdtype(c.dtype), device="cuda") if H0 is None else H0
        ws = torch.empty(dg4.dg4_layer_workspace_bytes(cfg, g), dtype=torch.uint8, device="cuda")
        ws.fill_(0xFF)
        dg4.dg4_layer_fwd(cfg, g, X, W, H, level_begin, level_end, workspace=ws)
        torch.cuda.synchronize()
        dg4.dg4_layer_status(cfg, g, ws)
        return H

    cfg = cfg_of(c, ffn=True)
    H = go(cfg)
    Hn = to_np(H)
    assert not np.isnan(Hn).any()
    ref = oracle.layer_fwd(og, w.x, w.wqkv, w.wo, w.rel_bias, c.heads, store=c.dtype, w1=w1, w2=w2)
    err = row_rel_err(Hn, ref)
    print(f"  max rel err {err.max():.3e}, max element err {elem_err(Hn, ref).max():.3e}", flush=True)
    assert err.max() <= TOL[c.dtype]
    H_pl = to_np(go(cfg_of(c, ffn=True, per_level=True)))
    assert row_rel_err(Hn, H_pl.astype(np.float64)).max() <= 2 * TOL[c.dtype]
    assert torch.equal(H, go(cfg_of(c, ffn=True, level_order=True)))
    mid = g.n_levels // 2
    H2 = go(cfg, mid, None, H0=go(cfg, 0, mid))
    assert torch.equal(H2, H)
