"""AIGs with inverters as NODES (the paper's own form, Section 3.2: in-degree 1 = NOT gate).

The synthetic workloads carry inverters as edge flags; `dg4_synth.not_as_nodes` rewrites one into the
paper's form. CPU part: the graph tables on such graphs, and the pin of reading R15: the fanout
counts of Eq. 2 computed on the edge-flag form equal the plain AND / NOT fanout counts of the
rewritten circuit. GPU part: the layer on the rewritten circuit against the oracle.
"""
import numpy as np
import pytest

import dg4_synth as synth
import oracle
import paper_2502_01681_amd as dg4


def rewritten(name, n_and):
    w = synth.make(name, n_and=n_and, features=False)
    n = w.cfg.n_nodes
    n2, src, dst, inv, not_node = synth.not_as_nodes(n, w.edge_src, w.edge_dst, w.edge_inv)
    return w, n, n2, src, dst, inv, not_node


@pytest.mark.parametrize("name,n_and", [("tiny", None), ("small", 6000), ("large", 30_000)])
def test_eq2_fanout_counts_match_the_rewritten_circuit(name, n_and):
    w, n, n2, src, dst, inv, not_node = rewritten(name, n_and)
    assert n2 > n and not inv.any()
    indeg = np.bincount(dst, minlength=n2)
    assert set(np.unique(indeg)) == {0, 1, 2} and (indeg[n:] == 1).all()
    # counted literally on the rewritten circuit: fanouts by type, no reading involved
    want_and = np.bincount(src[indeg[dst] == 2], minlength=n2)
    want_not = np.bincount(src[indeg[dst] == 1], minlength=n2)
    oa2, on2 = oracle.out_degrees(n2, src, dst, inv)
    assert (oa2 == want_and).all() and (on2 == want_not).all()
    # reading R15 on the edge-flag form gives the same numbers for the original gates
    oa, on = oracle.out_degrees(n, w.edge_src, w.edge_dst, w.edge_inv)
    assert (oa == want_and[:n]).all() and (on == want_not[:n]).all()
    assert on.max() == 1 and (on == (not_node >= 0)).all()
    # a NOT node feeds exactly the ANDs that read its signal inverted
    sig = np.nonzero(not_node >= 0)[0]
    inverted_uses = np.bincount(w.edge_src[w.edge_inv == 1], minlength=n)
    assert (want_and[not_node[sig]] == inverted_uses[sig]).all()


@pytest.mark.parametrize("name,n_and,hops", [("tiny", None, 2), ("small", 6000, 3), ("large", 30_000, 2)])
def test_graph_tables_on_the_rewritten_circuit(name, n_and, hops):
    w, n, n2, src, dst, inv, not_node = rewritten(name, n_and)
    g = dg4.dg4_build_levels(n2, src, dst, inv, hops)
    og = oracle.build_levels(n2, src, dst, inv, hops)
    for a in ("level", "order", "level_ptr", "nbr_ptr", "nbr_idx", "nbr_rel"):
        assert (g.array(a) == getattr(og, a)).all(), a
    # a NOT node sits one level above its signal, and its row is its signal's row plus itself
    lev = og.level
    sig = np.nonzero(not_node >= 0)[0]
    assert (lev[not_node[sig]] == lev[sig] + 1).all()
    oa, on = oracle.out_degrees(n2, src, dst, inv)
    assert (g.array("out_and") == oa).all() and (g.array("out_not") == on).all()


@pytest.mark.gpu
@pytest.mark.parametrize("name,n_and,ffn", [("tiny", None, False), ("tiny", None, True), ("large", 30_000, False),
                                            ("large", 30_000, True), ("stress", 10_000, False)])
def test_layer_on_the_rewritten_circuit(name, n_and, ffn):
    import torch
    from gpu_utils import TOL, cfg_of, row_rel_err, tdtype, to_dev, to_np
    print(f"NOT nodes: layer_fwd {name} n_and={n_and} ffn={ffn}", flush=True)
    w, n, n2, src, dst, inv, not_node = rewritten(name, n_and)
    c = w.cfg
    bf = c.dtype == "bf16"
    x = synth.normal(c.seed, synth.STREAM_X, (n2, c.hidden), 1.0, bf)
    w1 = w2 = None
    if ffn:
        w1, w2 = synth.ffn_weights(c)
    g = dg4.dg4_build_levels(n2, src, dst, inv, c.hops)
    og = oracle.build_levels(n2, src, dst, inv, c.hops)
    cfg = cfg_of(c, ffn=ffn)
    W = []
    for l in range(c.n_layers):
        lw = (to_dev(w.wqkv[l], c.dtype), to_dev(w.wo[l], c.dtype), to_dev(w.rel_bias[l], "f32"))
        W.append(lw + ((to_dev(w1[l], c.dtype), to_dev(w2[l], c.dtype)) if ffn else ()))
    H = torch.full((n2, c.hidden), float("nan"), dtype=tdtype(c.dtype), device="cuda")
    dg4.dg4_layer_fwd(cfg, g, to_dev(x, c.dtype), W, H)
    torch.cuda.synchronize()
    Hn = to_np(H)
    assert not np.isnan(Hn).any()
    ref = oracle.layer_fwd(og, x, w.wqkv, w.wo, w.rel_bias, c.heads, store=c.dtype, w1=w1, w2=w2)
    err = row_rel_err(Hn, ref)
    print(f"  {n2 - n} NOT nodes of {n2}; max rel err {err.max():.3e}", flush=True)
    assert err.max() <= TOL[c.dtype]
