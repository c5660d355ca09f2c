"""Host side of the C ABI (no GPU): the library loads, exports every declared
symbol, and dg4_build_levels matches the oracle bit for bit."""
import ctypes
import os
import re

import numpy as np
import pytest

import dg4_synth as synth
import oracle
import paper_2502_01681_amd as dg4
from helpers import load_hand_graphs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "dg4.h")).read()
    names = set(re.findall(r"^(?:int|int64_t|void|const char\*)\s+(dg4_[a-z_]+)\s*\(", hdr, flags=re.M))
    assert len(names) == 22
    assert {"dg4_build_levels", "dg4_qkv_proj", "dg4_sparse_attn_fwd", "dg4_layer_fwd", "dg4_struct_encode"} <= names
    L = ctypes.CDLL(dg4.library_path()) if os.path.exists(dg4.library_path()) else dg4.lib()
    for n in sorted(names):
        assert hasattr(L, n), n


def same_tables(g, og):
    for a in ("level", "order", "level_ptr", "nbr_ptr", "nbr_idx", "nbr_rel"):
        mine, ref = g.array(a), getattr(og, a)
        assert mine.dtype == ref.dtype and mine.shape == ref.shape and (mine == ref).all(), a


@pytest.mark.parametrize("gr", load_hand_graphs(), ids=lambda g: g["name"])
def test_hand_graphs(gr):
    g = dg4.dg4_build_levels(gr["n"], gr["src"], gr["dst"], gr["inv"], gr["hops"])
    assert g.array("level").tolist() == gr["level"]
    ptr, idx, rel = g.array("nbr_ptr"), g.array("nbr_idx"), g.array("nbr_rel")
    for v, row in gr["rows"].items():
        assert list(zip(idx[ptr[v]:ptr[v + 1]].tolist(), rel[ptr[v]:ptr[v + 1]].tolist())) == row


@pytest.mark.parametrize("name,n_and,hops", [("tiny", None, 1), ("tiny", None, 2), ("tiny", None, 3),
                                             ("tiny", None, 4), ("tiny", None, 8), ("small", 3000, 6), ("stress", 2000, 8),
                                              ("small", None, 2), ("medium", 50_000, 2),
                                              ("large", 60_000, 2), ("stress", 60_000, 3)])
def test_tables_bit_exact_against_oracle(name, n_and, hops):
    w = synth.make(name, n_and=n_and, features=False)
    n = w.cfg.n_nodes
    for hint in ([None, w.level_hint] if w.level_hint is not None else [None]):
        g = dg4.dg4_build_levels(n, w.edge_src, w.edge_dst, w.edge_inv, hops, hint)
        og = oracle.build_levels(n, w.edge_src, w.edge_dst, w.edge_inv, hops, hint)
        same_tables(g, og)
        assert g.n == n and g.n_levels == og.n_levels and g.nnz == len(og.nbr_idx)


@pytest.mark.parametrize("name,n_and,hops,hint", [("tiny", None, 2, False), ("small", None, 2, False),
                                                   ("large", 60_000, 2, True), ("large", 60_000, 2, False),
                                                   ("stress", 40_000, 3, True)])
def test_dataflow_order_is_a_valid_schedule(name, n_and, hops, hint):
    # the order of whole-graph sweeps on the device: every gate once, in tiles of at most 16, and
    # every gate of a neighbour row in a strictly earlier tile than the row's own gate
    w = synth.make(name, n_and=n_and, features=False)
    n = w.cfg.n_nodes
    g = dg4.dg4_build_levels(n, w.edge_src, w.edge_dst, w.edge_inv, hops, w.level_hint if hint else None)
    order, tp = g.array("flow_order"), g.array("flow_tile_ptr")
    assert sorted(order.tolist()) == list(range(n))
    assert tp[0] == 0 and tp[-1] == n
    rows = np.diff(tp)
    cap = int(rows.max())                                  # the tile size the scheduler chose for this circuit
    assert rows.min() >= 1 and cap in (2, 4, 8, 16)
    tile_of = np.empty(n, dtype=np.int64)
    tile_of[order] = np.repeat(np.arange(len(rows)), rows)
    ptr, idx = g.array("nbr_ptr"), g.array("nbr_idx")
    dst = np.repeat(np.arange(n), np.diff(ptr))
    other = idx != dst
    assert (tile_of[idx[other]] < tile_of[dst[other]]).all()
    # a primary input has no source: all of them fit into the leading tiles, which are full
    n_pi = int((np.diff(ptr) == 1).sum())
    assert (rows[: n_pi // cap] == cap).all()
    # the same graph gives the same order again
    g2 = dg4.dg4_build_levels(n, w.edge_src, w.edge_dst, w.edge_inv, hops, w.level_hint if hint else None)
    assert (g2.array("flow_order") == order).all()


def test_tile_size_follows_the_width_of_the_circuit():
    # deep and narrow (a few hundred gates per dependency level): small tiles, so that a gate waits for its
    # own sources and little else; wide: full tiles of 16 (pairs: 8 and 16)
    deep = synth.make("medium", n_and=100_000, features=False)
    wide = synth.make("large", n_and=200_000, features=False)
    sizes = {}
    for tag, w in (("deep", deep), ("wide", wide)):
        g = dg4.dg4_build_levels(w.cfg.n_nodes, w.edge_src, w.edge_dst, w.edge_inv, 2, w.level_hint)
        sizes[tag] = (int(np.diff(g.array("flow_tile_ptr")).max()), int(np.diff(g.array("pair_tile_ptr")).max()))
    assert sizes["deep"] == (2, 8) and sizes["wide"] == (16, 16), sizes


@pytest.mark.parametrize("name,n_and,hint", [("tiny", None, False), ("medium", 30_000, False), ("large", 40_000, True)])
def test_pair_order_is_a_valid_schedule(name, n_and, hint):
    # the order of sweeps with the feed-forward sub-block: tiles in pairs (2k, 2k+1), at most 16 gates
    # each, the second possibly empty; every gate of a neighbour row in a strictly earlier PAIR
    w = synth.make(name, n_and=n_and, features=False)
    n = w.cfg.n_nodes
    g = dg4.dg4_build_levels(n, w.edge_src, w.edge_dst, w.edge_inv, 2, w.level_hint if hint else None)
    order, tp = g.array("pair_order"), g.array("pair_tile_ptr")
    assert sorted(order.tolist()) == list(range(n))
    assert tp[0] == 0 and tp[-1] == n and (len(tp) - 1) % 2 == 0
    rows = np.diff(tp)
    cap = int(rows.max())
    assert rows.min() >= 0 and cap in (8, 16)
    assert (rows[0::2] >= 1).all()                         # only a second tile may be empty ...
    assert (rows[1::2][rows[0::2] < cap] == 0).all()       # ... and is, unless the first one is full
    pair_of = np.empty(n, dtype=np.int64)
    pair_of[order] = np.repeat(np.arange(len(rows)), rows) // 2
    ptr, idx = g.array("nbr_ptr"), g.array("nbr_idx")
    dst = np.repeat(np.arange(n), np.diff(ptr))
    other = idx != dst
    assert (pair_of[idx[other]] < pair_of[dst[other]]).all()


@pytest.mark.parametrize("name,n_and", [("tiny", None), ("small", None), ("large", 40_000)])
def test_fanout_counts_of_the_structural_encoding(name, n_and):
    # OutAND / OutNOT of Eq. 2, bit for bit against the oracle; also on a graph with in-degree-1 nodes
    w = synth.make(name, n_and=n_and, features=False)
    n = w.cfg.n_nodes
    g = dg4.dg4_build_levels(n, w.edge_src, w.edge_dst, w.edge_inv, 2, w.level_hint)
    oa, on = oracle.out_degrees(n, w.edge_src, w.edge_dst, w.edge_inv)
    assert (g.array("out_and") == oa).all() and (g.array("out_not") == on).all()
    # drop the second fanin of every third AND: those gates become NOT/buffer nodes
    keep = np.ones(len(w.edge_src), dtype=bool)
    keep[np.arange(1, len(w.edge_src), 6)] = False
    src, dst, inv = w.edge_src[keep], w.edge_dst[keep], w.edge_inv[keep]
    g = dg4.dg4_build_levels(n, src, dst, inv, 2)
    oa, on = oracle.out_degrees(n, src, dst, inv)
    assert (g.array("out_and") == oa).all() and (g.array("out_not") == on).all()
    assert on.max() >= 2                                       # a NOT node and the signal's own inverter


def test_shuffled_edges_and_relabelled_nodes():
    w = synth.make("small", n_and=5000, features=False)
    n = w.cfg.n_nodes
    rng = np.random.default_rng(1)
    perm, eperm = rng.permutation(n).astype(np.int32), rng.permutation(len(w.edge_src))
    src, dst, inv = perm[w.edge_src][eperm], perm[w.edge_dst][eperm], w.edge_inv[eperm]
    same_tables(dg4.dg4_build_levels(n, src, dst, inv, 2), oracle.build_levels(n, src, dst, inv, 2))


def test_in_degree_one_nodes():
    # NOT/buffer nodes of the paper's AIG representation (in-degree 1)
    src, dst, inv = [0, 1, 2, 3, 3], [2, 2, 3, 4, 5], [0, 1, 1, 0, 1]
    same_tables(dg4.dg4_build_levels(6, src, dst, inv, 3), oracle.build_levels(6, src, dst, inv, 3))


@pytest.mark.parametrize("src,dst,inv,err", [
    ([0, 1, 2], [3, 3, 3], [0, 0, 0], "EFANIN"),
    ([0, 0], [3, 3], [0, 1], "EFANIN"),
    ([0, 5], [3, 3], [0, 0], "ERANGE"),
    ([0, -1], [3, 3], [0, 0], "ERANGE"),
    ([0, 1], [3, 3], [0, 2], "EINVAL"),
    ([3, 1], [3, 3], [0, 0], "ECYCLE"),
    ([0, 3, 2, 4], [3, 4, 4, 3], [0, 0, 0, 0], "ECYCLE"),
])
def test_invalid_graphs_agree_with_oracle(src, dst, inv, err):
    with pytest.raises(dg4.DG4Error) as e:
        dg4.dg4_build_levels(5, src, dst, inv, 2)
    assert e.value.name == err
    with pytest.raises(oracle.OracleError, match=err):
        oracle.build_levels(5, src, dst, inv, 2)


def test_bad_hint_hops_and_empty():
    with pytest.raises(dg4.DG4Error) as e:
        dg4.dg4_build_levels(3, [0, 1], [2, 2], [0, 0], 2, level_hint=[0, 0, 0])
    assert e.value.name == "EHINT"
    with pytest.raises(dg4.DG4Error) as e:
        dg4.dg4_build_levels(3, [0, 1], [2, 2], [0, 0], 2, level_hint=[0, 1, 2])
    assert e.value.name == "EHINT"
    for hops in (0, 9):
        with pytest.raises(dg4.DG4Error) as e:
            dg4.dg4_build_levels(3, [0, 1], [2, 2], [0, 0], hops)
        assert e.value.name == "EUNSUPPORTED"
    g = dg4.dg4_build_levels(0, [], [], [], 2)
    assert g.n == 0 and g.n_levels == 1 and g.array("level_ptr").tolist() == [0, 0]
    g = dg4.dg4_build_levels(3, [0, 1], [2, 2], [0, 0], 2, level_hint=[0, 0, 5])
    assert g.n_levels == 6 and g.array("level_ptr").tolist() == [0, 2, 2, 2, 2, 2, 3]


def test_config_errors_without_a_device():
    g = dg4.dg4_build_levels(3, [0, 1], [2, 2], [0, 0], 2)
    for bad in (dict(hidden=64, heads=2), dict(hidden=128, heads=8), dict(hidden=128, heads=4, n_layers=17),
                dict(hidden=128, heads=4, hops=3)):
        kw = dict(hidden=128, heads=4, hops=2, n_layers=1, dtype="f32")
        kw.update(bad)
        with pytest.raises(dg4.DG4Error):
            dg4.dg4_layer_workspace_bytes(dg4.LayerConfig(**kw), g)
    assert dg4.dg4_layer_workspace_bytes(dg4.LayerConfig(128, 4, 2, 1, "f32"), g) > 0
    assert dg4.dg4_proj_workspace_bytes(dg4.LayerConfig(256, 8, 2, 1, "bf16")) == 256 * 768 * 2


def test_misaligned_tensors_are_refused_before_any_device_work():
    # rows travel as 16-byte pieces: a tensor that does not start on a 16-byte boundary is an
    # argument error, found before anything is queued (so this needs no GPU: the addresses are never used)
    L = dg4.lib()
    cfg = dg4.LayerConfig(128, 4, 2, 1, "f32").c()
    ok, odd = 0x10000, 0x10008
    P = ctypes.c_void_p
    rc = L.dg4_qkv_proj(ctypes.byref(cfg), P(odd), 0, 4, P(ok), P(ok), P(ok), P(ok), P(ok), 1 << 20, None)
    assert rc == -1
    rc = L.dg4_qkv_proj(ctypes.byref(cfg), P(ok), 0, 4, P(ok), P(ok), P(odd), P(ok), P(ok), 1 << 20, None)
    assert rc == -1
    rc = L.dg4_ffn_fwd(ctypes.byref(cfg), P(ok), 0, 4, P(ok), P(ok), P(odd), P(ok), 1 << 20, None)
    assert rc == -1
    g = dg4.dg4_build_levels(3, [0, 1], [2, 2], [0, 0], 2)
    rc = L.dg4_sparse_attn_fwd(ctypes.byref(cfg), g.handle, 0, 3, P(ok), P(odd), P(ok), P(ok), P(ok), None)
    assert rc == -1
    W = (P * 3)(P(ok), P(ok), P(ok))
    rc = L.dg4_layer_fwd(ctypes.byref(cfg), g.handle, P(ok), W, 0, 1, P(odd), P(ok), 1 << 30, None)
    assert rc == -1
