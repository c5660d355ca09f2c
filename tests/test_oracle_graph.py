"""Pins of the oracle's integer part: levels (Eq. 1), (level,id) order, cone CSR.

Pinned against hand-worked graphs (tests/golden/hand_graphs.txt), the paper's
size bound |cone_k| <= 2^(k+1)-1 with equality on a complete binary fan-in tree
(Section 3.2), boolean matrix powers of the adjacency matrix, and a
longest-path recursion written independently.
"""
import numpy as np
import pytest

import dg4_synth as synth
import oracle
from helpers import dense_masks, load_hand_graphs


@pytest.mark.parametrize("g", load_hand_graphs(), ids=lambda g: g["name"])
def test_hand_graphs(g):
    og = oracle.build_levels(g["n"], g["src"], g["dst"], g["inv"], g["hops"])
    assert og.level.tolist() == g["level"]
    for v, row in g["rows"].items():
        lo, hi = og.nbr_ptr[v], og.nbr_ptr[v + 1]
        assert list(zip(og.nbr_idx[lo:hi].tolist(), og.nbr_rel[lo:hi].tolist())) == row, v
    # order: ids by (level, id)
    expect = sorted(range(g["n"]), key=lambda v: (g["level"][v], v))
    assert og.order.tolist() == expect
    counts = np.bincount(g["level"])
    assert og.level_ptr.tolist() == [0] + np.cumsum(counts).tolist()


def complete_tree(depth):
    """Complete binary fan-in tree: root id 0, children of i are 2i+1, 2i+2 (heap layout)."""
    n = 2 ** (depth + 1) - 1
    src, dst = [], []
    for i in range(2 ** depth - 1):
        src += [2 * i + 1, 2 * i + 2]
        dst += [i, i]
    return n, src, dst, [0] * len(src)


@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_cone_size_bound_is_tight_on_complete_tree(k):
    n, src, dst, inv = complete_tree(5)
    g = oracle.build_levels(n, src, dst, inv, k)
    sizes = np.diff(g.nbr_ptr)
    assert sizes.max() == 2 ** (k + 1) - 1 == sizes[0]
    assert g.level[0] == 5 and (g.level[-32:] == 0).all()


def longest_path_levels(n, src, dst):
    fanin = [[] for _ in range(n)]
    for s, t in zip(src, dst):
        fanin[t].append(s)
    memo = {}

    def lev(v):
        stack = [v]
        while stack:
            u = stack[-1]
            todo = [w for w in fanin[u] if w not in memo]
            if todo:
                stack.extend(todo)
            else:
                memo[u] = 0 if not fanin[u] else 1 + max(memo[w] for w in fanin[u])
                stack.pop()
        return memo[v]
    return [lev(v) for v in range(n)]


def test_levels_against_recursion_and_csr_against_matrix_powers():
    w = synth.make("tiny", features=False)
    n = w.cfg.n_nodes
    for hops in (1, 2, 3):
        g = oracle.build_levels(n, w.edge_src, w.edge_dst, w.edge_inv, hops)
        if hops == 1:
            assert g.level.tolist() == longest_path_levels(n, w.edge_src, w.edge_dst)
        _, reach, rel = dense_masks(n, w.edge_src, w.edge_dst, w.edge_inv, hops)
        for v in range(n):
            lo, hi = g.nbr_ptr[v], g.nbr_ptr[v + 1]
            ids = g.nbr_idx[lo:hi]
            assert (np.diff(ids) > 0).all()
            assert ids.tolist() == np.nonzero(reach[v])[0].tolist()
            assert g.nbr_rel[lo:hi].tolist() == rel[v, ids].tolist()
        assert np.diff(g.nbr_ptr).max() <= 2 ** (hops + 1) - 1


def test_csr_does_not_depend_on_edge_list_order():
    w = synth.make("tiny", features=False)
    n = w.cfg.n_nodes
    g0 = oracle.build_levels(n, w.edge_src, w.edge_dst, w.edge_inv, 2)
    perm = np.random.default_rng(0).permutation(len(w.edge_src))
    g1 = oracle.build_levels(n, w.edge_src[perm], w.edge_dst[perm], w.edge_inv[perm], 2)
    for a in ("level", "order", "level_ptr", "nbr_ptr", "nbr_idx", "nbr_rel"):
        assert (getattr(g0, a) == getattr(g1, a)).all(), a


def test_small_config_depth_and_density():
    # The small configuration is stated to give about 150 topological levels.
    w = synth.make("small", features=False)
    g = oracle.build_levels(w.cfg.n_nodes, w.edge_src, w.edge_dst, w.edge_inv, 2)
    assert 110 <= g.n_levels <= 200, g.n_levels
    assert 6.0 < len(g.nbr_idx) / w.cfg.n_nodes <= 7.0


def test_hint_schedule():
    w = synth.make("large", n_and=20_000, features=False)
    n = w.cfg.n_nodes
    g = oracle.build_levels(n, w.edge_src, w.edge_dst, w.edge_inv, 2, level_hint=w.level_hint)
    assert (g.level == w.level_hint).all()
    asap = oracle.levels(n, w.edge_src, w.edge_dst)
    assert (asap <= w.level_hint).all() and asap.max() < w.level_hint.max()
    bad = w.level_hint.copy()
    bad[w.edge_dst[0]] = 0
    with pytest.raises(oracle.OracleError, match="EHINT"):
        oracle.build_levels(n, w.edge_src, w.edge_dst, w.edge_inv, 2, level_hint=bad)
    bad = w.level_hint.copy()
    bad[0] = 1                                   # a primary input must sit at level 0
    with pytest.raises(oracle.OracleError, match="EHINT"):
        oracle.build_levels(n, w.edge_src, w.edge_dst, w.edge_inv, 2, level_hint=bad)


@pytest.mark.parametrize("src,dst,inv,err", [
    ([0, 1, 2], [3, 3, 3], [0, 0, 0], "EFANIN"),      # in-degree 3
    ([0, 0], [3, 3], [0, 1], "EFANIN"),               # same pair twice
    ([0, 5], [3, 3], [0, 0], "ERANGE"),
    ([0, -1], [3, 3], [0, 0], "ERANGE"),
    ([0, 1], [3, 3], [0, 2], "EINVAL"),
    ([3, 1], [3, 3], [0, 0], "ECYCLE"),               # self loop
    ([0, 3, 2, 4], [3, 4, 4, 3], [0, 0, 0, 0], "ECYCLE"),
])
def test_invalid_graphs(src, dst, inv, err):
    with pytest.raises(oracle.OracleError, match=err):
        oracle.build_levels(5, src, dst, inv, 2)


def test_empty_and_edgeless():
    g = oracle.build_levels(0, [], [], [], 2)
    assert g.n_levels == 1 and len(g.nbr_idx) == 0
    g = oracle.build_levels(3, [], [], [], 2)
    assert g.level.tolist() == [0, 0, 0] and g.nbr_idx.tolist() == [0, 1, 2] and g.nbr_rel.tolist() == [0, 0, 0]
