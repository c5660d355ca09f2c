"""Host side of dg4_build_partitioned (no GPU): Algorithm 1's lists, the mini-batch of every gate
and the neighbour rows equal, bit for bit, what the oracle's literal run of Algorithms 1 and 2
uses (Sections 3.3 and 3.4); the processing orders built from such rows stay valid schedules."""
import numpy as np
import pytest

import dg4_synth as synth
import oracle
import paper_2502_01681_amd as dg4
from test_oracle_partition import irregular, layered, load_partition_cases, problem


def oracle_run(n, src, dst, inv, k, delta, batch, hint=None):
    og = oracle.build_levels(n, src, dst, inv, k, level_hint=hint)
    cones = oracle.partition(og, src, delta)
    x, wqkv, wo, rb = problem(n, d=4, heads=1)
    _, rows, stage, work = oracle.partitioned_fwd(og, cones, batch, x, wqkv, wo, rb, 1)
    assert work == n
    return og, cones, rows, stage


def same_partition(g, og, cones, rows, stage):
    assert (g.array("level") == og.level).all() and (g.array("order") == og.order).all()
    assert (g.array("cone_root") == cones.cone_root).all()
    assert (g.array("cone_group_level") == cones.group_level).all()
    assert (g.array("cone_group_ptr") == cones.group_ptr).all()
    assert (g.array("stage") == stage).all()
    for name, ref in zip(("nbr_ptr", "nbr_idx", "nbr_rel"), rows):
        mine = g.array(name)
        assert mine.dtype == ref.dtype and mine.shape == ref.shape and (mine == ref).all(), name
    assert g.nnz == len(rows[1])


@pytest.mark.parametrize("case", load_partition_cases(), ids=lambda c: c["name"])
def test_hand_worked_cases(case):
    g = dg4.dg4_build_partitioned(case["n"], case["src"], case["dst"], case["inv"], case["k"], case["delta"],
                                  case["batch"], level_hint=case["hint"])
    ptr, idx, rel = g.array("nbr_ptr"), g.array("nbr_idx"), g.array("nbr_rel")
    for v, row in case["rows"].items():
        assert list(zip(idx[ptr[v]:ptr[v + 1]].tolist(), rel[ptr[v]:ptr[v + 1]].tolist())) == row
    assert g.array("stage").tolist() == case["stage"]
    assert g.array("cone_root").tolist() == [r for _, roots in case["groups"] for r in roots]
    assert g.array("cone_group_level").tolist() == [l for l, _ in case["groups"]]


@pytest.mark.parametrize("seed,k,delta,batch,cap", [
    (1, 3, 2, 1, 0), (2, 3, 2, 4, 0), (3, 3, 1, 3, 0), (4, 2, 1, 128, 0), (7, 3, 2, 3, 30), (9, 3, 2, 2, -1),
    (10, 3, 2, 128, -1), (11, 3, 1, 5, -1), (12, 8, 6, 128, 0), (13, 8, 6, 4, -1), (14, 5, 3, 16, 40), (15, 8, 7, 1, 0),
])
def test_small_graphs_bit_for_bit(seed, k, delta, batch, cap):
    n, src, dst, inv, hint = irregular(seed, n_and=300, window=24, cap=cap)
    g = dg4.dg4_build_partitioned(n, src, dst, inv, k, delta, batch, level_hint=hint)
    same_partition(g, *oracle_run(n, src, dst, inv, k, delta, batch, hint))


@pytest.mark.parametrize("cfg,k,delta,batch", [("tiny", 3, 2, 128), ("small", 3, 2, 128), ("medium", 2, 1, 16),
                                               ("tiny", 8, 6, 128), ("stress", 8, 6, 128)])
def test_configs_bit_for_bit(cfg, k, delta, batch):
    w = synth.make(cfg, n_and=None if cfg == "tiny" else 3000 if k > 3 else 20000, features=False)
    n, src, dst, inv = w.cfg.n_nodes, w.edge_src, w.edge_dst, w.edge_inv
    g = dg4.dg4_build_partitioned(n, src, dst, inv, k, delta, batch, level_hint=w.level_hint)
    og, cones, rows, stage = oracle_run(n, src, dst, inv, k, delta, batch, w.level_hint)
    same_partition(g, og, cones, rows, stage)
    full = dg4.dg4_build_levels(n, src, dst, inv, k, level_hint=w.level_hint)
    assert g.nnz <= full.nnz


def test_layered_circuit():
    n, src, dst, inv = layered(31, 6, 10)
    g = dg4.dg4_build_partitioned(n, src, dst, inv, 3, 2, 4)
    same_partition(g, *oracle_run(n, src, dst, inv, 3, 2, 4))


def test_arguments():
    n, src, dst, inv, _ = irregular(1)
    for k, delta, batch in [(3, 3, 1), (3, 0, 1), (2, 2, 8), (3, 2, 0), (1, 1, 1)]:
        with pytest.raises(dg4.DG4Error) as e:
            dg4.dg4_build_partitioned(n, src, dst, inv, k, delta, batch)
        assert e.value.name == "EINVAL"
    with pytest.raises(dg4.DG4Error) as e:
        dg4.dg4_build_partitioned(n, src, dst, inv, 9, 2, 8)
    assert e.value.name == "EUNSUPPORTED"
    plain = dg4.dg4_build_levels(n, src, dst, inv, 3)
    with pytest.raises(dg4.DG4Error):
        plain.array("stage")
    empty = dg4.dg4_build_partitioned(0, [], [], [], 3, 2, 8)
    assert empty.array("cone_root").size == 0 and empty.array("cone_group_ptr").tolist() == [0]


@pytest.mark.parametrize("which", ["flow", "pair"])
def test_processing_orders_put_every_source_in_an_earlier_tile(which):
    """Rows cut by the partition may keep a distant source while losing the fanin in between: the
    orders must wait for every source of a row, not only for the direct fanins."""
    n, src, dst, inv, hint = irregular(9, n_and=3000, window=48, cap=-1)
    g = dg4.dg4_build_partitioned(n, src, dst, inv, 3, 2, 8, level_hint=hint)
    order, tile_ptr = g.array(which + "_order"), g.array(which + "_tile_ptr")
    assert sorted(order.tolist()) == list(range(n))
    tile_of = np.empty(n, dtype=np.int64)
    for t in range(len(tile_ptr) - 1):
        tile_of[order[tile_ptr[t]:tile_ptr[t + 1]]] = t // 2 if which == "pair" else t
    ptr, idx, rel = g.array("nbr_ptr"), g.array("nbr_idx"), g.array("nbr_rel")
    fanins = {}
    for s, t in zip(src.tolist(), dst.tolist()):
        fanins.setdefault(t, []).append(s)
    lost = 0
    for v in range(n):
        row = idx[ptr[v]:ptr[v + 1]]
        for u in row:
            assert u == v or tile_of[u] < tile_of[v]
        lost += any(u not in row for u in fanins.get(v, [])) and (rel[ptr[v]:ptr[v + 1]] == 3).any()
    assert lost > 20            # the case this test is about does occur


def members_of_batches(cones, batch):
    out = []
    for i in range(len(cones.group_level)):
        for b in range(cones.group_ptr[i], cones.group_ptr[i + 1], batch):
            cs = range(b, min(b + batch, cones.group_ptr[i + 1]))
            out.append((sorted(set(v for c in cs for v in cones.cone(c).tolist())), [set(cones.cone(c).tolist()) for c in cs]))
    return out


@pytest.mark.parametrize("seed,k,delta,batch,cap", [
    (1, 3, 2, 1, 0), (2, 3, 2, 4, 0), (5, 2, 1, 16, 0), (9, 3, 2, 2, -1), (12, 8, 6, 128, 0), (13, 5, 3, 3, -1),
])
def test_without_marks_one_copy_per_mini_batch_and_gate(seed, k, delta, batch, cap):
    n, src, dst, inv, hint = irregular(seed, n_and=150, window=16, cap=cap)
    g = dg4.dg4_build_partitioned(n, src, dst, inv, k, delta, batch, level_hint=hint, marks=False)
    og = oracle.build_levels(n, src, dst, inv, k, level_hint=hint)
    cones = oracle.partition(og, src, delta)
    x, wqkv, wo, rb = problem(n, d=4, heads=1)
    _, rows, last_stage, work = oracle.partitioned_fwd(og, cones, batch, x, wqkv, wo, rb, 1, mark=False)
    assert g.n == work and (g.array("cone_root") == cones.cone_root).all()
    copy_of, last_copy = g.array("copy_of"), g.array("last_copy")
    ptr, idx, rel, level = g.array("nbr_ptr"), g.array("nbr_idx"), g.array("nbr_rel"), g.array("level")
    assert (level == og.level[copy_of]).all()
    full = {v: dict(zip(og.nbr_idx[og.nbr_ptr[v]:og.nbr_ptr[v + 1]].tolist(), og.nbr_rel[og.nbr_ptr[v]:og.nbr_ptr[v + 1]].tolist()))
            for v in range(n)}
    c = 0
    for members, cone_sets in members_of_batches(cones, batch):
        first = c
        assert copy_of[c:c + len(members)].tolist() == members
        for v in members:
            want = sorted(u for u in full[v] if any(u in cs and v in cs for cs in cone_sets))
            got = idx[ptr[c]:ptr[c + 1]]
            assert ((got >= first) & (got < first + len(members))).all()          # copies of the same mini-batch
            assert copy_of[got].tolist() == want
            assert rel[ptr[c]:ptr[c + 1]].tolist() == [full[v][u] for u in want]
            c += 1
    assert c == g.n
    # the copy that stands: the one of the last mini-batch holding the gate, with the row the oracle used last
    for v in range(n):
        cp = last_copy[v]
        assert copy_of[cp] == v and not (copy_of[cp + 1:] == v).any()
        assert copy_of[idx[ptr[cp]:ptr[cp + 1]]].tolist() == rows[1][rows[0][v]:rows[0][v + 1]].tolist()
    with pytest.raises(dg4.DG4Error):
        g.array("stage")
    marked = dg4.dg4_build_partitioned(n, src, dst, inv, k, delta, batch, level_hint=hint)
    with pytest.raises(dg4.DG4Error):
        marked.array("copy_of")
    assert g.n > marked.n


def test_degenerate_circuits():
    # nothing at all; primary inputs only (each is read by nothing: one cone per input, in the list of level 0)
    for marks in (True, False):
        empty = dg4.dg4_build_partitioned(0, [], [], [], 3, 2, 8, marks=marks)
        assert empty.n == 0 and empty.array("cone_root").size == 0 and empty.array("cone_group_ptr").tolist() == [0]
        g = dg4.dg4_build_partitioned(5, [], [], [], 8, 6, 2, marks=marks)
        assert g.n == 5 and g.array("cone_root").tolist() == [0, 1, 2, 3, 4]
        assert g.array("cone_group_level").tolist() == [0] and g.array("cone_group_ptr").tolist() == [0, 5]
        assert g.array("nbr_idx").tolist() == [0, 1, 2, 3, 4] and g.array("nbr_rel").tolist() == [0] * 5
        if marks:
            assert g.array("stage").tolist() == [0, 0, 1, 1, 2]
        else:
            assert g.array("copy_of").tolist() == [0, 1, 2, 3, 4] and g.array("last_copy").tolist() == [0, 1, 2, 3, 4]
    og = oracle.build_levels(5, [], [], [], 8)
    cones = oracle.partition(og, [], 6)
    assert cones.cone_root.tolist() == [0, 1, 2, 3, 4] and cones.group_level.tolist() == [0]
    # a single AND: level 1 < k, so its cone comes from the "read by nothing" rule and covers the inputs
    g = dg4.dg4_build_partitioned(3, [0, 1], [2, 2], [0, 1], 3, 2, 4)
    assert g.array("cone_root").tolist() == [2] and g.array("cone_group_level").tolist() == [1]
    assert g.array("stage").tolist() == [0, 0, 0] and g.nnz == 5
    og = oracle.build_levels(3, [0, 1], [2, 2], [0, 1], 3)
    assert oracle.partition(og, [0, 1], 2).cone_root.tolist() == [2]
