"""Pins of the oracle's graph partition (Section 3.3, Algorithm 1) and updating strategy
(Section 3.4, Algorithm 2, at inference; the ablation without marks of Section 4.4).

The paper prints no worked partition, so the pins are: two cases worked by hand from the two
algorithms (tests/golden/partition_hand.txt), a brute force with Python sets and dense
N x N masks in another schedule, a closed form on strictly layered circuits (every edge
climbs one level: the neighbourhood is the k-hop cone cut at "root level - k", whatever the
mini-batch size), stride 1 reducing to the plain level sweep from level k on, the count
"every gate once" with marks against the recount without, and, without marks, a cone
recomputed alone being the plain sweep of that cone's sub-circuit.
"""
import os

import numpy as np
import pytest

import dg4_synth as synth
import oracle
from helpers import GOLDEN, dense_masks, dense_partitioned, set_partition


def load_partition_cases():
    cases, cur = [], None
    with open(os.path.join(GOLDEN, "partition_hand.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            tok = line.split()
            if tok[0] == "graph":
                cur = dict(name=tok[1], n=int(tok[2]), k=int(tok[3]), delta=int(tok[4]), batch=int(tok[5]),
                           src=[], dst=[], inv=[], hint=None, groups=[], cones={}, rows={})
            elif tok[0] == "edge":
                cur["src"].append(int(tok[1])); cur["dst"].append(int(tok[2])); cur["inv"].append(int(tok[3]))
            elif tok[0] == "level":
                cur["level"] = [int(t) for t in tok[1:]]
            elif tok[0] == "hint":
                cur["hint"] = [int(t) for t in tok[1:]]
                cur["level"] = cur["hint"]
            elif tok[0] == "group":
                cur["groups"].append((int(tok[1]), [int(t) for t in tok[2:]]))
            elif tok[0] == "cone":
                cur["cones"][int(tok[1])] = [int(t) for t in tok[2:]]
            elif tok[0] == "row":
                cur["rows"][int(tok[1])] = [tuple(int(a) for a in t.split(":")) for t in tok[2:]]
            elif tok[0] == "stage":
                cur["stage"] = [int(t) for t in tok[1:]]
            elif tok[0] == "end":
                cases.append(cur); cur = None
    return cases


def problem(n, d=16, heads=2, layers=1, seed=23):
    x = synth.normal(seed, 4, (n, d))
    s = d ** -0.5
    wqkv = [synth.normal(seed, 100 + 3 * l, (d, 3 * d), s) for l in range(layers)]
    wo = [synth.normal(seed, 101 + 3 * l, (d, d), s) for l in range(layers)]
    rb = [synth.normal(seed, 102 + 3 * l, (heads, 4)) for l in range(layers)]
    return x, wqkv, wo, rb


def rows_of(rows, v):
    ptr, idx, rel = rows
    return list(zip(idx[ptr[v]:ptr[v + 1]].tolist(), rel[ptr[v]:ptr[v + 1]].tolist()))


@pytest.mark.parametrize("case", load_partition_cases(), ids=lambda c: c["name"])
def test_hand_worked_partition_and_rows(case):
    n, k = case["n"], case["k"]
    g = oracle.build_levels(n, case["src"], case["dst"], case["inv"], k, level_hint=case["hint"])
    assert g.level.tolist() == case["level"]
    cones = oracle.partition(g, case["src"], case["delta"])
    assert cones.group_level.tolist() == [l for l, _ in case["groups"]]
    for i, (_, roots) in enumerate(case["groups"]):
        assert cones.cone_root[cones.group_ptr[i]:cones.group_ptr[i + 1]].tolist() == roots
    for c, r in enumerate(cones.cone_root.tolist()):
        assert cones.cone(c).tolist() == case["cones"][r]
    x, wqkv, wo, rb = problem(n)
    H, rows, stage, work = oracle.partitioned_fwd(g, cones, case["batch"], x, wqkv, wo, rb, 2)
    for v in range(n):
        assert rows_of(rows, v) == case["rows"][v], v
    assert stage.tolist() == case["stage"]
    assert work == n and np.isfinite(H).all()


def irregular(seed, n_pi=5, n_and=45, window=12, cap=0):
    """cap > 0: the generator's own stretched levelling; cap < 0: twice the Eq. 1 level, plus one
    for an eighth of the gates, so that most gates sit between the root levels and some are left
    in no cone by the two loops of Algorithm 1."""
    src, dst, inv, hint = synth.aig(seed, n_pi, n_and, window, 0.8 if cap > 0 else 1.0, max(cap, 0))
    n = n_pi + n_and
    if cap < 0:
        lev = oracle.levels(n, src, dst)
        odd = np.array([synth.rand_u64(seed, 6, v) % 8 == 0 for v in range(n)]) & (lev > 0)
        hint = (2 * lev + odd).astype(np.int32)
    return n, src, dst, inv, hint


@pytest.mark.parametrize("seed,k,delta,batch,mark,layers,ffn,cap", [
    (1, 3, 2, 1, True, 1, False, 0),
    (2, 3, 2, 4, True, 2, False, 0),
    (3, 3, 1, 3, True, 1, True, 0),
    (4, 2, 1, 128, True, 1, False, 0),
    (5, 3, 2, 2, False, 1, False, 0),
    (6, 3, 2, 128, False, 2, False, 0),
    (7, 3, 2, 3, True, 1, False, 30),      # a stretched levelling: gates left in no cone
    (8, 3, 2, 5, False, 1, True, 30),
    (9, 3, 2, 2, True, 1, False, -1),      # most gates between the root levels
    (10, 3, 2, 4, False, 1, False, -1),
])
def test_against_brute_force_with_sets_and_dense_masks(seed, k, delta, batch, mark, layers, ffn, cap):
    n, src, dst, inv, hint = irregular(seed, n_and=60 if cap < 0 else 45, cap=cap)
    g = oracle.build_levels(n, src, dst, inv, k, level_hint=hint)
    x, wqkv, wo, rb = problem(n, layers=layers)
    d = x.shape[1]
    w1 = [synth.normal(seed, 200 + 2 * l, (d, 4 * d), d ** -0.5) for l in range(layers)] if ffn else None
    w2 = [synth.normal(seed, 201 + 2 * l, (4 * d, d), (4 * d) ** -0.5) for l in range(layers)] if ffn else None
    cones = oracle.partition(g, src, delta)
    H, rows, stage, work = oracle.partitioned_fwd(g, cones, batch, x, wqkv, wo, rb, 2, mark=mark, w1=w1, w2=w2, memo=False)
    H2, rows2, stage2, work2 = oracle.partitioned_fwd(g, cones, batch, x, wqkv, wo, rb, 2, mark=mark, w1=w1, w2=w2, memo=True)
    assert (H == H2).all() and (stage == stage2).all() and work == work2       # the K|V cache changes no bit
    assert all((a == b).all() for a, b in zip(rows, rows2))
    ref, masks, ref_work = dense_partitioned(n, src, dst, inv, g.level.tolist(), k, delta, batch, x, wqkv, wo, rb, 2,
                                             mark=mark, w1=w1, w2=w2)
    # Algorithm 1: the same lists
    _, reach, _ = dense_masks(n, src, dst, inv, k)
    lists = set_partition(n, src, g.level.tolist(), reach, k, delta)
    assert cones.group_level.tolist() == sorted(lists)
    for i, l in enumerate(cones.group_level.tolist()):
        assert cones.cone_root[cones.group_ptr[i]:cones.group_ptr[i + 1]].tolist() == lists[l]
    for c, r in enumerate(cones.cone_root.tolist()):
        assert cones.cone(c).tolist() == np.nonzero(reach[r])[0].tolist()
    # Algorithm 2: the same neighbourhoods, the same count, the same embeddings
    for v in range(n):
        assert [u for u, _ in rows_of(rows, v)] == np.nonzero(masks[v])[0].tolist(), v
    assert work == ref_work
    assert np.abs(H - ref).max() < 1e-10
    if cap < 0:
        # cones of all three kinds: from the stride loop, of gates nothing reads, of gates left over
        read = set(src.tolist())
        kinds = [0, 0, 0]
        for r in cones.cone_root.tolist():
            on_stride = g.level[r] >= k and (g.level[r] - k) % delta == 0
            kinds[0 if on_stride else 1 if r not in read else 2] += 1
        assert min(kinds) >= 2, kinds


def layered(seed, width, depth):
    """Every edge climbs exactly one level; gate j of a level reads gate j of the level below
    (so every gate below the top is read one level up) and one other gate of that level."""
    src, dst, inv = [], [], []
    for lev in range(1, depth + 1):
        for j in range(width):
            v = lev * width + j
            other = (j + 1 + synth.rand_u64(seed, 7, v) % (width - 1)) % width
            for u, s in ((j, 8), (other, 9)):
                src.append((lev - 1) * width + u); dst.append(v); inv.append(synth.rand_u64(seed, s, v) & 1)
    return width * (depth + 1), np.array(src, np.int32), np.array(dst, np.int32), np.array(inv, np.uint8)


@pytest.mark.parametrize("k,delta,depth", [(3, 2, 9), (3, 1, 6), (2, 1, 5), (3, 2, 10)])
def test_layered_circuits_cut_the_cone_at_root_level_minus_k(k, delta, depth):
    n, src, dst, inv = layered(31, 6, depth)
    g = oracle.build_levels(n, src, dst, inv, k)
    assert g.level.tolist() == [v // 6 for v in range(n)]
    x, wqkv, wo, rb = problem(n)
    cones = oracle.partition(g, src, delta)
    root_levels = list(range(k, depth + 1, delta))
    if root_levels[-1] != depth:
        root_levels.append(depth)                      # the top level: read by nothing
    assert cones.group_level.tolist() == root_levels
    results = []
    for batch in (1, 4, 128):
        H, rows, stage, work = oracle.partitioned_fwd(g, cones, batch, x, wqkv, wo, rb, 2)
        assert work == n
        for v in range(n):
            first = min(l for l in root_levels if l >= g.level[v])
            full = list(zip(g.nbr_idx[g.nbr_ptr[v]:g.nbr_ptr[v + 1]].tolist(), g.nbr_rel[g.nbr_ptr[v]:g.nbr_ptr[v + 1]].tolist()))
            assert rows_of(rows, v) == [(u, c) for u, c in full if g.level[u] >= first - k], (batch, v)
        results.append(H)
    assert (results[0] == results[1]).all() and (results[0] == results[2]).all()
    # some rows really are cut when the stride is above one
    if delta > 1:
        assert rows[0][-1] < g.nbr_ptr[-1]


@pytest.mark.parametrize("seed,k", [(11, 2), (12, 3)])
def test_stride_one_is_the_level_sweep_from_level_k_on(seed, k):
    n, src, dst, inv, _ = irregular(seed, n_and=120, window=16)
    g = oracle.build_levels(n, src, dst, inv, k)
    x, wqkv, wo, rb = problem(n, layers=2)
    cones = oracle.partition(g, src, 1)
    H, rows, _, work = oracle.partitioned_fwd(g, cones, 7, x, wqkv, wo, rb, 2)
    assert work == n
    # every gate at level >= k roots a cone, so it sees its whole k-hop cone
    deep = g.level >= k
    assert deep.sum() > n // 2
    cnt = np.diff(rows[0])
    assert (cnt[deep] == np.diff(g.nbr_ptr)[deep]).all()
    # where all rows are whole the result is the plain sweep's, bit for bit
    if (cnt == np.diff(g.nbr_ptr)).all():
        assert (H == oracle.layer_fwd(g, x, wqkv, wo, rb, 2)).all()
    else:
        whole = oracle.layer_fwd(g, x, wqkv, wo, rb, 2)
        assert (H[g.level == 0] == whole[g.level == 0]).all()


def test_stride_one_on_a_layered_circuit_equals_the_level_sweep_bit_for_bit():
    n, src, dst, inv = layered(5, 5, 7)
    g = oracle.build_levels(n, src, dst, inv, 3)
    x, wqkv, wo, rb = problem(n, layers=2)
    H, rows, _, _ = oracle.partitioned_fwd(g, oracle.partition(g, src, 1), 3, x, wqkv, wo, rb, 2)
    assert (np.diff(rows[0]) == np.diff(g.nbr_ptr)).all()
    assert (H == oracle.layer_fwd(g, x, wqkv, wo, rb, 2)).all()


def test_marks_compute_every_gate_once_and_the_ablation_recomputes_overlaps():
    n, src, dst, inv, _ = irregular(21, n_and=200, window=16)
    g = oracle.build_levels(n, src, dst, inv, 3)
    x, wqkv, wo, rb = problem(n)
    cones = oracle.partition(g, src, 2)
    for batch in (1, 16):
        _, _, stage, work = oracle.partitioned_fwd(g, cones, batch, x, wqkv, wo, rb, 2)
        assert work == n and (stage >= 0).all()
        # a gate is computed by the first mini-batch that holds it
        first = np.full(n, -1)
        s = 0
        recount = 0
        for i in range(len(cones.group_level)):
            for b in range(cones.group_ptr[i], cones.group_ptr[i + 1], batch):
                members = set()
                for c in range(b, min(b + batch, cones.group_ptr[i + 1])):
                    members.update(cones.cone(c).tolist())
                recount += len(members)
                for v in members:
                    if first[v] < 0:
                        first[v] = s
                s += 1
        assert (stage == first).all()
        _, _, last, work0 = oracle.partitioned_fwd(g, cones, batch, x, wqkv, wo, rb, 2, mark=False)
        assert work0 == recount and recount > n
        assert (last >= stage).all() and (last > stage).any()


def test_without_marks_a_cone_alone_is_the_sweep_of_its_sub_circuit():
    """Layered circuit, mini-batches of one cone, no marks: the root of the last cone that is
    processed is computed from a from-scratch sweep over exactly that cone."""
    k = 3
    n, src, dst, inv = layered(9, 5, 8)
    g = oracle.build_levels(n, src, dst, inv, k)
    x, wqkv, wo, rb = problem(n)
    cones = oracle.partition(g, src, 2)
    H, _, _, _ = oracle.partitioned_fwd(g, cones, 1, x, wqkv, wo, rb, 2, mark=False)
    for c in (len(cones.cone_root) - 1, len(cones.cone_root) // 2):
        members = cones.cone(c).tolist()
        r = int(cones.cone_root[c])
        new = {v: i for i, v in enumerate(members)}
        keep = [i for i in range(len(src)) if src[i] in new and dst[i] in new]
        s2 = [new[int(src[i])] for i in keep]; d2 = [new[int(dst[i])] for i in keep]; i2 = [int(inv[i]) for i in keep]
        g2 = oracle.build_levels(len(members), s2, d2, i2, k)
        H2 = oracle.layer_fwd(g2, x[members], wqkv, wo, rb, 2)
        later = [c2 for c2 in range(c + 1, len(cones.cone_root)) if r in cones.cone(c2).tolist()]
        if not later:
            assert np.abs(H[r] - H2[new[r]]).max() < 1e-12
