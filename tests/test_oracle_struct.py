"""Pins of the oracle's structural encoding (Section 3.5, Eq. 2): hand-worked counts, an independent
recount, closed forms of the linear embeddings."""
import os

import numpy as np
import pytest

import dg4_synth as synth
import oracle

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "struct_encoding.txt")


def load():
    graphs, cur = [], None
    for line in open(GOLDEN):
        tok = line.split("#")[0].split()
        if not tok:
            continue
        if tok[0] == "graph":
            cur = dict(name=tok[1], n=int(tok[2]), src=[], dst=[], inv=[])
        elif tok[0] == "edge":
            cur["src"].append(int(tok[1])); cur["dst"].append(int(tok[2])); cur["inv"].append(int(tok[3]))
        elif tok[0] in ("outand", "outnot"):
            cur[tok[0]] = [int(t) for t in tok[1:]]
        elif tok[0] == "end":
            graphs.append(cur)
    return graphs


@pytest.mark.parametrize("gr", load(), ids=lambda g: g["name"])
def test_hand_counts(gr):
    oa, on = oracle.out_degrees(gr["n"], gr["src"], gr["dst"], gr["inv"])
    assert oa.tolist() == gr["outand"] and on.tolist() == gr["outnot"]


def recount(n, src, dst, inv):
    """The same reading, written differently: set-based, one fanout gate at a time."""
    indeg = np.bincount(dst, minlength=n)
    and_gates = [set() for _ in range(n)]
    not_gates = [set() for _ in range(n)]
    for s, t, i in zip(src.tolist(), dst.tolist(), inv.tolist()):
        if indeg[t] == 1:
            not_gates[s].add(("node", t))
        elif i:
            not_gates[s].add(("inverter of", s))
        else:
            and_gates[s].add(t)
    return np.array([len(a) for a in and_gates]), np.array([len(b) for b in not_gates])


@pytest.mark.parametrize("name,n_and", [("tiny", None), ("small", None), ("large", 30_000)])
def test_counts_against_recount_and_totals(name, n_and):
    w = synth.make(name, n_and=n_and, features=False)
    n = w.cfg.n_nodes
    oa, on = oracle.out_degrees(n, w.edge_src, w.edge_dst, w.edge_inv)
    ra, rn = recount(n, w.edge_src, w.edge_dst, w.edge_inv)
    assert (oa == ra).all() and (on == rn).all()
    # every gate here is a PI or an AND: plain edges are counted one by one, inverted ones once per source
    assert oa.sum() == int((w.edge_inv == 0).sum())
    assert on.sum() == len(np.unique(w.edge_src[w.edge_inv == 1]))
    assert on.max() <= 1
    # shuffling the edge list changes nothing
    p = np.random.default_rng(0).permutation(len(w.edge_src))
    oa2, on2 = oracle.out_degrees(n, w.edge_src[p], w.edge_dst[p], w.edge_inv[p])
    assert (oa2 == oa).all() and (on2 == on).all()


def test_linear_embeddings_closed_forms():
    rng = np.random.default_rng(1)
    n, d = 40, 8
    x = rng.standard_normal((n, d)).astype(np.float32)
    level = rng.integers(0, 30, n).astype(np.int32)
    oa = rng.integers(0, 5, n).astype(np.int32)
    on = rng.integers(0, 2, n).astype(np.int32)
    emb = rng.standard_normal((6, d)).astype(np.float32)
    zero = np.zeros((6, d), dtype=np.float32)
    # no embedding: the features pass through
    assert (oracle.struct_encode(x, level, oa, on, zero) == x.astype(np.float64)).all()
    # biases only: one constant vector for every gate
    b = zero.copy(); b[1], b[3], b[5] = emb[1], emb[3], emb[5]
    out = oracle.struct_encode(x, level, oa, on, b)
    assert np.allclose(out - x, (emb[1].astype(np.float64) + emb[3] + emb[5])[None, :], rtol=0, atol=1e-12)
    # the full formula with matrices: [level, 1, OutAND, 1, OutNOT, 1] @ emb
    F = np.stack([level, np.ones(n), oa, np.ones(n), on, np.ones(n)], axis=1).astype(np.float64)
    assert np.allclose(oracle.struct_encode(x, level, oa, on, emb), x + F @ emb.astype(np.float64), rtol=0, atol=1e-10)
    # each term alone scales with its own count only
    only_l = zero.copy(); only_l[0] = emb[0]
    out = oracle.struct_encode(x, level, np.zeros_like(oa), np.zeros_like(on), only_l)
    assert np.allclose(out - x, level[:, None] * emb[0].astype(np.float64)[None, :], rtol=0, atol=1e-12)
    assert (oracle.struct_encode(x, level, oa, on, only_l) == out).all()     # counts do not leak into the level term
    # stored as bfloat16: every value has at most 8 significant bits and is the nearest such value
    ob = oracle.struct_encode(x, level, oa, on, emb, store="bf16")
    assert (ob.astype(np.float32).view(np.uint32) & 0xFFFF == 0).all()
    ex = oracle.struct_encode(x, level, oa, on, emb)
    assert (np.abs(ob - ex) <= np.abs(ex) * 2.0 ** -8 + 1e-30).all()
