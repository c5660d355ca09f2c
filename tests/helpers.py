"""Shared test helpers: golden-file parser and an independent dense reference.

Nothing here is used by the product. The dense reference derives the attention
neighbourhood from boolean matrix powers of the adjacency matrix and processes
nodes one at a time in a depth-first topological order, so it shares neither the
neighbourhood derivation nor the schedule with the oracle it pins.
"""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def load_hand_graphs():
    graphs, cur = [], None
    with open(os.path.join(GOLDEN, "hand_graphs.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            tok = line.split()
            if tok[0] == "graph":
                cur = dict(name=tok[1], n=int(tok[2]), hops=int(tok[3]), src=[], dst=[], inv=[], rows={})
            elif tok[0] == "edge":
                cur["src"].append(int(tok[1])); cur["dst"].append(int(tok[2])); cur["inv"].append(int(tok[3]))
            elif tok[0] == "level":
                cur["level"] = [int(t) for t in tok[1:]]
            elif tok[0] == "row":
                cur["rows"][int(tok[1])] = [tuple(int(a) for a in t.split(":")) for t in tok[2:]]
            elif tok[0] == "end":
                graphs.append(cur); cur = None
    return graphs


def dense_masks(n, src, dst, inv, hops):
    """reach[v,u] = u in cone_hops(v); rel[v,u] relation code (0 self, 1/2 direct, 3 virtual)."""
    A = np.zeros((n, n), dtype=bool)          # A[v,u] = edge u -> v
    I = np.zeros((n, n), dtype=np.int64)
    for s, t, i in zip(src, dst, inv):
        A[t, s] = True
        I[t, s] = i
    reach = np.eye(n, dtype=bool)
    P = np.eye(n, dtype=bool)
    for _ in range(hops):
        P = (P.astype(np.int64) @ A.astype(np.int64)) > 0
        reach |= P
    rel = np.full((n, n), 3, dtype=np.int64)
    if hops >= 1:
        rel[A] = 1 + I[A]
    rel[np.eye(n, dtype=bool)] = 0
    return A, reach, rel


def dfs_topological(n, A):
    """A depth-first post-order: every fanin before its fanout, not level by level."""
    seen, out = np.zeros(n, dtype=bool), []

    def visit(v):
        stack = [(v, iter(np.nonzero(A[v])[0]))]
        seen[v] = True
        while stack:
            node, it = stack[-1]
            for u in it:
                if not seen[u]:
                    seen[u] = True
                    stack.append((u, iter(np.nonzero(A[u])[0])))
                    break
            else:
                out.append(node); stack.pop()
    for v in reversed(range(n)):
        if not seen[v]:
            visit(v)
    return out


def layer_norm(t, eps):
    mu = t.mean()
    var = ((t - mu) ** 2).mean()
    return (t - mu) / np.sqrt(var + eps)


def dense_layer(n, src, dst, inv, hops, x, wqkv, wo, rel_bias, heads, eps=1e-5, epilogue=True, w1=None, w2=None):
    """Brute-force dense masked attention, float64, one node at a time.

    Multi-layer nesting: a node finishes all its layers before any fanout starts;
    sources are read at their final embedding in every layer. With w1 / w2 (per-layer
    lists) every layer ends with the feed-forward sub-block LN(h + relu(h W1) W2).
    """
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[1]
    dh = d // heads
    A, reach, rel = dense_masks(n, src, dst, inv, hops)
    H = np.full((n, d), np.nan)
    for v in dfs_topological(n, A):
        s = x[v].copy()
        for l, (W, Wo, B) in enumerate(zip(wqkv, wo, rel_bias)):
            W, Wo, B = (np.asarray(t, dtype=np.float64) for t in (W, Wo, B))
            Wq, Wk, Wv = W[:, :d], W[:, d:2 * d], W[:, 2 * d:]
            state = H.copy()
            state[v] = s
            state[~reach[v]] = 0.0                       # never read; avoid NaN * 0
            q = s @ Wq
            K = state @ Wk
            V = state @ Wv
            a = np.zeros(d)
            for h in range(heads):
                sl = slice(h * dh, (h + 1) * dh)
                sc = K[:, sl] @ q[sl] / np.sqrt(dh) + B[h][rel[v]]
                sc = np.where(reach[v], sc, -np.inf)
                p = np.exp(sc - sc.max())
                p /= p.sum()
                a[sl] = p @ V[:, sl]
            o = a @ Wo
            s = layer_norm(s + o, eps) if epilogue else o
            if w1 is not None:
                hid = np.maximum(s @ np.asarray(w1[l], dtype=np.float64), 0.0)
                s = layer_norm(s + hid @ np.asarray(w2[l], dtype=np.float64), eps)
        H[v] = s
    return H
