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


def dense_node(v, mask, relrow, x, H, wqkv, wo, rel_bias, heads, eps=1e-5, epilogue=True, w1=None, w2=None):
    """All layers of node v over the sources selected by the boolean row `mask` (v included),
    sources at their final embeddings in H: dense masked attention in float64."""
    d = x.shape[1]
    dh = d // heads
    s = x[v].copy()
    for l, (W, Wo, B) in enumerate(zip(wqkv, wo, rel_bias)):
        W, Wo, B = (np.asarray(t, dtype=np.float64) for t in (W, Wo, B))
        Wq, Wk, Wv = W[:, :d], W[:, d:2 * d], W[:, 2 * d:]
        state = H.copy()
        state[v] = s
        state[~mask] = 0.0                           # never read; avoid NaN * 0
        q = s @ Wq
        K = state @ Wk
        V = state @ Wv
        a = np.zeros(d)
        for h in range(heads):
            sl = slice(h * dh, (h + 1) * dh)
            sc = K[:, sl] @ q[sl] / np.sqrt(dh) + B[h][relrow]
            sc = np.where(mask, sc, -np.inf)
            p = np.exp(sc - sc.max())
            p /= p.sum()
            a[sl] = p @ V[:, sl]
        o = a @ Wo
        s = layer_norm(s + o, eps) if epilogue else o
        if w1 is not None:
            hid = np.maximum(s @ np.asarray(w1[l], dtype=np.float64), 0.0)
            s = layer_norm(s + hid @ np.asarray(w2[l], dtype=np.float64), eps)
    return s


def dense_layer(n, src, dst, inv, hops, x, wqkv, wo, rel_bias, heads, eps=1e-5, epilogue=True, w1=None, w2=None):
    """Brute-force dense masked attention, float64, one node at a time.

    Multi-layer nesting: a node finishes all its layers before any fanout starts;
    sources are read at their final embedding in every layer. With w1 / w2 (per-layer
    lists) every layer ends with the feed-forward sub-block LN(h + relu(h W1) W2).
    """
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[1]
    A, reach, rel = dense_masks(n, src, dst, inv, hops)
    H = np.full((n, d), np.nan)
    for v in dfs_topological(n, A):
        H[v] = dense_node(v, reach[v], rel[v], x, H, wqkv, wo, rel_bias, heads, eps, epilogue, w1, w2)
    return H


def set_partition(n, src, level, reach, k, delta):
    """Algorithm 1 with Python sets over the dense k-hop reachability: {level: [roots]}.
    Roots of the stride loop by ascending id, then the gates nothing reads, then (one
    decision for all of them) the gates that lie in no cone so far."""
    lists = {}
    top = max(level) if n else 0
    l = k
    while l <= top:
        lists[l] = [v for v in range(n) if level[v] == l]
        l += delta
    read = set(int(s) for s in src)
    for v in range(n):
        if v not in read and v not in lists.get(level[v], []):
            lists.setdefault(level[v], []).append(v)
    covered = np.zeros(n, dtype=bool)
    for roots in lists.values():
        for r in roots:
            covered |= reach[r]
    for v in range(n):
        if not covered[v]:
            lists.setdefault(level[v], []).append(v)
    return {l: r for l, r in lists.items() if r}


def dense_partitioned(n, src, dst, inv, level, k, delta, batch, x, wqkv, wo, rel_bias, heads, mark=True,
                      eps=1e-5, w1=None, w2=None):
    """Algorithm 2 at inference by brute force: per mini-batch a dense N x N mask (the union
    over the batch's cones of "both ends in the cone, and u within k hops of v"), members
    computed in a depth-first topological order. Returns (H, masks, computations) with
    masks[v] the mask row v was last computed with."""
    x = np.asarray(x, dtype=np.float64)
    A, reach, rel = dense_masks(n, src, dst, inv, k)
    lists = set_partition(n, src, level, reach, k, delta)
    topo = dfs_topological(n, A)
    H = np.full((n, x.shape[1]), np.nan)
    masks = np.zeros((n, n), dtype=bool)
    updated = np.zeros(n, dtype=bool)
    work = 0
    for l in sorted(lists):
        roots = lists[l]
        for b in range(0, len(roots), batch):
            M = np.zeros((n, n), dtype=bool)
            members = np.zeros(n, dtype=bool)
            for r in roots[b:b + batch]:
                M |= np.outer(reach[r], reach[r]) & reach
                members |= reach[r]
            for v in topo:
                if members[v] and not (mark and updated[v]):
                    H[v] = dense_node(v, M[v], rel[v], x, H, wqkv, wo, rel_bias, heads, eps, True, w1, w2)
                    masks[v] = M[v]
                    work += 1
            updated |= members
    return H, masks, work
