"""Pins of the oracle's floating-point part.

The paper prints no embedding value, so the numbers are pinned by mathematics:
brute-force dense masked attention (independent neighbourhood derivation and
schedule), closed forms that reduce to library GEMMs, softmax row sums,
invariance to relabelling, schedule independence, and the receptive-field
statement of Section 3.4 (a gate sees exactly {u : u <=_inf v}).
"""
import numpy as np
import pytest

import dg4_synth as synth
import oracle
from helpers import dense_layer, layer_norm


def small_problem(n_and=40, n_pi=6, d=16, heads=2, layers=1, seed=11, window=8, hops=2):
    src, dst, inv, _ = synth.aig(seed, n_pi, n_and, window)
    n = n_pi + n_and
    x = synth.normal(seed, 4, (n, d))
    s = d ** -0.5
    wqkv = [synth.normal(seed, 100 + 3 * l, (d, 3 * d), s) for l in range(layers)]
    wo = [synth.normal(seed, 101 + 3 * l, (d, d), s) for l in range(layers)]
    rb = [synth.normal(seed, 102 + 3 * l, (heads, 4)) for l in range(layers)]
    g = oracle.build_levels(n, src, dst, inv, hops)
    return n, src, dst, inv, x, wqkv, wo, rb, g


@pytest.mark.parametrize("hops,layers,epilogue", [(2, 1, True), (3, 1, True), (2, 3, True), (1, 2, False), (3, 4, True)])
def test_layer_against_dense_brute_force(hops, layers, epilogue):
    n, src, dst, inv, x, wqkv, wo, rb, g = small_problem(layers=layers, hops=hops)
    ref = dense_layer(n, src, dst, inv, hops, x, wqkv, wo, rb, heads=2, epilogue=epilogue)
    for memo in (False, True):
        H = oracle.layer_fwd(g, x, wqkv, wo, rb, 2, epilogue=epilogue, memo=memo)
        assert np.abs(H - ref).max() < 1e-10 * max(1.0, np.abs(ref).max())


def test_memo_and_thread_count_do_not_change_a_bit(monkeypatch):
    n, src, dst, inv, x, wqkv, wo, rb, g = small_problem(n_and=300, layers=2)
    a = oracle.layer_fwd(g, x, wqkv, wo, rb, 2, memo=False)
    b = oracle.layer_fwd(g, x, wqkv, wo, rb, 2, memo=True)
    assert (a == b).all()
    c = oracle.layer_nodes(g, x, wqkv, wo, rb, 2, a.astype(np.float32), np.arange(n))
    # sources rounded to float32 there: equal only approximately
    assert np.abs(c - a).max() < 1e-5


def test_qkv_proj_is_three_gemms():
    rng = np.random.default_rng(3)
    S = rng.standard_normal((37, 24)).astype(np.float32)
    W = rng.standard_normal((24, 72)).astype(np.float32)
    Q, K, V = oracle.qkv_proj(S, W)
    ref = S.astype(np.float64) @ W.astype(np.float64)
    assert np.allclose(Q, ref[:, :24], rtol=0, atol=1e-12)
    assert np.allclose(K, ref[:, 24:48], rtol=0, atol=1e-12)
    assert np.allclose(V, ref[:, 48:], rtol=0, atol=1e-12)
    # a transposed weight must not pass
    assert not np.allclose(Q, S.astype(np.float64) @ W[:, :24].astype(np.float64).T, atol=1e-3)


def test_softmax_rows_sum_to_one_and_attention_matches_dense():
    n, src, dst, inv, x, wqkv, wo, rb, g = small_problem(n_and=200, d=32, heads=4)
    d, heads, dh = 32, 4, 8
    rng = np.random.default_rng(5)
    Q, K, V = (rng.standard_normal((n, d)).astype(np.float32) * 2 for _ in range(3))
    bias = synth.normal(5, 102, (heads, 4))
    A, alpha = oracle.sparse_attn(g, heads, Q, K, V, bias, want_alpha=True)
    B = bias.astype(np.float64)
    assert ((alpha > 0) & (alpha <= 1)).all()
    for v in range(n):
        lo, hi = g.nbr_ptr[v], g.nbr_ptr[v + 1]
        assert np.abs(alpha[lo:hi].sum(axis=0) - 1).max() < 1e-12
        ids, rel = g.nbr_idx[lo:hi], g.nbr_rel[lo:hi]
        for h in range(heads):
            sl = slice(h * dh, (h + 1) * dh)
            sc = K[ids][:, sl].astype(np.float64) @ Q[v, sl].astype(np.float64) / np.sqrt(dh) + B[h][rel]
            p = np.exp(sc - sc.max()); p /= p.sum()
            assert np.abs(p - alpha[lo:hi, h]).max() < 1e-12
            assert np.abs(p @ V[ids][:, sl].astype(np.float64) - A[v, sl]).max() < 1e-12


def test_row_range_leaves_other_rows_untouched():
    n, src, dst, inv, x, wqkv, wo, rb, g = small_problem(n_and=50)
    rng = np.random.default_rng(6)
    Q, K, V = (rng.standard_normal((n, 16)).astype(np.float32) for _ in range(3))
    full = oracle.sparse_attn(g, 2, Q, K, V, rb[0])
    part = oracle.sparse_attn(g, 2, Q, K, V, rb[0], row_begin=10, row_end=30)
    assert (part[10:30] == full[10:30]).all() and (part[:10] == 0).all() and (part[30:] == 0).all()


def test_closed_form_single_source_rows():
    # A row with one source has alpha = 1 (Section 3.7): primary inputs attend to
    # themselves only, so H = LN(x + x Wv Wo), two library GEMMs.
    n, src, dst, inv, x, wqkv, wo, rb, g = small_problem()
    H = oracle.layer_fwd(g, x, wqkv, wo, rb, 2)
    xd = x.astype(np.float64)
    Wv = wqkv[0][:, 32:].astype(np.float64)
    t = xd + xd @ Wv @ wo[0].astype(np.float64)
    for v in range(6):
        assert np.abs(H[v] - layer_norm(t[v], 1e-5)).max() < 1e-12
    # hops = 0: every node is alone in its cone
    g0 = oracle.build_levels(n, src, dst, inv, 0)
    H0 = oracle.layer_fwd(g0, x, wqkv, wo, rb, 2)
    for v in range(n):
        assert np.abs(H0[v] - layer_norm(t[v], 1e-5)).max() < 1e-12


def test_closed_form_uniform_attention_and_hard_selection():
    n, src, dst, inv, x, wqkv, wo, rb, g = small_problem(d=16, heads=2)
    d = 16
    # Wq = 0 and zero bias: alpha = 1/|N(v)|, aggregation is a plain mean of V rows
    W = wqkv[0].copy(); W[:, :d] = 0
    zero_b = [np.zeros((2, 4), dtype=np.float32)]
    H = oracle.layer_fwd(g, x, [W], wo, zero_b, 2, epilogue=False)
    Wv, Wo = W[:, 2 * d:].astype(np.float64), wo[0].astype(np.float64)
    ref = np.zeros((n, d))
    for v in g.order:                                   # level order
        ids = g.nbr_idx[g.nbr_ptr[v]:g.nbr_ptr[v + 1]]
        states = np.stack([x[u].astype(np.float64) if u == v else ref[u] for u in ids])
        ref[v] = (states @ Wv).mean(axis=0) @ Wo
    assert np.abs(H - ref).max() < 1e-12
    # bias +1e4 on the self relation: every node attends to itself only
    hard = [np.array([[1e4, 0, 0, 0]] * 2, dtype=np.float32)]
    Hs = oracle.layer_fwd(g, x, wqkv, wo, hard, 2)
    xd = x.astype(np.float64)
    t = xd + xd @ wqkv[0][:, 2 * d:].astype(np.float64) @ Wo
    for v in range(n):
        assert np.abs(Hs[v] - layer_norm(t[v], 1e-5)).max() < 1e-9
    # bias +1e4 on "direct fanin, not inverted": ANDs with exactly one such fanin copy its V
    sel = [np.array([[0, 1e4, 0, 0]] * 2, dtype=np.float32)]
    Hh = oracle.layer_fwd(g, x, wqkv, wo, sel, 2, epilogue=False)
    checked = 0
    for v in range(6, n):
        lo, hi = g.nbr_ptr[v], g.nbr_ptr[v + 1]
        direct = g.nbr_idx[lo:hi][g.nbr_rel[lo:hi] == 1]
        if len(direct) == 1:
            u = direct[0]
            assert np.abs(Hh[v] - Hh[u] @ wqkv[0][:, 2 * d:].astype(np.float64) @ Wo).max() < 1e-9
            checked += 1
    assert checked > 5


def test_equal_value_rows_make_alpha_irrelevant():
    n, src, dst, inv, x, wqkv, wo, rb, g = small_problem(n_and=60)
    rng = np.random.default_rng(8)
    Q, K = (rng.standard_normal((n, 16)).astype(np.float32) for _ in range(2))
    V = np.tile(rng.standard_normal((1, 16)).astype(np.float32), (n, 1))
    A = oracle.sparse_attn(g, 2, Q, K, V, rb[0])
    assert np.abs(A - V.astype(np.float64)).max() < 1e-12


def test_relabelling_invariance():
    n, src, dst, inv, x, wqkv, wo, rb, g = small_problem(n_and=120, layers=2)
    H = oracle.layer_fwd(g, x, wqkv, wo, rb, 2)
    perm = np.random.default_rng(9).permutation(n)       # new id of old node i is perm[i]
    eperm = np.random.default_rng(10).permutation(len(src))
    src2, dst2, inv2 = perm[src][eperm], perm[dst][eperm], inv[eperm]
    x2 = np.empty_like(x); x2[perm] = x
    g2 = oracle.build_levels(n, src2, dst2, inv2, 2)
    H2 = oracle.layer_fwd(g2, x2, wqkv, wo, rb, 2)
    assert np.abs(H2[perm] - H).max() < 1e-11            # summation order inside rows changed
    assert (g2.level[perm] == g.level).all()


def test_schedule_independence_and_resume():
    w = synth.make("large", n_and=3000, features=False)
    n = w.cfg.n_nodes
    d, heads = 16, 2
    x = synth.normal(1, 4, (n, d))
    wqkv = [synth.normal(1, 100, (d, 3 * d), d ** -0.5)]
    wo = [synth.normal(1, 101, (d, d), d ** -0.5)]
    rb = [synth.normal(1, 102, (heads, 4))]
    g_asap = oracle.build_levels(n, w.edge_src, w.edge_dst, w.edge_inv, 2)
    g_hint = oracle.build_levels(n, w.edge_src, w.edge_dst, w.edge_inv, 2, level_hint=w.level_hint)
    assert g_hint.n_levels > 3 * g_asap.n_levels
    Ha = oracle.layer_fwd(g_asap, x, wqkv, wo, rb, heads, store="bf16")
    Hh = oracle.layer_fwd(g_hint, x, wqkv, wo, rb, heads, store="bf16")
    assert (Ha == Hh).all()                              # per-node arithmetic is fixed
    # unwritten rows are never read: poison them
    poison = np.full((n, d), np.nan)
    Hp = oracle.layer_fwd(g_hint, x, wqkv, wo, rb, heads, store="bf16", H_init=poison)
    assert (Hp == Hh).all()
    # split sweep = whole sweep
    mid = g_hint.n_levels // 3
    H1 = oracle.layer_fwd(g_hint, x, wqkv, wo, rb, heads, store="bf16", H_init=poison, level_end=mid)
    assert np.isnan(H1[g_hint.level >= mid]).all() and not np.isnan(H1[g_hint.level < mid]).any()
    H2 = oracle.layer_fwd(g_hint, x, wqkv, wo, rb, heads, store="bf16", H_init=H1, level_begin=mid)
    assert (H2 == Hh).all()
    # stored values sit on the bf16 grid
    assert (Hh.astype(np.float32).view(np.uint32) & 0xFFFF == 0).all()
    assert (Hh.astype(np.float32) == Hh).all()


def test_receptive_field_is_the_transitive_fanin():
    # Section 3.4: through the historical embeddings a gate aggregates from
    # {u : u <=_inf v}; so changing one primary input changes exactly its fan-out cone.
    n, src, dst, inv, x, wqkv, wo, rb, g = small_problem(n_and=150, n_pi=10, window=12)
    H = oracle.layer_fwd(g, x, wqkv, wo, rb, 2)
    pi = int(src[0])                                     # a primary input that has fan-out
    assert pi < 10
    x2 = x.copy(); x2[pi] += 1.0
    H2 = oracle.layer_fwd(g, x2, wqkv, wo, rb, 2)
    changed = np.abs(H2 - H).max(axis=1) > 0
    A = np.zeros((n, n), dtype=bool); A[dst, src] = True
    reach = np.zeros(n, dtype=bool); reach[pi] = True
    for _ in range(n):
        new = reach | (A[:, reach].any(axis=1))
        if (new == reach).all():
            break
        reach = new
    assert (changed == reach).all() and reach.sum() > 5 and (~reach).sum() > 5


def test_bf16_store_rounding_is_nearest_even():
    # checked through the public path: epilogue off, Wo = I, Wv = I, self-only graph
    d = 8
    vals = np.array([1.0, 1.00390625, 1.01171875, 1.005859375, -3.14159, 1e-3, 255.5, 0.0], dtype=np.float32)
    x = vals[None, :]
    W = np.concatenate([np.zeros((d, d)), np.zeros((d, d)), np.eye(d)], axis=1).astype(np.float32)
    g = oracle.build_levels(1, [], [], [], 2)
    H = oracle.layer_fwd(g, x, [W], [np.eye(d, dtype=np.float32)], [np.zeros((1, 4), np.float32)], 1,
                         store="bf16", epilogue=False)[0]
    # bf16 spacing above 1 is 2^-7. Ties go to the even significand: 1+2^-8 -> 1, 1+3*2^-8 -> 1+2^-6
    assert H[0] == 1.0 and H[1] == 1.0 and H[2] == 1.015625 and H[3] == 1.0078125
    def ref(v):
        u = np.float32(v).view(np.uint32).astype(np.uint64)
        u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
        return np.uint32(u).view(np.float32)
    assert [float(h) for h in H] == [float(ref(v)) for v in vals]
