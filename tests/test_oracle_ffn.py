"""Pins of the oracle's feed-forward sub-block (the post-norm encoder block that Section 3.5's
unchanged rest of the transformer layer is read as: s' = LN(h + relu(h W1) W2) after the
attention sub-block).

Pinned by mathematics, as the paper prints no value: the dense brute force (library
matrix products, another schedule), a closed form on rows that attend to themselves only,
selector weights that turn the sub-block into a plain rectifier, the positive
homogeneity that only a rectifier has, and the degenerate W2 = 0.
"""
import numpy as np
import pytest

import dg4_synth as synth
import oracle
from helpers import dense_layer, layer_norm
from test_oracle_layer import small_problem


def ffn_weights(d, layers, seed=11):
    w1 = [synth.normal(seed, 200 + 2 * l, (d, 4 * d), d ** -0.5) for l in range(layers)]
    w2 = [synth.normal(seed, 201 + 2 * l, (4 * d, d), (4 * d) ** -0.5) for l in range(layers)]
    return w1, w2


@pytest.mark.parametrize("hops,layers", [(2, 1), (3, 2), (1, 3)])
def test_ffn_layer_against_dense_brute_force(hops, layers):
    n, src, dst, inv, x, wqkv, wo, rb, g = small_problem(layers=layers, hops=hops)
    w1, w2 = ffn_weights(x.shape[1], layers)
    ref = dense_layer(n, src, dst, inv, hops, x, wqkv, wo, rb, heads=2, w1=w1, w2=w2)
    for memo in (False, True):
        H = oracle.layer_fwd(g, x, wqkv, wo, rb, 2, memo=memo, w1=w1, w2=w2)
        assert np.abs(H - ref).max() < 1e-10
    # and the sub-block is not a no-op
    assert np.abs(H - oracle.layer_fwd(g, x, wqkv, wo, rb, 2)).max() > 1e-2


def test_closed_form_on_self_only_rows():
    """A primary input attends to itself alone (alpha = 1), so its embedding is two
    LayerNorms around library matrix products."""
    n, src, dst, inv, x, wqkv, wo, rb, g = small_problem()
    d = x.shape[1]
    w1, w2 = ffn_weights(d, 1)
    H = oracle.layer_fwd(g, x, wqkv, wo, rb, 2, w1=w1, w2=w2)
    X = x.astype(np.float64)
    Wv, Wo = wqkv[0][:, 2 * d:].astype(np.float64), wo[0].astype(np.float64)
    W1, W2 = w1[0].astype(np.float64), w2[0].astype(np.float64)
    pis = np.nonzero(g.level == 0)[0]
    assert len(pis) >= 3
    for v in pis:
        h = layer_norm(X[v] + X[v] @ Wv @ Wo, 1e-5)
        want = layer_norm(h + np.maximum(h @ W1, 0.0) @ W2, 1e-5)
        assert np.abs(H[v] - want).max() < 1e-12
        # transposed or swapped operands must not pass
        assert np.abs(H[v] - layer_norm(h + np.maximum(h @ W2.T, 0.0) @ W1.T, 1e-5)).max() > 1e-3


def test_selector_weights_make_the_block_a_rectifier():
    """W1 = [I 0 0 0], W2 = [I; 0; 0; 0]: the sub-block adds relu(h) to h. Every gate of a
    real graph, sources given: H = LN(h + relu(h)) with h the attention sub-block alone."""
    n, src, dst, inv, x, wqkv, wo, rb, g = small_problem(n_and=120)
    d = x.shape[1]
    w1 = [np.zeros((d, 4 * d), dtype=np.float32)]; w1[0][:, :d] = np.eye(d)
    w2 = [np.zeros((4 * d, d), dtype=np.float32)]; w2[0][:d] = np.eye(d)
    Hsrc = synth.normal(5, 9, (n, d))
    nodes = np.arange(n)
    h = oracle.layer_nodes(g, x, wqkv, wo, rb, 2, Hsrc, nodes)
    H = oracle.layer_nodes(g, x, wqkv, wo, rb, 2, Hsrc, nodes, w1=w1, w2=w2)
    want = np.stack([layer_norm(r + np.maximum(r, 0.0), 1e-5) for r in h])
    assert np.abs(H - want).max() < 1e-12
    # the selector in the second quarter of the hidden units works alike
    w1b = [np.roll(w1[0], d, axis=1)]; w2b = [np.roll(w2[0], d, axis=0)]
    Hb = oracle.layer_nodes(g, x, wqkv, wo, rb, 2, Hsrc, nodes, w1=w1b, w2=w2b)
    assert np.abs(Hb - want).max() < 1e-12


def test_positive_homogeneity_only():
    """relu(c t) = c relu(t) for c > 0 only: (c W1, W2 / c) leaves H unchanged for c = 4
    and changes it for c = -4."""
    n, src, dst, inv, x, wqkv, wo, rb, g = small_problem(layers=2)
    w1, w2 = ffn_weights(x.shape[1], 2)
    H = oracle.layer_fwd(g, x, wqkv, wo, rb, 2, w1=w1, w2=w2)
    Hp = oracle.layer_fwd(g, x, wqkv, wo, rb, 2, w1=[4 * w for w in w1], w2=[w / 4 for w in w2])
    Hn = oracle.layer_fwd(g, x, wqkv, wo, rb, 2, w1=[-4 * w for w in w1], w2=[w / -4 for w in w2])
    assert np.abs(Hp - H).max() < 1e-12          # powers of two: exact scaling
    assert np.abs(Hn - H).max() > 1e-2


def test_zero_second_weight_leaves_a_second_layernorm():
    n, src, dst, inv, x, wqkv, wo, rb, g = small_problem()
    d = x.shape[1]
    w1, _ = ffn_weights(d, 1)
    Hsrc = synth.normal(5, 9, (n, d))
    nodes = np.arange(n)
    h = oracle.layer_nodes(g, x, wqkv, wo, rb, 2, Hsrc, nodes)
    H = oracle.layer_nodes(g, x, wqkv, wo, rb, 2, Hsrc, nodes, w1=w1, w2=[np.zeros((4 * d, d), dtype=np.float32)])
    want = np.stack([layer_norm(r, 1e-5) for r in h])
    assert np.abs(H - want).max() < 1e-12


def test_row_oracle_is_two_library_products_between_layernorms():
    rng = np.random.default_rng(8)
    d = 24
    S = rng.standard_normal((19, d)).astype(np.float32)
    W1 = (rng.standard_normal((d, 4 * d)) / 5).astype(np.float32)
    W2 = (rng.standard_normal((4 * d, d)) / 10).astype(np.float32)
    got = oracle.ffn(S, W1, W2, ln_eps=1e-3)
    S64 = S.astype(np.float64)
    t = S64 + np.maximum(S64 @ W1.astype(np.float64), 0.0) @ W2.astype(np.float64)
    mu = t.mean(axis=1, keepdims=True)
    want = (t - mu) / np.sqrt(((t - mu) ** 2).mean(axis=1, keepdims=True) + 1e-3)
    assert np.abs(got - want).max() < 1e-12
    # eps sits inside the root, the variance is the biased one
    assert np.abs(got - (t - mu) / (t.std(axis=1, ddof=1, keepdims=True))).max() > 1e-3
    # and the layer applies the same function after its attention sub-block
    n, src, dst, inv, x, wqkv, wo, rb, g = small_problem()
    w1, w2 = ffn_weights(x.shape[1], 1)
    h = oracle.layer_fwd(g, x, wqkv, wo, rb, 2)
    pis = np.nonzero(g.level == 0)[0]
    H = oracle.layer_fwd(g, x, wqkv, wo, rb, 2, w1=w1, w2=w2)
    # float32 rows in, so agreement to float32 rounding of h only
    assert np.abs(oracle.ffn(h[pis], w1[0], w2[0]) - H[pis]).max() < 1e-5


def test_ffn_needs_the_epilogue_and_both_weights():
    n, src, dst, inv, x, wqkv, wo, rb, g = small_problem()
    w1, w2 = ffn_weights(x.shape[1], 1)
    with pytest.raises(oracle.OracleError):
        oracle.layer_fwd(g, x, wqkv, wo, rb, 2, epilogue=False, w1=w1, w2=w2)
    with pytest.raises(AssertionError):
        oracle.layer_fwd(g, x, wqkv, wo, rb, 2, w1=w1)


def test_bf16_store_applies_to_the_final_embedding_only():
    n, src, dst, inv, x, wqkv, wo, rb, g = small_problem()
    w1, w2 = ffn_weights(x.shape[1], 1)
    Hsrc = synth.normal(5, 9, (n, x.shape[1]))
    nodes = np.arange(n)
    a = oracle.layer_nodes(g, x, wqkv, wo, rb, 2, Hsrc, nodes, w1=w1, w2=w2)
    b = oracle.layer_nodes(g, x, wqkv, wo, rb, 2, Hsrc, nodes, w1=w1, w2=w2, store="bf16")
    # b is a rounded to 8 significant bits, nothing else
    m, e = np.frexp(a)
    assert np.array_equal(b, np.ldexp(np.rint(np.ldexp(m, 8)), e - 8))
