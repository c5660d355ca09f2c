"""The seeded input generators: determinism and the shapes the configurations state."""
import numpy as np

import dg4_synth as synth


def test_rng_is_a_pure_function():
    a = synth.rand_u64(1, 2, 3)
    assert a == synth.rand_u64(1, 2, 3)
    assert len({synth.rand_u64(1, 2, i) for i in range(1000)}) == 1000
    assert synth.rand_u64(1, 2, 3) != synth.rand_u64(1, 3, 2)


def test_normal_moments_and_bf16_grid():
    z = synth.normal(7, 4, (200_000,), 1.0)
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1.0) < 0.01
    assert abs(((z - z.mean()) ** 3).mean()) < 0.03
    b = synth.normal(7, 4, (1000,), 1.0, bf16=True)
    assert (b.view(np.uint32) & 0xFFFF == 0).all()          # exactly representable in bf16
    assert np.abs(b - z[:1000]).max() <= np.abs(z[:1000]).max() * 2.0 ** -8
    assert (synth.normal(7, 4, (1000,)) == z[:1000]).all()  # prefix-stable and deterministic


def test_tiny_graph_shape():
    w = synth.make("tiny")
    c = w.cfg
    assert c.n_nodes == 1032 and len(w.edge_src) == 2000
    j = np.arange(c.n_and)
    assert (w.edge_dst[0::2] == c.n_pi + j).all() and (w.edge_dst[1::2] == c.n_pi + j).all()
    assert (w.edge_src[0::2] != w.edge_src[1::2]).all()              # two distinct fanins
    assert (w.edge_src < w.edge_dst).all()
    assert (w.edge_dst - w.edge_src <= c.window).all()                # windowed
    assert 0.45 < w.edge_inv.mean() < 0.55
    assert w.x.shape == (1032, 128) and w.wqkv[0].shape == (128, 384) and w.rel_bias[0].shape == (4, 4)
    assert abs(w.wqkv[0].std() * 128 ** 0.5 - 1.0) < 0.02             # variance 1/hidden


def test_medium_generator_mixture():
    w = synth.make("medium", features=False)
    far = (w.edge_dst - w.edge_src) > w.cfg.window
    late = w.edge_dst > 50_000
    assert 0.15 < far[late].mean() < 0.21       # ~20% global draws, a few of which land in the window
    assert (w.edge_src[0::2] != w.edge_src[1::2]).all()


def test_large_generator_levels_are_a_valid_capped_schedule():
    w = synth.make("large", n_and=100_000, features=False)
    h = w.level_hint
    assert h.max() <= 1000 and (h[: w.cfg.n_pi] == 0).all() and (h[w.cfg.n_pi:] >= 1).all()
    assert (h[w.edge_src] < h[w.edge_dst]).all()
    assert (w.edge_src[0::2] != w.edge_src[1::2]).all()
    counts = np.bincount(h[w.cfg.n_pi:], minlength=1001)[1:]
    assert counts.min() > 50 and counts.max() < 160                   # ~100 per level, uniform
