"""The seeded generators: determinism, stated shapes, guard bands, tree limits."""
import numpy as np

from mars_inputs import CONFIGS, bf16_bits_to_f32, f32_to_bf16_bits, make_config, make_workload, random_tree


def test_bf16_round_trip_and_rounding():
    x = np.array([1.0, 3.140625, -2.0, 22.37, 0.1], np.float32)
    b = f32_to_bf16_bits(x)
    assert b[:3].tolist() == [0x3F80, 0x4049, 0xC000]
    y = bf16_bits_to_f32(b)
    assert y[3] == 22.375 and abs(y[4] - 0.1) < 0.1 * 2 ** -8
    assert np.array_equal(f32_to_bf16_bits(y), b)


def test_configs_have_the_stated_shapes():
    want = {0: (1, 9, 32000, "f32"), 1: (1, 60, 151936, "bf16"), 2: (16, 60, 151936, "bf16"),
            3: (64, 9, 128256, "bf16"), 4: (256, 26, 151936, "f32")}
    for k, (B, N, V, dt) in want.items():
        c = CONFIGS[k]
        assert (c["B"], c["N"], c["V"], c["dtype"]) == (B, N, V, dt)
    assert CONFIGS[2]["dense_q"] and CONFIGS[2]["temperature"] == 0.7
    assert CONFIGS[4]["B"] * CONFIGS[4]["N"] * CONFIGS[4]["V"] * 4 == 4_045_144_064


def test_generation_is_deterministic_and_thread_independent():
    a = make_config(1, V=4096, N=12, tree={"kind": "tree", "depth": 3, "max_children": 4}, threads=1)
    b = make_config(1, V=4096, N=12, tree={"kind": "tree", "depth": 3, "max_children": 4}, threads=4)
    for k in ("logits", "draft_tokens", "tree_parent", "uniforms", "theta"):
        assert np.array_equal(getattr(a, k), getattr(b, k))


def test_guard_band_on_the_stored_ratio_and_token_recipe():
    w = make_config(3, B=16, V=8192)
    z = w.logits_f32().astype(np.float64)
    top = np.sort(z, axis=2)[:, :, -2:]
    ratio = top[:, :, 0] / top[:, :, 1]
    assert (np.abs(ratio - w.theta[:, None].astype(np.float64)) >= 1e-4).all()
    assert {round(float(t), 2) for t in np.unique(w.theta)} <= {0.85, 0.9, 0.95}
    # most draft tokens are the parent's arg-max or runner-up
    order = np.argsort(-z, axis=2, kind="stable")
    hits = 0
    for b in range(w.B):
        for i in range(1, w.N):
            hits += w.draft_tokens[b, i] in order[b, w.tree_parent[b, i], :2]
    assert hits / (w.B * (w.N - 1)) > 0.7


def test_trees_respect_depth_and_fanout_and_are_topological():
    rng = np.random.default_rng(0)
    for N, depth, fan in ((60, 6, 4), (26, 5, 4), (9, 8, 1)):
        p = random_tree(rng, N, depth, fan)
        assert p[0] == -1 and all(0 <= p[i] < i for i in range(1, N))
        d = np.zeros(N, int)
        for i in range(1, N):
            d[i] = d[p[i]] + 1
        assert d.max() == depth and np.bincount(p[1:], minlength=N).max() <= fan


def test_dense_draft_distribution_is_a_distribution_and_siblings_differ():
    w = make_workload("t", B=2, N=10, V=3000, dtype="bf16", temperature=0.7,
                      tree={"kind": "tree", "depth": 3, "max_children": 4}, dense_q=True, seed=5)
    assert np.allclose(w.draft_probs.sum(axis=2), 1.0, atol=1e-4) and (w.draft_probs >= 0).all()
    assert w.uniforms.shape == (2, 11) and (w.uniforms >= 0).all() and (w.uniforms < 1).all()
    for b in range(2):
        for p in range(10):
            kids = [w.draft_tokens[b, i] for i in range(1, 10) if w.tree_parent[b, i] == p]
            assert len(set(kids)) == len(kids)


def test_random_tree_rejects_shapes_that_cannot_exist():
    import numpy as np
    import pytest
    from mars_inputs import random_tree
    rng = np.random.default_rng(0)
    with pytest.raises(ValueError):
        random_tree(rng, 33, 2, 3)          # 1 + 3 + 9 = 13 nodes at most
    with pytest.raises(ValueError):
        random_tree(rng, 5, 7, 2)           # five nodes cannot be seven deep
    p = random_tree(rng, 13, 2, 3)          # exactly full
    assert p[0] == -1 and len(p) == 13
