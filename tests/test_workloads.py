"""The seeded input generators: shapes, determinism, tree well-formedness."""
import numpy as np
import pytest

from workloads import (CONFIGS, chain_tree, gen_draft_tokens, gen_logits, gen_qkv, gen_trees,
                       gen_uniforms, round_to_bf16)


@pytest.mark.parametrize("n,depth,topk", [(1, 3, 2), (2, 1, 1), (26, 5, 4), (26, 6, 4), (60, 6, 10), (64, 6, 10)])
def test_tree_shape(n, depth, topk):
    parent, n_nodes = gen_trees(5, 3, 64, depth, topk, n_nodes=[n] * 3)
    assert n_nodes.tolist() == [n] * 3
    assert not np.array_equal(parent[0], parent[1]) or n <= 2
    for b in range(3):
        p = parent[b]
        assert p[0] == -1 and np.all(p[n:] == -1)
        level = np.zeros(n, int)
        for i in range(1, n):
            assert 0 <= p[i] < i
            level[i] = level[p[i]] + 1
        assert level.max() <= depth
        assert np.all(np.diff(level) >= 0)               # breadth-first numbering
        assert np.bincount(p[1:n], minlength=1).max(initial=0) <= topk


def test_determinism_and_value_types():
    a = gen_qkv(3, 1, 4, 2, 1, 8, 5, "bf16")
    b = gen_qkv(3, 1, 4, 2, 1, 8, 5, "bf16")
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)
        assert np.all((x.view(np.uint32) & 0xFFFF) == 0)   # exactly representable in bf16
    assert a[0].shape == (1, 4, 2, 8) and a[1].shape == (1, 4, 1, 8) and a[3].shape == (1, 1, 5, 8)
    u = gen_uniforms(1, 2, 7)
    assert u.shape == (2, 2, 7) and u.dtype == np.float32 and u.min() >= 0 and u.max() < 1


def test_round_to_bf16_ties_to_even():
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -7, -3.14159], np.float32)
    r = round_to_bf16(x)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.0 + 2.0 ** -6 and r[3] == 1.0 + 2.0 ** -7
    assert abs(r[4] + 3.14159) < 2.0 ** -7


def test_draft_tokens_are_distinct_per_parent():
    parent, n_nodes = gen_trees(9, 2, 60, 6, 10)
    logits = gen_logits(9, 2, 60, 500)
    for mode in ("greedy", "sample"):
        tok = gen_draft_tokens(9, logits, parent, n_nodes, mode)
        assert tok.min() >= 0 and tok.max() < 500
        for b in range(2):
            for p in range(60):
                kids = tok[b, 1:][parent[b, 1:] == p]
                assert len(set(kids.tolist())) == len(kids)


def test_config_byte_counts_match_stated_sizes():
    c1, c3 = CONFIGS["c1"], CONFIGS["c3"]
    assert abs(c1.step_bytes() / 1e6 - 37.7) < 0.2       # Vicuna-7B layer: 37.7 MB per step
    assert abs(c3.step_bytes() / 1e9 - 26.97) < 0.1      # Vicuna-33B stack: 26.97 GB per step
    assert abs(CONFIGS["c4"].step_flops() / 1e12 - 2.586) < 0.01
    assert chain_tree(4).tolist() == [-1, 0, 1, 2]


def test_sampled_drafts_are_distinct_per_parent_and_repeatable():
    from workloads import gen_logits, gen_sampled_drafts, gen_trees
    B, N, V = 3, 20, 50
    parent, n_nodes = gen_trees(5, B, N, 4, 4, n_nodes=[20, 7, 1])
    logits = gen_logits(5, B, N, V)
    dl, tok = gen_sampled_drafts(5, logits, parent, n_nodes, 0.8)
    dl2, tok2 = gen_sampled_drafts(5, logits, parent, n_nodes, 0.8)
    assert np.array_equal(dl, dl2) and np.array_equal(tok, tok2)
    assert dl.dtype == np.float32 and dl.shape == logits.shape and tok.dtype == np.int32
    assert not np.array_equal(dl, logits)
    for b in range(B):
        for p in range(int(n_nodes[b])):
            kids = [c for c in range(p + 1, int(n_nodes[b])) if parent[b, c] == p]
            assert len(set(tok[b, kids].tolist())) == len(kids)       # drawn without replacement
            assert all(0 <= t < V for t in tok[b, kids])


def test_draft_layer_inputs_are_bf16_values_with_unit_scale():
    from workloads import gen_draft_layer, round_to_bf16, tree_depths, gen_trees
    d = gen_draft_layer(3, 2, 5, 256, 512, 4, 2, 64, 16)
    assert d["w_qkv"].shape == (8 * 64, 256) and d["w_down"].shape == (512, 512) and d["k_cache"].shape == (2, 2, 16, 64)
    for k, a in d.items():
        assert a.dtype == np.float32 and np.array_equal(a, round_to_bf16(a)), k
    assert 0.8 < d["eta"].std() < 1.2
    assert 0.8 < (d["eta"][0] @ d["w_qkv"].T).std() < 1.2           # projections keep O(1) entries
    parent, n_nodes = gen_trees(3, 2, 5, 3, 2, n_nodes=[5, 2])
    depth = tree_depths(parent, n_nodes)
    assert depth[0, 0] == 0 and all(depth[0, i] == depth[0, parent[0, i]] + 1 for i in range(1, 5))
    assert depth[1, 2:].tolist() == [0, 0, 0]
