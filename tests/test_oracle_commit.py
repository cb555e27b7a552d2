"""CPU pins of the oracle's KV-cache commit (no GPU).

The commit has a plain definition (rows of the accepted nodes appended to the prefix in path
order), so the pins are: a hand-worked example, the chain special case (full acceptance appends
the tree rows as they are), the attention oracle itself (a node's tree-attention output equals
plain decode over the committed cache) and the emitted-token bookkeeping across two steps."""
import numpy as np

import oracle
from workloads import chain_tree, gen_draft_tokens, gen_logits, gen_qkv, gen_trees


def test_hand_worked_example():
    # B=1, Hkv=1, D=2, a root with two children; the walk accepted child 2.  Prefix of 2 tokens.
    k_tree = np.array([[[[10., 11.]], [[20., 21.]], [[30., 31.]]]])
    v_tree = -k_tree
    k_cache = np.array([[[[1., 1.], [2., 2.], [0., 0.], [0., 0.], [0., 0.]]]])
    v_cache = k_cache + 100
    path = np.array([[0, 2, -1]], np.int32)
    k2, v2, len2 = oracle.kv_commit(k_tree, v_tree, k_cache, v_cache, [2], path, np.array([2], np.int32))
    assert k2.tolist() == [[[[1., 1.], [2., 2.], [10., 11.], [30., 31.], [0., 0.]]]]
    assert v2.tolist() == [[[[101., 101.], [102., 102.], [-10., -11.], [-30., -31.], [100., 100.]]]]
    assert len2.tolist() == [4]
    assert k_cache[0, 0, 2].tolist() == [0., 0.]      # inputs are not modified


def test_chain_with_full_acceptance_appends_the_tree_rows_in_order():
    B, N, Hq, Hkv, D, L = 2, 9, 4, 2, 64, 37
    q, kt, vt, kc, vc = gen_qkv(3, B, N, Hq, Hkv, D, L + N, "f32")
    path = np.tile(np.arange(N, dtype=np.int32), (B, 1))
    lens = np.array([N, 4], np.int32)
    k2, v2, len2 = oracle.kv_commit(kt, vt, kc, vc, [L, L - 5], path, lens)
    assert np.array_equal(k2[0, :, L:L + N], kt[0].transpose(1, 0, 2))
    assert np.array_equal(v2[1, :, L - 5:L - 1], vt[1, :4].transpose(1, 0, 2))
    untouched = np.ones(kc.shape[:3], bool)
    untouched[0, :, L:L + N] = False
    untouched[1, :, L - 5:L - 1] = False
    assert np.array_equal(k2[untouched], kc[untouched]) and np.array_equal(v2[untouched], vc[untouched])
    assert len2.tolist() == [L + N, L - 1]


def test_decode_over_the_committed_cache_equals_the_tree_row():
    """Node p = path[-1] sees the prefix and its ancestors, which are exactly the path: after the
    commit, a single-node step whose root carries p's q/k/v and whose prefix is the committed cache
    without p must give p's row of the tree-attention output."""
    B, N, Hq, Hkv, D, L = 3, 26, 4, 2, 64, 50
    parent, n_nodes = gen_trees(5, B, N, 6, 10)
    q, kt, vt, kc, vc = gen_qkv(5, B, N, Hq, Hkv, D, L + N, "f32")
    kv_len = np.array([L, L - 7, 3], np.int32)
    logits = gen_logits(5, B, N, 500, peak=4.0)
    tokens = gen_draft_tokens(5, logits, parent, n_nodes, "greedy")
    path, path_len, _, _ = oracle.accept_greedy(logits, tokens, parent, n_nodes)
    assert path_len.max() >= 3
    tree_out = oracle.tree_attn(q, kt, vt, kc, vc, kv_len, n_nodes, parent)
    k2, v2, len2 = oracle.kv_commit(kt, vt, kc, vc, kv_len, path, path_len)
    last = path[np.arange(B), path_len - 1]
    one = np.full((B, 1), -1, np.int32)
    sel = np.arange(B)
    dec = oracle.tree_attn(q[sel, last][:, None], kt[sel, last][:, None], vt[sel, last][:, None], k2, v2,
                           len2 - 1, np.ones(B, np.int32), one)
    assert np.abs(dec[:, 0] - tree_out[sel, last]).max() < 1e-12


def test_two_chained_steps_grow_the_prefix_by_the_emitted_count():
    B, N, Hkv, D, L = 2, 12, 2, 64, 20
    lens = np.array([L, L], np.int32)
    _, kt, vt, kc, vc = gen_qkv(8, B, N, 2, Hkv, D, L + 2 * N, "f32")
    total = 0
    for step in range(2):
        parent = np.tile(chain_tree(N), (B, 1))
        n_nodes = np.full(B, N, np.int32)
        logits = gen_logits(20 + step, B, N, 300, peak=5.0)
        tokens = gen_draft_tokens(20 + step, logits, parent, n_nodes, "greedy")
        path, path_len, _, n_tok = oracle.accept_greedy(logits, tokens, parent, n_nodes)
        kc, vc, new_lens = oracle.kv_commit(kt, vt, kc, vc, lens, path, path_len)
        assert np.array_equal(new_lens - lens, n_tok)   # one cached position per emitted token
        for b in range(B):
            assert np.array_equal(kc[b, :, lens[b]:new_lens[b]], kt[b, path[b, :path_len[b]]].transpose(1, 0, 2))
        lens, total = new_lens, total + int(n_tok.sum())
    assert int(lens.sum()) == 2 * L + total
