"""Pins of the CPU oracle's tree attention against things fixed by the mathematics.

None of these retype the oracle's loop: the references are PyTorch's own
scaled_dot_product_attention (a library routine), closed forms, and a case worked
by hand with rational probabilities (tests/golden/attn_rational_case.json).
"""
import json
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from workloads import chain_tree, gen_qkv, gen_trees

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _sdpa_causal_last_rows(q_new, k_all, v_all, scale):
    """Library causal attention: q_new [H,n,D] are the queries of the LAST n positions of
    a sequence whose keys/values are k_all, v_all [H,S,D]; returns [H,n,D] (fp64)."""
    H, n, D = q_new.shape
    S = k_all.shape[1]
    q_full = torch.zeros(H, S, D, dtype=torch.float64)
    q_full[:, S - n:] = torch.from_numpy(q_new)
    out = F.scaled_dot_product_attention(q_full[None], torch.from_numpy(k_all)[None],
                                         torch.from_numpy(v_all)[None], is_causal=True, scale=scale)
    return out[0, :, S - n:].numpy()


def _inputs(seed, B, N, Hq, Hkv, D, L, dtype="f32"):
    q, kt, vt, kc, vc = gen_qkv(seed, B, N, Hq, Hkv, D, max(L, 1), dtype)
    return [a.astype(np.float64) for a in (q, kt, vt, kc, vc)]


def _ancestors(parent, i):
    out = []
    while i >= 0:
        out.append(i)
        i = int(parent[i])
    return out[::-1]  # root .. i


def test_single_node_is_standard_decode(oracle):
    # one node = the not-yet-cached last token: softmax attention over L+1 keys
    B, N, Hq, Hkv, D, L = 2, 1, 4, 4, 16, 37
    q, kt, vt, kc, vc = _inputs(1, B, N, Hq, Hkv, D, L)
    parent = np.full((B, 1), -1, np.int32)
    out = oracle.tree_attn(q, kt, vt, kc, vc, [L] * B, [1] * B, parent)
    for b in range(B):
        k_all = np.concatenate([kc[b, :, :L], kt[b].transpose(1, 0, 2)], axis=1)  # [H,L+1,D]
        v_all = np.concatenate([vc[b, :, :L], vt[b].transpose(1, 0, 2)], axis=1)
        ref = F.scaled_dot_product_attention(torch.from_numpy(q[b].transpose(1, 0, 2))[None],
                                             torch.from_numpy(k_all)[None], torch.from_numpy(v_all)[None],
                                             scale=1 / np.sqrt(D))[0].numpy()  # [H,1,D]
        np.testing.assert_allclose(out[b].transpose(1, 0, 2), ref, rtol=0, atol=1e-12)


@pytest.mark.parametrize("L", [0, 5, 64])
def test_chain_tree_is_causal_attention(oracle, L):
    B, N, Hq, Hkv, D = 1, 9, 3, 3, 8
    q, kt, vt, kc, vc = _inputs(2 + L, B, N, Hq, Hkv, D, L)
    parent = chain_tree(N)[None]
    out = oracle.tree_attn(q, kt, vt, kc, vc, [L], [N], parent)
    k_all = np.concatenate([kc[0, :, :L], kt[0].transpose(1, 0, 2)], axis=1)
    v_all = np.concatenate([vc[0, :, :L], vt[0].transpose(1, 0, 2)], axis=1)
    ref = _sdpa_causal_last_rows(np.ascontiguousarray(q[0].transpose(1, 0, 2)), k_all, v_all, 1 / np.sqrt(D))
    np.testing.assert_allclose(out[0].transpose(1, 0, 2), ref, rtol=0, atol=1e-12)


def test_path_linearisation_on_random_trees(oracle):
    """Row i of tree attention == last row of causal attention over prefix + path(root..i)."""
    B, N, Hq, Hkv, D, L = 2, 26, 4, 2, 16, 19
    q, kt, vt, kc, vc = _inputs(3, B, N, Hq, Hkv, D, L)
    parent, n_nodes = gen_trees(3, B, N, 5, 4)
    out = oracle.tree_attn(q, kt, vt, kc, vc, [L] * B, n_nodes, parent, scale=0.3)
    G = Hq // Hkv
    for b in range(B):
        for i in range(N):
            path = _ancestors(parent[b], i)
            for h in range(Hq):
                g = h // G
                k_all = np.concatenate([kc[b, g, :L], kt[b, path, g]], axis=0)[None]  # [1,S,D]
                v_all = np.concatenate([vc[b, g, :L], vt[b, path, g]], axis=0)[None]
                ref = _sdpa_causal_last_rows(q[b, i, h][None, None], k_all, v_all, 0.3)
                np.testing.assert_allclose(out[b, i, h], ref[0, 0], rtol=0, atol=1e-12)


def test_zero_query_gives_mean_of_visible_values(oracle):
    """Closed form: Q = 0 => uniform weights => mean over prefix rows and ancestors-or-self."""
    B, N, Hq, Hkv, D, L = 1, 26, 2, 1, 8, 11
    q, kt, vt, kc, vc = _inputs(4, B, N, Hq, Hkv, D, L)
    q[:] = 0.0
    parent, n_nodes = gen_trees(4, B, N, 5, 4)
    out = oracle.tree_attn(q, kt, vt, kc, vc, [L], n_nodes, parent)
    for i in range(N):
        anc = _ancestors(parent[0], i)
        expect = (vc[0, 0, :L].sum(0) + vt[0, anc, 0].sum(0)) / (L + len(anc))
        for h in range(Hq):
            np.testing.assert_allclose(out[0, i, h], expect, rtol=0, atol=1e-13)


def test_rational_hand_case(oracle):
    """Scores that are logs of integers make every probability a ratio of integers; the
    expected outputs in the fixture were worked out by hand from those ratios."""
    with open(os.path.join(GOLDEN, "attn_rational_case.json")) as f:
        case = json.load(f)
    a_prefix = np.array(case["prefix_weight"], dtype=np.float64)   # exp(score) of prefix keys
    a_tree = np.array(case["tree_weight"], dtype=np.float64)       # exp(score) of tree keys
    v_prefix = np.array(case["prefix_value"], dtype=np.float64)    # [L,D]
    v_tree = np.array(case["tree_value"], dtype=np.float64)        # [N,D]
    parent = np.array(case["parent"], dtype=np.int32)[None]
    L, N, D = len(a_prefix), len(a_tree), v_prefix.shape[1]
    # q = (1, 0): the score of a key is its first coordinate; scale = 1
    q = np.zeros((1, N, 1, D)); q[..., 0] = 1.0
    kc = np.zeros((1, 1, L, D)); kc[0, 0, :, 0] = np.log(a_prefix)
    kt = np.zeros((1, N, 1, D)); kt[0, :, 0, 0] = np.log(a_tree)
    out = oracle.tree_attn(q, kt, v_tree[None, :, None, :], kc, v_prefix[None, None], [L], [N], parent, scale=1.0)
    expect = np.array([[num / case["expected_den"][i] for num in row]
                       for i, row in enumerate(case["expected_num"])])
    np.testing.assert_allclose(out[0, :, 0, :], expect, rtol=0, atol=1e-14)


def test_empty_prefix_root_row_is_root_value(oracle):
    B, N, Hq, Hkv, D = 1, 7, 2, 2, 8
    q, kt, vt, kc, vc = _inputs(5, B, N, Hq, Hkv, D, 0)
    parent, n_nodes = gen_trees(5, B, N, 3, 3)
    out = oracle.tree_attn(q, kt, vt, None, None, [0], n_nodes, parent)
    np.testing.assert_array_equal(out[0, 0], vt[0, 0])


def test_gqa_equals_mha_with_replicated_kv(oracle):
    B, N, Hq, Hkv, D, L = 1, 12, 8, 2, 8, 23
    q, kt, vt, kc, vc = _inputs(6, B, N, Hq, Hkv, D, L)
    parent, n_nodes = gen_trees(6, B, N, 4, 3)
    out = oracle.tree_attn(q, kt, vt, kc, vc, [L], n_nodes, parent)
    G = Hq // Hkv
    out_mha = oracle.tree_attn(q, np.repeat(kt, G, axis=2), np.repeat(vt, G, axis=2),
                               np.repeat(kc, G, axis=1), np.repeat(vc, G, axis=1), [L], n_nodes, parent)
    np.testing.assert_array_equal(out, out_mha)


def test_non_ancestor_keys_do_not_matter_and_bounds(oracle):
    B, N, Hq, Hkv, D, L = 1, 26, 2, 2, 8, 9
    q, kt, vt, kc, vc = _inputs(7, B, N, Hq, Hkv, D, L)
    parent, n_nodes = gen_trees(7, B, N, 5, 4)
    out = oracle.tree_attn(q, kt, vt, kc, vc, [L], n_nodes, parent)
    i = N - 1
    anc = set(_ancestors(parent[0], i))
    other = [t for t in range(N) if t not in anc]
    kt2, vt2 = kt.copy(), vt.copy()
    kt2[0, other] += 100.0
    vt2[0, other] -= 55.0
    out2 = oracle.tree_attn(q, kt2, vt2, kc, vc, [L], n_nodes, parent)
    np.testing.assert_array_equal(out[0, i], out2[0, i])
    assert not np.array_equal(out[0, other[0]], out2[0, other[0]])
    # a convex combination of visible value rows stays inside their range
    vis = np.concatenate([vc[0, :, :L], vt[0, sorted(anc)].transpose(1, 0, 2)], axis=1)  # [H,*,D]
    assert np.all(out[0, i] <= vis.max(axis=1) + 1e-12) and np.all(out[0, i] >= vis.min(axis=1) - 1e-12)


def test_ragged_batch_and_padding_rows(oracle):
    B, N, Hq, Hkv, D, L = 3, 10, 2, 1, 8, 30
    q, kt, vt, kc, vc = _inputs(8, B, N, Hq, Hkv, D, L)
    n_nodes = np.array([10, 4, 1], np.int32)
    kv_len = np.array([30, 0, 17], np.int32)
    parent, _ = gen_trees(8, B, N, 3, 3, n_nodes=n_nodes)
    out = oracle.tree_attn(q, kt, vt, kc, vc, kv_len, n_nodes, parent)
    for b in range(B):
        n, l = int(n_nodes[b]), int(kv_len[b])
        assert np.all(out[b, n:] == 0)
        solo = oracle.tree_attn(q[b:b + 1, :n], kt[b:b + 1, :n], vt[b:b + 1, :n], kc[b:b + 1, :, :max(l, 1)],
                                vc[b:b + 1, :, :max(l, 1)], [l], [n], parent[b:b + 1, :n])
        np.testing.assert_array_equal(out[b, :n], solo[0])


def test_packed_mask_is_checked_against_tree(oracle):
    B, N, Hq, Hkv, D, L = 1, 6, 1, 1, 8, 3
    q, kt, vt, kc, vc = _inputs(9, B, N, Hq, Hkv, D, L)
    parent = np.array([[-1, 0, 0, 1, 1, 2]], np.int32)
    # transitive closure written out by hand: 0; 0,1; 0,2; 0,1,3; 0,1,4; 0,2,5
    good = np.array([[0b1, 0b11, 0b101, 0b1011, 0b10011, 0b100101]], np.uint64)
    oracle.tree_attn(q, kt, vt, kc, vc, [L], [N], parent, packed_mask=good)
    bad = good.copy()
    bad[0, 4] |= np.uint64(0b100)  # node 4 must not see its uncle 2
    with pytest.raises(ValueError):
        oracle.tree_attn(q, kt, vt, kc, vc, [L], [N], parent, packed_mask=bad)
    # popcount = depth + 1, own bit set, nothing above own bit
    m = oracle.dense_mask(parent[0])
    depth = [0, 1, 1, 2, 2, 2]
    for i in range(N):
        assert m[i].sum() == depth[i] + 1 and m[i, i] == 1 and m[i, i + 1:].sum() == 0
    with pytest.raises(ValueError):
        oracle.dense_mask([-1, 1])  # parent must precede child


def test_threads_do_not_change_results(oracle):
    B, N, Hq, Hkv, D, L = 2, 8, 4, 2, 8, 40
    q, kt, vt, kc, vc = _inputs(10, B, N, Hq, Hkv, D, L)
    parent, n_nodes = gen_trees(10, B, N, 3, 3)
    a = oracle.tree_attn(q, kt, vt, kc, vc, [L] * B, n_nodes, parent, nthreads=1)
    b = oracle.tree_attn(q, kt, vt, kc, vc, [L] * B, n_nodes, parent, nthreads=4)
    np.testing.assert_array_equal(a, b)
