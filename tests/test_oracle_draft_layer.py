"""CPU pins of the oracle's draft decoder layer (no GPU): the library's LLaMA decoder layer on a
chain, on a tree (through its additive mask) and with a prefix; the equivalence of a tree node
with the chain of its ancestors; incremental decoding against one pass over the whole sequence;
the two halves of the doubled MLP output; rotary encoding and RMSNorm against closed forms."""
import numpy as np
import pytest
import torch

import oracle
from workloads import gen_trees, tree_depths


def _weights(rng, Hd, I, Hq, Hkv, D):
    return dict(
        w_qkv=rng.standard_normal(((Hq + 2 * Hkv) * D, Hd)) / np.sqrt(Hd),
        w_o=rng.standard_normal((Hd, Hq * D)) / np.sqrt(Hq * D),
        w_gate=rng.standard_normal((I, Hd)) / np.sqrt(Hd),
        w_up=rng.standard_normal((I, Hd)) / np.sqrt(Hd),
        w_down=rng.standard_normal((2 * Hd, I)) / np.sqrt(I),
        gain_attn=1.0 + 0.1 * rng.standard_normal(Hd),
        gain_mlp=1.0 + 0.1 * rng.standard_normal(Hd),
    )


def _library_layer(w, Hd, I, Hq, Hkv, D, eps, theta, half):
    """transformers' LLaMA decoder layer in fp64 carrying the same weights; its down projection is
    one half of the doubled one."""
    from transformers import LlamaConfig
    from transformers.models.llama.modeling_llama import LlamaDecoderLayer, LlamaRotaryEmbedding
    cfg = LlamaConfig(hidden_size=Hd, intermediate_size=I, num_attention_heads=Hq, num_key_value_heads=Hkv,
                      head_dim=D, rms_norm_eps=eps, rope_theta=theta, attention_bias=False, mlp_bias=False,
                      num_hidden_layers=1, vocab_size=8)
    cfg._attn_implementation = "eager"
    layer = LlamaDecoderLayer(cfg, 0).double()
    T = lambda a: torch.from_numpy(np.ascontiguousarray(a))
    with torch.no_grad():
        layer.self_attn.q_proj.weight.copy_(T(w["w_qkv"][: Hq * D]))
        layer.self_attn.k_proj.weight.copy_(T(w["w_qkv"][Hq * D:(Hq + Hkv) * D]))
        layer.self_attn.v_proj.weight.copy_(T(w["w_qkv"][(Hq + Hkv) * D:]))
        layer.self_attn.o_proj.weight.copy_(T(w["w_o"]))
        layer.mlp.gate_proj.weight.copy_(T(w["w_gate"]))
        layer.mlp.up_proj.weight.copy_(T(w["w_up"]))
        layer.mlp.down_proj.weight.copy_(T(w["w_down"][half * Hd:(half + 1) * Hd]))
        layer.input_layernorm.weight.copy_(T(w["gain_attn"]))
        layer.post_attention_layernorm.weight.copy_(T(w["gain_mlp"]))
    return layer.eval(), LlamaRotaryEmbedding(cfg)


def _run_library(layer, rot, x, pos, allowed):
    """x [S,Hd], pos [S], allowed [S,S] bool -> [S,Hd]"""
    xt = torch.from_numpy(x)[None]
    pt = torch.from_numpy(np.asarray(pos, dtype=np.int64))[None]
    mask = torch.zeros(allowed.shape, dtype=torch.float64)
    mask[~torch.from_numpy(allowed)] = float("-inf")
    with torch.no_grad():
        cos, sin = rot(xt, pt)
        out = layer(xt, attention_mask=mask[None, None], position_ids=pt, position_embeddings=(cos, sin))
    return (out[0] if isinstance(out, tuple) else out)[0].numpy()


GEOM = dict(Hd=32, I=48, Hq=4, Hkv=2, D=8)


def _call(w, eta, pos, kc, vc, kv_len, n_nodes, parent, eps=1e-5, theta=10000.0, g=GEOM):
    return oracle.draft_layer(eta, pos, w["w_qkv"], w["w_o"], w["w_gate"], w["w_up"], w["w_down"], w["gain_attn"],
                              w["gain_mlp"], kc, vc, kv_len, n_nodes, parent, g["Hq"], g["Hkv"], g["D"], eps, theta)


def test_chain_without_prefix_is_the_librarys_causal_layer():
    rng = np.random.default_rng(11)
    g = GEOM
    w = _weights(rng, **g)
    S = 7
    eta = rng.standard_normal((1, S, g["Hd"]))
    parent = np.arange(-1, S - 1, dtype=np.int32)[None]
    pos = np.arange(S, dtype=np.int32)[None]
    ft, f, k, v = _call(w, eta, pos, None, None, [0], [S], parent)
    causal = np.tril(np.ones((S, S), dtype=bool))
    for half, got in ((0, ft), (1, f)):
        layer, rot = _library_layer(w, g["Hd"], g["I"], g["Hq"], g["Hkv"], g["D"], 1e-5, 10000.0, half)
        ref = _run_library(layer, rot, eta[0], pos[0], causal)
        np.testing.assert_allclose(got[0], ref, rtol=1e-6, atol=1e-6)


def test_tree_with_prefix_is_the_librarys_layer_under_the_tree_mask():
    # The prefix is produced by the layer itself: the oracle runs once over the L prefix tokens as
    # a chain, its keys / values become the cache, then it runs over the tree.  The library sees
    # all L + N tokens at once under the mask "prefix causal, tree rows see the prefix and their
    # ancestors", with positions L + depth.
    rng = np.random.default_rng(12)
    g = GEOM
    w = _weights(rng, **g)
    L, N = 5, 9
    parent, n_nodes = gen_trees(5, 1, N, 4, 3)
    depth = tree_depths(parent, n_nodes)
    x_pre = rng.standard_normal((1, L, g["Hd"]))
    x_tree = rng.standard_normal((1, N, g["Hd"]))
    chain = np.arange(-1, L - 1, dtype=np.int32)[None]
    _, _, kp, vp = _call(w, x_pre, np.arange(L, dtype=np.int32)[None], None, None, [0], [L], chain)
    kc = np.ascontiguousarray(kp.transpose(0, 2, 1, 3))     # [B,Hkv,L,D]
    vc = np.ascontiguousarray(vp.transpose(0, 2, 1, 3))
    ft, f, _, _ = _call(w, x_tree, L + depth, kc, vc, [L], n_nodes, parent)
    allowed = np.zeros((L + N, L + N), dtype=bool)
    allowed[:L, :L] = np.tril(np.ones((L, L), dtype=bool))
    allowed[L:, :L] = True
    allowed[L:, L:] = oracle.dense_mask(parent[0]).astype(bool)
    pos = np.concatenate([np.arange(L), L + depth[0]])
    for half, got in ((0, ft), (1, f)):
        layer, rot = _library_layer(w, g["Hd"], g["I"], g["Hq"], g["Hkv"], g["D"], 1e-5, 10000.0, half)
        ref = _run_library(layer, rot, np.concatenate([x_pre[0], x_tree[0]]), pos, allowed)
        np.testing.assert_allclose(got[0], ref[L:], rtol=1e-6, atol=1e-6)


def test_a_tree_node_equals_the_chain_of_its_ancestors():
    rng = np.random.default_rng(13)
    g = GEOM
    w = _weights(rng, **g)
    L, N = 6, 12
    parent, n_nodes = gen_trees(8, 1, N, 5, 3)
    depth = tree_depths(parent, n_nodes)
    eta = rng.standard_normal((1, N, g["Hd"]))
    kc = rng.standard_normal((1, g["Hkv"], L, g["D"]))
    vc = rng.standard_normal((1, g["Hkv"], L, g["D"]))
    ft, f, k, v = _call(w, eta, L + depth, kc, vc, [L], n_nodes, parent)
    for node in range(N):
        path = [node]
        while parent[0, path[-1]] >= 0:
            path.append(int(parent[0, path[-1]]))
        path = path[::-1]
        n = len(path)
        cp = np.arange(-1, n - 1, dtype=np.int32)[None]
        cft, cf, ck, cv = _call(w, eta[:, path], L + np.arange(n, dtype=np.int32)[None], kc, vc, [L], [n], cp)
        np.testing.assert_allclose(ft[0, node], cft[0, -1], rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(f[0, node], cf[0, -1], rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(k[0, node], ck[0, -1], rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(v[0, node], cv[0, -1], rtol=1e-10, atol=1e-12)


def test_incremental_decoding_equals_one_pass():
    # keys / values of the first L tokens in the cache, the rest as a chain on top
    rng = np.random.default_rng(14)
    g = GEOM
    w = _weights(rng, **g)
    S, L = 10, 6
    eta = rng.standard_normal((1, S, g["Hd"]))
    chain = lambda n: np.arange(-1, n - 1, dtype=np.int32)[None]
    ft_all, f_all, k_all, v_all = _call(w, eta, np.arange(S, dtype=np.int32)[None], None, None, [0], [S], chain(S))
    kc = np.ascontiguousarray(k_all[:, :L].transpose(0, 2, 1, 3))
    vc = np.ascontiguousarray(v_all[:, :L].transpose(0, 2, 1, 3))
    ft, f, k, v = _call(w, eta[:, L:], np.arange(L, S, dtype=np.int32)[None], kc, vc, [L], [S - L], chain(S - L))
    np.testing.assert_allclose(ft, ft_all[:, L:], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(f, f_all[:, L:], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(k, k_all[:, L:], rtol=1e-10, atol=1e-12)


def test_the_two_features_share_the_residual():
    rng = np.random.default_rng(15)
    g = GEOM
    w = _weights(rng, **g)
    N = 5
    eta = rng.standard_normal((2, N, g["Hd"]))
    parent, n_nodes = gen_trees(3, 2, N, 3, 2, n_nodes=[5, 3])
    pos = tree_depths(parent, n_nodes)
    ft, f, _, _ = _call(w, eta, pos, None, None, [0, 0], n_nodes, parent)
    # zero second half of the down projection: f is the state after attention, the same residual
    # both features start from; swapping the halves swaps the features
    w0 = dict(w); w0["w_down"] = w["w_down"].copy(); w0["w_down"][g["Hd"]:] = 0.0
    ft0, h, _, _ = _call(w0, eta, pos, None, None, [0, 0], n_nodes, parent)
    np.testing.assert_allclose(ft0, ft, rtol=1e-12, atol=1e-14)
    ws = dict(w); ws["w_down"] = np.concatenate([w["w_down"][g["Hd"]:], w["w_down"][: g["Hd"]]])
    fts, fs, _, _ = _call(ws, eta, pos, None, None, [0, 0], n_nodes, parent)
    np.testing.assert_allclose(fts, f, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(fs, ft, rtol=1e-12, atol=1e-14)
    # doubling the down projection doubles what each feature adds to the shared residual
    w2 = dict(w); w2["w_down"] = 2.0 * w["w_down"]
    ft2, f2, _, _ = _call(w2, eta, pos, None, None, [0, 0], n_nodes, parent)
    np.testing.assert_allclose(ft2 - h, 2.0 * (ft - h), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(f2 - h, 2.0 * (f - h), rtol=1e-9, atol=1e-12)
    # unused tree slots come back as zeros
    assert np.all(ft[1, 3:] == 0.0) and np.all(f[1, 3:] == 0.0)


def test_rotary_encoding_closed_forms():
    rng = np.random.default_rng(16)
    D = 8
    u = rng.standard_normal((3, D))
    np.testing.assert_array_equal(oracle.rope(u, np.zeros(3), 10000.0), u)            # position 0: identity
    # theta = 1: every pair turns by the position itself
    r = oracle.rope(u, np.full(3, 2.0), 1.0)
    np.testing.assert_allclose(r[:, :4], u[:, :4] * np.cos(2.0) - u[:, 4:] * np.sin(2.0), rtol=1e-14)
    np.testing.assert_allclose(r[:, 4:], u[:, 4:] * np.cos(2.0) + u[:, :4] * np.sin(2.0), rtol=1e-14)
    # pair i turns by position * theta^(-2i/D): a unit vector in pair 1, theta = 16, D = 8 -> angle p / 2
    e = np.zeros((1, D)); e[0, 1] = 1.0
    r = oracle.rope(e, np.array([3.0]), 16.0)
    np.testing.assert_allclose(r[0, [1, 5]], [np.cos(1.5), np.sin(1.5)], rtol=1e-14)
    assert np.count_nonzero(r) == 2
    # rotations keep lengths and compose: scores depend on the position difference only
    a, b = rng.standard_normal(D), rng.standard_normal(D)
    s1 = oracle.rope(a, 7, 10000.0) @ oracle.rope(b, 3, 10000.0)
    s2 = oracle.rope(a, 104, 10000.0) @ oracle.rope(b, 100, 10000.0)
    np.testing.assert_allclose(s1, s2, rtol=1e-10)
    np.testing.assert_allclose(np.linalg.norm(oracle.rope(a, 55, 10000.0)), np.linalg.norm(a), rtol=1e-13)


def test_rms_norm_closed_forms():
    x = np.array([[3.0, -4.0, 0.0, 0.0]])             # mean square 25/4
    np.testing.assert_allclose(oracle.rms_norm(x, np.ones(4), 0.0), x / 2.5, rtol=1e-15)
    np.testing.assert_allclose(oracle.rms_norm(x, np.array([2.0, 1.0, 1.0, 1.0]), 0.75), x / np.sqrt(7.0) * [2, 1, 1, 1], rtol=1e-15)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (4,), torch.ones(4, dtype=torch.float64), 1e-3)
    np.testing.assert_allclose(oracle.rms_norm(x, np.ones(4), 1e-3), ref.numpy(), rtol=1e-14)
