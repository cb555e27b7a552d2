"""CPU pins of the oracle's greedy validation from hidden states (no GPU).

The logits have a plain definition (a matrix product), the rest is the greedy walk.  Pins: a
hand-worked example with integer data, exact integer brute force in pure Python, one-hot hidden
states (a logit row is then a column of the weight matrix, which catches a transposed operand),
ties, the separately pinned C oracle of the walk on the same (exactly representable) logits, and
a chain whose every token is planted so that the whole tree is accepted."""
import numpy as np

import oracle
from workloads import chain_tree, gen_draft_tokens, gen_lm_head, gen_trees


def test_hand_worked_example():
    # V=4, Hd=2.  Rows of W: token 0..3.  Tree: root 0 with children 1 (token 2) and 2 (token 3);
    # node 2 has child 3 (token 1).
    w = np.array([[1., 0.], [0., 1.], [-1., 0.], [1., 1.]])
    hidden = np.array([[[2., 1.],     # logits 2,1,-2,3  -> target 3 -> child 2 matches
                        [9., 9.],     # never visited
                        [-1., 3.],    # logits -1,3,1,2  -> target 1 -> child 3 matches
                        [-5., -4.]]])  # logits -5,-4,5,-9 -> target 2 (bonus)
    parent = np.array([[-1, 0, 0, 2]], np.int32)
    tokens_in = np.array([[7, 2, 3, 1]], np.int32)
    path, plen, toks, ntok, target, top, margin = oracle.lm_head_greedy(hidden, w, tokens_in, parent, [4])
    assert path.tolist() == [[0, 2, 3, -1]] and plen.tolist() == [3]
    assert toks.tolist() == [[3, 1, 2, -1]] and ntok.tolist() == [3]
    assert target.tolist() == [[3, 3, 1, 2]]
    assert top.tolist() == [[3., 18., 3., 5.]]
    assert margin.tolist() == [[1., 9., 1., 9.]]


def test_integer_brute_force():
    rng = np.random.default_rng(5)
    B, N, Hd, V = 2, 7, 5, 11
    hidden = rng.integers(-4, 5, size=(B, N, Hd))
    w = rng.integers(-4, 5, size=(V, Hd))
    parent, n_nodes = gen_trees(9, B, N, 3, 3)
    draft = rng.integers(0, V, size=(B, N)).astype(np.int32)
    _, _, _, _, target, top, margin = oracle.lm_head_greedy(hidden, w, draft, parent, n_nodes)
    for b in range(B):
        for i in range(int(n_nodes[b])):
            logits = [sum(int(hidden[b, i, k]) * int(w[v, k]) for k in range(Hd)) for v in range(V)]
            best = max(logits)
            assert target[b, i] == logits.index(best)          # first index among equals
            assert top[b, i] == best
            rest = logits[:target[b, i]] + logits[target[b, i] + 1:]
            assert margin[b, i] == best - max(rest)
        assert (target[b, int(n_nodes[b]):] == -1).all()


def test_one_hot_hidden_reads_a_column_of_the_weights():
    rng = np.random.default_rng(6)
    V, Hd, N = 13, 6, 6
    w = rng.standard_normal((V, Hd))
    hidden = np.zeros((1, N, Hd))
    for i in range(N):
        hidden[0, i, i] = 1.0
    parent, n_nodes = chain_tree(N)[None], [N]
    _, _, _, _, target, top, _ = oracle.lm_head_greedy(hidden, w, np.zeros((1, N), np.int32), parent, n_nodes)
    assert target[0].tolist() == [int(np.argmax(w[:, i])) for i in range(N)]
    assert np.array_equal(top[0], w.max(axis=0))


def test_ties_take_the_lowest_token():
    w = np.array([[1., 0.], [2., 0.], [2., 0.], [0., 5.]])
    hidden = np.array([[[1., 0.]]])
    out = oracle.lm_head_greedy(hidden, w, np.zeros((1, 1), np.int32), np.array([[-1]], np.int32), [1])
    assert out[4].tolist() == [[1]] and out[6].tolist() == [[0.]]
    assert out[0].tolist() == [[0]] and out[2].tolist() == [[1]] and out[1].tolist() == [1]


def test_walk_agrees_with_the_logit_oracle_on_exact_logits():
    # small integers: the products and sums are exact in fp32, so the C oracle of the walk (pinned
    # on its own) sees exactly the logits that the definition gives
    rng = np.random.default_rng(7)
    B, N, Hd, V = 3, 20, 8, 40
    hidden = rng.integers(-3, 4, size=(B, N, Hd)).astype(np.float64)
    w = rng.integers(-3, 4, size=(V, Hd)).astype(np.float64)
    parent, n_nodes = gen_trees(11, B, N, 4, 3)
    logits = np.einsum("bik,vk->biv", hidden, w).astype(np.float32)
    # children carry the first-argmax token of their parent half of the time, so that walks go deep
    draft = rng.integers(0, V, size=(B, N)).astype(np.int32)
    for b in range(B):
        seen = set()
        for c in range(1, int(n_nodes[b])):
            p = int(parent[b, c])
            if p not in seen and rng.random() < 0.7:
                draft[b, c] = int(np.argmax(logits[b, p]))
                seen.add(p)
    a = oracle.lm_head_greedy(hidden, w, draft, parent, n_nodes)
    r = oracle.accept_greedy(logits, draft, parent, n_nodes)
    assert a[1].max() > 2                                      # some walk went below the root's children
    for x, y in zip(a[:4], r):
        assert np.array_equal(x, y)


def test_planted_chain_is_accepted_whole():
    B, N, Hd, V = 2, 12, 64, 500
    hidden, w = gen_lm_head(3, B, N, Hd, V)
    parent = np.tile(chain_tree(N), (B, 1))
    n_nodes = np.array([N, 5], np.int32)
    _, _, _, _, target, _, margin = oracle.lm_head_greedy(hidden, w, np.zeros((B, N), np.int32), parent, n_nodes)
    draft = np.zeros((B, N), np.int32)
    draft[:, 1:] = np.where(target[:, :-1] >= 0, target[:, :-1], 0)   # node i+1 carries target[i]
    path, plen, toks, ntok = oracle.lm_head_greedy(hidden, w, draft, parent, n_nodes)[:4]
    assert plen.tolist() == [N, 5] and ntok.tolist() == [N, 5]
    assert path[0].tolist() == list(range(N)) and path[1, :5].tolist() == list(range(5))
    assert np.array_equal(toks[0], target[0]) and np.array_equal(toks[1, :5], target[1, :5])
    assert (path[1, 5:] == -1).all() and (toks[1, 5:] == -1).all()
    assert np.nanmin(margin) > 0


def test_sampling_from_hidden_states_is_the_sampling_oracle_on_the_defined_logits():
    # integer data: the logits are exact in fp32, so the composition can be checked against logits
    # written out by hand (einsum in integers), with the separately pinned sampling walk
    from workloads import gen_uniforms
    rng = np.random.default_rng(8)
    B, N, Hd, V = 2, 14, 6, 30
    hidden = rng.integers(-2, 3, size=(B, N, Hd)).astype(np.float64)
    w = rng.integers(-2, 3, size=(V, Hd)).astype(np.float64)
    parent, n_nodes = gen_trees(13, B, N, 4, 3)
    logits = np.einsum("bik,vk->biv", hidden.astype(np.int64), w.astype(np.int64)).astype(np.float32)
    assert np.array_equal(oracle.lm_head_logits(hidden, w), logits)
    draft = gen_draft_tokens(13, logits, parent, n_nodes, "sample")
    uni = gen_uniforms(13, B, N)
    a = oracle.lm_head_sample(hidden, w, draft, parent, n_nodes, 0.7, uni)
    r = oracle.accept_sample(logits, draft, parent, n_nodes, 0.7, uni)
    for x, y in zip(a, r):
        assert np.array_equal(x, y)


def test_cold_sampling_from_hidden_states_is_the_greedy_walk():
    from workloads import gen_uniforms
    B, N, Hd, V = 3, 20, 64, 400
    hidden, w = gen_lm_head(21, B, N, Hd, V)
    parent, n_nodes = gen_trees(21, B, N, 5, 4)
    draft = gen_draft_tokens(21, oracle.lm_head_logits(hidden, w), parent, n_nodes, "greedy", 0.5)
    g = oracle.lm_head_greedy(hidden, w, draft, parent, n_nodes)
    s = oracle.lm_head_sample(hidden, w, draft, parent, n_nodes, 1e-3, gen_uniforms(21, B, N))
    assert g[6][g[4] >= 0].min() > 0.02          # the argmaxes are decided far beyond a temperature of 1e-3
    for x, y in zip(g[:4], s[:4]):
        assert np.array_equal(x, y)
    assert g[1].max() >= 2
