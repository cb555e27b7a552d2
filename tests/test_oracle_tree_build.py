"""CPU pins of the oracle's dynamic-tree selection (no GPU): a hand-worked example, brute force
over every ancestor-closed subset on tiny candidate sets, structural invariants on
EAGLE-2-shaped candidate sets, a closure and a validator written out here as independent checks of
the emitted arrays, and tie handling. Nothing of the GPU library is used."""
import itertools

import numpy as np

import oracle
from workloads import gen_candidates


def _well_formed(parent, tokens, n_nodes, V):
    """parent[0] = -1, every later parent precedes its child, tokens in range, siblings distinct."""
    for b in range(parent.shape[0]):
        n = int(n_nodes[b])
        if n < 1 or parent[b, 0] != -1:
            return False
        seen = set()
        for i in range(1, n):
            p, t = int(parent[b, i]), int(tokens[b, i])
            if not (0 <= p < i) or not (0 <= t < V) or (p, t) in seen:
                return False
            seen.add((p, t))
    return True


def _ancestor_words(parent, n_nodes):
    """bit t of word [b,i] <=> t is i or one of its ancestors, by walking up from every node."""
    words = np.zeros(parent.shape, dtype=np.uint64)
    for b in range(parent.shape[0]):
        for i in range(int(n_nodes[b])):
            w, a = 0, i
            while a >= 0:
                w |= 1 << a
                a = int(parent[b, a])
            words[b, i] = w
    return words


def test_hand_worked_example():
    # root 0; children 1 (p=.6), 2 (p=.3); grandchildren 3 (of 1, .5 -> .30 joint), 4 (of 1, .1 -> .06),
    # 5 (of 2, .9 -> .27).  Joint: 1:.6  2:.3  3:.3(-)  4:.06  5:.27.  log(.6*.5) < log(.3) by rounding? use
    # explicit logs that are exact in binary so that the order is beyond doubt.
    par = np.array([[-1, 0, 0, 1, 1, 2]], np.int32)
    tok = np.array([[100, 11, 12, 13, 14, 15]], np.int32)
    logp = np.array([[0.0, -0.5, -1.25, -0.5, -3.0, -0.125]], np.float32)   # joints: -.5 -1.25 -1.0 -3.5 -1.375
    parent, tokens, n_nodes, mask, cand = oracle.tree_build(par, tok, logp, [6], 4, 5)
    # best three non-root: 1 (-.5), 3 (-1.0), 2 (-1.25); candidate 5 (-1.375) and 4 are out
    assert n_nodes.tolist() == [4]
    assert cand[0].tolist() == [0, 1, 2, 3, -1]
    assert parent[0].tolist() == [-1, 0, 0, 1, -1]
    assert tokens[0].tolist() == [100, 11, 12, 13, -1]
    assert [int(x) for x in mask[0]] == [0b1, 0b11, 0b101, 0b1011, 0]


def test_brute_force_best_closed_subset():
    """With scores that fall along every path, the kept set is the ancestor-closed set of its size
    with the largest total score."""
    rng = np.random.default_rng(3)
    for trial in range(40):
        m = int(rng.integers(2, 11))
        par = np.array([[-1] + [int(rng.integers(0, c)) for c in range(1, m)]], np.int32)
        logp = np.concatenate([[0.0], -rng.uniform(0.05, 2.0, m - 1)]).astype(np.float32)[None]
        tok = np.arange(m, dtype=np.int32)[None]
        n_keep = int(rng.integers(1, m + 1))
        _, _, n_nodes, _, cand = oracle.tree_build(par, tok, logp, [m], n_keep, 16)
        joint = np.zeros(m, np.float32)
        for c in range(1, m):
            joint[c] = np.float32(joint[par[0, c]] + logp[0, c])
        best, best_set = None, None
        for sub in itertools.combinations(range(1, m), n_keep - 1):
            s = set(sub) | {0}
            if any(par[0, c] not in s for c in sub):
                continue
            tot = float(sum(np.float64(joint[c]) for c in sub))
            if best is None or tot > best + 1e-12:
                best, best_set = tot, s
        assert n_nodes[0] == n_keep
        assert set(cand[0, :n_keep].tolist()) == best_set


def test_invariants_on_shaped_candidates():
    par, tok, logp, n_cand = gen_candidates(11, 5, 6, 10, 32000)
    for n_keep, n_max in ((60, 64), (26, 26), (1, 8)):
        parent, tokens, n_nodes, mask, cand = oracle.tree_build(par, tok, logp, n_cand, n_keep, n_max)
        assert np.array_equal(n_nodes, np.minimum(n_cand, n_keep))
        assert _well_formed(parent, tokens, n_nodes, 32000)
        assert np.array_equal(mask, _ancestor_words(parent, n_nodes))               # independent closure
        for b in range(par.shape[0]):
            n = int(n_nodes[b])
            c = cand[b, :n]
            assert np.all(np.diff(c) > 0) and c[0] == 0                             # candidate order kept
            assert np.array_equal(tokens[b, :n], tok[b, c])
            assert np.array_equal(c[parent[b, 1:n]], par[b, c[1:]])                 # parents map back
            assert np.all(parent[b, n:] == -1) and np.all(cand[b, n:] == -1) and np.all(mask[b, n:] == 0)
            joint = np.zeros(int(n_cand[b]), np.float32)
            for k in range(1, int(n_cand[b])):
                joint[k] = np.float32(joint[par[b, k]] + logp[b, k])
            dropped = np.setdiff1d(np.arange(int(n_cand[b])), c)
            if n > 1 and dropped.size:
                assert joint[c[1:]].min() >= joint[dropped].max()                   # nothing better was left out


def test_ties_go_to_the_lower_index_and_nan_ranks_last():
    par = np.array([[-1, 0, 0, 0, 0]], np.int32)
    tok = np.arange(5, dtype=np.int32)[None]
    logp = np.array([[0.0, -1.0, -1.0, np.nan, -1.0]], np.float32)
    _, _, n_nodes, _, cand = oracle.tree_build(par, tok, logp, [5], 3, 4)
    assert n_nodes.tolist() == [3] and cand[0].tolist() == [0, 1, 2, -1]
    _, _, n_nodes, _, cand = oracle.tree_build(par, tok, logp, [5], 4, 4)
    assert cand[0].tolist() == [0, 1, 2, 4]
    par, tok, logp, n_cand = gen_candidates(12, 3, 5, 4, 1000, ties=True)
    parent, tokens, n_nodes, mask, cand = oracle.tree_build(par, tok, logp, n_cand, 26, 26)
    assert _well_formed(parent, tokens, n_nodes, 1000)
