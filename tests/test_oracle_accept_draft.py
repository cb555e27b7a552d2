"""CPU pins of the oracle's acceptance for sampled drafts (no GPU): the emitted token follows the
target distribution exactly (the lossless property, by exhaustive enumeration of the drafter's draws
and a fine grid of uniforms); a point-mass draft distribution reduces it to the top-k acceptance
oracle; a drafter equal to the target is always accepted; hand-worked thresholds."""
import itertools

import numpy as np
import pytest

import oracle


def _one_node_distribution(p_logits, q_logits, m, grid):
    """Distribution of the emitted token at a root with m children: the drafter draws the children
    from q without replacement (every ordered draw enumerated with its probability), the uniforms run
    over the midpoints of a grid^(m+1) lattice."""
    V = len(p_logits)
    q = np.exp(q_logits - np.max(q_logits)); q /= q.sum()
    parent = np.array([[-1] + [0] * m], dtype=np.int32)
    us = (np.arange(grid) + 0.5) / grid
    out = np.zeros(V)
    for draw in itertools.permutations(range(V), m):
        prob, rest = 1.0, 1.0
        for x in draw:
            prob *= q[x] / rest
            rest -= q[x]
        if prob == 0.0:
            continue
        tokens = np.array([[0] + list(draw)], dtype=np.int32)
        for u in itertools.product(us, repeat=m + 1):
            uni = np.zeros((1, 2, m + 1))
            uni[0, 0, 1:] = u[:m]
            uni[0, 1, :] = u[m]        # the draw uniform of whichever node the walk stops at
            _, _, emitted, _, _ = oracle.accept_sample_draft(p_logits[None, None, :].repeat(m + 1, 1),
                                                             q_logits[None, None, :].repeat(m + 1, 1),
                                                             tokens, parent, [m + 1], 1.0, uni)
            out[emitted[0, 0]] += prob / grid ** (m + 1)
    return out


@pytest.mark.parametrize("m,grid", [(1, 60), (2, 24)])
def test_first_emitted_token_follows_the_target(m, grid):
    p_logits = np.log(np.array([0.5, 0.3, 0.15, 0.05]))
    q_logits = np.log(np.array([0.2, 0.1, 0.3, 0.4]))          # a drafter far from the target
    got = _one_node_distribution(p_logits, q_logits, m, grid)
    np.testing.assert_allclose(got.sum(), 1.0, rtol=1e-9)
    # a grid of g points per uniform resolves every threshold to 1/g
    np.testing.assert_allclose(got, [0.5, 0.3, 0.15, 0.05], atol=1.5 / grid)


def _log_rows(*rows):
    return np.log(np.array(rows, dtype=np.float64))[None]          # [1, nodes, V]


def test_exact_counts_on_a_rational_case_one_level():
    """Target p = (1/2, 1/4, 1/8, 1/8) against drafter q = (1/8, 1/8, 1/4, 1/2): every threshold of the
    rule (min(1, p/q) in {1, 1/2, 1/4}; the residual after one rejection (3/4, 1/4, 0, 0); after two
    (7/8, 1/8, 0, 0) or (1, 0, 0, 0); the running sums of every distribution a draw can see) is a
    multiple of 1/8, so with every uniform on the midpoints of an 8-cell grid the emitted-token counts,
    weighted with the exact probability of each ordered draw of the drafter, must equal p as
    fractions -- no tolerance."""
    from fractions import Fraction as F
    p = [F(1, 2), F(1, 4), F(1, 8), F(1, 8)]
    q = [F(1, 8), F(1, 8), F(1, 4), F(1, 2)]
    grid = 8
    us = (np.arange(grid) + 0.5) / grid
    for m in (1, 2):
        rows = _log_rows(*([[float(x) for x in p]] * (m + 1)))
        qrows = _log_rows(*([[float(x) for x in q]] * (m + 1)))
        parent = np.array([[-1] + [0] * m], dtype=np.int32)
        total = [F(0)] * 4
        for draw in itertools.permutations(range(4), m):
            prob, rest = F(1), F(1)
            for x in draw:
                prob *= q[x] / rest
                rest -= q[x]
            tokens = np.array([[0] + list(draw)], dtype=np.int32)
            counts = [0] * 4
            for u in itertools.product(us, repeat=m + 1):
                uni = np.zeros((1, 2, m + 1))
                uni[0, 0, 1:] = u[:m]
                uni[0, 1, :] = u[m]
                _, _, emitted, _, margin = oracle.accept_sample_draft(rows, qrows, tokens, parent, [m + 1], 1.0, uni)
                assert margin[0] > 1e-3          # no walk sits on a threshold
                counts[int(emitted[0, 0])] += 1
            for y in range(4):
                total[y] += prob * F(counts[y], grid ** (m + 1))
        assert total == p, (m, total)


def test_exact_counts_on_a_two_level_tree():
    """Root -> A -> B, A drawn from the root's drafter row, B from A's. Given that A (token x) was
    accepted, the second emitted token must follow A's own target row exactly:
        sum_y q_A(y) * #(walks through A that emit b second | x, y) / grid^3 = min(1, p(x)/q(x)) * p_A(b)
    as fractions, for every x and b; every threshold is again a multiple of 1/8."""
    from fractions import Fraction as F
    p0 = [F(1, 2), F(1, 4), F(1, 8), F(1, 8)]; q0 = [F(1, 8), F(1, 8), F(1, 4), F(1, 2)]
    pA = [F(1, 8), F(1, 8), F(1, 4), F(1, 2)]; qA = [F(1, 2), F(1, 4), F(1, 8), F(1, 8)]
    pB = p0                                     # the leaf's own row: running sums 1/2, 3/4, 7/8
    f = lambda r: [float(x) for x in r]
    rows, qrows = _log_rows(f(p0), f(pA), f(pB)), _log_rows(f(q0), f(qA), f(q0))
    parent = np.array([[-1, 0, 1]], dtype=np.int32)
    grid = 8
    us = (np.arange(grid) + 0.5) / grid
    first = [F(0)] * 4                          # distribution of the first emitted token, over everything
    for x in range(4):
        second = [F(0)] * 4
        through_a = F(0)
        for y in range(4):
            tokens = np.array([[0, x, y]], dtype=np.int32)
            cnt_first, cnt_second, cnt_a = [0] * 4, [0] * 4, 0
            for ua, ub, ud in itertools.product(us, repeat=3):
                uni = np.zeros((1, 2, 3))
                uni[0, 0, 1], uni[0, 0, 2], uni[0, 1, :] = ua, ub, ud
                path, plen, emitted, _, margin = oracle.accept_sample_draft(rows, qrows, tokens, parent, [3], 1.0, uni)
                assert margin[0] > 1e-3
                cnt_first[int(emitted[0, 0])] += 1
                if plen[0] >= 2:
                    assert path[0, 1] == 1 and emitted[0, 0] == x
                    cnt_a += 1
                    cnt_second[int(emitted[0, 1])] += 1
            for b in range(4):
                second[b] += qA[y] * F(cnt_second[b], grid ** 3)
                first[b] += q0[x] * qA[y] * F(cnt_first[b], grid ** 3)
            through_a += qA[y] * F(cnt_a, grid ** 3)
        accept_x = min(F(1), p0[x] / q0[x])
        assert through_a == accept_x, (x, through_a)
        assert second == [accept_x * pb for pb in pA], (x, second)
    assert first == p0, first


def test_point_mass_drafts_are_the_topk_acceptance():
    rng = np.random.default_rng(3)
    B, N, V = 3, 9, 50
    from workloads import gen_trees, gen_draft_tokens, gen_uniforms
    parent, n_nodes = gen_trees(3, B, N, 4, 3)
    logits = (3.0 * rng.standard_normal((B, N, V))).astype(np.float32)
    tokens = gen_draft_tokens(3, logits, parent, n_nodes, "sample", 0.5)
    # q of node i: all mass on ... there is one q per parent but several children; a point mass on the
    # FIRST child reproduces the top-k rule for that child only, so compare chains (one child per node)
    chain = np.tile(np.arange(-1, N - 1, dtype=np.int32), (B, 1))
    nn = np.full(B, N, dtype=np.int32)
    ql = np.full((B, N, V), -1e30, dtype=np.float32)
    for b in range(B):
        for c in range(1, N):
            ql[b, c - 1, tokens[b, c]] = 0.0
    for seed in range(5):
        uni = gen_uniforms(seed, B, N)
        a = oracle.accept_sample(logits, tokens, chain, nn, 0.8, uni)
        d = oracle.accept_sample_draft(logits, ql, tokens, chain, nn, 0.8, uni)
        for x, y in zip(a[:4], d[:4]):
            np.testing.assert_array_equal(x, y)


def test_a_drafter_equal_to_the_target_is_always_accepted():
    rng = np.random.default_rng(4)
    B, N, V = 2, 6, 30
    logits = rng.standard_normal((B, N, V)).astype(np.float32)
    chain = np.tile(np.arange(-1, N - 1, dtype=np.int32), (B, 1))
    tokens = rng.integers(0, V, (B, N)).astype(np.int32)
    uni = rng.uniform(0, 0.999, (B, 2, N))
    path, path_len, emitted, n_tok, _ = oracle.accept_sample_draft(logits, logits, tokens, chain, [N, N], 1.3, uni)
    assert path_len.tolist() == [N, N]
    np.testing.assert_array_equal(emitted[:, : N - 1], tokens[:, 1:])


def test_hand_worked_thresholds_and_residual():
    # p = (0.5, 0.3, 0.2), q = (0.2, 0.2, 0.6); the root has children with tokens 2 then 0
    p, q = np.array([0.5, 0.3, 0.2]), np.array([0.2, 0.2, 0.6])
    lp, lq = np.log(p)[None, None, :].repeat(3, 1), np.log(q)[None, None, :].repeat(3, 1)
    parent = np.array([[-1, 0, 0]], dtype=np.int32)
    tokens = np.array([[0, 2, 0]], dtype=np.int32)

    def run(u1, u2, ud):
        uni = np.zeros((1, 2, 3)); uni[0, 0, 1], uni[0, 0, 2], uni[0, 1, :] = u1, u2, ud
        path, plen, emitted, _, _ = oracle.accept_sample_draft(lp, lq, tokens, parent, [3], 1.0, uni)
        return path[0, :plen[0]].tolist(), emitted[0, :plen[0]].tolist()

    # child 1 (token 2): accepted iff u < p/q = 1/3
    assert run(0.33, 0.0, 0.0)[0] == [0, 1]
    assert run(0.34, 0.0, 0.0)[0][:2] != [0, 1]
    # after rejecting token 2: p' = max(p - q, 0)/0.4 = (0.75, 0.25, 0), q' = (0.5, 0.5, 0)
    # child 2 (token 0): accepted iff u * 0.5 < 0.75: always
    assert run(0.9, 0.999, 0.0)[0] == [0, 2]
    # with the second child's token changed to 1: accepted iff u * 0.5 < 0.25
    tokens[0, 2] = 1
    assert run(0.9, 0.49, 0.0)[0] == [0, 2]
    path, emitted = run(0.9, 0.51, 0.74)
    # both rejected: p'' = max(p' - q', 0) = (0.25, 0, 0) -> token 0 whatever the uniform
    assert path == [0] and emitted == [0]
    # a leaf draws from its own p: cumulative 0.5, 0.8, 1.0
    tokens[0, 2] = 0
    assert run(0.0, 0.0, 0.79) == ([0, 1], [2, 1])
    assert run(0.0, 0.0, 0.81) == ([0, 1], [2, 2])
