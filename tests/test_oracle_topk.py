"""CPU pins of the oracle's per-step top-k cut (no GPU).

Plain definition (sort + log-softmax), pinned against the library routines (torch.topk,
torch.log_softmax), a hand-worked row, ties / NaN / -inf, k == V (probabilities sum to one) and
shift invariance."""
import numpy as np
import torch

import oracle


def test_hand_worked_row():
    # softmax of (0, ln 2, ln 5) = (1/8, 2/8, 5/8)
    logits = np.array([[0.0, np.log(2.0), np.log(5.0), -np.inf]], np.float32)
    tok, lp = oracle.draft_topk(logits, 3)
    assert tok.tolist() == [[2, 1, 0]]
    np.testing.assert_allclose(np.exp(lp.astype(np.float64))[0], [5 / 8, 2 / 8, 1 / 8], rtol=1e-6)


def test_against_library_routines():
    rng = np.random.default_rng(1)
    x = (rng.standard_normal((7, 5000)) * 4).astype(np.float32)
    tok, lp = oracle.draft_topk(x, 10)
    t = torch.from_numpy(x).double()
    vals, idx = torch.topk(t, 10, dim=-1)                       # no ties in continuous data
    assert np.array_equal(tok, idx.numpy())
    ref = torch.log_softmax(t, dim=-1).gather(1, idx).numpy()
    np.testing.assert_allclose(lp, ref, rtol=0, atol=1e-6)


def test_ties_nan_and_minus_infinity():
    x = np.array([[1.0, 3.0, 3.0, np.nan, 3.0, -np.inf, 2.0]], np.float32)
    tok, lp = oracle.draft_topk(x, 7)
    assert tok.tolist() == [[1, 2, 4, 6, 0, 3, 5]]              # equal logits by token; NaN == -inf, by token
    assert lp[0, 0] == lp[0, 1] == lp[0, 2] and np.isneginf(lp[0, 5]) and np.isneginf(lp[0, 6])
    tok, lp = oracle.draft_topk(np.full((1, 4), -np.inf, np.float32), 2)
    assert tok.tolist() == [[0, 1]] and np.isneginf(lp).all()


def test_all_entries_kept_sum_to_one_and_shift_invariance():
    rng = np.random.default_rng(2)
    x = (rng.standard_normal((3, 300)) * 3).astype(np.float32)
    tok, lp = oracle.draft_topk(x, 300)
    np.testing.assert_allclose(np.exp(lp.astype(np.float64)).sum(axis=1), 1.0, rtol=1e-5)
    assert (np.diff(lp.astype(np.float64), axis=1) <= 0).all()
    tok2, lp2 = oracle.draft_topk(x + np.float32(8.0), 300)     # a power of two: the sums stay exact enough
    assert np.array_equal(tok, tok2)
    np.testing.assert_allclose(lp, lp2, rtol=0, atol=2e-6)


def test_feeds_the_tree_build():
    """The cut is what the tree build consumes: k children per expanded node, conditional
    log-probabilities <= 0, siblings distinct and in falling order."""
    rng = np.random.default_rng(3)
    x = (rng.standard_normal((4, 1000)) * 3).astype(np.float32)
    tok, lp = oracle.draft_topk(x, 4)
    m = 1 + 4
    par = np.array([[-1, 0, 0, 0, 0]], np.int32)
    out = oracle.tree_build(par, np.concatenate([[7], tok[0]])[None].astype(np.int32),
                            np.concatenate([[0.0], lp[0]])[None].astype(np.float32), [m], 3, 8)
    assert out[2].tolist() == [3] and out[1][0, :3].tolist() == [7, int(tok[0, 0]), int(tok[0, 1])]
    assert (lp <= 0).all() and all(len(set(r)) == 4 for r in tok.tolist())
