"""GPU parity of the dynamic-tree selection against the CPU oracle, through the C ABI.
Bar: every output array bit-identical (the scores are fp32 on both sides, one addition per edge)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2408_15562_amd as fspad
from workloads import gen_candidates

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _run(par, tok, logp, n_cand, n_keep, n_max):
    out = fspad.fspad_tree_build(*[torch.from_numpy(np.ascontiguousarray(a)).to(DEV) for a in (par, tok, logp, n_cand)],
                                 n_keep, n_max)
    torch.cuda.synchronize()
    parent, tokens, n_nodes, mask, cand = [t.cpu().numpy() for t in out]
    return parent, tokens, n_nodes, mask.view(np.uint64), cand


@pytest.mark.parametrize("B,depth,topk,n_keep,n_max", [(1, 1, 1, 1, 1), (3, 5, 4, 26, 26), (4, 6, 10, 60, 64), (2, 6, 10, 64, 64),
                                                       (5, 6, 10, 7, 60), (130, 3, 4, 26, 32), (2, 11, 10, 60, 60)])
@pytest.mark.parametrize("ties", [False, True])
def test_tree_build_matches_oracle(B, depth, topk, n_keep, n_max, ties):
    par, tok, logp, n_cand = gen_candidates(900 + B + depth + topk, B, depth, topk, 32000, ties=ties)
    assert par.shape[1] <= 1024
    ref = oracle.tree_build(par, tok, logp, n_cand, n_keep, n_max)
    got = _run(par, tok, logp, n_cand, n_keep, n_max)
    for name, g, r in zip(("parent", "tokens", "n_nodes", "anc_mask", "node_cand"), got, ref):
        np.testing.assert_array_equal(g, r, err_msg=name)


def test_padding_chain_and_nan():
    # a chain of 40 candidates (as deep as it gets), padded candidate rows, a NaN score
    m = 40
    par = np.full((2, 64), -1, np.int32)
    par[:, 1:m] = np.arange(0, m - 1)
    tok = np.tile(np.arange(64, dtype=np.int32), (2, 1))
    logp = np.full((2, 64), -0.25, np.float32)
    logp[1, 17] = np.nan
    n_cand = np.array([m, m], np.int32)
    ref = oracle.tree_build(par, tok, logp, n_cand, 30, 32)
    got = _run(par, tok, logp, n_cand, 30, 32)
    for g, r in zip(got, ref):
        np.testing.assert_array_equal(g, r)
    assert got[2].tolist() == [30, 30]      # a NaN edge ranks its subtree last (-infinity), it does not remove it


def test_built_tree_feeds_the_verification_calls():
    """The emitted arrays are exactly what attention and acceptance take: run both on them and
    compare with the oracle fed from the oracle's own tree."""
    from tests import _harness as H
    from workloads import gen_logits, gen_qkv
    B, N, Hq, Hkv, D, L, V = 2, 26, 4, 2, 64, 200, 1000
    par, tok, logp, n_cand = gen_candidates(77, B, 5, 4, V)
    d_parent, d_tokens, d_n, d_mask, _ = fspad.fspad_tree_build(
        *[torch.from_numpy(a).to(DEV) for a in (par, tok, logp, n_cand)], N, N)
    torch.cuda.synchronize()
    r_parent, r_tokens, r_n, r_mask, _ = oracle.tree_build(par, tok, logp, n_cand, N, N)
    host = gen_qkv(78, B, N, Hq, Hkv, D, L, "bf16")
    q, kt, vt, kc, vc = [H.to_dev(a, "bf16") for a in host]
    kv_len = np.array([L, L - 33], np.int32)
    out = fspad.fspad_tree_attn(q, kt, vt, kc, vc, kv_len, d_n.cpu().numpy(), d_mask, out_dtype=torch.float32)
    logits = gen_logits(78, B, N, V, peak=4.0)
    acc = fspad.fspad_tree_accept_greedy(torch.from_numpy(logits).to(DEV), d_tokens, d_parent, d_n)
    torch.cuda.synchronize()
    ref = oracle.tree_attn(*host, kv_len, r_n, r_parent, packed_mask=r_mask, nthreads=4)
    assert H.rel_err(out, ref) <= H.TOL["bf16"]
    for a, b in zip(acc, oracle.accept_greedy(logits, r_tokens, r_parent, r_n)):
        np.testing.assert_array_equal(a.cpu().numpy(), b)
