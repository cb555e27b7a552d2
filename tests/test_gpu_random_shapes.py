"""Seeded random sweep over shapes inside the documented limits: every draw is a fresh combination of
batch, tree size, head geometry, head dimension, ragged prefix lengths and node counts, cache
strides and workgroup count (attention), of batch, tree size, vocabulary and row padding
(acceptance, from logits and from hidden states), or of rows, vocabulary, k and layer sizes (top-k
cut, Feature Sampler). Same bars as the fixed cases."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    from tests import _harness
    return _harness


@pytest.mark.parametrize("draw", range(24))
def test_attention_random_shape(H, draw):
    rng = np.random.default_rng([2408, draw])
    D = int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2, 3, 4, 8]))
    G = int(rng.choice([1, 1, 2, 4, 7, 8]))
    B = int(rng.integers(1, 5))
    N = int(rng.integers(1, 65))
    Lmax = int(rng.choice([0, 1, 31, 32, 33, 100, 257, 700, 1500]))
    kv_len = rng.integers(0, Lmax + 1, B).astype(np.int32)
    kv_len[int(rng.integers(0, B))] = Lmax
    n_nodes = rng.integers(1, N + 1, B).astype(np.int32)
    n_nodes[int(rng.integers(0, B))] = N
    splits = int(rng.choice([0, 0, 1, 5, 37, 300]))
    case = H.AttnCase(9000 + draw, B, N, Hkv * G, Hkv, D, Lmax, "bf16", kv_len=kv_len, n_nodes=n_nodes,
                      l_cap=max(1, Lmax + int(rng.integers(0, 9))), interleave=bool(rng.integers(0, 2)))
    out = case.run_gpu(out_dtype=torch.float32, splits=splits)
    ref = case.run_oracle(nthreads=8)
    assert H.rel_err(out, ref) <= H.TOL["bf16"], (B, N, Hkv, G, D, kv_len.tolist(), n_nodes.tolist(), splits)
    for b in range(B):                                   # rows of unused tree slots are written as zeros
        assert not out[b, int(n_nodes[b]):].any()


@pytest.mark.parametrize("draw", range(16))
def test_acceptance_random_shape(H, draw):
    rng = np.random.default_rng([15562, draw])
    B = int(rng.integers(1, 6))
    N = int(rng.integers(1, 65))
    V = int(rng.choice([2, 17, 1000, 1024, 4097, 32000, 50257]))
    topk = int(min(10, max(1, min(N - 1, V - 1))))      # siblings carry distinct tokens
    N = min(N, 1 + topk + 5 * topk * topk)              # what a depth-6 generator tree can hold
    n_nodes = rng.integers(1, N + 1, B).astype(np.int32)
    mode = str(rng.choice(["greedy", "sample"]))
    case = H.AcceptCase(9100 + draw, B, N, V, mode, peak=float(rng.choice([0.0, 3.0])), n_nodes=n_nodes,
                        row_pad=int(rng.choice([0, 0, 1, 3, 8])), topk=topk)
    H.assert_accept_equal(case.gpu_greedy(), case.cpu_greedy())
    T = float(rng.choice([0.5, 1.0, 1.7]))
    cpu = case.cpu_sample(T)
    keep = cpu[4] >= H.MARGIN
    H.assert_accept_equal(case.gpu_sample(T), cpu, keep=keep)


@pytest.mark.parametrize("draw", range(12))
def test_lm_head_acceptance_random_shape(H, draw):
    """Greedy and sampling acceptance from hidden states: batch, tree size, ragged node counts, hidden
    size (multiples of 256), vocabulary (ragged slices of 128) at random."""
    rng = np.random.default_rng([26, draw])
    B = int(rng.integers(1, 7))
    N = int(rng.integers(2, 65))
    Hd = 256 * int(rng.integers(1, 7))
    V = int(rng.choice([2, 100, 129, 1000, 4097, 20000]))
    topk = int(min(10, max(1, min(N - 1, V - 1))))
    N = min(N, 1 + topk + 5 * topk * topk)
    n_nodes = rng.integers(1, N + 1, B).astype(np.int32)
    n_nodes[int(rng.integers(0, B))] = N
    case = H.LmHeadCase(9200 + draw, B, N, Hd, V, topk=topk, n_nodes=n_nodes, noise=0.5)
    H.assert_lm_head_equal(case.gpu(), case.cpu(), require_decided=False)
    T = float(rng.choice([0.5, 1.0, 1.5]))
    # every draw compares at least one sequence: uniforms are redrawn (a few times at most) until one is decided
    compared = 0
    for useed in range(draw, draw + 8):
        compared += H.assert_lm_head_sample_equal(case.gpu_sample(T, useed), case.cpu_sample(T, useed), min_compared=0.0)
        if compared:
            break
    assert compared >= 1


@pytest.mark.parametrize("draw", range(10))
def test_draft_side_random_shape(draw):
    """Top-k cut, tree build on its output, Feature Sampler: rows, vocabulary, k, sizes at random."""
    import oracle
    import paper_2408_15562_amd as fspad
    from workloads import gen_feature_sampler, gen_logits
    rng = np.random.default_rng([2024, draw])
    rows = int(rng.integers(1, 41))
    V = int(rng.choice([5, 100, 1023, 5000, 33000]))
    k = int(min(V, rng.integers(1, 17)))
    x = gen_logits(9300 + draw, 1, rows, V, peak=float(rng.choice([0.0, 4.0])))[0]
    tok, lp = fspad.fspad_draft_topk(torch.from_numpy(x).to("cuda:0"), k)
    torch.cuda.synchronize()
    r_tok, r_lp = oracle.draft_topk(x, k)
    np.testing.assert_array_equal(tok.cpu().numpy(), r_tok)
    np.testing.assert_allclose(lp.cpu().numpy(), r_lp, rtol=0, atol=4e-6)

    Hd, I = 256 * int(rng.integers(1, 5)), 256 * int(rng.integers(1, 9))
    host = gen_feature_sampler(9400 + draw, rows, Hd, I)
    residual = bool(rng.integers(0, 2))
    out = fspad.fspad_feature_sampler(*[torch.from_numpy(a).to("cuda:0", dtype=torch.bfloat16) for a in host], residual=residual)
    torch.cuda.synchronize()
    ref = oracle.feature_sampler(*host, residual=residual)
    err = np.abs(out.float().cpu().numpy().astype(np.float64) - ref)
    bound = np.abs(ref) * 2.0 ** -8 + 1e-2 * np.sqrt(np.mean(ref ** 2))
    assert (err <= bound).all(), (rows, Hd, I, residual, float((err / bound).max()))
