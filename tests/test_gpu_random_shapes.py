"""Seeded random sweep over shapes inside the documented limits: every draw is a fresh combination of
batch, tree size, head geometry, head dimension, ragged prefix lengths and node counts, cache
strides and workgroup count (attention), or of batch, tree size, vocabulary and row padding
(acceptance). Same bars as the fixed cases: 2e-2 x RMS for bf16 attention, bit-exact acceptance."""
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
