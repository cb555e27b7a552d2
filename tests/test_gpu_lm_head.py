"""GPU parity of fspad_tree_accept_greedy_lm_head against the CPU oracle, through the C ABI.

Bar: target tokens, path and emitted tokens bit-exact wherever the oracle's winning logit leads
the runner-up by more than 1e-3 (the kernel sums in fp32, the oracle in fp64; the seeded inputs
are required to be decided everywhere), winning logits within 2e-4 x the largest logit."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from workloads import CONFIGS  # noqa: E402


@pytest.fixture(scope="module")
def H():
    from tests import _harness
    return _harness


@pytest.mark.parametrize("B,N,Hd,V", [
    (1, 1, 256, 1), (1, 2, 256, 127), (1, 16, 512, 128), (1, 17, 256, 129), (1, 26, 1024, 1000),
    (1, 33, 768, 4097), (1, 60, 512, 2000), (1, 64, 256, 640), (2, 26, 512, 999), (3, 22, 256, 3000),
    (2, 60, 1024, 1500), (5, 26, 512, 777), (4, 60, 256, 1111), (3, 60, 512, 1500), (5, 60, 256, 900),
    (9, 58, 768, 300), (1, 26, 256, 40000), (2, 60, 256, 70001),
])
def test_shapes(H, B, N, Hd, V):
    """One to sixteen 16-row tiles (both workgroup shapes), more than 256 rows (several passes over
    the weights), vocabularies that are not multiples of a workgroup's 128 rows and ones with more
    slices than the merge takes in one turn (256), hidden sizes of 1 to 4 times 256."""
    case = H.LmHeadCase(1000 + 7 * N + V, B, N, Hd, V, topk=min(10, max(1, V // 2)))
    H.assert_lm_head_equal(case.gpu(), case.cpu())


def test_ragged_trees(H):
    case = H.LmHeadCase(77, 4, 40, 512, 5000, n_nodes=[40, 1, 17, 33])
    gpu, cpu = case.gpu(), case.cpu()
    H.assert_lm_head_equal(gpu, cpu)
    assert gpu[1].tolist() == cpu[1].tolist() and gpu[1][1] == 1


def test_walks_go_deep_and_results_repeat(H):
    case = H.LmHeadCase(5, 2, 60, 1024, 8000, noise=0.3)
    gpu, cpu = case.gpu(), case.cpu()
    H.assert_lm_head_equal(gpu, cpu)
    assert cpu[1].max() >= 3
    again = case.gpu()
    for a, b in zip(gpu, again):
        assert np.array_equal(a, b)


def test_equal_logits_take_the_lowest_token(H):
    """Duplicate weight rows inside one aligned group of 128 tokens are summed in the same order and
    give bit-identical logits: the lower token wins, within a wavefront's 16 rows and across the
    wavefronts of a workgroup."""
    import paper_2408_15562_amd as fspad
    B, N, Hd, V = 1, 8, 512, 700
    case = H.LmHeadCase(9, B, N, Hd, V)
    hidden = case.hidden.astype(np.float64)
    w = case.w.copy()
    _, _, _, _, target, _, _ = case.cpu()
    # give every node's winning row a twin in the same group: 1, 3, 17, 40, ... rows further (wrapping)
    picks = {}
    for i, off in zip(range(N), (1, 40, 100, 3, 17, 64, 127, 5)):
        t = int(target[0, i])
        base = t // 128 * 128
        twin = base + (t - base + off) % 128
        if twin >= V or twin in picks or twin in target[0] or t in picks:
            continue
        w[twin] = w[t]
        picks[twin] = t
    w_dev = H.to_dev(w, "bf16")
    out = fspad.fspad_tree_accept_greedy_lm_head(case.hidden_dev, w_dev, case.tokens_dev, case.parent_dev, case.n_nodes_dev)
    torch.cuda.synchronize()
    ref = np.einsum("ik,vk->iv", hidden[0], w.astype(np.float64))
    got = out[4].cpu().numpy()[0]
    assert len(picks) >= 5
    for i in range(N):
        assert got[i] == int(np.argmax(ref[i]))      # numpy's argmax is the first maximum


def test_config1_vicuna7b_head_full(H):
    c = CONFIGS["c1"]
    case = H.LmHeadCase(2024, c.batch, c.n_nodes, 4096, c.vocab, depth=c.tree_depth, topk=c.tree_topk)
    H.assert_lm_head_equal(case.gpu(), case.cpu())


def test_config3_four_sequences_33b_head(H):
    c = CONFIGS["c3"]
    case = H.LmHeadCase(2025, c.batch, c.n_nodes, 6656, c.vocab, depth=c.tree_depth, topk=c.tree_topk)
    H.assert_lm_head_equal(case.gpu(), case.cpu())


def test_missing_workspace_is_an_error(H):
    import paper_2408_15562_amd as fspad
    case = H.LmHeadCase(3, 1, 8, 256, 500)
    ws = torch.empty(16, dtype=torch.uint8, device=H.DEV)
    with pytest.raises(fspad.FspadError):
        fspad.fspad_tree_accept_greedy_lm_head(case.hidden_dev, case.w_dev, case.tokens_dev, case.parent_dev,
                                               case.n_nodes_dev, workspace=ws)


@pytest.mark.parametrize("B,N,Hd,V", [
    (1, 1, 256, 1), (1, 2, 256, 127), (2, 16, 512, 128), (3, 17, 256, 129), (4, 26, 1024, 1000),
    (2, 33, 768, 4097), (4, 60, 512, 2000), (2, 64, 256, 640), (8, 26, 512, 999), (3, 60, 512, 1500),
    (5, 60, 256, 900), (2, 26, 256, 40000), (2, 60, 256, 70001),
])
@pytest.mark.parametrize("temperature", [1.0, 0.5])
def test_sampling_shapes(H, B, N, Hd, V, temperature):
    """Tree rejection sampling from hidden states over the same shapes as the greedy form (every
    workgroup shape, several passes, ragged vocabularies, more slices than one scan turn)."""
    case = H.LmHeadCase(3000 + 7 * N + V, B, N, Hd, V, topk=min(10, max(1, V // 2)), noise=0.5)
    for seed in (1, 2):
        H.assert_lm_head_sample_equal(case.gpu_sample(temperature, seed), case.cpu_sample(temperature, seed),
                                      min_compared=0.5 if B < 4 else 0.7)


def test_sampling_walks_accept_reject_and_draw(H):
    """Many sequences at once: accepted chains, rejections with siblings left, draws from the residual."""
    case = H.LmHeadCase(88, 16, 40, 512, 3000, noise=0.3)
    lens = []
    for seed in range(4):
        gpu, cpu = case.gpu_sample(0.7, seed), case.cpu_sample(0.7, seed)
        H.assert_lm_head_sample_equal(gpu, cpu, min_compared=0.8)
        lens += cpu[1].tolist()
    assert max(lens) >= 3 and min(lens) == 1
    again = case.gpu_sample(0.7, 3)
    for a, b in zip(gpu, again):
        assert np.array_equal(a, b)


def test_sampling_config2_llama3_8b_head_full(H):
    c = CONFIGS["c2"]
    case = H.LmHeadCase(2026, c.batch, c.n_nodes, 4096, c.vocab, depth=c.tree_depth, topk=c.tree_topk, noise=0.5)
    compared = 0
    for seed in range(3):       # B = 1: a seed either is decided or is not; two of the three must be
        gpu, cpu = case.gpu_sample(1.0, seed), case.cpu_sample(1.0, seed)
        compared += H.assert_lm_head_sample_equal(gpu, cpu, min_compared=0.0)
    assert compared >= 2


@pytest.mark.parametrize("B,N,V,T,seeds", [(16, 40, 3000, 1.0, (2, 3, 11)), (8, 60, 1500, 0.5, (0, 1, 3)),
                                           (4, 26, 8000, 2.0, (1, 4, 6))])
def test_sampling_on_exactly_representable_logits_has_no_exclusions(H, B, N, V, T, seeds):
    """Hidden states and weights whose products and partial sums are multiples of 1/8 below 2^8: the
    kernel's fp32 logit sums are exact in any order and equal the oracle's, so what is left between
    the two sides is the fp32 exponential and its fp32 argument (a few 1e-7 relative on the sums).
    Every sequence is compared, bit for bit, with no margin exclusion; the uniform seeds were chosen
    on the oracle alone so that every decision stays 2e-5 away from its threshold."""
    case = H.LmHeadCase(600 + N, B, N, 256, V, noise=0.3, exact=True)
    for seed in seeds:
        gpu, cpu = case.gpu_sample(T, seed), case.cpu_sample(T, seed)
        assert cpu[4].min() >= 2e-5, "a decision within 2e-5 of its threshold: pick another seed"
        H.assert_accept_equal(gpu, cpu)


def test_sampling_exclusions_are_counted(H):
    """Runs last among the sampling tests of this file: over everything they compared, the sequences
    left out for a small margin are counted and so are those of them that really differ."""
    s = H.LM_HEAD_SAMPLE_STATS
    print("lm_head sampling totals:", s)
    assert s["compared"] >= 0.5 * s["sequences"] > 0
    assert s["excluded_that_differ"] <= s["excluded"]


def test_sampling_rejects_bad_temperature(H):
    import paper_2408_15562_amd as fspad
    case = H.LmHeadCase(3, 1, 8, 256, 500)
    uni = torch.zeros((1, 2, 8), dtype=torch.float32, device=H.DEV)
    for t in (0.0, -1.0, float("inf"), float("nan")):
        with pytest.raises(fspad.FspadError):
            fspad.fspad_tree_accept_sample_lm_head(case.hidden_dev, case.w_dev, case.tokens_dev, case.parent_dev,
                                                   case.n_nodes_dev, t, uni)


@pytest.mark.parametrize("B,N,Hd,V", [
    (1, 2, 256, 127), (1, 17, 256, 129), (1, 26, 1024, 1000), (1, 33, 768, 4097), (2, 60, 1024, 1500),
    (5, 60, 256, 900), (9, 58, 768, 300), (2, 60, 256, 70001), (1, 26, 4096, 32000),
])
def test_tile_order_weights_give_the_same_bits(H, B, N, Hd, V):
    """The LM head in the tile order of fspad_pack_weight: every output of the greedy form (winning
    logits included) and of the sampling form equals, bit for bit, the one from row-major weights --
    the order of the sums does not change. Vocabularies that leave the last tile row ragged included."""
    case = H.LmHeadCase(4000 + 7 * N + V, B, N, Hd, V, topk=min(10, max(1, V // 2)), noise=0.5)
    for a, b in zip(case.gpu(), case.gpu(packed=True)):
        assert np.array_equal(a, b, equal_nan=True)
    for seed in (1, 2):
        for a, b in zip(case.gpu_sample(0.8, seed), case.gpu_sample(0.8, seed, packed=True)):
            assert np.array_equal(a, b)
