"""GPU parity of the acceptance passes against the CPU oracle, through the C ABI.

Bar: path, lengths and emitted tokens bit-exact. For sampling, a sequence whose
closest decision sits within 1e-9 (relative) of its threshold is not compared: there
the answer depends on fp64 rounding order (such seeds are counted and must be rare)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from workloads import CONFIGS  # noqa: E402


@pytest.fixture(scope="module")
def H():
    from tests import _harness
    return _harness


@pytest.mark.parametrize("B,N,V", [(1, 1, 7), (3, 2, 1000), (2, 26, 1000), (1, 26, 32000), (2, 60, 32000),
                                   (1, 64, 8192), (1, 60, 128256), (4, 33, 8193), (2, 17, 1001)])
@pytest.mark.parametrize("peak", [0.0, 4.0])
def test_greedy_matches_oracle(H, B, N, V, peak):
    case = H.AcceptCase(1000 + B + N + V, B, N, V, "greedy", peak=peak)
    gpu, cpu = case.gpu_greedy(), case.cpu_greedy()
    H.assert_accept_equal(gpu, cpu)
    if peak and N >= 26:
        assert cpu[1].max() >= 3   # the peaked variant exercises deep walks


@pytest.mark.parametrize("B,N,V", [(1, 1, 7), (3, 2, 1000), (2, 26, 1000), (1, 26, 32000), (2, 60, 32000),
                                   (1, 64, 8192), (1, 60, 128256), (4, 33, 8193), (2, 17, 1001)])
@pytest.mark.parametrize("peak,mode", [(0.0, "sample"), (2.0, "sample"), (4.0, "greedy")])
@pytest.mark.parametrize("T", [1.0, 0.7])
def test_sampling_matches_oracle(H, B, N, V, peak, mode, T):
    case = H.AcceptCase(2000 + B + N + V, B, N, V, mode, peak=peak)
    gpu, cpu = case.gpu_sample(T), case.cpu_sample(T)
    keep = cpu[4] >= H.MARGIN
    assert keep.sum() >= max(1, B - 1)
    H.assert_accept_equal(gpu, cpu, keep)


def test_many_seeds_sampling_walk_depths(H):
    """Peaked logits + drafts from the perturbed target give multi-level walks with rejections."""
    B, N, V = 64, 60, 4096
    case = H.AcceptCase(2500, B, N, V, "sample", peak=1.5)
    gpu, cpu = case.gpu_sample(1.0), case.cpu_sample(1.0)
    keep = cpu[4] >= H.MARGIN
    assert keep.sum() >= B - 2
    H.assert_accept_equal(gpu, cpu, keep)
    assert len(np.unique(cpu[1])) >= 3


def test_ragged_n_nodes_and_padded_rows(H):
    case = H.AcceptCase(2600, 5, 60, 5000, "sample", peak=2.0, n_nodes=[60, 1, 17, 33, 2], row_pad=3)
    H.assert_accept_equal(case.gpu_greedy(), case.cpu_greedy())
    gpu, cpu = case.gpu_sample(1.0), case.cpu_sample(1.0)
    H.assert_accept_equal(gpu, cpu, cpu[4] >= H.MARGIN)


def test_argmax_ties_nan_and_signed_zero(H):
    parent = np.array([[-1, 0, 0]], np.int32)
    V = 9000
    logits = np.full((1, 3, V), -1.0, np.float32)
    logits[0, 0, [10, 8500, 4000]] = 5.0       # three-way tie across chunks -> lowest index
    logits[0, 0, 3] = np.nan
    logits[0, 1, :] = -0.0
    logits[0, 1, 8191] = 0.0                   # -0 == +0 -> index 0 wins
    logits[0, 2, :] = np.nan                   # nothing comparable -> token 0
    tokens = np.array([[1, 10, 4000]], np.int32)
    case = H.AcceptCase(0, 1, 3, V, parent=parent, logits=logits, tokens=tokens)
    gpu, cpu = case.gpu_greedy(), case.cpu_greedy()
    H.assert_accept_equal(gpu, cpu)
    assert gpu[0][0].tolist() == [0, 1, -1] and gpu[2][0].tolist() == [10, 0, -1]


def test_sampling_enumeration_on_gpu(H):
    """The two-level, 4-token-vocabulary case of the oracle pins on a 10-point midpoint grid:
    the GPU must agree with the oracle on every one of the 10^4 walks, and the counts of the two
    drafted first tokens (whose thresholds 4/10 and 1/2 lie on the grid) are exact."""
    M = 10
    rows = np.array([[1, 3, 2, 4], [4, 3, 2, 1], [3, 1, 4, 2], [1, 2, 3, 4], [2, 3, 1, 4]], np.float64) / 10
    parent = np.array([-1, 0, 0, 1, 2], np.int32)
    tokens = np.array([7, 3, 1, 0, 2], np.int32)
    grid = ((np.arange(M) + 0.5) / M).astype(np.float32)
    u1, u2, u3, ub = [g.ravel() for g in np.meshgrid(grid, grid, grid, grid, indexing="ij")]
    B = u1.size
    uni = np.zeros((B, 2, 5), np.float32)
    uni[:, 0, 1], uni[:, 0, 2], uni[:, 0, 3], uni[:, 0, 4] = u1, u2, u3, u3
    uni[:, 1, :] = ub[:, None]
    logits = np.ascontiguousarray(np.broadcast_to(np.log(rows).astype(np.float32), (B, 5, 4)))
    case = H.AcceptCase(0, B, 5, 4, parent=np.broadcast_to(parent, (B, 5)), logits=logits,
                        tokens=np.ascontiguousarray(np.broadcast_to(tokens, (B, 5))), uniforms=uni)
    gpu, cpu = case.gpu_sample(1.0), case.cpu_sample(1.0)
    assert cpu[4].min() > 1e-3
    H.assert_accept_equal(gpu, cpu)
    first = gpu[2][:, 0]
    assert int((first == 3).sum()) == 4000 and int((first == 1).sum()) == 3000


@pytest.mark.parametrize("name", ["c0", "c1", "c2", "c3", "c4"])
def test_config_vocabulary_and_tree_full_size(H, name):
    """Acceptance at the full logits size of every configuration, both modes."""
    c = CONFIGS[name]
    peak = 3.0
    case = H.AcceptCase(3000 + c.vocab + c.n_nodes, c.batch, c.n_nodes, c.vocab, "sample", depth=c.tree_depth,
                        topk=c.tree_topk, peak=peak)
    H.assert_accept_equal(case.gpu_greedy(), case.cpu_greedy())
    gpu, cpu = case.gpu_sample(c.temperature), case.cpu_sample(c.temperature)
    H.assert_accept_equal(gpu, cpu, cpu[4] >= H.MARGIN)
    flat = H.AcceptCase(3100 + c.vocab, c.batch, c.n_nodes, c.vocab, c.accept, depth=c.tree_depth, topk=c.tree_topk)
    H.assert_accept_equal(flat.gpu_greedy(), flat.cpu_greedy())
    gpu, cpu = flat.gpu_sample(1.0), flat.cpu_sample(1.0)
    H.assert_accept_equal(gpu, cpu, cpu[4] >= H.MARGIN)


def test_deterministic_and_reusable_workspace(H):
    import paper_2408_15562_amd as fspad
    case = H.AcceptCase(3200, 2, 60, 32000, "sample", peak=2.0)
    ws = torch.empty(fspad.fspad_tree_accept_workspace_bytes(2, 60, 32000), dtype=torch.uint8, device=H.DEV)
    ws.fill_(0xFF)  # garbage on entry is ignored
    a = fspad.fspad_tree_accept_sample(case.logits_dev, case.tokens_dev, case.parent_dev, case.n_nodes_dev, 1.0,
                                       case.uniforms_dev, workspace=ws)
    g = fspad.fspad_tree_accept_greedy(case.logits_dev, case.tokens_dev, case.parent_dev, case.n_nodes_dev, workspace=ws)
    b = fspad.fspad_tree_accept_sample(case.logits_dev, case.tokens_dev, case.parent_dev, case.n_nodes_dev, 1.0,
                                       case.uniforms_dev, workspace=ws)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x, y)
    H.assert_accept_equal([t.cpu().numpy() for t in g], case.cpu_greedy())


@pytest.mark.parametrize("V", [1024, 5000, 128256])
def test_draw_finds_a_point_mass_at_lane_wavefront_and_chunk_edges(V):
    """A root without children draws its token from the target's distribution. With all the mass on one
    entry the draw must return that entry whatever the uniform is (closed form); the entries sit on both
    sides of the borders of the draw's running sums: lanes 15|16, 31|32, 63|64, thread, wavefront and
    chunk edges, the first and the last entry of the vocabulary. The same through the sampled-draft entry point."""
    import paper_2408_15562_amd as fspad
    from workloads import gen_uniforms
    spots = sorted({i for i in (0, 1, 15, 16, 31, 32, 63, 64, 255, 256, 1023, 1024, 4095, 4096, 8191, 8192, 65535, 65536,
                                V // 2, V - 2, V - 1) if i < V})
    B = len(spots)
    logits = np.full((B, 1, V), -30000.0, np.float32)
    for b, i in enumerate(spots):
        logits[b, 0, i] = 3.0
    tokens = np.zeros((B, 1), np.int32)
    parent = np.full((B, 1), -1, np.int32)
    n_nodes = np.ones(B, np.int32)
    dev = "cuda:0"
    for useed in range(3):
        uni = torch.from_numpy(gen_uniforms(useed, B, 1)).to(dev)
        args = [torch.from_numpy(a).to(dev) for a in (tokens, parent, n_nodes)]
        lg = torch.from_numpy(logits).to(dev)
        out = fspad.fspad_tree_accept_sample(lg, *args, 0.8, uni)
        out2 = fspad.fspad_tree_accept_sample_draft(lg, lg.clone(), *args, 0.8, uni)
        torch.cuda.synchronize()
        for o in (out, out2):
            assert o[1].cpu().tolist() == [1] * B and o[3].cpu().tolist() == [1] * B
            assert o[2].cpu().numpy()[:, 0].tolist() == spots


@pytest.mark.parametrize("V", [5000, 128256])
def test_draw_splits_two_equal_masses_at_every_border(V):
    """Two neighbouring entries with half of the mass each, on the two sides of a border of the draw's running
    sums: a uniform of 0.25 must give the first, 0.75 the second (closed form), through both sampling entry points."""
    import paper_2408_15562_amd as fspad
    firsts = sorted({i for i in (0, 15, 31, 63, 255, 1023, 4095, 8191, 65535, V // 2, V - 2) if i + 1 < V})
    B = 2 * len(firsts)
    logits = np.full((B, 1, V), -30000.0, np.float32)
    uni = np.zeros((B, 2, 1), np.float32)
    want = []
    for k, i in enumerate(firsts):
        for half in (0, 1):
            b = 2 * k + half
            logits[b, 0, i] = logits[b, 0, i + 1] = -1.5
            uni[b, 1, 0] = 0.25 + 0.5 * half
            want.append(i + half)
    dev = "cuda:0"
    args = [torch.from_numpy(a).to(dev) for a in (np.zeros((B, 1), np.int32), np.full((B, 1), -1, np.int32), np.ones(B, np.int32))]
    lg, u = torch.from_numpy(logits).to(dev), torch.from_numpy(uni).to(dev)
    out = fspad.fspad_tree_accept_sample(lg, *args, 1.3, u)
    out2 = fspad.fspad_tree_accept_sample_draft(lg, lg.clone(), *args, 1.3, u)
    torch.cuda.synchronize()
    assert out[2].cpu().numpy()[:, 0].tolist() == want
    assert out2[2].cpu().numpy()[:, 0].tolist() == want
