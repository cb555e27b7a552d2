"""GPU parity of fspad_tree_accept_sample_draft (acceptance for sampled drafts) against the CPU
oracle, through the C ABI.

Bar: path, lengths and emitted tokens bit-exact. Both sides decide in fp64 but sum in different
orders: a sequence whose closest decision sits within 1e-9 of its threshold is not compared
(such sequences must be rare)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import oracle  # noqa: E402
from workloads import gen_logits, gen_sampled_drafts, gen_trees, gen_uniforms  # noqa: E402

DEV = "cuda:0"
MARGIN = 1e-9


def _case(seed, B, N, V, T, peak=0.0, noise=1.0, n_nodes=None, row_pad=0, depth=6, topk=10):
    topk = min(topk, max(1, N - 1))
    parent, n_nodes = gen_trees(seed, B, N, depth, topk, n_nodes=n_nodes)
    logits = gen_logits(seed, B, N, V, peak=peak)
    draft_logits, tokens = gen_sampled_drafts(seed, logits, parent, n_nodes, T, noise)
    return parent, n_nodes, logits, draft_logits, tokens


def _padded(a, pad):
    if not pad:
        return torch.from_numpy(a).to(DEV)
    B, N, V = a.shape
    buf = torch.full((B, N, V + pad), float("nan"), dtype=torch.float32, device=DEV)
    buf[:, :, :V] = torch.from_numpy(a).to(DEV)
    return buf[:, :, :V]


def _run(seed, B, N, V, T, useed=0, min_compared=None, **kw):
    import paper_2408_15562_amd as fspad
    parent, n_nodes, logits, draft_logits, tokens = _case(seed, B, N, V, T, **kw)
    uni = gen_uniforms(useed, B, N)
    pad = kw.get("row_pad", 0)
    out = fspad.fspad_tree_accept_sample_draft(_padded(logits, pad), _padded(draft_logits, pad), torch.from_numpy(tokens).to(DEV),
                                               torch.from_numpy(parent).to(DEV), torch.from_numpy(n_nodes).to(DEV), T,
                                               torch.from_numpy(uni).to(DEV))
    torch.cuda.synchronize()
    ref = oracle.accept_sample_draft(logits, draft_logits, tokens, parent, n_nodes, T, uni)
    keep = ref[4] >= MARGIN
    assert keep.sum() >= (max(1, B - 1) if min_compared is None else min_compared), ref[4]
    for name, g, c in zip(("path", "path_len", "tokens", "n_tokens"), out, ref[:4]):
        np.testing.assert_array_equal(g.cpu().numpy()[keep], c[keep], err_msg=name)
    return ref


@pytest.mark.parametrize("B,N,V", [(1, 1, 7), (3, 2, 1000), (2, 26, 1000), (1, 26, 32000), (2, 60, 32000),
                                   (1, 64, 8192), (1, 60, 128256), (4, 33, 8193), (2, 17, 1001), (3, 9, 1023)])
@pytest.mark.parametrize("peak,noise", [(0.0, 1.0), (3.0, 0.5)])
@pytest.mark.parametrize("T", [1.0, 0.7])
def test_matches_oracle(B, N, V, peak, noise, T):
    _run(5000 + B + N + V, B, N, V, T, peak=peak, noise=noise)


@pytest.mark.parametrize("B,N,V", [(260, 4, 600), (1, 6, 200000), (1, 5, 300001), (40, 8, 5000), (256, 3, 700)])
def test_both_launch_forms(B, N, V):
    """The library spreads a sequence over several workgroups when the shape allows it and keeps one
    workgroup a sequence otherwise: more sequences than the chip-wide form takes; vocabularies that
    put 16 and 32 entries into a thread; batches that leave a sequence five workgroups, or one."""
    _run(6100 + B + V, B, N, V, 0.9, peak=2.0, noise=0.5, min_compared=B - max(1, B // 40))


def test_one_workspace_call_after_call():
    """The chip-wide form keeps its arrival counts in the workspace and has the streaming pass of every
    call set them to zero: calls that follow one another through one workspace (a larger problem, then a
    smaller one, then the first again) each match the oracle."""
    import paper_2408_15562_amd as fspad
    shapes = [(2, 40, 20000), (1, 12, 3000), (2, 40, 20000)]
    ws = torch.empty(max(fspad.fspad_tree_accept_sample_draft_workspace_bytes(*sh) for sh in shapes), dtype=torch.uint8, device=DEV)
    ws.fill_(0xAB)   # nothing in it is assumed to be zero
    for i, (B, N, V) in enumerate(shapes):
        parent, n_nodes, logits, draft_logits, tokens = _case(6400 + i, B, N, V, 0.8, peak=2.0, noise=0.5)
        uni = gen_uniforms(i, B, N)
        out = fspad.fspad_tree_accept_sample_draft(torch.from_numpy(logits).to(DEV), torch.from_numpy(draft_logits).to(DEV),
                                                   torch.from_numpy(tokens).to(DEV), torch.from_numpy(parent).to(DEV),
                                                   torch.from_numpy(n_nodes).to(DEV), 0.8, torch.from_numpy(uni).to(DEV), workspace=ws)
        torch.cuda.synchronize()
        ref = oracle.accept_sample_draft(logits, draft_logits, tokens, parent, n_nodes, 0.8, uni)
        keep = ref[4] >= MARGIN
        assert keep.sum() >= 1
        for name, g, c in zip(("path", "path_len", "tokens", "n_tokens"), out, ref[:4]):
            np.testing.assert_array_equal(g.cpu().numpy()[keep], c[keep], err_msg=f"call {i}: {name}")


def test_walks_accept_reject_and_draw():
    """A drafter close to a peaked target: accepted chains several levels deep, rejections with
    siblings left (the residual max(p - q, 0) applied more than once at a node), draws at inner
    nodes and at leaves."""
    lens = []
    for useed in range(4):
        ref = _run(77, 32, 40, 3000, 1.0, useed=useed, peak=3.0, noise=0.3, min_compared=30)
        lens += ref[1].tolist()
    assert max(lens) >= 4 and len(set(lens)) >= 3


def test_ragged_trees_and_padded_rows():
    _run(78, 5, 60, 5000, 0.9, peak=2.0, n_nodes=[60, 1, 17, 33, 2], row_pad=4, min_compared=4)


def test_drafter_equal_to_the_target_accepts_whole_chains():
    import paper_2408_15562_amd as fspad
    B, N, V = 3, 12, 2000
    logits = gen_logits(9, B, N, V)
    chain = np.tile(np.arange(-1, N - 1, dtype=np.int32), (B, 1))
    tokens = np.random.default_rng(9).integers(0, V, (B, N)).astype(np.int32)
    uni = gen_uniforms(9, B, N)
    dl = torch.from_numpy(logits).to(DEV)
    out = fspad.fspad_tree_accept_sample_draft(dl, dl.clone(), torch.from_numpy(tokens).to(DEV), torch.from_numpy(chain).to(DEV),
                                               torch.full((B,), N, dtype=torch.int32, device=DEV), 1.0,
                                               torch.from_numpy(uni).to(DEV))
    torch.cuda.synchronize()
    assert out[1].cpu().tolist() == [N] * B
    assert np.array_equal(out[2].cpu().numpy()[:, : N - 1], tokens[:, 1:])


def test_point_mass_drafts_agree_with_the_topk_acceptance_on_gpu():
    """On chains whose draft distribution is a point mass on the drafted token, the call gives what
    fspad_tree_accept_sample gives."""
    import paper_2408_15562_amd as fspad
    B, N, V = 4, 10, 3000
    logits = gen_logits(11, B, N, V, peak=3.0)
    chain = np.tile(np.arange(-1, N - 1, dtype=np.int32), (B, 1))
    nn = torch.full((B,), N, dtype=torch.int32, device=DEV)
    tokens = np.argsort(-logits, axis=2)[:, :, 0].astype(np.int32)          # child c carries its parent's best token
    tokens = np.concatenate([np.zeros((B, 1), np.int32), tokens[:, :-1]], axis=1)
    ql = np.full((B, N, V), -1e30, dtype=np.float32)
    for b in range(B):
        for c in range(1, N):
            ql[b, c - 1, tokens[b, c]] = 0.0
    for useed in range(3):
        uni = torch.from_numpy(gen_uniforms(useed, B, N)).to(DEV)
        args = (torch.from_numpy(tokens).to(DEV), torch.from_numpy(chain).to(DEV), nn, 0.8, uni)
        a = fspad.fspad_tree_accept_sample(torch.from_numpy(logits).to(DEV), *args)
        d = fspad.fspad_tree_accept_sample_draft(torch.from_numpy(logits).to(DEV), torch.from_numpy(ql).to(DEV), *args)
        torch.cuda.synchronize()
        ref = oracle.accept_sample(logits, tokens, chain, np.full(B, N, np.int32), 0.8, uni.cpu().numpy())
        keep = torch.from_numpy(ref[4] >= MARGIN).to(DEV)
        for x, y in zip(a, d):
            assert torch.equal(x[keep], y[keep])


def test_bad_arguments_are_errors():
    import paper_2408_15562_amd as fspad
    B, N, V = 1, 4, 100
    logits = torch.zeros((B, N, V), dtype=torch.float32, device=DEV)
    tok = torch.zeros((B, N), dtype=torch.int32, device=DEV)
    par = torch.tensor([[-1, 0, 0, 1]], dtype=torch.int32, device=DEV)
    nn = torch.tensor([4], dtype=torch.int32, device=DEV)
    uni = torch.zeros((B, 2, N), dtype=torch.float32, device=DEV)
    for t in (0.0, -1.0, float("inf"), float("nan")):
        with pytest.raises(fspad.FspadError):
            fspad.fspad_tree_accept_sample_draft(logits, logits, tok, par, nn, t, uni)
    with pytest.raises(fspad.FspadError):
        fspad.fspad_tree_accept_sample_draft(logits, logits, tok, par, nn, 1.0, uni,
                                             workspace=torch.empty(16, dtype=torch.uint8, device=DEV))
    torch.cuda.synchronize()


@pytest.mark.parametrize("draw", range(10))
def test_random_shape(draw):
    """Batch, tree size, vocabulary, temperature, drafter noise and target peakedness at random."""
    rng = np.random.default_rng([616, draw])
    B = int(rng.integers(1, 7))
    N = int(rng.integers(1, 65))
    V = int(rng.choice([3, 64, 65, 1000, 4097, 20000, 50257]))
    T = float(rng.choice([0.5, 1.0, 1.7]))
    n_nodes = [int(rng.integers(1, N + 1)) for _ in range(B)]
    _run(6000 + draw, B, N, V, T, useed=draw, peak=float(rng.choice([0.0, 2.0, 4.0])), noise=float(rng.choice([0.2, 1.0, 3.0])),
         n_nodes=n_nodes, row_pad=int(rng.choice([0, 0, 4])), depth=8, topk=int(rng.integers(3, 11)), min_compared=max(1, B - 1))


def test_captured_call_replays_like_eager():
    import paper_2408_15562_amd as fspad
    B, N, V, T = 3, 30, 5000, 1.0
    parent, n_nodes, logits, draft_logits, tokens = _case(91, B, N, V, T, peak=2.0, noise=0.5)
    dev = [torch.from_numpy(a).to(DEV) for a in (logits, draft_logits, tokens, parent, n_nodes, gen_uniforms(1, B, N))]
    outs = tuple(torch.empty(s, dtype=torch.int32, device=DEV) for s in ((B, N), (B,), (B, N), (B,)))
    ws = torch.empty(fspad.fspad_tree_accept_sample_draft_workspace_bytes(B, N, V), dtype=torch.uint8, device=DEV)

    def step():
        fspad.fspad_tree_accept_sample_draft(dev[0], dev[1], dev[2], dev[3], dev[4], T, dev[5], outputs=outs, workspace=ws)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in outs]

    def scrub():
        for t in outs:
            t.fill_(-9)
        ws.random_()
        torch.cuda.synchronize()

    step()
    eager = snapshot()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        scrub()
        with torch.cuda.graph(graph, stream=side):
            step()
    for _ in range(3):
        scrub()
        graph.replay()
        for a, b in zip(eager, snapshot()):
            assert torch.equal(a, b)
