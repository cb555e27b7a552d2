"""The library enqueues kernels only (no allocation, no memset, no synchronisation), so a whole
verification step can be captured into a HIP graph. Every replay must reproduce the eager result,
with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

import paper_2408_15562_amd as fspad
from workloads import gen_draft_tokens, gen_logits, gen_qkv, gen_trees, gen_uniforms

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    from tests import _harness
    return _harness


@pytest.mark.parametrize("Hq,Hkv,N,L", [(8, 8, 26, 700), (8, 2, 60, 333)])
def test_captured_step_replays_like_eager(H, Hq, Hkv, N, L):
    B, D, V, cap = 2, 128, 4000, L + N
    dev = H.DEV
    parent, n_nodes = gen_trees(5, B, N, 6, min(10, N - 1))
    mask = torch.from_numpy(fspad.fspad_tree_build_mask(parent, n_nodes).view(np.int64)).to(dev)
    kv_len = np.array([L, L - 50], np.int32)
    q, kt, vt, kc, vc = [H.to_dev(a, "bf16") for a in gen_qkv(5, B, N, Hq, Hkv, D, cap, "bf16")]
    logits_h = gen_logits(5, B, N, V, peak=3.0)
    logits = torch.from_numpy(logits_h).to(dev)
    tokens = torch.from_numpy(gen_draft_tokens(5, logits_h, parent, n_nodes, "sample")).to(dev)
    uni = torch.from_numpy(gen_uniforms(5, B, N)).to(dev)
    parent_d, n_nodes_d = torch.from_numpy(parent).to(dev), torch.from_numpy(n_nodes).to(dev)
    out = torch.empty((B, N, Hq, D), dtype=torch.float32, device=dev)
    desc = fspad.make_attn_desc(q, kt, kc, torch.float32)
    ws_attn = torch.empty(max(16, fspad.fspad_tree_attn_workspace_bytes(desc, L)), dtype=torch.uint8, device=dev)
    ws_acc = torch.empty(fspad.fspad_tree_accept_workspace_bytes(B, N, V), dtype=torch.uint8, device=dev)
    acc_g = tuple(torch.empty(s, dtype=torch.int32, device=dev) for s in ((B, N), (B,), (B, N), (B,)))
    acc_s = tuple(torch.empty(s, dtype=torch.int32, device=dev) for s in ((B, N), (B,), (B, N), (B,)))
    new_len = torch.empty(B, dtype=torch.int32, device=dev)
    cache0 = (kc.clone(), vc.clone())

    def step():
        fspad.fspad_tree_attn(q, kt, vt, kc, vc, kv_len, n_nodes, mask, out=out, workspace=ws_attn, desc=desc)
        fspad.fspad_tree_accept_greedy(logits, tokens, parent_d, n_nodes_d, outputs=acc_g, workspace=ws_acc)
        fspad.fspad_tree_accept_sample(logits, tokens, parent_d, n_nodes_d, 0.8, uni, outputs=acc_s, workspace=ws_acc)
        fspad.fspad_kv_commit(kt, vt, kc, vc, kv_len, acc_s[0], acc_s[1], new_len)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (out, *acc_g, *acc_s, new_len, kc, vc)]

    def scrub():   # eager work between replays; also proves the replay rewrites everything it should
        out.fill_(7.0)
        for t in (*acc_g, *acc_s, new_len):
            t.fill_(-9)
        kc.copy_(cache0[0]); vc.copy_(cache0[1])
        ws_attn.random_(); ws_acc.random_()
        torch.cuda.synchronize()

    step()
    eager = snapshot()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        scrub()
        with torch.cuda.graph(graph, stream=side):
            step()
    for _ in range(4):
        scrub()
        graph.replay()
        for a, b in zip(eager, snapshot()):
            assert torch.equal(a, b)


def test_captured_draft_cut_tree_build_and_fused_acceptance_replay_like_eager(H):
    """The calls around the verification step are captured the same way: top-k cut of a draft step,
    tree selection from the candidates, attention with the tree just built (its node counts read
    back once, before the capture: the attention call takes them on the host), greedy acceptance
    from hidden states."""
    from workloads import gen_candidates, gen_lm_head
    B, N, Hq, Hkv, D, L, V, Hd, k = 2, 26, 8, 2, 128, 500, 3000, 512, 4
    dev = H.DEV
    draft_logits = torch.from_numpy(gen_logits(6, 1, B * k, V)[0]).to(dev)
    cands = [torch.from_numpy(a).to(dev) for a in gen_candidates(6, B, 5, k, V)]
    q, kt, vt, kc, vc = [H.to_dev(a, "bf16") for a in gen_qkv(6, B, N, Hq, Hkv, D, L, "bf16")]
    hidden_h, w_h = gen_lm_head(6, B, N, Hd, V)
    hidden, w = H.to_dev(hidden_h, "bf16"), H.to_dev(w_h, "bf16")
    kv_len = np.array([L, L - 7], np.int32)
    topk_out = (torch.empty((B * k, k), dtype=torch.int32, device=dev), torch.empty((B * k, k), dtype=torch.float32, device=dev))
    ws_topk = torch.empty(fspad.fspad_draft_topk_workspace_bytes(B * k, V, k), dtype=torch.uint8, device=dev)
    ws_lm = torch.empty(fspad.fspad_tree_accept_lm_head_workspace_bytes(B, N, V), dtype=torch.uint8, device=dev)
    acc = tuple(torch.empty(s, dtype=torch.int32, device=dev) for s in ((B, N), (B,), (B, N), (B,)))
    node = (torch.empty((B, N), dtype=torch.int32, device=dev), torch.empty((B, N), dtype=torch.float32, device=dev))
    out = torch.empty((B, N, Hq, D), dtype=torch.float32, device=dev)
    desc = fspad.make_attn_desc(q, kt, kc, torch.float32)
    ws_attn = torch.empty(max(16, fspad.fspad_tree_attn_workspace_bytes(desc, L)), dtype=torch.uint8, device=dev)

    built = fspad.fspad_tree_build(*cands, N, N)        # also the buffers the captured call rewrites
    torch.cuda.synchronize()
    n_nodes_h = built[2].cpu().numpy()
    parent_d, tokens_d, n_nodes_d, mask_d, _ = built

    def step():
        fspad.fspad_draft_topk(draft_logits, k, outputs=topk_out, workspace=ws_topk)
        fspad.fspad_tree_build(*cands, N, N, outputs=built)
        fspad.fspad_tree_attn(q, kt, vt, kc, vc, kv_len, n_nodes_h, mask_d, out=out, workspace=ws_attn, desc=desc)
        fspad.fspad_tree_accept_greedy_lm_head(hidden, w, tokens_d, parent_d, n_nodes_d, outputs=acc, node_outputs=node,
                                               workspace=ws_lm)

    watched = (*topk_out, parent_d, tokens_d, n_nodes_d, mask_d, out, *acc, *node)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in watched]

    def scrub():
        for t in watched:
            t.fill_(-9) if t.dtype != torch.float32 else t.fill_(7.0)
        ws_topk.random_(); ws_lm.random_(); ws_attn.random_()
        torch.cuda.synchronize()

    step()
    eager = snapshot()
    assert np.array_equal(eager[4].cpu().numpy(), n_nodes_h)
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
