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
