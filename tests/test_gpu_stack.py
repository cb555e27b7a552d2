"""The layer stacks of the two large configurations run the way the benchmark runs them: several
layers back to back over distinct K/V, query and output buffers, all through ONE workspace, prepared
calls on one stream with no synchronisation in between, then a single synchronisation.

Checked against the CPU oracle: ALL query heads of the first, the middle and the last layer for one
sequence, and two sampled heads of every other (layer, sequence) pair -- so a partial result that one
layer's call left in the shared workspace and a later call picked up, or a buffer mixed up between
layers, cannot pass. Bar: max-abs-error <= 2e-2 x RMS(oracle output), as for the single calls."""
import numpy as np
import pytest
import torch

import paper_2408_15562_amd as fspad
from workloads import CONFIGS

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    from tests import _harness
    return _harness


@pytest.mark.parametrize("name,n_layers", [("c3", 5), ("c4", 5)])
def test_stack_of_layers_through_one_workspace(H, name, n_layers):
    c = CONFIGS[name]
    cases = [H.AttnCase(7000 + 11 * layer + (0 if name == "c3" else 500), c.batch, c.n_nodes, c.n_q_heads, c.n_kv_heads,
                        c.head_dim, c.kv_len, "bf16", depth=c.tree_depth, topk=c.tree_topk) for layer in range(n_layers)]
    # the benchmark's launch sequence: one descriptor, one workspace, one prepared call per layer
    first = cases[0]
    desc = fspad.make_attn_desc(first.q, first.k_tree, first.k_cache, torch.float32)
    ws = torch.empty(max(16, fspad.fspad_tree_attn_workspace_bytes(desc, c.kv_len)), dtype=torch.uint8, device=H.DEV)
    ws.random_()                                            # whatever an earlier user left there
    outs = [torch.full(case.q.shape, float("nan"), dtype=torch.float32, device=H.DEV) for case in cases]
    calls = [fspad.fspad_tree_attn(case.q, case.k_tree, case.v_tree, case.k_cache, case.v_cache, case.kv_len, case.n_nodes,
                                   case.mask_dev, out=out, workspace=ws, desc=desc, prepare=True)
             for case, out in zip(cases, outs)]
    for _ in range(2):                                      # twice: the second pass starts from the first one's workspace
        for call in calls:
            call()
    torch.cuda.synchronize()

    rng = np.random.default_rng(7 if name == "c3" else 8)
    full_layers = {0, n_layers // 2, n_layers - 1}
    seq_full = int(rng.integers(0, c.batch))
    worst = 0.0
    for layer, (case, out) in enumerate(zip(cases, outs)):
        assert torch.isfinite(out).all()
        if layer in full_layers:
            # every head of one sequence (run as a batch of one so that the oracle does only that work)
            h = case.host
            import oracle
            b = seq_full
            ref = oracle.tree_attn(h["q"][b:b + 1], h["k_tree"][b:b + 1], h["v_tree"][b:b + 1], h["k_cache"][b:b + 1],
                                   h["v_cache"][b:b + 1], case.kv_len[b:b + 1], case.n_nodes[b:b + 1], case.parent[b:b + 1],
                                   packed_mask=case.mask[b:b + 1], nthreads=16)
            worst = max(worst, H.rel_err(out[b:b + 1], ref))
        heads = sorted(rng.choice(c.n_q_heads, size=2, replace=False).tolist())
        ref = case.run_oracle(heads=heads)                  # two sampled heads, all sequences
        worst = max(worst, H.rel_err(out[:, :, heads], ref))
        print(f"{name} layer {layer}: worst rel err so far {worst:.3e}", flush=True)
    assert worst <= H.TOL["bf16"], worst
