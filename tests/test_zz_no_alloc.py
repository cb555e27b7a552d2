"""The greedy acceptance that keeps its scratch in the library's own fixed device array
(fspad_tree_accept_greedy_static, for callers that cannot allocate) against the entry point that
takes a caller workspace: bit-identical outputs through the C ABI, on two calls in a row that share
the array, the second on a smaller input."""
import numpy as np
import pytest
import torch

import paper_2408_15562_amd as fspad
from workloads import gen_draft_tokens, gen_logits, gen_trees

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _inputs(seed, B, N, V, depth, topk):
    parent, n_nodes = gen_trees(seed, B, N, depth, topk)
    logits = gen_logits(seed, B, N, V, peak=4.0)          # peaked rows: walks several levels deep
    tokens = gen_draft_tokens(seed, logits, parent, n_nodes, "greedy")
    return [torch.from_numpy(np.ascontiguousarray(a)).to(DEV) for a in (logits, tokens, parent, n_nodes)]


def _outputs(B, N):
    return (torch.full((B, N), -7, dtype=torch.int32, device=DEV), torch.full((B,), -7, dtype=torch.int32, device=DEV),
            torch.full((B, N), -7, dtype=torch.int32, device=DEV), torch.full((B,), -7, dtype=torch.int32, device=DEV))


def test_static_scratch_matches_workspace_entry_point_on_two_calls_in_a_row():
    big = _inputs(71, 4, 60, 32000, 6, 10)       # 240 rows x 32 chunks of statistics
    small = _inputs(72, 1, 26, 1000, 5, 4)       # the next call reuses the array with fewer, shorter rows
    seen = []
    for args, (B, N) in ((big, (4, 60)), (small, (1, 26))):
        out_static = _outputs(B, N)
        fspad.fspad_tree_accept_greedy_static(*args, outputs=out_static)     # straight after the previous call
        seen.append(out_static)
    torch.cuda.synchronize()
    for args, (B, N), got in ((big, (4, 60), seen[0]), (small, (1, 26), seen[1])):
        ref = fspad.fspad_tree_accept_greedy(*args, outputs=_outputs(B, N))
        torch.cuda.synchronize()
        for g, r in zip(got, ref):
            assert torch.equal(g, r)
        assert int(got[1].min()) >= 1
    assert int(seen[0][1].max()) >= 2            # the peaked case does accept drafts


def test_static_scratch_rejects_sizes_beyond_the_array():
    B, N, V = 16, 64, 128256
    assert fspad.fspad_tree_accept_workspace_bytes(B, N, V) > (1 << 20)
    logits = torch.zeros((B, N, V), dtype=torch.float32, device=DEV)
    ints = torch.zeros((B, N), dtype=torch.int32, device=DEV)
    n_nodes = torch.ones((B,), dtype=torch.int32, device=DEV)
    with pytest.raises(fspad.FspadError) as err:
        fspad.fspad_tree_accept_greedy_static(logits, ints, ints, n_nodes, outputs=_outputs(B, N))
    assert err.value.status == 5
