"""Prepared calls (arguments marshalled once) issue exactly the call they were made from."""
import numpy as np
import pytest
import torch

import paper_2408_15562_amd as fspad

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    from tests import _harness
    return _harness


def test_prepared_attention_and_acceptance_repeat_the_direct_calls(H):
    case = H.AttnCase(77, 2, 26, 8, 2, 128, 300, "bf16", kv_len=[300, 123])
    direct = case.run_gpu(out_dtype=torch.float32)
    out = torch.zeros_like(direct)
    call = fspad.fspad_tree_attn(case.q, case.k_tree, case.v_tree, case.k_cache, case.v_cache, case.kv_len,
                                 case.n_nodes, case.mask_dev, out=out, out_dtype=torch.float32, prepare=True)
    assert isinstance(call, fspad.PreparedCall)
    torch.cuda.synchronize()
    assert not out.any()                    # preparing issues nothing
    for _ in range(2):
        out.zero_()
        assert call() is out
        torch.cuda.synchronize()
        assert torch.equal(out, direct)

    acc = H.AcceptCase(78, 2, 26, 1000, "sample", peak=2.0)
    for direct, prepared in ((acc.gpu_greedy(), fspad.fspad_tree_accept_greedy(acc.logits_dev, acc.tokens_dev, acc.parent_dev, acc.n_nodes_dev, prepare=True)),
                             (acc.gpu_sample(0.9), fspad.fspad_tree_accept_sample(acc.logits_dev, acc.tokens_dev, acc.parent_dev, acc.n_nodes_dev, 0.9,
                                                                                  acc.uniforms_dev, prepare=True))):
        for _ in range(2):
            res = prepared()
            torch.cuda.synchronize()
            for a, b in zip(direct, res):
                assert np.array_equal(a if isinstance(a, np.ndarray) else a.cpu().numpy(), b.cpu().numpy())
