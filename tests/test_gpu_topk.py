"""GPU parity of fspad_draft_topk against the CPU oracle, through the C ABI.

Bar: tokens bit-exact (order included; ties to the lower token), log-probabilities within 4e-6
absolute (fp32 exponentials summed in fp64 on the GPU, fp64 throughout in the oracle)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import oracle  # noqa: E402
from workloads import gen_logits  # noqa: E402

DEV = "cuda:0"
ATOL = 4e-6


def _run(x, k, **kw):
    import paper_2408_15562_amd as fspad
    tok, lp = fspad.fspad_draft_topk(x, k, **kw)
    torch.cuda.synchronize()
    return tok.cpu().numpy(), lp.cpu().numpy()


def _check(host, k, dev=None):
    tok, lp = _run(torch.from_numpy(host).to(DEV) if dev is None else dev, k)
    r_tok, r_lp = oracle.draft_topk(host, k)
    np.testing.assert_array_equal(tok, r_tok)
    fin = np.isfinite(r_lp)
    np.testing.assert_allclose(lp[fin], r_lp[fin], rtol=0, atol=ATOL)
    assert np.array_equal(np.isneginf(lp), np.isneginf(r_lp))


@pytest.mark.parametrize("rows,V,k", [
    (1, 1, 1), (1, 5, 5), (3, 1000, 4), (4, 1024, 10), (2, 1025, 16), (10, 32000, 10), (40, 32000, 4),
    (1, 32000, 16), (10, 128256, 10), (100, 4099, 10), (700, 777, 3),
])
def test_shapes(rows, V, k):
    """One chunk and many, chunk tails, every chunk size the planner picks, k from 1 to the maximum."""
    x = gen_logits(50 + rows + V, 1, rows, V)[0]
    _check(x, k)


def test_ties_resolve_to_the_lower_token():
    rng = np.random.default_rng(4)
    x = rng.integers(-3, 4, size=(6, 20000)).astype(np.float32)     # seven distinct values: ties everywhere
    x[:, ::7] *= -0.0                                                # zeros of both signs
    _check(x, 16)


def test_nan_and_infinite_entries():
    x = gen_logits(9, 1, 5, 9000)[0]
    x[0, :] = -np.inf                       # nothing finite: tokens 0..k-1, logp -inf
    x[1, 100:8000] = np.nan                 # NaN ranks as -inf and adds nothing to the normaliser
    x[2, :8990] = -np.inf                   # fewer finite entries (10) than k in all chunks but one
    x[3, 5] = np.nan
    _check(x, 12)


def test_strided_and_unaligned_rows():
    host = gen_logits(10, 1, 7, 3001)[0]
    buf = torch.full((7, 3001 + 6), float("nan"), dtype=torch.float32, device=DEV)
    buf[:, 1:3002] = torch.from_numpy(host).to(DEV)
    _check(host, 10, dev=buf[:, 1:3002])    # rows start 4 bytes off a 16-byte boundary


def test_peaked_rows_and_large_values():
    x = gen_logits(11, 1, 8, 32000, peak=12.0)[0]
    x[4] *= 20.0                             # logits in the hundreds: the shift by the maximum matters
    x[5] -= 1000.0
    _check(x, 10)


def test_output_feeds_the_tree_build():
    """A draft step on the device: cut each expanded node's output, append the candidates, build."""
    import paper_2408_15562_amd as fspad
    V, k, n_keep = 5000, 4, 12
    x = gen_logits(12, 1, 1 + k, V)[0]                     # outputs at the root and at its k children
    tok, lp = _run(torch.from_numpy(x).to(DEV), k)
    r_tok, r_lp = oracle.draft_topk(x, k)
    m = 1 + k + k * k
    par = np.full((1, m), -1, np.int32)
    par[0, 1:1 + k] = 0
    for j in range(k):
        par[0, 1 + k + j * k:1 + k + (j + 1) * k] = 1 + j

    def cands(t, l):
        return (np.concatenate([[0], t[0], t[1:].reshape(-1)])[None].astype(np.int32),
                np.concatenate([[0.0], l[0], l[1:].reshape(-1)])[None].astype(np.float32))
    g_tok, g_lp = cands(tok, lp)
    o_tok, o_lp = cands(r_tok, r_lp)
    dev = [torch.from_numpy(a).to(DEV) for a in (par, g_tok, g_lp, np.array([m], np.int32))]
    out = fspad.fspad_tree_build(*dev, n_keep, 16)
    torch.cuda.synchronize()
    ref = oracle.tree_build(par, o_tok, o_lp, [m], n_keep, 16)
    # the two candidate sets differ by rounding in logp only; with continuous data the kept set is the same
    assert np.array_equal(out[0].cpu().numpy(), ref[0]) and np.array_equal(out[1].cpu().numpy(), ref[1])


def test_missing_workspace_is_an_error():
    import paper_2408_15562_amd as fspad
    x = torch.zeros((2, 5000), dtype=torch.float32, device=DEV)
    with pytest.raises(fspad.FspadError):
        fspad.fspad_draft_topk(x, 4, workspace=torch.empty(16, dtype=torch.uint8, device=DEV))
