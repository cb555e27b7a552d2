"""GPU parity of fspad_tree_attn against the CPU oracle, through the C ABI.

Bar: max-abs-error <= 2e-2 x RMS(oracle output) for bf16 inputs, <= 1e-5 x RMS for fp32.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from workloads import CONFIGS, chain_tree  # noqa: E402


@pytest.fixture(scope="module")
def H():
    from tests import _harness
    return _harness


def _check(H, case, tol, **kw):
    out = case.run_gpu(**kw)
    ref = case.run_oracle(scale=kw.get("scale") or None)
    err = H.rel_err(out, ref)
    assert err <= tol, f"rel err {err:.3e} > {tol}"
    # rows of unused tree slots are written as zeros
    for b, n in enumerate(case.n_nodes):
        assert torch.all(out[b, int(n):] == 0)
    return out, ref, err


def test_config0_tiny_fp32(H):
    c = CONFIGS["c0"]
    case = H.AttnCase(100, c.batch, c.n_nodes, c.n_q_heads, c.n_kv_heads, c.head_dim, c.kv_len, "f32",
                      depth=c.tree_depth, topk=c.tree_topk)
    _check(H, case, H.TOL["f32"])


@pytest.mark.parametrize("N,L,Hq,Hkv,D", [
    (1, 0, 2, 2, 64), (2, 1, 4, 1, 64), (26, 15, 4, 4, 128), (31, 17, 8, 2, 64), (33, 255, 2, 1, 128),
    (60, 256, 8, 8, 64), (64, 100, 4, 2, 128),
])
def test_fp32_sweep(H, N, L, Hq, Hkv, D):
    case = H.AttnCase(101 + N + L, 2, N, Hq, Hkv, D, L, "f32", l_cap=L + 3)
    _check(H, case, H.TOL["f32"])


@pytest.mark.parametrize("N", [1, 2, 16, 17, 26, 31, 32, 33, 48, 60, 63, 64])
@pytest.mark.parametrize("L", [0, 1, 31, 32, 33, 255, 1000])
def test_bf16_mha_sweep_nodes_and_lengths(H, N, L):
    case = H.AttnCase(7 * N + L, 2, N, 2, 2, 128, L, "bf16", l_cap=L + 5)
    _check(H, case, H.TOL["bf16"])


@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (4, 1), (8, 2), (8, 1), (16, 2)])
@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("N", [5, 26, 60])
def test_bf16_gqa_and_head_dim(H, Hq, Hkv, D, N):
    case = H.AttnCase(13 * Hq + D + N, 1, N, Hq, Hkv, D, 200, "bf16")
    _check(H, case, H.TOL["bf16"])


@pytest.mark.parametrize("N,Hq,Hkv,D", [(60, 8, 2, 128), (40, 4, 1, 64), (26, 16, 2, 128), (64, 8, 1, 64)])
@pytest.mark.parametrize("L,splits", [(0, 0), (33, 0), (200, 0), (1000, 0), (1000, 7), (3000, 64)])
def test_bf16_shared_stage_kernel(H, N, Hq, Hkv, D, L, splits):
    """Grouped-query shapes with more than 128 rows per KV head take the kernel whose wavefronts
    share K/V blocks through LDS."""
    case = H.AttnCase(31 * N + L + 4, 2, N, Hq, Hkv, D, L, "bf16", l_cap=L + 9)
    _check(H, case, H.TOL["bf16"], **({"splits": splits} if splits else {}))


@pytest.mark.parametrize("splits", [1, 2, 3, 7, 16, 50, 333, 4096])
def test_bf16_workgroup_counts(H, splits):
    """Any number of workgroups cuts the flat block list differently (whole units, units cut in
    two or many segments, more workgroups than blocks); the result must not depend on it."""
    case = H.AttnCase(300 + splits, 2, 26, 4, 4, 128, 777, "bf16", kv_len=[777, 40])
    out, ref, _ = _check(H, case, H.TOL["bf16"], splits=splits)
    # run-to-run determinism (no floating-point atomics, fixed merge order)
    for _ in range(3):
        again = case.run_gpu(splits=splits)
        assert torch.equal(out, again)


@pytest.mark.parametrize("N,splits", [(26, 0), (26, 300), (26, 511), (17, 400), (26, 256)])
def test_bf16_small_tiles_above_and_below_one_workgroup_per_cu(H, N, splits):
    """32-row tiles with one workgroup per compute unit at most, and with two (more than 256
    workgroups), on a problem long enough for either: streams of 4 to 30 blocks per wave."""
    case = H.AttnCase(500 + N + splits, 2, N, 8, 8, 128, 2100, "bf16", kv_len=[2100, 1500])
    _check(H, case, H.TOL["bf16"], splits=splits)


@pytest.mark.parametrize("dtype,N,Hq,Hkv", [("bf16", 9, 2, 2), ("bf16", 40, 4, 1), ("f32", 9, 2, 2)])
def test_more_sequences_than_one_launch_takes(H, dtype, N, Hq, Hkv):
    """Sequences go to the kernels in slices of 128 (their lengths travel as kernel arguments): 130
    ragged sequences take two launches that reuse one workspace in stream order."""
    B = 130
    rng = np.random.default_rng(130 + N)
    kv_len = rng.integers(0, 90, B).astype(np.int32)
    n_nodes = rng.integers(1, N + 1, B).astype(np.int32)
    case = H.AttnCase(1300 + N, B, N, Hq, Hkv, 64, 90, dtype, kv_len=kv_len, n_nodes=n_nodes, topk=4)
    _check(H, case, H.TOL[dtype])


def test_bf16_shared_workspace_sees_no_stale_partials(H):
    """Two different problems of one shape alternate on one workspace, launched back to back: a
    merge that picked up the other problem's leftovers would not reproduce the result obtained
    on a private workspace."""
    import paper_2408_15562_amd as fspad
    cases = [H.AttnCase(340 + i, 1, 26, 8, 8, 128, 1500, "bf16") for i in range(2)]
    desc = fspad.make_attn_desc(cases[0].q, cases[0].k_tree, cases[0].k_cache, torch.float32, 0.0)
    shared = torch.empty(fspad.fspad_tree_attn_workspace_bytes(desc, 1500), dtype=torch.uint8, device=H.DEV)
    private = [c.run_gpu() for c in cases]
    for i, c in enumerate(cases):
        assert H.rel_err(private[i], c.run_oracle()) <= H.TOL["bf16"]
    for rep in range(6):
        for i, c in enumerate(cases):   # no host synchronisation in between: back-to-back launches
            out = fspad.fspad_tree_attn(c.q, c.k_tree, c.v_tree, c.k_cache, c.v_cache, c.kv_len, c.n_nodes,
                                        c.mask_dev, workspace=shared, out_dtype=torch.float32)
            assert torch.equal(out, private[i]), f"repetition {rep}, problem {i}"


@pytest.mark.parametrize("N,Hq,Hkv", [(26, 2, 2), (60, 2, 2), (60, 8, 2), (40, 4, 1)])
@pytest.mark.parametrize("splits", [0, 1])
def test_bf16_scores_that_keep_growing(H, N, Hq, Hkv, splits):
    """Keys whose scores climb along the prefix (by far more than the slack the kernel leaves before
    it moves a row's softmax shift) force the shift to move again and again in the middle of the
    stream, in some row tiles and not in others; a ramp in the other direction never moves it."""
    L = 1500
    for direction in (1.0, -1.0):
        case = H.AttnCase(900 + N + Hq, 1, N, Hq, Hkv, 128, L, "bf16")
        ramp = np.linspace(-1.0, 1.0, L)[None, None, :, None] * direction
        k = case.host["k_cache"]
        # rows of Q get different signs, so that growth happens for some rows only
        q = case.host["q"]
        q_dir = np.sign(q.sum(axis=-1, keepdims=True)) * np.ones_like(q) * 0.25
        k_new = (k * 0.3 + 4.0 * ramp * np.ones_like(k)).astype(np.float32)
        q_new = (q * 0.3 + q_dir).astype(np.float32)
        # round to bf16 on both sides
        case.host["k_cache"] = torch.from_numpy(k_new).to(torch.bfloat16).float().numpy()
        case.host["q"] = torch.from_numpy(q_new).to(torch.bfloat16).float().numpy()
        case.k_cache = H.to_dev(case.host["k_cache"], "bf16")
        case.q = H.to_dev(case.host["q"], "bf16")
        _check(H, case, H.TOL["bf16"], splits=splits)


def test_bf16_ragged_batch_and_strided_cache(H):
    case = H.AttnCase(400, 4, 60, 8, 2, 128, 0, "bf16", kv_len=[513, 0, 64, 1], n_nodes=[60, 1, 33, 17],
                      l_cap=600, interleave=True)
    _check(H, case, H.TOL["bf16"])
    _check(H, case, H.TOL["bf16"], splits=4)
    _check(H, case, H.TOL["bf16"], splits=40)


def test_bf16_output_is_rounded_fp32_output(H):
    case = H.AttnCase(401, 1, 26, 4, 4, 128, 300, "bf16")
    o32 = case.run_gpu(out_dtype=torch.float32)
    o16 = case.run_gpu(out_dtype=torch.bfloat16)
    assert torch.equal(o16, o32.to(torch.bfloat16))
    o16s = case.run_gpu(out_dtype=torch.bfloat16, splits=3)
    assert torch.equal(o16s, case.run_gpu(out_dtype=torch.float32, splits=3).to(torch.bfloat16))


def test_custom_scale(H):
    case = H.AttnCase(402, 1, 26, 4, 2, 64, 100, "bf16")
    _check(H, case, H.TOL["bf16"], scale=0.05)
    case32 = H.AttnCase(403, 1, 26, 4, 2, 64, 100, "f32")
    _check(H, case32, H.TOL["f32"], scale=0.05)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_zero_query_closed_form_on_gpu(H, dtype):
    """Q = 0 => every row is the plain mean of the visible value rows: catches mask and stride
    mistakes that a tolerance could hide."""
    case = H.AttnCase(404, 1, 60, 2, 1, 128, 100, dtype)
    case.q.zero_()
    out = case.run_gpu().double().cpu().numpy()
    v_pre = case.host["v_cache"][0, 0, :100].astype(np.float64)
    v_tree = case.host["v_tree"][0, :, 0].astype(np.float64)
    for i in range(60):
        anc, a = [], i
        while a >= 0:
            anc.append(a)
            a = int(case.parent[0, a])
        expect = (v_pre.sum(0) + v_tree[anc].sum(0)) / (100 + len(anc))
        tol = 2e-2 * np.sqrt(np.mean(expect ** 2)) if dtype == "bf16" else 1e-5
        assert np.abs(out[0, i] - expect).max() <= tol


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_chain_tree_is_causal_attention_on_gpu(H, dtype):
    import torch.nn.functional as F
    N, L, Hh, D = 33, 70, 2, 64
    case = H.AttnCase(405, 1, N, Hh, Hh, D, L, dtype, parent=chain_tree(N))
    out = case.run_gpu().double().cpu()
    h = case.host
    k_all = torch.from_numpy(np.concatenate([h["k_cache"][0, :, :L], h["k_tree"][0].transpose(1, 0, 2)], axis=1)).double()
    v_all = torch.from_numpy(np.concatenate([h["v_cache"][0, :, :L], h["v_tree"][0].transpose(1, 0, 2)], axis=1)).double()
    q_full = torch.zeros(Hh, L + N, D, dtype=torch.float64)
    q_full[:, L:] = torch.from_numpy(h["q"][0].transpose(1, 0, 2)).double()
    ref = F.scaled_dot_product_attention(q_full[None], k_all[None], v_all[None], is_causal=True)[0, :, L:]
    ref = ref.permute(1, 0, 2)
    rms = ref.pow(2).mean().sqrt().item()
    assert (out[0] - ref).abs().max().item() <= H.TOL[dtype] * rms


def test_config1_vicuna7b_layer_full(H):
    c = CONFIGS["c1"]
    case = H.AttnCase(500, c.batch, c.n_nodes, c.n_q_heads, c.n_kv_heads, c.head_dim, c.kv_len, "bf16",
                      depth=c.tree_depth, topk=c.tree_topk)
    _check(H, case, H.TOL["bf16"])
    out16 = case.run_gpu(out_dtype=torch.bfloat16)
    # bf16 output: the fp32 bound plus half a bf16 ulp of the largest output
    ref = case.run_oracle()
    assert H.rel_err(out16.float(), ref) <= H.TOL["bf16"] + 2.0 ** -8 * np.abs(ref).max() / np.sqrt(np.mean(ref ** 2))


def test_config2_llama3_8b_gqa_layer_full(H):
    c = CONFIGS["c2"]
    case = H.AttnCase(501, c.batch, c.n_nodes, c.n_q_heads, c.n_kv_heads, c.head_dim, c.kv_len, "bf16",
                      depth=c.tree_depth, topk=c.tree_topk)
    _check(H, case, H.TOL["bf16"])


def test_config3_one_layer_four_sequences_sampled_heads(H):
    """One layer of the Vicuna-33B-shaped stack at full size (B=4, 52 heads, L=4096, N=60), in the
    launch configuration the benchmark uses; the oracle checks all rows of 6 sampled heads."""
    c = CONFIGS["c3"]
    case = H.AttnCase(502, c.batch, c.n_nodes, c.n_q_heads, c.n_kv_heads, c.head_dim, c.kv_len, "bf16",
                      depth=c.tree_depth, topk=c.tree_topk)
    out = case.run_gpu()
    heads = [0, 7, 19, 33, 44, 51]
    ref = case.run_oracle(heads=heads)
    assert H.rel_err(out[:, :, heads], ref) <= H.TOL["bf16"]
    assert torch.isfinite(out).all()


def test_config4_one_layer_long_context_sampled_heads(H):
    """One layer of the LLaMA3-70B-shaped stack (64/8 GQA, L=16384, N=60); oracle on 4 sampled heads."""
    c = CONFIGS["c4"]
    case = H.AttnCase(503, c.batch, c.n_nodes, c.n_q_heads, c.n_kv_heads, c.head_dim, c.kv_len, "bf16",
                      depth=c.tree_depth, topk=c.tree_topk)
    out = case.run_gpu()
    heads = [0, 13, 38, 63]
    ref = case.run_oracle(heads=heads)
    assert H.rel_err(out[:, :, heads], ref) <= H.TOL["bf16"]
    assert torch.isfinite(out).all()


def test_very_long_prefix(H):
    """150 000 prefix keys of one kv head under two query heads (4 689 blocks per unit, cut over every
    compute unit): the flat block arithmetic and the merge at the far end of their ranges."""
    case = H.AttnCase(505, 1, 64, 2, 1, 128, 150_000, "bf16")
    _check(H, case, H.TOL["bf16"])


def test_token_stride_of_two_megabytes(H):
    """A cache whose tokens lie 2^20 elements apart (the largest strides the descriptor accepts are of
    that order): byte offsets inside one sequence pass 4 GB, so every address has to be formed in 64
    bits. The keys and values themselves are the usual ones, viewed through the wide stride."""
    L, stride = 2100, 1 << 20
    case = H.AttnCase(506, 1, 40, 4, 2, 128, L, "bf16")
    wide = []
    for t in (case.k_cache, case.v_cache):          # [1, 2, L, 128] contiguous
        buf = torch.empty((2 * L * stride,), dtype=torch.bfloat16, device=H.DEV)
        view = buf.as_strided((1, 2, L, 128), (2 * L * stride, L * stride, stride, 1))
        view.copy_(t)
        wide.append(view)
    case.k_cache, case.v_cache = wide
    assert case.k_cache.stride(2) == stride and (L - 1) * stride * 2 > 4 * 2 ** 30
    _check(H, case, H.TOL["bf16"])
    del wide, case
    torch.cuda.empty_cache()


def test_missing_workspace_is_an_error_not_a_crash(H):
    import paper_2408_15562_amd as fspad
    case = H.AttnCase(504, 1, 26, 32, 32, 128, 2048, "bf16")
    tiny = torch.empty(16, dtype=torch.uint8, device=H.DEV)
    with pytest.raises(fspad.FspadError) as e:
        fspad.fspad_tree_attn(case.q, case.k_tree, case.v_tree, case.k_cache, case.v_cache, case.kv_len,
                              case.n_nodes, case.mask_dev, workspace=tiny)
    assert e.value.status == 5
