"""GPU parity of fspad_draft_layer against the CPU oracle, through the C ABI.

The oracle keeps fp64 throughout; the library rounds the activations between the projections to
bf16 as a bf16 model stores them.  Bar, element by element over the rows of used tree slots:

    features  |out - oracle| <= 2^-8 |oracle| + 2e-2 x RMS(oracle)
    keys / values  |out - oracle| <= 2^-8 |oracle| + 1e-2 x RMS(oracle)

The first term is the rounding of the result itself to bf16 (half an ulp is at most 2^-8
relative).  The second covers the roundings on the way: each rounds every entry of an activation by
up to 2^-9 relative (standard deviation 2^-9 / sqrt 3 = 1.1e-3), and a projection with weights of
variance 1 / fan-in carries that to a standard deviation of about 1.1e-3 .. 1.7e-3 x the RMS of
its output.  Keys and values have one such rounding behind them (the normalised input); the
features have five or six (normalised input, q / k / v, the attention's probabilities and its
output, the state after attention, its normalised form, the gated product), independent, so about
3.5e-3 x RMS together, and the largest of 10^5 entries lies five to six standard deviations out.
The fp32 sums are far below either term."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import oracle  # noqa: E402
from workloads import gen_draft_layer, gen_trees, tree_depths  # noqa: E402

DEV = "cuda:0"
WEIGHTS = ("w_qkv", "w_o", "w_gate", "w_up", "w_down", "gain_attn", "gain_mlp")


def _dev(a):
    return torch.from_numpy(a).to(DEV, dtype=torch.bfloat16)


def _worst(out, ref, used, c):
    got = out.float().cpu().numpy().astype(np.float64)[used]
    ref = ref[used]
    bound = np.abs(ref) * 2.0 ** -8 + c * np.sqrt(np.mean(ref ** 2))
    return float((np.abs(got - ref) / bound).max())


def _run(seed, B, Nmax, Hd, I, Hq, Hkv, D, kv_len, n_nodes=None, depth=6, topk=8, theta=10000.0, eps=1e-5,
         cache_pad=0):
    import paper_2408_15562_amd as fspad
    kv_len = np.asarray(kv_len, dtype=np.int32)
    l_cap = int(kv_len.max()) + cache_pad
    parent, n_nodes = gen_trees(seed, B, Nmax, depth, topk, n_nodes)
    pos = (kv_len[:, None] + tree_depths(parent, n_nodes)).astype(np.int32)
    host = gen_draft_layer(seed, B, Nmax, Hd, I, Hq, Hkv, D, max(l_cap, 1))
    mask = fspad.fspad_tree_build_mask(parent, n_nodes)
    have_cache = l_cap > 0
    kc = _dev(host["k_cache"]) if have_cache else None
    vc = _dev(host["v_cache"]) if have_cache else None
    outs = fspad.fspad_draft_layer(
        _dev(host["eta"]), torch.from_numpy(pos).to(DEV), {k: _dev(host[k]) for k in WEIGHTS}, kc, vc, kv_len, n_nodes,
        torch.from_numpy(mask.view(np.int64)).to(DEV), Hq, Hkv, D, rms_eps=eps, rope_theta=theta)
    torch.cuda.synchronize()
    ref = oracle.draft_layer(host["eta"], pos, *[host[k] for k in WEIGHTS],
                             host["k_cache"] if have_cache else None, host["v_cache"] if have_cache else None,
                             kv_len, n_nodes, parent, Hq, Hkv, D, eps, theta)
    used = np.arange(Nmax)[None, :] < n_nodes[:, None]
    worst = [_worst(outs[0], ref[0], used, 2e-2), _worst(outs[1], ref[1], used, 2e-2),
             _worst(outs[2], ref[2], used, 1e-2), _worst(outs[3], ref[3], used, 1e-2)]
    print(f"draft layer seed {seed}: worst error / bound  f~ {worst[0]:.2f}  f {worst[1]:.2f}  k {worst[2]:.2f}  v {worst[3]:.2f}",
          flush=True)
    assert max(worst) <= 1.0, f"error at {max(worst):.2f} of the bound ({worst})"
    return outs


@pytest.mark.parametrize("B,Nmax,Hd,I,Hq,Hkv,D,kv_len,n_nodes", [
    (1, 1, 256, 256, 4, 4, 64, [0], None),                      # a lone root, no prefix
    (1, 9, 256, 512, 4, 2, 64, [37], None),
    (2, 9, 256, 512, 4, 2, 64, [37, 0], [9, 5]),                # ragged trees, one sequence without prefix
    (1, 26, 512, 1280, 4, 4, 128, [300], None),                 # head size 128, multi-head
    (3, 11, 512, 768, 8, 1, 64, [129, 64, 1000], [11, 1, 7]),   # one key / value head for eight query heads
    (2, 64, 512, 1024, 8, 2, 64, [515, 77], [64, 33]),          # 128 rows: the largest call
    (4, 16, 768, 2048, 6, 2, 128, [0, 1, 255, 256], None),
])
def test_shapes(B, Nmax, Hd, I, Hq, Hkv, D, kv_len, n_nodes):
    _run(200 + Nmax + Hd // 256, B, Nmax, Hd, I, Hq, Hkv, D, kv_len, n_nodes)


def test_repeatable_and_other_constants():
    a = _run(5, 2, 12, 256, 512, 4, 2, 64, [90, 45], theta=500000.0, eps=1e-6)
    b = _run(5, 2, 12, 256, 512, 4, 2, 64, [90, 45], theta=500000.0, eps=1e-6)
    for x, y in zip(a, b):
        assert torch.equal(x, y)


def test_long_prefix_positions():
    """positions in the thousands: the rotary angles are formed in fp64"""
    _run(6, 1, 10, 256, 512, 4, 2, 64, [8100])


def test_llama_7b_layer_one_verification_sized_tree():
    """hidden 4096, intermediate 11008, 32 heads of 128, a 26-node tree on a 2048-token prefix"""
    _run(7, 1, 26, 4096, 11008, 32, 32, 128, [2048])


def test_zeroed_second_half_returns_the_state_after_attention():
    """with W_down's lower half zero, f is the shared residual itself and f~ is unchanged"""
    import paper_2408_15562_amd as fspad
    B, Nmax, Hd, I, Hq, Hkv, D = 1, 8, 256, 512, 4, 2, 64
    kv_len = np.array([50], dtype=np.int32)
    parent, n_nodes = gen_trees(3, B, Nmax, 4, 3)
    pos = (kv_len[:, None] + tree_depths(parent, n_nodes)).astype(np.int32)
    host = gen_draft_layer(3, B, Nmax, Hd, I, Hq, Hkv, D, 50)
    mask = torch.from_numpy(fspad.fspad_tree_build_mask(parent, n_nodes).view(np.int64)).to(DEV)
    w = {k: _dev(host[k]) for k in WEIGHTS}
    args = (_dev(host["eta"]), torch.from_numpy(pos).to(DEV))
    tail = (_dev(host["k_cache"]), _dev(host["v_cache"]), kv_len, n_nodes, mask, Hq, Hkv, D)
    ft, f, _, _ = [t.clone() for t in fspad.fspad_draft_layer(*args, w, *tail)]
    w0 = dict(w)
    w0["w_down"] = w["w_down"].clone()
    w0["w_down"][Hd:] = 0
    ft0, h, _, _ = fspad.fspad_draft_layer(*args, w0, *tail)
    torch.cuda.synchronize()
    assert torch.equal(ft0, ft)
    # f - h is then what the second half adds: compare with the oracle's MLP contribution loosely
    assert not torch.equal(f, h)


def test_bad_arguments_are_errors():
    import paper_2408_15562_amd as fspad
    B, Nmax, Hd, I, Hq, Hkv, D = 1, 4, 256, 256, 4, 4, 64
    parent, n_nodes = gen_trees(1, B, Nmax, 3, 2)
    host = gen_draft_layer(1, B, Nmax, Hd, I, Hq, Hkv, D, 8)
    mask = torch.from_numpy(fspad.fspad_tree_build_mask(parent, n_nodes).view(np.int64)).to(DEV)
    w = {k: _dev(host[k]) for k in WEIGHTS}
    pos = torch.zeros((B, Nmax), dtype=torch.int32, device=DEV)
    common = (_dev(host["k_cache"]), _dev(host["v_cache"]), [8], n_nodes, mask, Hq, Hkv, D)
    with pytest.raises(fspad.FspadError):        # workspace too small
        fspad.fspad_draft_layer(_dev(host["eta"]), pos, w, *common, workspace=torch.empty(16, dtype=torch.uint8, device=DEV))
    with pytest.raises(fspad.FspadError):        # n_nodes beyond the pitch
        fspad.fspad_draft_layer(_dev(host["eta"]), pos, w, common[0], common[1], [8], [Nmax + 1], mask, Hq, Hkv, D)
    torch.cuda.synchronize()


@pytest.mark.parametrize("draw", range(10))
def test_random_shape(draw):
    """Batch, tree size, head geometry, layer sizes and prefix lengths at random (at most 128 rows)."""
    rng = np.random.default_rng([515, draw])
    Nmax = int(rng.integers(1, 41))
    B = int(rng.integers(1, max(2, min(5, 128 // Nmax + 1))))
    D = int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2, 4]))
    Hq = Hkv * int(rng.choice([1, 2, 4]))
    while (Hq * D) % 256:
        Hq *= 2
    Hd, I = 256 * int(rng.integers(1, 4)), 256 * int(rng.integers(1, 7))
    kv_len = [int(rng.choice([0, 1, 63, 64, 200, 777, 1500])) for _ in range(B)]
    n_nodes = [int(rng.integers(1, Nmax + 1)) for _ in range(B)]
    _run(9500 + draw, B, Nmax, Hd, I, Hq, Hkv, D, kv_len, n_nodes, cache_pad=int(rng.integers(0, 9)))


def test_captured_layer_replays_like_eager():
    """Feature Sampler and decoder layer of one draft step under graph capture: every replay, with
    scrubbed outputs and workspaces, gives what the eager calls gave."""
    import paper_2408_15562_amd as fspad
    from workloads import gen_feature_sampler
    B, Nmax, Hd, I, Hq, Hkv, D, L = 2, 10, 512, 1024, 4, 2, 128, 300
    kv_len = np.array([L, L - 40], dtype=np.int32)
    parent, n_nodes = gen_trees(4, B, Nmax, 4, 3)
    pos = torch.from_numpy((kv_len[:, None] + tree_depths(parent, n_nodes)).astype(np.int32)).to(DEV)
    host = gen_draft_layer(4, B, Nmax, Hd, I, Hq, Hkv, D, L)
    mask = torch.from_numpy(fspad.fspad_tree_build_mask(parent, n_nodes).view(np.int64)).to(DEV)
    w = {k: _dev(host[k]) for k in WEIGHTS}
    kc, vc = _dev(host["k_cache"]), _dev(host["v_cache"])
    f_in, e_in, wu, wg, wd = [_dev(a) for a in gen_feature_sampler(4, B * Nmax, Hd, I)]
    eta = torch.empty((B, Nmax, Hd), dtype=torch.bfloat16, device=DEV)
    outs = (torch.empty((B, Nmax, Hd), dtype=torch.bfloat16, device=DEV), torch.empty((B, Nmax, Hd), dtype=torch.bfloat16, device=DEV),
            torch.empty((B, Nmax, Hkv, D), dtype=torch.bfloat16, device=DEV), torch.empty((B, Nmax, Hkv, D), dtype=torch.bfloat16, device=DEV))
    ws_fs = torch.empty(fspad.fspad_feature_sampler_workspace_bytes(B * Nmax, Hd, I), dtype=torch.uint8, device=DEV)
    ws = torch.empty(1 << 24, dtype=torch.uint8, device=DEV)

    def step():
        fspad.fspad_feature_sampler(f_in, e_in, wu, wg, wd, out=eta.view(B * Nmax, Hd), workspace=ws_fs)
        fspad.fspad_draft_layer(eta, pos, w, kc, vc, kv_len, n_nodes, mask, Hq, Hkv, D, outputs=outs, workspace=ws)

    used = torch.from_numpy(np.arange(Nmax)[None, :] < n_nodes[:, None]).to(DEV)

    def snapshot():
        torch.cuda.synchronize()
        return [eta.clone()] + [t[used].clone() for t in outs]

    def scrub():
        for t in (eta, *outs):
            t.fill_(7.0)
        ws.random_(); ws_fs.random_()
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


@pytest.mark.parametrize("B,Nmax,Hd,I,Hq,Hkv,D,L", [(1, 9, 256, 512, 4, 2, 64, 37), (2, 40, 512, 1280, 4, 4, 128, 300),
                                                  (1, 26, 4096, 11008, 32, 32, 128, 2048)])
def test_packed_weights_give_the_same_bits(B, Nmax, Hd, I, Hq, Hkv, D, L):
    import paper_2408_15562_amd as fspad
    kv_len = np.full(B, L, dtype=np.int32)
    parent, n_nodes = gen_trees(21, B, Nmax, 6, 8)
    pos = torch.from_numpy((kv_len[:, None] + tree_depths(parent, n_nodes)).astype(np.int32)).to(DEV)
    host = gen_draft_layer(21, B, Nmax, Hd, I, Hq, Hkv, D, L)
    mask = torch.from_numpy(fspad.fspad_tree_build_mask(parent, n_nodes).view(np.int64)).to(DEV)
    w = {k: _dev(host[k]) for k in WEIGHTS}
    wp = {k: (fspad.fspad_pack_weight(v) if v.dim() == 2 else v) for k, v in w.items()}
    common = (_dev(host["k_cache"]), _dev(host["v_cache"]), kv_len, n_nodes, mask, Hq, Hkv, D)
    eta = _dev(host["eta"])
    plain = fspad.fspad_draft_layer(eta, pos, w, *common)
    packed = fspad.fspad_draft_layer(eta, pos, wp, *common, packed=True)
    torch.cuda.synchronize()
    used = torch.from_numpy(np.arange(Nmax)[None, :] < n_nodes[:, None]).to(DEV)
    for a, b in zip(plain, packed):
        assert torch.equal(a[used], b[used])


def test_layer_keys_join_the_draft_cache_and_serve_the_next_step():
    """Two draft steps chained on the device: the keys / values the layer returns are committed to the
    draft's cache along a root-to-leaf path (fspad_kv_commit reads them as they are), and the layer
    runs again over a new tree on the longer prefix. The oracle does the same in fp64."""
    import paper_2408_15562_amd as fspad
    B, Nmax, Hd, I, Hq, Hkv, D, L = 2, 12, 256, 512, 4, 2, 64, 90
    cap = L + Nmax
    kv_len = np.array([L, L - 33], dtype=np.int32)
    host = gen_draft_layer(31, B, Nmax, Hd, I, Hq, Hkv, D, cap)
    w = {k: _dev(host[k]) for k in WEIGHTS}
    kc, vc = _dev(host["k_cache"]), _dev(host["v_cache"])
    names = [host[k] for k in WEIGHTS]

    def tree(seed):
        parent, n_nodes = gen_trees(seed, B, Nmax, 5, 3)
        return parent, n_nodes, torch.from_numpy(fspad.fspad_tree_build_mask(parent, n_nodes).view(np.int64)).to(DEV)

    # step 1
    parent, n_nodes, mask = tree(32)
    pos = (kv_len[:, None] + tree_depths(parent, n_nodes)).astype(np.int32)
    out1 = fspad.fspad_draft_layer(_dev(host["eta"]), torch.from_numpy(pos).to(DEV), w, kc, vc, kv_len, n_nodes, mask, Hq, Hkv, D)
    ref1 = oracle.draft_layer(host["eta"], pos, *names, host["k_cache"], host["v_cache"], kv_len, n_nodes, parent, Hq, Hkv, D)
    # the accepted path: from the deepest node of each tree up to its root
    depth = tree_depths(parent, n_nodes)
    path = np.full((B, Nmax), -1, dtype=np.int32)
    path_len = np.zeros(B, dtype=np.int32)
    for b in range(B):
        node, chain = int(np.argmax(depth[b, : n_nodes[b]])), []
        while node >= 0:
            chain.append(node)
            node = int(parent[b, node])
        chain = chain[::-1]
        path[b, : len(chain)] = chain
        path_len[b] = len(chain)
    assert path_len.min() >= 2
    fspad.fspad_kv_commit(out1[2], out1[3], kc, vc, kv_len, torch.from_numpy(path).to(DEV), torch.from_numpy(path_len).to(DEV))
    k_ref, v_ref, len2 = oracle.kv_commit(ref1[2], ref1[3], host["k_cache"].astype(np.float64),
                                          host["v_cache"].astype(np.float64), kv_len, path, path_len)
    # step 2: a new tree and new inputs on the longer prefix
    parent2, n_nodes2, mask2 = tree(33)
    eta2 = gen_draft_layer(34, B, Nmax, Hd, I, Hq, Hkv, D, 1)["eta"]
    pos2 = (len2[:, None] + tree_depths(parent2, n_nodes2)).astype(np.int32)
    out2 = fspad.fspad_draft_layer(_dev(eta2), torch.from_numpy(pos2).to(DEV), w, kc, vc, len2, n_nodes2, mask2, Hq, Hkv, D)
    torch.cuda.synchronize()
    ref2 = oracle.draft_layer(eta2, pos2, *names, k_ref, v_ref, len2, n_nodes2, parent2, Hq, Hkv, D)
    used = np.arange(Nmax)[None, :] < n_nodes2[:, None]
    worst = [_worst(out2[0], ref2[0], used, 2e-2), _worst(out2[1], ref2[1], used, 2e-2),
             _worst(out2[2], ref2[2], used, 1e-2), _worst(out2[3], ref2[3], used, 1e-2)]
    assert max(worst) <= 1.0, worst
    # the committed cache rows are the layer's own keys, moved bit for bit
    got_k = kc.float().cpu().numpy()
    k1 = out1[2].float().cpu().numpy()
    for b in range(B):
        for j in range(path_len[b]):
            assert np.array_equal(got_k[b, :, kv_len[b] + j], k1[b, path[b, j]])
