"""CPU-only checks of the boundary: the library loads, exports what include/fspad.h declares,
and the host-side logic (mask builder, validator, argument checks) behaves as documented.
No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2408_15562_amd as fspad
from paper_2408_15562_amd import binding
from workloads import gen_trees

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return ctypes.CDLL(fspad.library_path())


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "fspad.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(fspad_[a-z_]+)\s*\(", header))
    assert declared == set(fspad.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    # ... and nothing beyond it: the dynamic symbol table holds no other fspad_* name
    import subprocess
    table = subprocess.run(["nm", "-D", "--defined-only", fspad.library_path()], capture_output=True, text=True, check=True).stdout
    exported = {line.split()[-1] for line in table.splitlines() if line.split() and line.split()[-1].startswith("fspad_")}
    assert exported == declared, sorted(exported ^ declared)


def test_status_strings():
    seen = {fspad.fspad_status_string(i) for i in range(8)}
    assert len(seen) == 8 and "unknown status" not in seen
    assert fspad.fspad_status_string(99) == "unknown status"


def _closure(parent, n):
    words = []
    for i in range(n):
        w, a = 0, i
        while a >= 0:
            w |= 1 << a
            a = int(parent[a])
        words.append(w)
    return words


def test_build_mask_is_transitive_closure():
    parent, n_nodes = gen_trees(21, 3, 64, 6, 10, n_nodes=[64, 26, 1])
    mask = fspad.fspad_tree_build_mask(parent, n_nodes)
    for b in range(3):
        n = int(n_nodes[b])
        assert [int(x) for x in mask[b, :n]] == _closure(parent[b], n)
        assert np.all(mask[b, n:] == 0)
        for i in range(n):
            depth = len(_closure(parent[b], n)) and bin(int(mask[b, i])).count("1") - 1
            assert (int(mask[b, i]) >> i) & 1 and int(mask[b, i]) >> (i + 1) == 0 and depth >= 0


def test_build_mask_and_validate_reject_bad_trees():
    good = np.array([[-1, 0, 0, 1]], np.int32)
    tok = np.array([[5, 1, 2, 1]], np.int32)
    assert fspad.fspad_tree_validate(good, tok, [4], 10) == 0
    assert fspad.fspad_tree_validate(good, None, [4], 10) == 0
    for bad in ([[0, 0, 0, 1]], [[-1, 1, 0, 1]], [[-1, 0, 3, 1]], [[-1, -1, 0, 1]]):
        bad = np.array(bad, np.int32)
        assert fspad.fspad_tree_validate(bad, tok, [4], 10) == 3
        with pytest.raises(fspad.FspadError) as e:
            fspad.fspad_tree_build_mask(bad, [4])
        assert e.value.status == 3
    assert fspad.fspad_tree_validate(good, np.array([[5, 1, 1, 1]], np.int32), [4], 10) == 3   # twin siblings
    assert fspad.fspad_tree_validate(good, np.array([[5, 1, 2, 10]], np.int32), [4], 10) == 3  # token out of range
    assert fspad.fspad_tree_validate(good, tok, [5], 10) == 2                                  # n_nodes > Nmax
    assert fspad.fspad_tree_validate(np.zeros((1, 65), np.int32), None, [1], 10) == 2          # Nmax > 64


def _desc(**kw):
    d = binding.fspad_attn_desc()
    d.batch, d.n_nodes_max, d.n_q_heads, d.n_kv_heads, d.head_dim = 1, 26, 32, 32, 128
    d.io_dtype = d.out_dtype = binding.FSPAD_BF16
    d.cache_stride_token, d.cache_stride_head, d.cache_stride_batch = 128, 128 * 2048, 128 * 2048 * 32
    for k, v in kw.items():
        setattr(d, k, v)
    return d


def test_attn_argument_checks_need_no_gpu(lib):
    f = lib.fspad_tree_attn
    f.restype = ctypes.c_int
    kv = (ctypes.c_int32 * 1)(2048)
    nn = (ctypes.c_int32 * 1)(26)
    fake = ctypes.c_void_p(0x1000)  # never dereferenced: every case below fails validation first

    def call(d, q=fake, kvp=kv, nnp=nn, ws=fake, wsb=1 << 30):
        return f(ctypes.byref(d), q, fake, fake, fake, fake, kvp, nnp, fake, fake, ws, ctypes.c_size_t(wsb), None)

    assert call(_desc(), q=None) == 1
    assert call(_desc(n_nodes_max=65)) == 2
    assert call(_desc(head_dim=96)) == 2
    assert call(_desc(n_kv_heads=5)) == 2
    assert call(_desc(io_dtype=3)) == 4
    assert call(_desc(io_dtype=0, out_dtype=1)) == 4
    assert call(_desc(cache_stride_token=100)) == 2
    assert call(_desc(), nnp=(ctypes.c_int32 * 1)(27)) == 2
    assert call(_desc(), kvp=(ctypes.c_int32 * 1)(-1)) == 2
    assert call(_desc(), wsb=16) == 5
    assert call(_desc(workgroups=-1)) == 2
    assert binding.fspad_tree_attn_workspace_bytes(_desc(), 2048) > 16
    assert binding.fspad_tree_attn_workspace_bytes(_desc(head_dim=96), 2048) == 0


def test_accept_argument_checks_need_no_gpu(lib):
    g, s = lib.fspad_tree_accept_greedy, lib.fspad_tree_accept_sample
    fake = ctypes.c_void_p(0x1000)
    i32, i64, sz = ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    need = fspad.fspad_tree_accept_workspace_bytes(1, 26, 32000)
    assert need >= 26 * 4 * 16

    def greedy(B=1, N=26, V=32000, logits=fake, stride=32000, ws=fake, wsb=need):
        return g(i32(B), i32(N), i32(V), logits, i64(stride), fake, fake, fake, fake, fake, fake, fake, ws, sz(wsb), None)

    assert greedy(logits=None) == 1
    assert greedy(N=65) == 2
    assert greedy(V=0) == 2
    assert greedy(stride=100) == 2
    assert greedy(wsb=need - 1) == 5
    assert greedy(ws=None) == 5

    # the variant that keeps its scratch in the library's own fixed array: sizes beyond it are refused
    # before anything touches the GPU
    gs = lib.fspad_tree_accept_greedy_static

    def greedy_static(B=1, N=26, V=32000, logits=fake, stride=32000):
        return gs(i32(B), i32(N), i32(V), logits, i64(stride), fake, fake, fake, fake, fake, fake, fake, None)

    assert greedy_static(logits=None) == 1
    assert greedy_static(N=65) == 2
    assert greedy_static(V=0) == 2
    assert fspad.fspad_tree_accept_workspace_bytes(16, 64, 128256) > (1 << 20)
    assert greedy_static(B=16, N=64, V=128256, stride=128256) == 5

    def sample(T, uni=fake):
        return s(i32(1), i32(26), i32(32000), fake, i64(32000), fake, fake, fake, ctypes.c_float(T), uni,
                 fake, fake, fake, fake, fake, sz(need), None)

    for t in (0.0, -1.0, float("inf"), float("nan")):
        assert sample(t) == 6
    assert sample(1.0, uni=None) == 1


def test_lm_head_argument_checks_need_no_gpu(lib):
    f = lib.fspad_tree_accept_greedy_lm_head
    fake = ctypes.c_void_p(0x1000)   # never dereferenced: every case below fails validation first
    i32, sz = ctypes.c_int32, ctypes.c_size_t
    need = fspad.fspad_tree_accept_lm_head_workspace_bytes(1, 26, 32000)
    assert need >= 26 * 250 * 8

    def call(B=1, N=26, V=32000, Hd=4096, hidden=fake, w=fake, ws=fake, wsb=need, flags=0):
        return f(i32(B), i32(N), i32(V), i32(Hd), hidden, w, i32(flags), fake, fake, fake, fake, fake, fake, fake, None, None,
                 ws, sz(wsb), None)

    assert call(hidden=None) == 1
    assert call(w=None) == 1
    assert call(N=65) == 2
    assert call(V=0) == 2
    assert call(Hd=4000) == 2          # not a multiple of 256
    assert call(Hd=128) == 2
    assert call(hidden=ctypes.c_void_p(0x1008)) == 2
    assert call(flags=1) == 2          # only "packed weights" (2) is a flag here
    assert call(flags=2, wsb=need - 1) == 5
    assert call(wsb=need - 1) == 5
    assert call(ws=None) == 5

    s = lib.fspad_tree_accept_sample_lm_head

    def sample(T=1.0, uni=fake, Hd=4096, wsb=need, flags=0):
        return s(i32(1), i32(26), i32(32000), i32(Hd), fake, fake, i32(flags), fake, fake, fake, ctypes.c_float(T), uni,
                 fake, fake, fake, fake, fake, sz(wsb), None)

    assert sample(flags=4) == 2

    for t in (0.0, -1.0, float("inf"), float("nan")):
        assert sample(T=t) == 6
    assert sample(uni=None) == 1
    assert sample(Hd=4000) == 2
    assert sample(wsb=need - 1) == 5


def test_sampled_draft_acceptance_argument_checks_need_no_gpu(lib):
    f = lib.fspad_tree_accept_sample_draft
    fake = ctypes.c_void_p(0x1000)   # never dereferenced: every case below fails validation first
    i32, i64, sz = ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    need = fspad.fspad_tree_accept_sample_draft_workspace_bytes(2, 26, 32000)
    assert need >= 2 * 3 * 32000 * 8

    def call(B=2, N=26, V=32000, logits=fake, dl=fake, stride=32000, T=1.0, uni=fake, ws=fake, wsb=need):
        return f(i32(B), i32(N), i32(V), logits, dl, i64(stride), fake, fake, fake, ctypes.c_float(T), uni,
                 fake, fake, fake, fake, ws, sz(wsb), None)

    assert call(logits=None) == 1
    assert call(dl=None) == 1
    assert call(uni=None) == 1
    assert call(N=65) == 2
    assert call(V=0) == 2
    assert call(stride=31999) == 2
    for t in (0.0, -1.0, float("inf"), float("nan")):
        assert call(T=t) == 6
    assert call(wsb=need - 1) == 5
    assert call(ws=None) == 5


def test_feature_sampler_argument_checks_need_no_gpu(lib):
    f = lib.fspad_feature_sampler
    fake = ctypes.c_void_p(0x1000)   # never dereferenced: every case below fails validation first
    i32, sz = ctypes.c_int32, ctypes.c_size_t
    need = fspad.fspad_feature_sampler_workspace_bytes(10, 4096, 11008)
    assert need >= 10 * 11008 * 2
    assert fspad.fspad_feature_sampler_workspace_bytes(129, 4096, 11008) == 0
    assert fspad.fspad_feature_sampler_workspace_bytes(10, 4096, 11000) == 0

    def call(rows=10, Hd=4096, I=11008, x=fake, w=fake, out=fake, ws=fake, wsb=need):
        return f(i32(rows), i32(Hd), i32(I), x, fake, w, fake, fake, i32(1), out, ws, sz(wsb), None)

    assert call(x=None) == 1
    assert call(w=None) == 1
    assert call(out=None) == 1
    assert call(rows=0) == 2
    assert call(rows=129) == 2
    assert call(Hd=4000) == 2
    assert call(I=11000) == 2
    assert call(x=ctypes.c_void_p(0x1008)) == 2
    assert call(wsb=need - 1) == 5
    assert call(ws=None) == 5
    # flags: residual = 1, packed weights = 2; anything else is refused
    assert f(i32(10), i32(4096), i32(11008), fake, fake, fake, fake, fake, i32(4), fake, fake, sz(need), None) == 2
    assert f(i32(10), i32(4096), i32(11008), fake, fake, fake, fake, fake, i32(3), fake, None, sz(need), None) == 5


def test_pack_weight_argument_checks_need_no_gpu(lib):
    fake = ctypes.c_void_p(0x1000)
    i32 = ctypes.c_int32
    assert fspad.fspad_packed_weight_bytes(4096, 11008) == 4096 * 11008 * 2
    assert fspad.fspad_packed_weight_bytes(40, 96) == 48 * 96 * 2          # last tile row padded
    assert fspad.fspad_packed_weight_bytes(40, 100) == 0
    assert fspad.fspad_packed_weight_bytes(0, 96) == 0
    f = lib.fspad_pack_weight
    assert f(i32(40), i32(96), None, fake, None) == 1
    assert f(i32(40), i32(96), fake, None, None) == 1
    assert f(i32(40), i32(100), fake, fake, None) == 2
    assert f(i32(0), i32(96), fake, fake, None) == 2
    assert f(i32(40), i32(96), ctypes.c_void_p(0x1008), fake, None) == 2


def test_draft_layer_argument_checks_need_no_gpu(lib):
    from paper_2408_15562_amd.binding import fspad_draft_layer_desc, fspad_draft_layer_weights
    f = lib.fspad_draft_layer
    fake = ctypes.c_void_p(0x1000)   # never dereferenced: every case below fails validation first
    sz = ctypes.c_size_t

    def desc(B=1, N=26, Hq=32, Hkv=32, D=128, Hd=4096, I=11008, dtype=1, eps=1e-6, theta=10000.0, packed=0):
        d = fspad_draft_layer_desc()
        a = d.attn
        a.batch, a.n_nodes_max, a.n_q_heads, a.n_kv_heads, a.head_dim = B, N, Hq, Hkv, D
        a.io_dtype = a.out_dtype = dtype
        a.cache_stride_batch, a.cache_stride_head, a.cache_stride_token = Hkv * 4096 * D, 4096 * D, D
        d.hidden_dim, d.intermediate_dim, d.rms_eps, d.rope_theta = Hd, I, eps, theta
        d.weights_packed = packed
        return d

    need = fspad.fspad_draft_layer_workspace_bytes(desc(), 2048)
    assert need >= 26 * 11008 * 2 + 26 * 4096 * 2 * 4
    for bad in (desc(N=65), desc(B=3, N=64), desc(Hd=4000), desc(I=11000), desc(D=96), desc(Hq=30, Hkv=4),
                desc(Hq=3, Hkv=3, D=64), desc(dtype=0), desc(theta=0.0), desc(eps=-1.0), desc(packed=2)):
        assert fspad.fspad_draft_layer_workspace_bytes(bad, 2048) == 0

    def weights(**over):
        w = fspad_draft_layer_weights()
        for name, _ in fspad_draft_layer_weights._fields_:
            setattr(w, name, over.get(name, 0x1000))
        return w

    kv = (ctypes.c_int32 * 1)(2048)
    nn = (ctypes.c_int32 * 1)(26)

    def call(d=None, w=None, eta=fake, pos=fake, kv_len=kv, n_nodes=nn, out=fake, ws=fake, wsb=need):
        d = d if d is not None else desc()
        w = w if w is not None else weights()
        return f(ctypes.byref(d), ctypes.byref(w), eta, pos, fake, fake, kv_len, n_nodes, fake, fake, fake, out, fake,
                 ws, sz(wsb), None)

    assert call(eta=None) == 1
    assert call(pos=None) == 1
    assert call(out=None) == 1
    assert call(w=weights(w_down=None)) == 1
    assert call(w=weights(gain_mlp=None)) == 1
    assert call(d=desc(dtype=0)) == 4
    assert call(d=desc(Hd=4000)) == 2
    assert call(d=desc(B=3, N=64)) == 2                    # more than 128 rows
    assert call(eta=ctypes.c_void_p(0x1008)) == 2
    assert call(w=weights(w_o=0x1004)) == 2
    assert call(n_nodes=(ctypes.c_int32 * 1)(27)) == 2
    assert call(kv_len=(ctypes.c_int32 * 1)(-1)) == 2
    assert call(wsb=need - 1) == 5
    assert call(ws=None) == 5


def test_topk_argument_checks_need_no_gpu(lib):
    f = lib.fspad_draft_topk
    fake = ctypes.c_void_p(0x1000)   # never dereferenced: every case below fails validation first
    i32, i64, sz = ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    need = fspad.fspad_draft_topk_workspace_bytes(10, 32000, 10)
    assert need >= 10 * 32 * (8 * 10 + 12)
    assert fspad.fspad_draft_topk_workspace_bytes(10, 32000, 17) == 0

    def call(rows=10, V=32000, k=10, logits=fake, stride=32000, tokens=fake, ws=fake, wsb=need):
        return f(i32(rows), i32(V), i32(k), logits, i64(stride), tokens, fake, ws, sz(wsb), None)

    assert call(logits=None) == 1
    assert call(tokens=None) == 1
    assert call(rows=0) == 2
    assert call(k=0) == 2
    assert call(k=17) == 2
    assert call(V=5, k=6, stride=5) == 2
    assert call(stride=100) == 2
    assert call(logits=ctypes.c_void_p(0x1002)) == 2
    assert call(wsb=need - 1) == 5
    assert call(ws=None) == 5


def test_commit_argument_checks_need_no_gpu(lib):
    f = lib.fspad_kv_commit
    f.restype = ctypes.c_int
    fake = ctypes.c_void_p(0x1000)   # never dereferenced: every case below fails validation first

    def call(d, kt=fake, cap=4096, kv=2048, path=fake):
        return f(ctypes.byref(d), kt, fake, fake, fake, ctypes.c_int32(cap), (ctypes.c_int32 * 1)(kv), path, fake,
                 None, None)

    assert call(_desc(), kt=None) == 1
    assert call(_desc(), path=None) == 1
    assert call(_desc(n_nodes_max=65)) == 2
    assert call(_desc(head_dim=96)) == 2
    assert call(_desc(io_dtype=2)) == 4
    assert call(_desc(cache_stride_token=100)) == 2
    assert call(_desc(), kv=-1) == 2
    assert call(_desc(), cap=2048 + 25) == 2        # no room for the longest possible path
    assert call(_desc(), kt=ctypes.c_void_p(0x1004)) == 2


def test_tree_build_argument_checks_need_no_gpu(lib):
    f = lib.fspad_tree_build
    f.restype = ctypes.c_int
    fake = ctypes.c_void_p(0x1000)   # never dereferenced: every case below fails validation first

    def call(B=1, M=511, N=60, keep=60, first=fake):
        return f(ctypes.c_int32(B), ctypes.c_int32(M), ctypes.c_int32(N), first, fake, fake, fake, ctypes.c_int32(keep),
                 fake, fake, fake, fake, fake, None)

    assert call(first=None) == 1
    assert call(M=1025) == 2
    assert call(N=65, keep=65) == 2
    assert call(keep=61) == 2
    assert call(keep=0) == 2
    assert call(B=0) == 2
