"""CPU oracle for tree verification -- TEST INFRASTRUCTURE, not product code.

Thin ctypes loader around ``fspad_oracle.c`` (plain C, fp64).  Only ``tests/``,
``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may import
this package; the GPU library never does and shares no code with it.

All functions take and return numpy arrays.  Floating-point inputs of the
attention oracle are converted to fp64 first (exact for fp32 and bf16 values).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fspad_oracle.c")
_LIB = os.path.join(_HERE, "libfspad_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no fast-math, OpenMP over heads only)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c11", "-fno-fast-math", "-ffp-contract=off", "-fopenmp",
               "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        for name in ("fspad_oracle_dense_mask", "fspad_oracle_tree_attn",
                     "fspad_oracle_accept_greedy", "fspad_oracle_accept_sample"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def dense_mask(parent) -> np.ndarray:
    """[N,N] uint8, M[i,t] = 1 iff t is i or an ancestor of i."""
    parent = _i32(parent)
    n = parent.shape[0]
    m = np.zeros((n, n), dtype=np.uint8)
    rc = _load().fspad_oracle_dense_mask(ctypes.c_int32(n), _ptr(parent), _ptr(m))
    if rc != 0:
        raise ValueError("ill-formed parent array")
    return m


def tree_attn(q, k_tree, v_tree, k_cache, v_cache, kv_len, n_nodes, parent,
              packed_mask=None, scale=None, nthreads: int = 1) -> np.ndarray:
    """fp64 tree attention by the plain definition.

    q [B,Nmax,Hq,D]; k_tree,v_tree [B,Nmax,Hkv,D]; k_cache,v_cache [B,Hkv,Lcap,D]
    (or None when every kv_len is 0); kv_len,n_nodes [B]; parent [B,Nmax];
    packed_mask [B,Nmax] uint64 or None (checked against the tree if given).
    Returns out [B,Nmax,Hq,D] fp64.
    """
    q = np.ascontiguousarray(q, dtype=np.float64)
    k_tree = np.ascontiguousarray(k_tree, dtype=np.float64)
    v_tree = np.ascontiguousarray(v_tree, dtype=np.float64)
    B, Nmax, Hq, D = q.shape
    Hkv = k_tree.shape[2]
    assert k_tree.shape == (B, Nmax, Hkv, D) and v_tree.shape == k_tree.shape
    if k_cache is not None:
        k_cache = np.ascontiguousarray(k_cache, dtype=np.float64)
        v_cache = np.ascontiguousarray(v_cache, dtype=np.float64)
        assert k_cache.shape[:2] == (B, Hkv) and k_cache.shape[3] == D
        assert v_cache.shape == k_cache.shape
        Lcap = k_cache.shape[2]
    else:
        Lcap = 0
    kv_len = _i32(kv_len)
    n_nodes = _i32(n_nodes)
    parent = _i32(parent)
    assert parent.shape == (B, Nmax) and kv_len.shape == (B,) and n_nodes.shape == (B,)
    if packed_mask is not None:
        packed_mask = np.ascontiguousarray(packed_mask, dtype=np.uint64)
        assert packed_mask.shape == (B, Nmax)
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    out = np.empty((B, Nmax, Hq, D), dtype=np.float64)
    rc = _load().fspad_oracle_tree_attn(
        ctypes.c_int32(B), ctypes.c_int32(Nmax), ctypes.c_int32(Hq), ctypes.c_int32(Hkv),
        ctypes.c_int32(D), ctypes.c_double(float(scale)),
        _ptr(q), _ptr(k_tree), _ptr(v_tree), _ptr(k_cache), _ptr(v_cache),
        ctypes.c_int64(Lcap), _ptr(kv_len), _ptr(n_nodes), _ptr(parent), _ptr(packed_mask),
        _ptr(out), ctypes.c_int32(nthreads))
    if rc == -2:
        raise ValueError("packed ancestor mask does not match the parent array")
    if rc != 0:
        raise ValueError(f"oracle tree_attn failed: {rc}")
    return out


def _accept_common(logits, draft_tokens, parent, n_nodes):
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    B, Nmax, V = logits.shape
    draft_tokens = _i32(draft_tokens)
    parent = _i32(parent)
    n_nodes = _i32(n_nodes)
    assert draft_tokens.shape == (B, Nmax) and parent.shape == (B, Nmax) and n_nodes.shape == (B,)
    path = np.empty((B, Nmax), dtype=np.int32)
    tokens = np.empty((B, Nmax), dtype=np.int32)
    path_len = np.empty((B,), dtype=np.int32)
    n_tokens = np.empty((B,), dtype=np.int32)
    return logits, B, Nmax, V, draft_tokens, parent, n_nodes, path, path_len, tokens, n_tokens


def accept_greedy(logits, draft_tokens, parent, n_nodes):
    """Returns (path [B,Nmax], path_len [B], tokens [B,Nmax], n_tokens [B]), int32."""
    (logits, B, Nmax, V, draft_tokens, parent, n_nodes,
     path, path_len, tokens, n_tokens) = _accept_common(logits, draft_tokens, parent, n_nodes)
    rc = _load().fspad_oracle_accept_greedy(
        ctypes.c_int32(B), ctypes.c_int32(Nmax), ctypes.c_int32(V), _ptr(logits),
        ctypes.c_int64(V), _ptr(draft_tokens), _ptr(parent), _ptr(n_nodes),
        _ptr(path), _ptr(path_len), _ptr(tokens), _ptr(n_tokens))
    if rc != 0:
        raise ValueError(f"oracle accept_greedy failed: {rc}")
    return path, path_len, tokens, n_tokens


def accept_sample(logits, draft_tokens, parent, n_nodes, temperature, uniforms):
    """Returns (path, path_len, tokens, n_tokens, min_margin [B] fp64)."""
    (logits, B, Nmax, V, draft_tokens, parent, n_nodes,
     path, path_len, tokens, n_tokens) = _accept_common(logits, draft_tokens, parent, n_nodes)
    uniforms = np.ascontiguousarray(uniforms, dtype=np.float32)
    assert uniforms.shape == (B, 2, Nmax)
    margin = np.empty((B,), dtype=np.float64)
    rc = _load().fspad_oracle_accept_sample(
        ctypes.c_int32(B), ctypes.c_int32(Nmax), ctypes.c_int32(V), _ptr(logits),
        ctypes.c_int64(V), _ptr(draft_tokens), _ptr(parent), _ptr(n_nodes),
        ctypes.c_float(float(temperature)), _ptr(uniforms),
        _ptr(path), _ptr(path_len), _ptr(tokens), _ptr(n_tokens), _ptr(margin))
    if rc != 0:
        raise ValueError(f"oracle accept_sample failed: {rc}")
    return path, path_len, tokens, n_tokens, margin


def kv_commit(k_tree, v_tree, k_cache, v_cache, kv_len, path, path_len):
    """Cache update after acceptance (Preliminaries: the validated tokens extend the prefix of
    the next cycle; the paper does not spell the update out). Position kv_len[b]+j of every kv
    head's cache row receives the key/value of tree node path[b,j], for j < path_len[b].

    k_tree,v_tree [B,Nmax,Hkv,D]; k_cache,v_cache [B,Hkv,Lcap,D] (any numpy dtype; values are
    moved, not converted). Returns (k_cache', v_cache', kv_len') as new arrays."""
    k_new, v_new = np.array(k_cache, copy=True), np.array(v_cache, copy=True)
    kv_len = _i32(kv_len)
    new_len = kv_len.copy()
    B, Nmax, Hkv, _ = k_tree.shape
    for b in range(B):
        for j in range(int(path_len[b])):
            node = int(path[b, j])
            for g in range(Hkv):
                k_new[b, g, kv_len[b] + j, :] = k_tree[b, node, g, :]
                v_new[b, g, kv_len[b] + j, :] = v_tree[b, node, g, :]
        new_len[b] = kv_len[b] + int(path_len[b])
    return k_new, v_new, new_len


def tree_build(cand_parent, cand_token, cand_logp, n_cand, n_keep, n_max):
    """Dynamic draft tree from its candidates (Preliminaries, last paragraph: each draft step's
    output is cut to its top-k, joint probabilities follow from the dependencies, and one more
    top-k over all tokens bounds the tree): joint[c] = joint[parent] + logp[c] accumulated in
    float32 down every path (joint[root] = 0); the n_keep-1 non-root candidates with the highest
    joint score are kept (ties: lower candidate index), a kept candidate whose parent is not
    kept is dropped with its descendants; kept candidates become the nodes in candidate order.

    Returns (parent [B,n_max], tokens [B,n_max], n_nodes [B], anc_mask [B,n_max] uint64,
    node_cand [B,n_max]); unused slots hold -1 (mask 0). NaN scores count as -infinity."""
    cand_parent, cand_token, n_cand = _i32(cand_parent), _i32(cand_token), _i32(n_cand)
    cand_logp = np.ascontiguousarray(cand_logp, dtype=np.float32)
    B = cand_parent.shape[0]
    parent = np.full((B, n_max), -1, np.int32)
    tokens = np.full((B, n_max), -1, np.int32)
    node_cand = np.full((B, n_max), -1, np.int32)
    mask = np.zeros((B, n_max), np.uint64)
    n_nodes = np.zeros(B, np.int32)
    for b in range(B):
        m = int(n_cand[b])
        joint = np.zeros(m, np.float32)
        for c in range(1, m):
            lp = cand_logp[b, c]
            lp = np.float32(-np.inf) if np.isnan(lp) else lp
            joint[c] = np.float32(joint[cand_parent[b, c]] + lp)      # one float32 addition per edge
        order = sorted(range(1, m), key=lambda c: (-float(joint[c]), c))
        kept = np.zeros(m, bool)
        kept[0] = True
        kept[order[: max(0, n_keep - 1)]] = True
        for c in range(1, m):                                          # parents come first
            kept[c] = kept[c] and kept[cand_parent[b, c]]
        new_id = {}
        for c in range(m):
            if not kept[c]:
                continue
            i = len(new_id)
            new_id[c] = i
            node_cand[b, i] = c
            tokens[b, i] = cand_token[b, c]
            if c == 0:
                mask[b, i] = np.uint64(1)
            else:
                parent[b, i] = new_id[int(cand_parent[b, c])]
                mask[b, i] = mask[b, parent[b, i]] | (np.uint64(1) << np.uint64(i))
        n_nodes[b] = len(new_id)
    return parent, tokens, n_nodes, mask, node_cand


def lm_head_greedy(hidden, lm_head, draft_tokens, parent, n_nodes):
    """Greedy validation straight from the target's last hidden states (Methodology, "LM Head":
    the final linear map from features to the vocabulary; Preliminaries, validation phase: the
    tree is compared strictly with the target's own choices and a differing token is dropped
    with its descendants; Experiments "Settings": temperature 0).

        logits[b,i,v] = sum_k hidden[b,i,k] * lm_head[v,k]        (fp64; the inputs are bf16 values)
        target[b,i]   = the v with the largest logit, lowest v among equals
        walk: cur = root; while some child c of cur (lowest index first) carries
              draft_tokens[c] == target[cur]: emit target[cur], cur = c;  finally emit target[cur].

    hidden [B,Nmax,Hd], lm_head [V,Hd] (any float dtype holding the values), draft_tokens/parent
    [B,Nmax], n_nodes [B].  Returns (path [B,Nmax], path_len [B], tokens [B,Nmax], n_tokens [B],
    target [B,Nmax] i32, top [B,Nmax] f64, margin [B,Nmax] f64): unused slots hold -1 (target -1,
    top/margin nan); margin = top logit minus the runner-up (inf when V == 1) -- what a test
    needs to tell a decided argmax from one that fp32 accumulation order may flip."""
    hidden = np.asarray(hidden, dtype=np.float64)
    lm_head = np.asarray(lm_head, dtype=np.float64)
    draft_tokens, parent, n_nodes = _i32(draft_tokens), _i32(parent), _i32(n_nodes)
    B, Nmax, Hd = hidden.shape
    V = lm_head.shape[0]
    assert lm_head.shape == (V, Hd) and draft_tokens.shape == (B, Nmax) and parent.shape == (B, Nmax)
    path = np.full((B, Nmax), -1, np.int32)
    tokens = np.full((B, Nmax), -1, np.int32)
    path_len = np.zeros(B, np.int32)
    n_tokens = np.zeros(B, np.int32)
    target = np.full((B, Nmax), -1, np.int32)
    top = np.full((B, Nmax), np.nan)
    margin = np.full((B, Nmax), np.nan)
    for b in range(B):
        n = int(n_nodes[b])
        logits = hidden[b, :n] @ lm_head.T                         # [n, V] fp64
        for i in range(n):
            row = logits[i]
            t = int(np.argmax(row))                                # first index of the maximum
            target[b, i] = t
            top[b, i] = row[t]
            margin[b, i] = row[t] - np.max(np.delete(row, t)) if V > 1 else np.inf
        cur, length = 0, 1
        path[b, 0] = 0
        while True:
            t = int(target[b, cur])
            tokens[b, length - 1] = t
            nxt = next((c for c in range(cur + 1, n) if parent[b, c] == cur and draft_tokens[b, c] == t), None)
            if nxt is None:
                break
            path[b, length] = nxt
            cur = nxt
            length += 1
        path_len[b] = length
        n_tokens[b] = length
    return path, path_len, tokens, n_tokens, target, top, margin


def draft_topk(logits, k):
    """Top-k cut of one draft step's output (Preliminaries, last paragraph: the output of every
    draft step is cut to its k most probable tokens, whose probabilities then feed the joint
    scores of the tree). Per row: the k entries with the largest logit, best first (equal logits:
    lower token first; NaN counts as -infinity), and their log-probabilities under the row's softmax,

        logp[v] = l[v] - log(sum_u exp(l[u]))        (fp64, rounded to float32 at the end).

    logits [R,V] float32 (finite, -inf or NaN), 1 <= k <= V.  Returns (tokens [R,k] int32,
    logp [R,k] float32).  A row without any finite entry yields tokens 0..k-1 and logp -inf."""
    x = np.array(logits, dtype=np.float64, copy=True)
    R, V = x.shape
    assert 1 <= k <= V
    x[np.isnan(x)] = -np.inf
    tokens = np.zeros((R, k), np.int32)
    logp = np.full((R, k), -np.inf, np.float32)
    for r in range(R):
        row = x[r]
        order = sorted(range(V), key=lambda v: (-row[v], v))[:k]
        tokens[r] = order
        m = row.max()
        if np.isfinite(m):
            lse = m + np.log(np.sum(np.exp(row - m)))
            logp[r] = (row[order] - lse).astype(np.float32)
    return tokens, logp


def lm_head_logits(hidden, lm_head):
    """logits[b,i,v] = sum_k hidden[b,i,k] * lm_head[v,k] in fp64 (Methodology, "LM Head"),
    rounded once to float32: the values a correctly rounded fp32 LM head would hand to the
    acceptance.  hidden [B,Nmax,Hd], lm_head [V,Hd]."""
    hidden = np.asarray(hidden, dtype=np.float64)
    lm_head = np.asarray(lm_head, dtype=np.float64)
    B, Nmax, Hd = hidden.shape
    return (hidden.reshape(B * Nmax, Hd) @ lm_head.T).reshape(B, Nmax, -1).astype(np.float32)


def lm_head_sample(hidden, lm_head, draft_tokens, parent, n_nodes, temperature, uniforms):
    """Tree rejection sampling straight from the target's last hidden states: the acceptance of
    `accept_sample` (Preliminaries, validation phase; Experiments "Settings": temperature 1,
    acceptance not relaxed) applied to `lm_head_logits`.  Returns what accept_sample returns,
    the smallest relative decision margin per sequence included."""
    return accept_sample(lm_head_logits(hidden, lm_head), draft_tokens, parent, n_nodes, temperature, uniforms)


def feature_sampler(f, e, w_up, w_gate, w_down, residual=True):
    """Feature Sampler of the draft model (Methodology, "Feature Sampling": three projectors and a
    sampling operation in the intermediate space): the Up Projector lifts the feature f, the Gate
    Projector lifts the token embedding e, the lifted embedding is activated with SiLU and
    multiplied element by element with the lifted feature, and the Down Projector maps the product
    back to the hidden size, where the feature path's residual connection is added:

        eta = W_down (SiLU(W_gate e) * (W_up f)) [+ f]           (fp64 throughout)

    f, e [rows,Hd]; w_up, w_gate [I,Hd]; w_down [Hd,I].  Returns eta [rows,Hd] float64."""
    f = np.asarray(f, dtype=np.float64)
    e = np.asarray(e, dtype=np.float64)
    up = f @ np.asarray(w_up, dtype=np.float64).T
    gate = e @ np.asarray(w_gate, dtype=np.float64).T
    sampled = gate / (1.0 + np.exp(-gate)) * up
    eta = sampled @ np.asarray(w_down, dtype=np.float64).T
    return eta + f if residual else eta


def rms_norm(x, gain, eps):
    """x / sqrt(mean(x^2) + eps) * gain over the last axis, fp64."""
    x = np.asarray(x, dtype=np.float64)
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * np.asarray(gain, dtype=np.float64)


def rope(u, positions, theta):
    """Rotary position encoding of head vectors u [..., D] at integer positions [...]: entry i of
    the first half and entry i of the second half form the pair that is rotated by the angle
    position * theta^(-2i/D)."""
    u = np.asarray(u, dtype=np.float64)
    D = u.shape[-1]
    half = D // 2
    inv_freq = float(theta) ** (-2.0 * np.arange(half, dtype=np.float64) / D)
    ang = np.asarray(positions, dtype=np.float64)[..., None] * inv_freq
    c, s = np.cos(ang), np.sin(ang)
    a, b = u[..., :half], u[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def draft_layer(eta, positions, w_qkv, w_o, w_gate, w_up, w_down, gain_attn, gain_mlp, k_cache, v_cache,
                kv_len, n_nodes, parent, n_q_heads, n_kv_heads, head_dim, rms_eps=1e-6, rope_theta=10000.0):
    """The draft model: one transformer decoder layer over the draft's token tree (Methodology,
    first paragraph: the draft model is a Transformer Decoder Layer; "Partial Alignment
    Distillation": the MLP's output dimension is doubled and both halves share one residual
    connection, giving the two features f~ and f), fp64 throughout:

        x   = eta                                             [B,Nmax,Hd]
        q,k,v = split(W_qkv rmsnorm(x)), rotary encoding of q and k at `positions`
        h   = x + W_o tree_attn(q, k, v | the draft's own cache, the tree mask)
        m   = W_down (SiLU(W_gate rmsnorm(h)) * (W_up rmsnorm(h)))        [B,Nmax,2 Hd]
        f~  = h + m[..., :Hd]        f = h + m[..., Hd:]

    The layer is LLaMA's (pre-normalisation with RMSNorm, rotary encoding, grouped-query
    attention, gated MLP, no biases).  w_qkv [(Hq+2Hkv) D, Hd] holds the query, key and value
    projections stacked in that order; w_o [Hd, Hq D]; w_gate, w_up [I, Hd]; w_down [2 Hd, I].
    positions [B,Nmax] int; the cache and tree arguments are those of `tree_attn`.
    Returns (f_tilde, f, k_tree, v_tree): [B,Nmax,Hd] twice, [B,Nmax,Hkv,D] twice, float64;
    rows of unused tree slots are zero."""
    x = np.asarray(eta, dtype=np.float64)
    B, Nmax, Hd = x.shape
    Hq, Hkv, D = n_q_heads, n_kv_heads, head_dim
    n_nodes = _i32(n_nodes)
    qkv = rms_norm(x, gain_attn, rms_eps) @ np.asarray(w_qkv, dtype=np.float64).T
    q = rope(qkv[..., :Hq * D].reshape(B, Nmax, Hq, D), np.asarray(positions)[..., None], rope_theta)
    k = rope(qkv[..., Hq * D:(Hq + Hkv) * D].reshape(B, Nmax, Hkv, D), np.asarray(positions)[..., None], rope_theta)
    v = qkv[..., (Hq + Hkv) * D:].reshape(B, Nmax, Hkv, D)
    a = tree_attn(q, k, v, k_cache, v_cache, kv_len, n_nodes, parent)
    h = x + a.reshape(B, Nmax, Hq * D) @ np.asarray(w_o, dtype=np.float64).T
    hn = rms_norm(h, gain_mlp, rms_eps)
    gate = hn @ np.asarray(w_gate, dtype=np.float64).T
    m = (gate / (1.0 + np.exp(-gate)) * (hn @ np.asarray(w_up, dtype=np.float64).T)) @ np.asarray(w_down, dtype=np.float64).T
    f_tilde, f = h + m[..., :Hd], h + m[..., Hd:]
    used = (np.arange(Nmax)[None, :] < n_nodes[:, None])
    for arr in (f_tilde, f):
        arr[~used] = 0.0
    k = np.where(used[..., None, None], k, 0.0)
    v = np.where(used[..., None, None], v, 0.0)
    return f_tilde, f, k, v


def pack_weight(w):
    """Tile order of a row-major [N,K] matrix (a storage format of the library's draft-side weights,
    not a step of the paper): tiles of 16 rows x 32 columns, tile rows one after another, within a
    tile row along k; inside a tile, slot n + 16 g holds w[16 t + n, 32 s + 8 g : 32 s + 8 g + 8].
    Rows past N in the last tile row are zeros.  Returns a flat array of ceil(N/16)*16*K entries."""
    w = np.asarray(w)
    N, K = w.shape
    assert K % 32 == 0
    T, S = (N + 15) // 16, K // 32
    padded = np.zeros((T * 16, K), dtype=w.dtype)
    padded[:N] = w
    tiles = padded.reshape(T, 16, S, 4, 8)               # [t, n, s, g, j]
    out = tiles.transpose(0, 2, 3, 1, 4)                 # [t, s, g, n, j]: slot n + 16 g
    return out.reshape(-1)


def accept_sample_draft(logits, draft_logits, draft_tokens, parent, n_nodes, temperature, uniforms):
    """Tree acceptance for drafts that were SAMPLED from a draft distribution q (Introduction: the
    draft-then-verify scheme of speculative sampling, which the method's lossless property rests
    on), in its multi-candidate form: at a node with target distribution p = softmax(l / T) and
    draft distribution q = softmax(l_draft / T), the children (drawn from q one after another,
    without replacement, in sibling order) are tested in that order:

        accept x    <=>  u * q(x) < p(x)                (probability min(1, p(x) / q(x)))
        reject x    :    p <- max(p - q, 0) / sum(max(p - q, 0));   q(x) <- 0, q <- q / sum(q)

    and when no child is accepted the step's last token is drawn from what p has become (inverse
    CDF with the node's second uniform, vocabulary order).  The token emitted at every position
    then follows the target's p exactly.  With q a point mass on each draft token this is
    `accept_sample`.  NaN logits carry no mass; tokens outside [0, V) are never accepted.

    logits, draft_logits [B,Nmax,V]; uniforms [B,2,Nmax] as for accept_sample.  fp64 throughout.
    Returns (path, path_len, tokens, n_tokens, min_margin): the margin is the smallest distance of
    any decision from its threshold (|u q(x) - p(x)| for a test; for the draw, the distance of the
    target from the two running sums that bracket it, relative to the total)."""
    logits = np.asarray(logits)
    draft_logits = np.asarray(draft_logits)
    B, Nmax, V = logits.shape
    assert draft_logits.shape == logits.shape
    if not (temperature > 0.0) or np.isinf(temperature):
        raise ValueError("temperature must be positive and finite")
    draft_tokens, parent, n_nodes = _i32(draft_tokens), _i32(parent), _i32(n_nodes)
    uniforms = np.asarray(uniforms, dtype=np.float64)
    assert uniforms.shape == (B, 2, Nmax)
    path = np.full((B, Nmax), -1, dtype=np.int32)
    tokens = np.full((B, Nmax), -1, dtype=np.int32)
    path_len = np.zeros(B, dtype=np.int32)
    margin = np.full(B, np.inf)

    def softmax(row):
        row = np.asarray(row, dtype=np.float64)
        ok = ~np.isnan(row)
        w = np.zeros(V)
        if ok.any():
            w[ok] = np.exp((row[ok] - row[ok].max()) / float(temperature))
        s = w.sum()
        return w / s if s > 0 else w

    for b in range(B):
        n = int(n_nodes[b])
        cur, length = 0, 1
        path[b, 0] = 0
        while True:
            p, q = softmax(logits[b, cur]), softmax(draft_logits[b, cur])
            nxt = -1
            for c in range(cur + 1, n):
                if parent[b, c] != cur:
                    continue
                x = int(draft_tokens[b, c])
                px, qx = (p[x], q[x]) if 0 <= x < V else (0.0, 0.0)
                lhs = uniforms[b, 0, c] * qx
                margin[b] = min(margin[b], abs(lhs - px))
                if lhs < px:
                    nxt = c
                    break
                r = np.maximum(p - q, 0.0)
                z = r.sum()
                if z > 0:
                    p = r / z
                if 0 <= x < V:
                    q[x] = 0.0
                s = q.sum()
                if s > 0:
                    q = q / s
            if nxt >= 0:
                tokens[b, length - 1] = draft_tokens[b, nxt]
                path[b, length] = nxt
                length += 1
                cur = nxt
                continue
            run = np.cumsum(p)
            total = run[-1] if V else 0.0
            t = uniforms[b, 1, cur] * total
            hit = np.nonzero(run > t)[0]
            if hit.size:
                v = int(hit[0])
                before = run[v - 1] if v > 0 else 0.0
                margin[b] = min(margin[b], (t - before) / total, (run[v] - t) / total)
            else:
                mass = np.nonzero(p > 0)[0]
                v = int(mass[-1]) if mass.size else 0
                margin[b] = 0.0
            tokens[b, length - 1] = v
            break
        path_len[b] = length
    return path, path_len, tokens, path_len.copy(), margin
