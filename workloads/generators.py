"""Seeded input generators (numpy, CPU).  Inputs only -- no method arithmetic."""
from __future__ import annotations

import numpy as np

GENERATOR_VERSION = 1


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even) and return them as fp32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    rounded = (bits >> np.uint32(16)) & np.uint32(1)      # 32-bit arithmetic: no finite value wraps around
    rounded += np.uint32(0x7FFF)
    rounded += bits
    rounded &= np.uint32(0xFFFF0000)
    return rounded.view(np.float32).reshape(x.shape)


def chain_tree(n: int) -> np.ndarray:
    """parent[i] = i-1: the tree of ordinary sequential decoding."""
    return np.arange(-1, n - 1, dtype=np.int32)


def gen_tree(rng: np.random.Generator, n_nodes: int, depth: int, topk: int) -> np.ndarray:
    """Parent array of a dynamic draft tree shaped the way EAGLE-2 builds one.

    Every expanded node proposes `topk` children whose conditional probabilities
    fall off geometrically (ratio rho ~ U(0.2, 0.7) per node); a candidate's joint
    probability is the product along its path.  At each level only the `topk`
    candidates with the highest joint probability are expanded further; after
    `depth` levels the n_nodes-1 candidates with the highest joint probability are
    kept (the set is ancestor-closed since a child's joint probability is below its
    parent's).  Nodes are renumbered breadth first, siblings by falling
    conditional probability, so parent[i] < i and node 0 is the root.
    """
    if n_nodes == 1:
        return np.array([-1], dtype=np.int32)
    # candidate records: (joint, level, parent_candidate_id, rank)
    joint = [1.0]
    level = [0]
    par = [-1]
    rank = [0]
    frontier = [0]
    for lev in range(1, depth + 1):
        new = []
        for p in frontier:
            rho = rng.uniform(0.2, 0.7)
            c = rho ** np.arange(topk)
            c = c / c.sum()
            for j in range(topk):
                joint.append(joint[p] * c[j])
                level.append(lev)
                par.append(p)
                rank.append(j)
                new.append(len(joint) - 1)
        new.sort(key=lambda i: (-joint[i], i))
        frontier = new[:topk]
    cand = list(range(1, len(joint)))
    cand.sort(key=lambda i: (-joint[i], i))
    if len(cand) < n_nodes - 1:
        raise ValueError("tree budget exceeds the number of candidates")
    keep = set(cand[: n_nodes - 1])
    keep.add(0)
    # a kept node's parent has a strictly larger joint probability, so it is kept as well
    assert all(par[i] in keep for i in keep if i != 0)
    # breadth-first renumbering
    children = {i: [] for i in keep}
    for i in keep:
        if i != 0:
            children[par[i]].append(i)
    order = [0]
    head = 0
    while head < len(order):
        node = order[head]
        head += 1
        order.extend(sorted(children[node], key=lambda i: rank[i]))
    new_id = {old: new for new, old in enumerate(order)}
    parent = np.full(n_nodes, -1, dtype=np.int32)
    for old in order[1:]:
        parent[new_id[old]] = new_id[par[old]]
    return parent


def gen_trees(seed: int, batch: int, n_max: int, depth: int, topk: int, n_nodes=None):
    """parent [B,Nmax] (unused slots -1) and n_nodes [B]; a different tree per sequence."""
    rng = np.random.default_rng([seed, 0x7EE])
    if n_nodes is None:
        n_nodes = [n_max] * batch
    parent = np.full((batch, n_max), -1, dtype=np.int32)
    for b in range(batch):
        parent[b, : n_nodes[b]] = gen_tree(rng, int(n_nodes[b]), depth, topk)
    return parent, np.asarray(n_nodes, dtype=np.int32)


def gen_qkv(seed: int, batch: int, n_max: int, n_q_heads: int, n_kv_heads: int, head_dim: int,
            l_cap: int, dtype: str = "bf16"):
    """q [B,N,Hq,D], k_tree/v_tree [B,N,Hkv,D], k_cache/v_cache [B,Hkv,Lcap,D], all N(0,1),
    returned as fp32 arrays holding values exactly representable in `dtype`."""
    rng = np.random.default_rng([seed, 0xA77])
    shapes = [(batch, n_max, n_q_heads, head_dim), (batch, n_max, n_kv_heads, head_dim),
              (batch, n_max, n_kv_heads, head_dim), (batch, n_kv_heads, l_cap, head_dim),
              (batch, n_kv_heads, l_cap, head_dim)]
    out = []
    for shp in shapes:
        x = rng.standard_normal(shp, dtype=np.float32)
        out.append(round_to_bf16(x) if dtype == "bf16" else x)
    return tuple(out)


def gen_logits(seed: int, batch: int, n_max: int, vocab: int, sigma: float = 3.0,
               peak: float = 0.0) -> np.ndarray:
    """fp32 logits [B,N,V] ~ N(0, sigma^2).  peak > 0 lifts one random entry of every row
    to (row max + peak) so that a single token carries most of the mass (deep accepted
    paths and multi-rejection residuals for the tests)."""
    rng = np.random.default_rng([seed, 0x106])
    x = rng.standard_normal((batch, n_max, vocab), dtype=np.float32) * np.float32(sigma)
    if peak > 0.0:
        idx = rng.integers(0, vocab, size=(batch, n_max))
        mx = x.max(axis=-1)
        b, i = np.meshgrid(np.arange(batch), np.arange(n_max), indexing="ij")
        x[b, i, idx] = mx + np.float32(peak)
    return x


def gen_draft_tokens(seed: int, logits: np.ndarray, parent: np.ndarray, n_nodes: np.ndarray,
                     mode: str = "greedy", noise: float = 1.0) -> np.ndarray:
    """Draft tokens [B,N] i32 from a perturbed copy of the target.

    The children of node p get distinct tokens, in sibling order: mode "greedy" --
    the top-m entries of logits[p] + N(0, noise^2); mode "sample" -- m draws
    without replacement from the categorical distribution with those perturbed
    logits (Gumbel top-m).  The root's own token is arbitrary."""
    rng = np.random.default_rng([seed, 0xD4A])
    batch, n_max, vocab = logits.shape
    tok = np.zeros((batch, n_max), dtype=np.int32)
    for b in range(batch):
        n = int(n_nodes[b])
        tok[b, 0] = rng.integers(0, vocab)
        for p in range(n):
            kids = [c for c in range(p + 1, n) if parent[b, c] == p]
            if not kids:
                continue
            key = logits[b, p].astype(np.float64) + noise * rng.standard_normal(vocab)
            if mode == "sample":
                key = key + rng.gumbel(size=vocab)
            elif mode != "greedy":
                raise ValueError(mode)
            m = len(kids)
            top = np.argpartition(-key, m - 1)[:m] if m < vocab else np.arange(vocab)
            top = top[np.argsort(-key[top], kind="stable")]
            tok[b, kids] = top[:m].astype(np.int32)
    return tok


def gen_uniforms(seed: int, batch: int, n_max: int) -> np.ndarray:
    """fp32 U[0,1) [B,2,N]: [:,0,:] acceptance tests, [:,1,:] bonus draws."""
    rng = np.random.default_rng([seed, 0x0F1])
    return rng.random((batch, 2, n_max), dtype=np.float32)


def gen_candidates(seed: int, batch: int, depth: int, topk: int, vocab: int, m_max: int = 0,
                   ties: bool = False):
    """Draft-tree candidates before selection, shaped like the output of `depth` draft steps that each
    keep `topk` continuations of `topk` expanded nodes: candidate 0 is the root; level 1 holds topk
    children of the root; every later level holds topk children of each of topk nodes of the level
    before (which ones are expanded is drawn at random here: no selection rule lives in this module).
    Returns cand_parent [B,M] int32 (-1 for the root, always < own index), cand_token [B,M] int32
    (distinct among siblings), cand_logp [B,M] float32 (conditional log-probabilities, <= 0; with
    `ties` drawn from a few values so that equal joint scores occur) and n_cand [B]."""
    rng = np.random.default_rng([seed, 0xCA9D])
    m = 1 + topk + (depth - 1) * topk * topk
    m_max = max(m_max, m)
    par = np.full((batch, m_max), -1, dtype=np.int32)
    tok = np.full((batch, m_max), -1, dtype=np.int32)
    logp = np.zeros((batch, m_max), dtype=np.float32)
    n_cand = np.zeros(batch, dtype=np.int32)
    for b in range(batch):
        d_b = int(rng.integers(1, depth + 1)) if b % 3 == 2 else depth   # some sequences stop early
        tok[b, 0] = rng.integers(0, vocab)
        count, frontier = 1, [0]
        for lev in range(1, d_b + 1):
            new = []
            for p in frontier:
                if ties:
                    c = np.log(rng.choice([0.5, 0.25, 0.125], size=topk)).astype(np.float32)
                else:
                    rho = rng.uniform(0.2, 0.7)
                    c = rho ** np.arange(topk)
                    c = np.log(c / c.sum() * rng.uniform(0.6, 1.0)).astype(np.float32)
                toks = rng.choice(vocab, size=topk, replace=False)
                for j in range(topk):
                    par[b, count], tok[b, count], logp[b, count] = p, toks[j], c[j]
                    new.append(count)
                    count += 1
            frontier = sorted(rng.choice(new, size=min(topk, len(new)), replace=False).tolist())
        n_cand[b] = count
    return par, tok, logp, n_cand


def gen_lm_head(seed: int, batch: int, n_max: int, hidden_dim: int, vocab: int, sigma: float = 3.0):
    """Last hidden states [B,N,Hd] ~ N(0,1) and LM-head weights [V,Hd] ~ N(0, sigma^2/Hd), both
    rounded to bf16 and returned as fp32: the logits they produce are ~ N(0, sigma^2), like the
    ones gen_logits draws."""
    rng = np.random.default_rng([seed, 0x1A4D])
    hidden = round_to_bf16(rng.standard_normal((batch, n_max, hidden_dim), dtype=np.float32))
    w = rng.standard_normal((vocab, hidden_dim), dtype=np.float32)
    w *= np.float32(sigma / np.sqrt(hidden_dim))
    return hidden, round_to_bf16(w)


def gen_lm_head_exact(seed: int, batch: int, n_max: int, hidden_dim: int, vocab: int):
    """Hidden states with entries in {-2..2} and LM-head weights with entries in {-1/8, 0, 1/8}: every
    product and every partial sum of a logit is a multiple of 1/8 below 2^8, so the logits are exact in
    fp32 whatever the order of summation (spread about 2.8 at hidden_dim 256)."""
    rng = np.random.default_rng([seed, 0xE8AC])
    hidden = rng.integers(-2, 3, (batch, n_max, hidden_dim)).astype(np.float32)
    w = rng.integers(-1, 2, (vocab, hidden_dim)).astype(np.float32) * np.float32(0.125)
    return hidden, w


def gen_feature_sampler(seed: int, rows: int, hidden_dim: int, intermediate_dim: int):
    """Inputs and projector weights of a Feature Sampler, all rounded to bf16 and returned as fp32:
    f, e [rows,Hd] ~ N(0,1); w_up, w_gate [I,Hd] ~ N(0, 1/Hd); w_down [Hd,I] ~ N(0, 1/I) -- the scales
    a trained layer keeps, so that every stage has O(1) entries."""
    rng = np.random.default_rng([seed, 0xF5A])
    f = round_to_bf16(rng.standard_normal((rows, hidden_dim), dtype=np.float32))
    e = round_to_bf16(rng.standard_normal((rows, hidden_dim), dtype=np.float32))
    w_up = round_to_bf16(rng.standard_normal((intermediate_dim, hidden_dim), dtype=np.float32) / np.float32(np.sqrt(hidden_dim)))
    w_gate = round_to_bf16(rng.standard_normal((intermediate_dim, hidden_dim), dtype=np.float32) / np.float32(np.sqrt(hidden_dim)))
    w_down = round_to_bf16(rng.standard_normal((hidden_dim, intermediate_dim), dtype=np.float32) / np.float32(np.sqrt(intermediate_dim)))
    return f, e, w_up, w_gate, w_down


def tree_depths(parent: np.ndarray, n_nodes: np.ndarray) -> np.ndarray:
    """depth [B,Nmax] of every node below its root (root 0; unused slots 0)."""
    depth = np.zeros(parent.shape, dtype=np.int32)
    for b in range(parent.shape[0]):
        for i in range(1, int(n_nodes[b])):
            depth[b, i] = depth[b, parent[b, i]] + 1
    return depth


def gen_draft_layer(seed: int, batch: int, n_max: int, hidden_dim: int, intermediate_dim: int,
                    n_q_heads: int, n_kv_heads: int, head_dim: int, l_cap: int):
    """Inputs, weights and cache of one draft decoder layer, all rounded to bf16 and returned as
    fp32 in a dict: eta [B,N,Hd] ~ N(0,1); projection weights ~ N(0, 1/fan_in) (w_qkv
    [(Hq+2Hkv)D,Hd], w_o [Hd,HqD], w_gate / w_up [I,Hd], w_down [2Hd,I]) so that every stage keeps
    O(1) entries; normalisation gains ~ 1 + 0.1 N(0,1); the draft's own cache k_cache / v_cache
    [B,Hkv,Lcap,D] ~ N(0,1)."""
    rng = np.random.default_rng([seed, 0xD1A7])

    def normal(shape, scale=1.0):
        return round_to_bf16(rng.standard_normal(shape, dtype=np.float32) * np.float32(scale))

    qkv_rows = (n_q_heads + 2 * n_kv_heads) * head_dim
    return {
        "eta": normal((batch, n_max, hidden_dim)),
        "w_qkv": normal((qkv_rows, hidden_dim), 1.0 / np.sqrt(hidden_dim)),
        "w_o": normal((hidden_dim, n_q_heads * head_dim), 1.0 / np.sqrt(n_q_heads * head_dim)),
        "w_gate": normal((intermediate_dim, hidden_dim), 1.0 / np.sqrt(hidden_dim)),
        "w_up": normal((intermediate_dim, hidden_dim), 1.0 / np.sqrt(hidden_dim)),
        "w_down": normal((2 * hidden_dim, intermediate_dim), 1.0 / np.sqrt(intermediate_dim)),
        "gain_attn": round_to_bf16(1.0 + 0.1 * rng.standard_normal(hidden_dim, dtype=np.float32)),
        "gain_mlp": round_to_bf16(1.0 + 0.1 * rng.standard_normal(hidden_dim, dtype=np.float32)),
        "k_cache": normal((batch, n_kv_heads, l_cap, head_dim)),
        "v_cache": normal((batch, n_kv_heads, l_cap, head_dim)),
    }


def gen_sampled_drafts(seed: int, logits: np.ndarray, parent: np.ndarray, n_nodes: np.ndarray,
                       temperature: float = 1.0, noise: float = 1.0):
    """A draft distribution per node and children drawn from it: draft_logits [B,N,V] fp32 =
    logits + N(0, noise^2) (a drafter that is close to the target), and tokens [B,N] i32 whose
    sibling groups are draws WITHOUT replacement, in sibling order, from softmax(draft_logits / T)
    of their parent (Gumbel top-m).  The root's own token is arbitrary."""
    rng = np.random.default_rng([seed, 0x5D4A])
    batch, n_max, vocab = logits.shape
    draft_logits = (logits + noise * rng.standard_normal(logits.shape)).astype(np.float32)
    tok = np.zeros((batch, n_max), dtype=np.int32)
    for b in range(batch):
        n = int(n_nodes[b])
        tok[b, 0] = rng.integers(0, vocab)
        for p in range(n):
            kids = [c for c in range(p + 1, n) if parent[b, c] == p]
            if not kids:
                continue
            key = draft_logits[b, p].astype(np.float64) / float(temperature) + rng.gumbel(size=vocab)
            m = min(len(kids), vocab)
            top = np.argsort(-key, kind="stable")[:m]
            tok[b, kids[:m]] = top.astype(np.int32)
            for extra in kids[m:]:          # more siblings than tokens: repeat the last (never accepted twice)
                tok[b, extra] = top[-1]
    return draft_logits, tok
