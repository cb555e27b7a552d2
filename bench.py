#!/usr/bin/env python3
"""Benchmark of the tree-verification hot path on one MI355X.

One *step* = tree-masked attention for every layer of the workload (one
fspad_tree_attn call per layer, each over its own KV buffers) followed by one
acceptance call over the per-node logits.  Inputs are synthetic, seeded, resident
in HBM before the timed region; single-layer workloads rotate through enough
independent buffer sets that they stream from HBM rather than the last-level cache.

Prints ONE JSON line.  Its top level is the headline workload (default c3, the Vicuna-33B-shaped
stack): metric / value / unit (steps per second), ms_per_step, the workload in `config`, the
event-timed attention and acceptance calls, `roofline` of the attention call, `step_roofline` of the
whole step and `cpu_baseline`.  `other_workloads` holds a short run of each of the other
configurations (same keys, fewer of them), `measured_roofs` what a plain streaming read and a
register-resident matrix-core loop reach on this machine; every roofline carries `frac` against the
published peak and `frac_vs_measured` against those.  `--only` prints the one workload alone.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0
TRAFFIC_PROFILE = os.path.join("profiles", "tree_verify_traffic.txt")


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="c3", choices=["c0", "c1", "c2", "c3", "c4"])
    ap.add_argument("--only", action="store_true",
                    help="run the one workload alone: no short runs of the other workloads, no measured roofs "
                         "(profiling runs; the extra options below imply it)")
    ap.add_argument("--accept", default=None, choices=["greedy", "sample", "sample-draft"],
                    help="override the workload's acceptance mode (sample-draft: drafts sampled from a draft distribution, "
                         "accepted against it with fspad_tree_accept_sample_draft)")
    ap.add_argument("--sets", type=int, default=None, help="independent buffer sets to rotate through")
    ap.add_argument("--splits", type=int, default=0,
                    help="fspad_attn_desc.workgroups: force the number of attention workgroups (0 = the library's choice)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--event-every", type=int, default=0,
                    help="bracket the attention calls of every n-th timed step with timing events (0 = every max(4, steps/12)-th)")
    ap.add_argument("--layers", type=int, default=None, help="profiling only: run fewer layers of a stack (the result line is then not the workload's)")
    ap.add_argument("--nodes", type=int, default=None, help="experiments only: override the tree size")
    ap.add_argument("--heads", type=int, default=None, help="experiments only: override the head count (MHA)")
    ap.add_argument("--kv-len", type=int, default=None, help="experiments only: override the prefix length")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="profiling only: before the timed region, copy a buffer of this many MiB three times with "
                         "roofs_copy_kernel (a kernel of known HBM traffic next to which rocprofv3 byte counters can be scaled)")
    ap.add_argument("--commit", action="store_true",
                    help="also append the accepted path's keys/values to every layer's cache after the acceptance "
                         "(fspad_kv_commit; the caches then carry room for one more tree)")
    ap.add_argument("--tree-build", action="store_true",
                    help="also select a tree from depth x top-k draft candidates at the top of every step "
                         "(fspad_tree_build; timing only: the step's other calls keep their pre-built tree)")
    ap.add_argument("--draft-topk", action="store_true",
                    help="also cut the outputs of the draft steps to their top-k at the top of every step: tree_depth calls "
                         "of fspad_draft_topk over B x top-k rows of V synthetic draft logits (timing only, like --tree-build)")
    ap.add_argument("--feature-sampler", default=None, choices=["fused", "library"],
                    help="also run the draft model's Feature Sampler at the top of every step: tree_depth calls over "
                         "B x top-k rows with the workload's hidden / intermediate sizes (timing only). fused = "
                         "fspad_feature_sampler; library = three library GEMMs + element-wise kernels (the comparison)")
    ap.add_argument("--draft-layer", default=None, choices=["fused", "library"],
                    help="also run the draft model's decoder layer (doubled MLP output) at the top of every step: "
                         "tree_depth calls, each over a top-k-node tree per sequence on a cache of kv_len tokens, with the "
                         "workload's head geometry and hidden / intermediate sizes (timing only; B x top-k <= 128). fused = "
                         "fspad_draft_layer; library = library GEMMs, attention and element-wise kernels (the comparison)")
    ap.add_argument("--lm-head", default=None, choices=["fused", "unfused"],
                    help="start the acceptance from the last hidden states instead of ready-made logits. "
                         "fused = fspad_tree_accept_{greedy,sample}_lm_head (logits never written); unfused = library GEMM "
                         "to bf16 logits, widened to fp32, then fspad_tree_accept_{greedy,sample} (the comparison)")
    ap.add_argument("--packed-weights", action="store_true",
                    help="with --feature-sampler fused / --draft-layer fused / --lm-head fused: the weight matrices are repacked once into "
                         "the tile order of fspad_pack_weight (same results, faster streaming)")
    ap.add_argument("--hidden-dim", type=int, default=None, help="hidden size for --lm-head (default: the workload's model)")
    ap.add_argument("--probe-overlap", action="store_true",
                    help="instead of a workload: time what one SIMD runs at the same time (a matrix instruction and vector "
                         "instructions of the same wavefront; a matrix wavefront next to a vector wavefront) and print it")
    ap.add_argument("--seed", type=int, default=2024)
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2408_15562_amd as fspad

    fspad.library_path()  # fail loudly if the HIP library is missing
    if not torch.cuda.is_available():
        raise RuntimeError("bench.py needs a GPU")
    torch.cuda.set_device(torch.device("cuda:0"))
    extras = any((args.commit, args.tree_build, args.draft_topk, args.feature_sampler, args.draft_layer, args.lm_head,
                  args.layers is not None, args.nodes is not None, args.heads is not None, args.kv_len is not None,
                  args.copy_calibration, args.accept is not None, args.splits))
    only = args.only or extras or args.workload == "c0"
    # everything runs on one side stream: the prepared calls, the timing events and the captured graph share it
    side = torch.cuda.Stream()
    if args.probe_overlap:
        with torch.cuda.stream(side):
            print(json.dumps(probe_overlap(torch, torch.cuda.current_stream().cuda_stream)))
        return
    with torch.cuda.stream(side):
        result = run_workload(args, args.workload, args.steps, args.warmup, primary=True)
        if not only:
            others = {}
            for name in ("c1", "c2", "c3", "c4"):
                if name == args.workload:
                    continue
                rec = run_workload(args, name, None, None, primary=False)
                others[name] = {k: rec[k] for k in ("value", "unit", "steps", "warmup", "ms_per_step", "config", "step_roofline",
                                                    "roofline", "accept_roofline", "attn_call_us", "accept_call_us", "steps_per_s_graph_replay",
                                                    "steps_per_s_one_buffer_set_cache_resident", "mean_tokens_per_step") if k in rec}
            result["other_workloads"] = others
            roofs = measure_roofs(torch, torch.cuda.current_stream().cuda_stream)
            result["measured_roofs"] = roofs
            for rec in [result] + list(others.values()):
                for key in ("roofline", "step_roofline"):
                    r = rec[key]
                    r["frac_vs_measured"] = r["achieved"] / (roofs["hbm_read_gb_per_s"] if r["bound"] == "hbm"
                                                            else roofs["mfma_bf16_tflops"])
    print(json.dumps(result))


def run_workload(args, workload, steps_arg, warmup_arg, primary):
    """Builds the workload's buffers, times its steps and returns its record. `primary`: the headline
    workload (honours every command-line option and carries cpu_baseline); otherwise a short plain run."""
    import numpy as np
    import torch

    import paper_2408_15562_amd as fspad
    from workloads import (CONFIGS, GENERATOR_VERSION, gen_candidates, gen_draft_tokens, gen_logits, gen_sampled_drafts, gen_trees,
                           gen_uniforms, tree_depths)

    if not primary:   # none of the command line's experiment options apply to the short runs
        args = argparse.Namespace(**{**vars(args), **dict(
            accept=None, sets=None, splits=0, layers=None, nodes=None, heads=None, kv_len=None, copy_calibration=0, commit=False,
            tree_build=False, draft_topk=False, feature_sampler=None, draft_layer=None, lm_head=None, packed_weights=False,
            hidden_dim=None, no_cpu_baseline=True, event_every=0)})
    dev = torch.device("cuda:0")
    cfg = CONFIGS[workload]
    if args.layers is not None:
        import dataclasses
        cfg = dataclasses.replace(cfg, layers=args.layers, name=cfg.name + f"-{args.layers}layers")
    if args.nodes is not None:
        import dataclasses
        cfg = dataclasses.replace(cfg, n_nodes=args.nodes, tree_topk=min(cfg.tree_topk, 4), name=cfg.name + f"-{args.nodes}nodes")
    if args.heads is not None:
        import dataclasses
        cfg = dataclasses.replace(cfg, n_q_heads=args.heads, n_kv_heads=args.heads, name=cfg.name + f"-{args.heads}heads")
    if args.kv_len is not None:
        import dataclasses
        cfg = dataclasses.replace(cfg, kv_len=args.kv_len, name=cfg.name + f"-{args.kv_len}prefix")
    default_shape = args.layers is None and args.nodes is None and args.heads is None and args.kv_len is None
    accept = args.accept or cfg.accept
    tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    B, N, Hq, Hkv, D, L, V = cfg.batch, cfg.n_nodes, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.kv_len, cfg.vocab

    # single-layer workloads are far smaller than the 256 MB last-level cache: rotate buffer sets
    set_bytes = cfg.step_bytes()
    n_sets = args.sets if args.sets is not None else (1 if set_bytes > 2e9 else max(2, int(np.ceil(1.0e9 / set_bytes))))
    steps = steps_arg if steps_arg is not None else (20 if set_bytes > 2e9 else 200)
    warmup = warmup_arg if warmup_arg is not None else (3 if set_bytes > 2e9 else 20)

    gen = torch.Generator(device=dev)
    gen.manual_seed(args.seed)
    parent, n_nodes = gen_trees(args.seed, B, N, cfg.tree_depth, cfg.tree_topk)
    mask = torch.from_numpy(fspad.fspad_tree_build_mask(parent, n_nodes).view(np.int64)).to(dev)
    kv_len = np.full(B, L, np.int32)

    sets = []
    for s in range(n_sets):
        layers = []
        for _ in range(cfg.layers):
            cap = L + N if (args.commit or args.draft_layer == "library") else L   # room behind the prefix
            kc = torch.empty((B, Hkv, cap, D), device=dev, dtype=tdt).normal_(generator=gen)
            vc = torch.empty((B, Hkv, cap, D), device=dev, dtype=tdt).normal_(generator=gen)
            q = torch.empty((B, N, Hq, D), device=dev, dtype=tdt).normal_(generator=gen)
            kt = torch.empty((B, N, Hkv, D), device=dev, dtype=tdt).normal_(generator=gen)
            vt = torch.empty((B, N, Hkv, D), device=dev, dtype=tdt).normal_(generator=gen)
            out = torch.empty((B, N, Hq, D), device=dev, dtype=tdt)
            layers.append((q, kt, vt, kc, vc, out))
        logits_h = gen_logits(args.seed + s, B, N, V)
        if accept == "sample-draft":
            draft_logits_h, tokens_h = gen_sampled_drafts(args.seed + s, logits_h, parent, n_nodes, cfg.temperature)
        else:
            draft_logits_h, tokens_h = None, gen_draft_tokens(args.seed + s, logits_h, parent, n_nodes, accept)
        sets.append(dict(layers=layers, logits=torch.from_numpy(logits_h).to(dev), tokens=torch.from_numpy(tokens_h).to(dev),
                         uniforms=torch.from_numpy(gen_uniforms(args.seed + s, B, N)).to(dev),
                         draft_logits=None if draft_logits_h is None else torch.from_numpy(draft_logits_h).to(dev)))
    parent_d = torch.from_numpy(parent).to(dev)
    n_nodes_d = torch.from_numpy(n_nodes).to(dev)
    hidden_dim = 0
    if args.lm_head:
        hidden_dim = args.hidden_dim or {"c0": 256, "c1": 4096, "c2": 4096, "c3": 6656, "c4": 8192}[workload]
        # the weights are streamed once per step; between two steps of a real model every layer's weights
        # pass through the caches, so a few copies are rotated to keep them out of the 256 MB last-level cache
        w_copies = [torch.empty((V, hidden_dim), device=dev, dtype=torch.bfloat16).normal_(generator=gen)
                    .mul_(3.0 / hidden_dim ** 0.5) for _ in range(min(n_sets, 4))]
        lm_packed = bool(args.packed_weights and args.lm_head == "fused")
        if lm_packed:
            w_copies = [fspad.fspad_pack_weight(w_).reshape(-1) for w_ in w_copies]
        for i, st in enumerate(sets):
            st["w"] = w_copies[i % len(w_copies)]
            st["hidden"] = torch.empty((B, N, hidden_dim), device=dev, dtype=torch.bfloat16).normal_(generator=gen)

    desc = fspad.make_attn_desc(sets[0]["layers"][0][0], sets[0]["layers"][0][1], sets[0]["layers"][0][3], tdt, 0.0,
                                workgroups=args.splits)
    ws_attn = torch.empty(max(16, fspad.fspad_tree_attn_workspace_bytes(desc, L)), dtype=torch.uint8, device=dev)
    ws_acc = torch.empty(fspad.fspad_tree_accept_workspace_bytes(B, N, V), dtype=torch.uint8, device=dev)
    ws_draft = (torch.empty(fspad.fspad_tree_accept_sample_draft_workspace_bytes(B, N, V), dtype=torch.uint8, device=dev)
                if accept == "sample-draft" else None)
    acc_out = (torch.empty((B, N), dtype=torch.int32, device=dev), torch.empty((B,), dtype=torch.int32, device=dev),
               torch.empty((B, N), dtype=torch.int32, device=dev), torch.empty((B,), dtype=torch.int32, device=dev))

    stream_handle = torch.cuda.current_stream().cuda_stream

    # Every call of a step is marshalled once (PreparedCall): in the timed loop Python only issues the
    # C calls, so the loop measures the GPU and not the binding's argument checks.
    for st in sets:
        st["attn"] = [fspad.fspad_tree_attn(q, kt, vt, kc, vc, kv_len, n_nodes, mask, out=out, workspace=ws_attn,
                                            desc=desc, prepare=True) for (q, kt, vt, kc, vc, out) in st["layers"]]
        if args.lm_head == "fused" and accept == "greedy":
            st["accept"] = fspad.fspad_tree_accept_greedy_lm_head(st["hidden"], st["w"], st["tokens"], parent_d, n_nodes_d,
                                                                  outputs=acc_out, prepare=True, packed=lm_packed, vocab=V)
        elif args.lm_head == "fused":
            st["accept"] = fspad.fspad_tree_accept_sample_lm_head(st["hidden"], st["w"], st["tokens"], parent_d, n_nodes_d,
                                                                  cfg.temperature, st["uniforms"], outputs=acc_out, prepare=True,
                                                                  packed=lm_packed, vocab=V)
        elif args.lm_head == "unfused":
            st["accept"] = unfused_lm_head_accept(torch, fspad, st, parent_d, n_nodes_d, acc_out, ws_acc, accept,
                                                  cfg.temperature)
        elif accept == "sample-draft":
            st["accept"] = fspad.fspad_tree_accept_sample_draft(st["logits"], st["draft_logits"], st["tokens"], parent_d,
                                                                n_nodes_d, cfg.temperature, st["uniforms"], outputs=acc_out,
                                                                workspace=ws_draft, prepare=True)
        elif accept == "greedy":
            st["accept"] = fspad.fspad_tree_accept_greedy(st["logits"], st["tokens"], parent_d, n_nodes_d, outputs=acc_out,
                                                          workspace=ws_acc, prepare=True)
        else:
            st["accept"] = fspad.fspad_tree_accept_sample(st["logits"], st["tokens"], parent_d, n_nodes_d, cfg.temperature,
                                                          st["uniforms"], outputs=acc_out, workspace=ws_acc, prepare=True)
        # the prefix length stays L from step to step: every step rewrites the same tail
        st["topk"] = []
        if args.draft_topk:
            rows = B * cfg.tree_topk
            draft_logits = torch.empty((rows, V), device=dev, dtype=torch.float32).normal_(generator=gen).mul_(3.0)
            st["topk"] = [fspad.fspad_draft_topk(draft_logits, min(cfg.tree_topk, 16), prepare=True)] * cfg.tree_depth
        st["sampler"] = []
        if args.feature_sampler:
            Hd_fs, I_fs = DRAFT_DIMS[workload]
            rows_fs = min(128, B * cfg.tree_topk)
            if "fs_w" not in sets[0]:
                sets[0]["fs_w"] = [[torch.empty(shape, device=dev, dtype=torch.bfloat16).normal_(generator=gen).mul_(shape[1] ** -0.5)
                                    for shape in ((I_fs, Hd_fs), (I_fs, Hd_fs), (Hd_fs, I_fs))] for _ in range(2)]
                if args.packed_weights and args.feature_sampler == "fused":
                    sets[0]["fs_w"] = [[fspad.fspad_pack_weight(w_) for w_ in ws_] for ws_ in sets[0]["fs_w"]]
            wu, wg, wd = sets[0]["fs_w"][len(sets[0].get("fs_n", [])) % 2]
            sets[0].setdefault("fs_n", []).append(1)
            f_in = torch.empty((rows_fs, Hd_fs), device=dev, dtype=torch.bfloat16).normal_(generator=gen)
            e_in = torch.empty((rows_fs, Hd_fs), device=dev, dtype=torch.bfloat16).normal_(generator=gen)
            if args.feature_sampler == "fused":
                st["sampler"] = [fspad.fspad_feature_sampler(f_in, e_in, wu, wg, wd, prepare=True,
                                                             packed=args.packed_weights)] * cfg.tree_depth
            else:
                st["sampler"] = [library_feature_sampler(torch, f_in, e_in, wu, wg, wd)] * cfg.tree_depth
            st["sampler_bytes"] = 2 * (3 * Hd_fs * I_fs + 3 * rows_fs * Hd_fs)
        st["layer"] = []
        if args.draft_layer:
            Hd_dl, I_dl = DRAFT_DIMS[workload]
            n_dl = cfg.tree_topk
            if B * n_dl > 128 or cfg.dtype != "bf16":
                raise SystemExit("--draft-layer: the layer takes at most 128 rows (batch x top-k) of bf16 per call")
            if "dl_w" not in sets[0]:
                dl_parent, dl_n = gen_trees(args.seed, B, n_dl, 2, n_dl)
                sets[0]["dl_tree"] = (dl_parent, dl_n, torch.from_numpy(
                    fspad.fspad_tree_build_mask(dl_parent, dl_n).view(np.int64)).to(dev),
                    torch.from_numpy((kv_len[:, None] + tree_depths(dl_parent, dl_n)).astype(np.int32)).to(dev))
                shapes = {"w_qkv": ((Hq + 2 * Hkv) * D, Hd_dl), "w_o": (Hd_dl, Hq * D), "w_gate": (I_dl, Hd_dl),
                          "w_up": (I_dl, Hd_dl), "w_down": (2 * Hd_dl, I_dl)}
                sets[0]["dl_w"] = []
                for _ in range(2):      # two copies, used in turn: 1 GB between two uses of a weight
                    wts = {k: torch.empty(shp, device=dev, dtype=torch.bfloat16).normal_(generator=gen).mul_(shp[1] ** -0.5)
                           for k, shp in shapes.items()}
                    if args.packed_weights and args.draft_layer == "fused":
                        wts = {k: fspad.fspad_pack_weight(w_) for k, w_ in wts.items()}
                    wts["gain_attn"] = torch.ones(Hd_dl, device=dev, dtype=torch.bfloat16)
                    wts["gain_mlp"] = torch.ones(Hd_dl, device=dev, dtype=torch.bfloat16)
                    sets[0]["dl_w"].append(wts)
            dl_parent, dl_n, dl_mask, dl_pos = sets[0]["dl_tree"]
            wts = sets[0]["dl_w"][len(sets[0].get("dl_n", [])) % 2]
            sets[0].setdefault("dl_n", []).append(1)
            eta_in = torch.empty((B, n_dl, Hd_dl), device=dev, dtype=torch.bfloat16).normal_(generator=gen)
            kc0, vc0 = st["layers"][0][3], st["layers"][0][4]    # the cache of the first layer stands in for the draft's
            if args.draft_layer == "fused":
                st["layer"] = [fspad.fspad_draft_layer(eta_in, dl_pos, wts, kc0, vc0, kv_len, dl_n, dl_mask, Hq, Hkv, D,
                                                       prepare=True, packed=args.packed_weights)] * cfg.tree_depth
            else:
                st["layer"] = [library_draft_layer(torch, eta_in, dl_pos, wts, kc0, vc0, L, dl_parent, dl_n, Hq, Hkv, D)] * cfg.tree_depth
            st["layer_bytes"] = 2 * (sum(w_.numel() for w_ in wts.values()) + 3 * B * n_dl * Hd_dl) + 4 * B * Hkv * L * D
        st["build"] = None
        if args.tree_build:
            cands = gen_candidates(args.seed, B, cfg.tree_depth, cfg.tree_topk, V)
            st["build"] = fspad.fspad_tree_build(*[torch.from_numpy(a).to(dev) for a in cands], N, N, prepare=True)
        st["commit"] = [fspad.fspad_kv_commit(kt, vt, kc, vc, kv_len, acc_out[0], acc_out[1], prepare=True)
                        for (q, kt, vt, kc, vc, out) in st["layers"]] if args.commit else []

    def step(i, timed=None):
        st = sets[i % n_sets]
        if st["sampler"] and timed is not None:
            e0, e1 = event_pool.pop(), event_pool.pop()
            e0.record()
            st["sampler"][0]()
            e1.record()
            sampler_events.append((e0, e1))
            for call in st["sampler"][1:]:
                call()
        else:
            for call in st["sampler"]:
                call()
        if st["layer"] and timed is not None:
            e0, e1 = event_pool.pop(), event_pool.pop()
            e0.record()
            st["layer"][0]()
            e1.record()
            layer_events.append((e0, e1))
            for call in st["layer"][1:]:
                call()
        else:
            for call in st["layer"]:
                call()
        for call in st["topk"]:
            call()
        if st["build"] is not None:
            st["build"]()
        if timed is None:
            for call in st["attn"]:
                call()
        else:  # bracket some attention calls of this step (eight at most) with a pair of timing events
            stride = -(-len(st["attn"]) // 8)
            for j, call in enumerate(st["attn"]):
                if j % stride:
                    call()
                    continue
                e0, e1 = event_pool.pop(), event_pool.pop()
                e0.record()
                call()
                e1.record()
                timed.append((e0, e1))
        if timed is None:
            st["accept"]()
        else:
            e0, e1 = event_pool.pop(), event_pool.pop()
            e0.record()
            st["accept"]()
            e1.record()
            accept_events.append((e0, e1))
        for call in st["commit"]:
            call()

    if args.copy_calibration:
        src = torch.empty(args.copy_calibration << 20, dtype=torch.uint8, device=dev).random_(generator=gen)
        dst = torch.empty_like(src)
        for _ in range(3):
            roofs_call("roofs_hbm_copy", src.data_ptr(), dst.data_ptr(), src.numel(), 2048, stream_handle)
        torch.cuda.synchronize()
        del src, dst

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    events = []
    event_every = args.event_every if args.event_every > 0 else max(4, steps // 12)
    # events are created ahead of the timed region (two per bracketed call)
    event_pool = [TimingEvent(stream_handle) for _ in range(2 * 11 * (steps // event_every + 1))]
    accept_events, sampler_events, layer_events = [], [], []
    t0 = time.perf_counter()
    # Recording an event costs the stream several microseconds, as much as a small kernel: only every
    # `event_every`-th step is bracketed, so that the timed region stays the workload's own.
    for i in range(steps):
        step(warmup + i, events if i % event_every == 0 else None)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    call_ms = np.array([a.elapsed_time(b) for a, b in events])  # one fspad_tree_attn call (all its kernels) each
    attn_ms = float(call_ms.mean())
    n_tokens_mean = float(acc_out[3].float().mean().item())
    accept_ms = np.array([a.elapsed_time(b) for a, b in accept_events])  # the step's acceptance call (all its kernels)

    # After the timed region: the same steps when the host reads the emitted-token counts back after
    # every step, as a decoding loop must (one device-to-host copy and synchronisation per step).
    sync_steps = max(1, steps // 4)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for i in range(sync_steps):
        step(warmup + steps + i)
        acc_out[3].cpu()
    t3 = time.perf_counter()
    ms_per_step_sync = (t3 - t2) * 1e3 / sync_steps

    # Also after the timed region: the same number of steps over ONE buffer set, i.e. with whatever fits
    # of a step's inputs resident in the 256 MB last-level cache (the headline value rotates the sets so
    # that every step streams from HBM). Reported separately and labelled as such.
    torch.cuda.synchronize()
    t4 = time.perf_counter()
    for i in range(steps):
        step(0)
    torch.cuda.synchronize()
    ms_per_step_resident = (time.perf_counter() - t4) * 1e3 / steps

    # And the same steps replayed from a captured graph (one graph holds a step over every buffer set, so
    # the replays stream from HBM like the timed loop): the launch cost of the 2 to 4 kernels of a small
    # step is then the graph's, not Python's and the runtime's. Only the verification calls are captured.
    graph_steps_per_s = None
    if not (args.feature_sampler or args.draft_layer or args.lm_head == "unfused"):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=torch.cuda.current_stream()):
            for i in range(n_sets):
                step(i)
        replays = max(1, steps // n_sets)
        for _ in range(2):
            graph.replay()
        torch.cuda.synchronize()
        t5 = time.perf_counter()
        for _ in range(replays):
            graph.replay()
        torch.cuda.synchronize()
        graph_steps_per_s = replays * n_sets / (time.perf_counter() - t5)
        del graph
    props = torch.cuda.get_device_properties(0)

    attn_bytes = cfg.attn_bytes_per_layer()
    attn_flops = cfg.attn_flops_per_layer()
    achieved_gbs = attn_bytes / (attn_ms * 1e-3) / 1e9
    achieved_tflops = attn_flops / (attn_ms * 1e-3) / 1e12
    flop_per_byte = attn_flops / attn_bytes
    mfma_bound = flop_per_byte > MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9) and cfg.dtype == "bf16"
    if mfma_bound:
        roofline = dict(bound="mfma", achieved=achieved_tflops, peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s",
                        frac=achieved_tflops / MFMA_BF16_PEAK_TFLOPS)
    else:
        roofline = dict(bound="hbm", achieved=achieved_gbs, peak=HBM_PEAK_GBS, unit="GB/s", frac=achieved_gbs / HBM_PEAK_GBS)
    traffic = read_profiled_traffic(workload) if (default_shape and not args.splits) else None
    roofline.update(kernel="fspad_tree_attn (split-KV kernel + merge kernel)", launch_ms=attn_ms,
                    algorithmic_bytes=attn_bytes, algorithmic_flops=attn_flops,
                    hbm_frac=achieved_gbs / HBM_PEAK_GBS, mfma_frac=achieved_tflops / MFMA_BF16_PEAK_TFLOPS,
                    traffic=traffic, traffic_source=TRAFFIC_PROFILE if traffic is not None else None)
    # the whole step (every layer's attention call and the acceptance call, launch gaps included) against the same roof
    step_s = ms_per_step * 1e-3
    if mfma_bound:
        step_roofline = dict(bound="mfma", achieved=cfg.step_flops() / step_s / 1e12, peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s")
    else:
        step_roofline = dict(bound="hbm", achieved=cfg.step_bytes() / step_s / 1e9, peak=HBM_PEAK_GBS, unit="GB/s")
    step_roofline["frac"] = step_roofline["achieved"] / step_roofline["peak"]
    step_roofline.update(algorithmic_bytes=cfg.step_bytes(), algorithmic_flops=cfg.step_flops())

    # the acceptance call (row pass + walk) against its own roofs: the logits are read once (HBM); the
    # sampling form also evaluates one fp64 exponential per logit: cast, scale, range reduction, an
    # 11-term polynomial, scaling and the sum: 27 fp64 vector operations of which 15 are fused
    # multiply-adds, counted as 42 flops, against the fp64 vector peak of 256 CUs x 4 SIMDs x 16 lanes
    # x 2 flops x 2.4 GHz = 78.6 TFLOP/s
    accept_s = float(np.percentile(accept_ms, 50)) * 1e-3
    accept_roofline = dict(bound="hbm", achieved=cfg.logit_bytes() / accept_s / 1e9, peak=HBM_PEAK_GBS, unit="GB/s")
    accept_roofline["frac"] = accept_roofline["achieved"] / HBM_PEAK_GBS
    if accept == "sample" and not args.lm_head:
        fp64_tflops = B * N * V * 42 / accept_s / 1e12
        accept_roofline.update(alu_fp64_tflops=fp64_tflops, alu_fp64_peak=78.6, alu_fp64_frac=fp64_tflops / 78.6)
    accept_roofline.update(kernel="acceptance call (row pass + walk)", call_us_p50=accept_s * 1e6, algorithmic_bytes=cfg.logit_bytes())

    result = {
        "metric": "tree-verify steps/s", "value": 1e3 / ms_per_step, "unit": "steps/s", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "layers": cfg.layers, "batch": B, "n_q_heads": Hq, "n_kv_heads": Hkv,
                   "head_dim": D, "kv_len": L, "tree_nodes": N, "vocab": V, "accept": accept, "buffer_sets": n_sets,
                   "kv_commit": bool(args.commit), "tree_build": bool(args.tree_build), "draft_topk": bool(args.draft_topk),
                   "seed": args.seed, "generator_version": GENERATOR_VERSION, "parallelism": "single-gpu"},
        "step_gb_per_s": cfg.step_bytes() / (ms_per_step * 1e-3) / 1e9,
        "step_hbm_frac": cfg.step_bytes() / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "step_roofline": step_roofline,
        "attn_tflops": achieved_tflops, "attn_gb_per_s": achieved_gbs,
        "attn_call_us": {"mean": attn_ms * 1e3, "p10": float(np.percentile(call_ms, 10)) * 1e3,
                         "p50": float(np.percentile(call_ms, 50)) * 1e3, "p90": float(np.percentile(call_ms, 90)) * 1e3,
                         "samples": int(call_ms.size)},
        "accept_call_us": {"mean": float(accept_ms.mean()) * 1e3, "p50": float(np.percentile(accept_ms, 50)) * 1e3,
                           "samples": int(accept_ms.size)},
        "steps_per_s_with_host_readback": 1e3 / ms_per_step_sync,
        "steps_per_s_one_buffer_set_cache_resident": 1e3 / ms_per_step_resident,
        "steps_per_s_graph_replay": graph_steps_per_s,
        "device": {"name": props.name, "arch": getattr(props, "gcnArchName", ""), "compute_units": props.multi_processor_count,
                   "hbm_bytes": props.total_memory, "clocks": read_clock_levels()},
        "mean_tokens_per_step": n_tokens_mean,
        "roofline": roofline,
        "accept_roofline": accept_roofline,
    }

    if args.feature_sampler:
        fs_ms = np.array([a.elapsed_time(b) for a, b in sampler_events])
        call_s = float(np.percentile(fs_ms, 50)) * 1e-3
        fs_bytes = sets[0]["sampler_bytes"]
        result["config"].update(feature_sampler=args.feature_sampler, packed_weights=bool(args.packed_weights))
        result["feature_sampler"] = {"mode": args.feature_sampler, "call_us_p50": call_s * 1e6, "calls_per_step": cfg.tree_depth,
                                     "algorithmic_bytes": fs_bytes, "gb_per_s": fs_bytes / call_s / 1e9,
                                     "hbm_frac": fs_bytes / call_s / 1e9 / HBM_PEAK_GBS}
    if args.draft_layer:
        dl_ms = np.array([a.elapsed_time(b) for a, b in layer_events])
        call_s = float(np.percentile(dl_ms, 50)) * 1e-3
        dl_bytes = sets[0]["layer_bytes"]
        result["config"].update(draft_layer=args.draft_layer, packed_weights=bool(args.packed_weights))
        result["draft_layer"] = {"mode": args.draft_layer, "call_us_p50": call_s * 1e6, "calls_per_step": cfg.tree_depth,
                                 "rows": B * cfg.tree_topk, "algorithmic_bytes": dl_bytes, "gb_per_s": dl_bytes / call_s / 1e9,
                                 "hbm_frac": dl_bytes / call_s / 1e9 / HBM_PEAK_GBS}
    if args.lm_head:
        # the LM head streams its V x Hd weights once (and the B*N x Hd hidden states); per group of rows when B*N > 256
        passes = -(-B * N // 256)
        head_bytes = 2 * hidden_dim * (V + B * N)
        call_s = float(np.percentile(accept_ms, 50)) * 1e-3
        result["config"].update(lm_head=args.lm_head, hidden_dim=hidden_dim, packed_weights=bool(args.packed_weights))
        result["lm_head"] = {"mode": args.lm_head, "call_us_p50": call_s * 1e6, "algorithmic_bytes": head_bytes,
                             "weight_passes": passes if args.lm_head == "fused" else 1,
                             "gb_per_s": head_bytes / call_s / 1e9, "hbm_frac": head_bytes / call_s / 1e9 / HBM_PEAK_GBS,
                             "tflops": 2.0 * B * N * hidden_dim * V / call_s / 1e12}
    if primary and not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, accept, sets[0], parent, n_nodes, kv_len, args.seed)
    del sets
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    return result


_ROOFS = None


def roofs_call(name, *call_args):
    """One call into libfspad_roofs.so (the benchmark's measurement kernels; not the verification library)."""
    import ctypes
    global _ROOFS
    if _ROOFS is None:
        from paper_2408_15562_amd.build import ROOFS_LIB_PATH
        if not os.path.exists(ROOFS_LIB_PATH):
            raise RuntimeError(f"{ROOFS_LIB_PATH} is missing: build it first (__graft_entry__.build())")
        lib = ctypes.CDLL(ROOFS_LIB_PATH)
        vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        lib.roofs_hbm_read.argtypes = [vp, sz, vp, i32, vp]
        lib.roofs_hbm_copy.argtypes = [vp, vp, sz, i32, vp]
        lib.roofs_mfma_bf16.argtypes = [i32, i32, i32, vp, vp]
        lib.roofs_overlap.argtypes = [i32, i32, i32, i32, vp, vp]
        _ROOFS = lib
    rc = getattr(_ROOFS, name)(*call_args)
    if rc != 0:
        raise RuntimeError(f"{name} failed: {rc}")


def measure_roofs(torch, stream_handle):
    """What this machine reaches on the two roofs, with the simplest kernels that can reach them: a
    streaming read of 4 GiB, 16 bytes per lane (HBM), and a register-resident loop of bf16 matrix-core
    instructions (both tile shapes; the better one counts). Event-timed, five launches each after two
    warm-up launches."""
    dev = torch.device("cuda:0")
    sink = torch.zeros(64, dtype=torch.float32, device=dev)

    def timed(launch, reps=5):
        for _ in range(2):
            launch()
        torch.cuda.synchronize()
        e0, e1 = TimingEvent(stream_handle), TimingEvent(stream_handle)
        e0.record()
        for _ in range(reps):
            launch()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    nbytes = 4 << 30
    buf = torch.empty(nbytes, dtype=torch.uint8, device=dev).random_()
    best_read = 0.0
    for wgs in (2048, 4096, 8192):
        t = timed(lambda: roofs_call("roofs_hbm_read", buf.data_ptr(), nbytes, sink.data_ptr(), wgs, stream_handle))
        best_read = max(best_read, nbytes / t / 1e9)
    del buf
    mfma = {}
    iters, wgs = 4096, 1024
    for shape, per_wave in ((16, 8 * 16 * 16 * 32 * 2), (32, 4 * 32 * 32 * 16 * 2)):
        t = timed(lambda: roofs_call("roofs_mfma_bf16", shape, iters, wgs, sink.data_ptr(), stream_handle))
        mfma[shape] = wgs * 4 * iters * per_wave / t / 1e12
    torch.cuda.empty_cache()
    return {"hbm_read_gb_per_s": best_read, "hbm_read_frac_of_published": best_read / HBM_PEAK_GBS,
            "hbm_read_bytes": nbytes, "mfma_bf16_tflops": max(mfma.values()),
            "mfma_bf16_frac_of_published": max(mfma.values()) / MFMA_BF16_PEAK_TFLOPS,
            "mfma_bf16_16x16x32_tflops": mfma[16], "mfma_bf16_32x32x16_tflops": mfma[32]}


def probe_overlap(torch, stream_handle):
    """Engine-clock cycles (at the nominal 2.4 GHz) per turn of the overlap kernels of libfspad_roofs.so: what a
    SIMD runs at the same time. The attention kernels' wavefront shapes follow from these figures."""
    sink = torch.zeros(64, dtype=torch.float32, device="cuda:0")
    iters = 20000

    def cycles(mode, nv, trans):
        for n_it in (200, iters):
            e0, e1 = TimingEvent(stream_handle), TimingEvent(stream_handle)
            e0.record()
            roofs_call("roofs_overlap", mode, nv, trans, n_it, sink.data_ptr(), stream_handle)
            e1.record()
            torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 * 2.4e9 / iters

    out = {"unit": "cycles per turn at 2.4 GHz", "same_wavefront_one_per_simd": {}, "two_wavefronts_per_simd": {}}
    for trans, name in ((0, "fma"), (1, "exp")):
        for nv in (0, 4, 8, 16):
            # a turn = 2 x (one 32x32x16 matrix instruction + nv vector instructions)
            out["same_wavefront_one_per_simd"][f"2x(mfma+{nv}{name})"] = cycles(0, nv, trans)
        out["two_wavefronts_per_simd"][f"2mfma_wave_alone"] = cycles(2, 16, trans)
        for nv in (4, 8, 16):   # wavefront B's vector instructions per turn
            out["two_wavefronts_per_simd"][f"{nv}{name}_wave_alone"] = cycles(3, nv, trans)
            out["two_wavefronts_per_simd"][f"2mfma_wave_beside_{nv}{name}_wave"] = cycles(1, nv, trans)
    return out


def read_profiled_traffic(workload):
    """HBM bytes of one fspad_tree_attn call as the profiler's byte counters measured them (not measured in
    this run): the line `traffic_bytes_per_call <workload> <bytes>` of profiles/tree_verify_traffic.txt,
    which is refreshed whenever the attention kernels or their work split change. None if there is none."""
    try:
        with open(os.path.join(ROOT, TRAFFIC_PROFILE)) as fh:
            for line in fh:
                m = re.match(r"\s*traffic_bytes_per_call\s+(\w+)\s+(\d+)", line)
                if m and m.group(1) == workload:
                    return int(m.group(2))
    except OSError:
        pass
    return None


def read_clock_levels():
    """Engine / memory clock levels of the first GPU as the driver lists them (the active level carries a
    '*'); None where the files cannot be read. Read after the timed region; changes nothing."""
    import glob
    out = {}
    for key, name in (("sclk", "pp_dpm_sclk"), ("mclk", "pp_dpm_mclk")):
        out[key] = None
        for path in sorted(glob.glob(f"/sys/class/drm/card*/device/{name}")):
            try:
                with open(path) as fh:
                    levels = [line.strip() for line in fh if line.strip()]
            except OSError:
                continue
            if levels:
                out[key] = levels
                break
    return out


def library_draft_layer(torch, eta, pos, w, k_cache, v_cache, L, parent, n_nodes, Hq, Hkv, D):
    """The comparison for --draft-layer: the same layer from library GEMMs, the library's fused attention
    under a dense mask and element-wise kernels. The tree's keys / values are written behind the prefix
    of the cache and the attention reads prefix and tree in one go. Temporaries come from torch's caching
    allocator (no device allocation after the warm-up)."""
    F = torch.nn.functional
    B, N, Hd = eta.shape
    dev = eta.device
    x = eta.view(B * N, Hd)
    half = D // 2
    inv_freq = 10000.0 ** (-torch.arange(half, device=dev, dtype=torch.float32) * 2.0 / D)
    ang = pos.view(B * N, 1).float() * inv_freq
    cos, sin = ang.cos()[:, None, :], ang.sin()[:, None, :]
    allowed = torch.zeros((B, 1, N, L + N), dtype=torch.bool, device=dev)
    allowed[..., :L] = True
    for b in range(B):
        for i in range(int(n_nodes[b])):
            j = i
            while j >= 0:
                allowed[b, 0, i, L + j] = True
                j = int(parent[b, j])
    kc = k_cache[:, :, :L + N]
    vc = v_cache[:, :, :L + N]
    w_down_a, w_down_b = w["w_down"][:Hd], w["w_down"][Hd:]

    def rope(u):
        a, b = u[..., :half].float(), u[..., half:].float()
        return torch.cat([a * cos - b * sin, b * cos + a * sin], dim=-1).to(torch.bfloat16)

    def call():
        xn = F.rms_norm(x, (Hd,), w["gain_attn"], 1e-6)
        qkv = torch.mm(xn, w["w_qkv"].t())
        q = rope(qkv[:, :Hq * D].view(B * N, Hq, D)).view(B, N, Hq, D).transpose(1, 2)
        k = rope(qkv[:, Hq * D:(Hq + Hkv) * D].view(B * N, Hkv, D)).view(B, N, Hkv, D)
        v = qkv[:, (Hq + Hkv) * D:].view(B, N, Hkv, D)
        kc[:, :, L:] = k.transpose(1, 2)
        vc[:, :, L:] = v.transpose(1, 2)
        a = F.scaled_dot_product_attention(q, kc, vc, attn_mask=allowed, enable_gqa=Hq != Hkv)
        h = x + torch.mm(a.transpose(1, 2).reshape(B * N, Hq * D), w["w_o"].t())
        hn = F.rms_norm(h, (Hd,), w["gain_mlp"], 1e-6)
        s = F.silu(torch.mm(hn, w["w_gate"].t())) * torch.mm(hn, w["w_up"].t())
        m = torch.mm(s, w["w_down"].t())
        return h + m[:, :Hd], h + m[:, Hd:]
    return call


def library_feature_sampler(torch, f_in, e_in, wu, wg, wd):
    """The comparison for --feature-sampler: library GEMMs and element-wise kernels, buffers allocated once."""
    rows, I = f_in.shape[0], wu.shape[0]
    up = torch.empty((rows, I), device=f_in.device, dtype=torch.bfloat16)
    gate = torch.empty_like(up)
    out = torch.empty_like(f_in)

    def call():
        torch.mm(f_in, wu.t(), out=up)
        torch.mm(e_in, wg.t(), out=gate)
        torch.nn.functional.silu(gate, inplace=True)
        gate.mul_(up)
        torch.mm(gate, wd.t(), out=out)
        out.add_(f_in)
    return call


def unfused_lm_head_accept(torch, fspad, st, parent_d, n_nodes_d, acc_out, ws_acc, accept, temperature):
    """The comparison for --lm-head: a library GEMM writes bf16 logits, they are widened to fp32 and the
    ordinary acceptance reads them. All buffers are allocated here, once."""
    B, N, Hd = st["hidden"].shape
    V = st["w"].shape[0]
    h2d = st["hidden"].view(B * N, Hd)
    wt = st["w"].t()
    logits_lp = torch.empty((B * N, V), device=h2d.device, dtype=torch.bfloat16)
    logits = torch.empty((B, N, V), device=h2d.device, dtype=torch.float32)
    if accept == "greedy":
        walk = fspad.fspad_tree_accept_greedy(logits, st["tokens"], parent_d, n_nodes_d, outputs=acc_out, workspace=ws_acc,
                                              prepare=True)
    else:
        walk = fspad.fspad_tree_accept_sample(logits, st["tokens"], parent_d, n_nodes_d, temperature, st["uniforms"],
                                              outputs=acc_out, workspace=ws_acc, prepare=True)

    def call():
        torch.mm(h2d, wt, out=logits_lp)
        logits.view(B * N, V).copy_(logits_lp)
        walk()
    return call


class TimingEvent:
    """HIP event that is only used for timing: created with hipEventDisableSystemFence, so that recording
    it neither writes back nor invalidates the caches around the kernels it brackets (the default event
    does, which costs the following kernel several microseconds)."""
    _hip = None
    _FLAGS = 0x20000000  # hipEventDisableSystemFence

    def __init__(self, stream_handle):
        import ctypes
        if TimingEvent._hip is None:
            TimingEvent._hip = ctypes.CDLL("libamdhip64.so")
        self._ev = ctypes.c_void_p()
        self._stream = ctypes.c_void_p(stream_handle)
        rc = TimingEvent._hip.hipEventCreateWithFlags(ctypes.byref(self._ev), ctypes.c_uint(self._FLAGS))
        if rc != 0:
            raise RuntimeError(f"hipEventCreateWithFlags failed: {rc}")

    def record(self):
        rc = TimingEvent._hip.hipEventRecord(self._ev, self._stream)
        if rc != 0:
            raise RuntimeError(f"hipEventRecord failed: {rc}")

    def elapsed_time(self, end) -> float:
        import ctypes
        ms = ctypes.c_float()
        rc = TimingEvent._hip.hipEventElapsedTime(ctypes.byref(ms), self._ev, end._ev)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return float(ms.value)

    def __del__(self):
        if self._ev and TimingEvent._hip is not None:
            TimingEvent._hip.hipEventDestroy(self._ev)


# hidden and intermediate size of the draft side per workload (the target model's own)
DRAFT_DIMS = {"c0": (256, 512), "c1": (4096, 11008), "c2": (4096, 14336), "c3": (6656, 17920), "c4": (8192, 28672)}


def cpu_baseline(cfg, accept, dev_set, parent, n_nodes, kv_len, seed):
    """The CPU oracle, as it stands, on this machine's host cores, on a bounded sample of the workload: once
    with OpenMP over the sampled heads (`value`, the figure of the contract) and once single-threaded on a
    smaller sample; both extrapolated linearly to the whole step where the sample is partial."""
    import numpy as np

    import oracle
    nproc = os.cpu_count() or 1
    cores = min(nproc, int(os.environ.get("OMP_NUM_THREADS", "16")), 16)
    B, N, Hq, Hkv = cfg.batch, cfg.n_nodes, cfg.n_q_heads, cfg.n_kv_heads
    G = Hq // Hkv
    q, kt, vt, kc, vc, _ = dev_set["layers"][0]
    logits = dev_set["logits"].cpu().numpy()
    tokens = dev_set["tokens"].cpu().numpy()
    uniforms = dev_set["uniforms"].cpu().numpy()
    work_per_head = 2.0 * N * (cfg.kv_len + N) * cfg.head_dim * 2 * B     # flops of one query head, all sequences

    def accept_once():
        if accept == "greedy":
            oracle.accept_greedy(logits, tokens, parent, n_nodes)
        elif accept == "sample-draft":
            oracle.accept_sample_draft(logits, dev_set["draft_logits"].cpu().numpy(), tokens, parent, n_nodes, cfg.temperature,
                                       uniforms)
        else:
            oracle.accept_sample(logits, tokens, parent, n_nodes, cfg.temperature, uniforms)

    def leg(threads, flop_budget, seconds):
        # sample: all sequences, a subset of the query heads of ONE layer, sized to a few seconds of CPU work
        heads = int(max(1, min(Hq, flop_budget // work_per_head)))
        head_ids = sorted(set(np.linspace(0, Hq - 1, heads).astype(int).tolist()))
        kvh = [h // G for h in head_ids]
        host = [q[:, :, head_ids].float().cpu().numpy(), kt[:, :, kvh].float().cpu().numpy(), vt[:, :, kvh].float().cpu().numpy(),
                kc[:, kvh].float().cpu().numpy(), vc[:, kvh].float().cpu().numpy()]
        t_attn, t_acc, reps = 0.0, 0.0, 0
        t_start = time.perf_counter()
        while reps < 1 or (time.perf_counter() - t_start < seconds and reps < 50):
            t0 = time.perf_counter()
            oracle.tree_attn(*host, kv_len, n_nodes, parent, nthreads=threads)
            t1 = time.perf_counter()
            accept_once()
            t2 = time.perf_counter()
            t_attn += t1 - t0
            t_acc += t2 - t1
            reps += 1
        # whole step = every head of every layer (attention extrapolated linearly from the sampled heads) + acceptance
        step_s = (t_attn / reps) * (Hq / len(head_ids)) * cfg.layers + t_acc / reps
        extrap = len(head_ids) < Hq or cfg.layers > 1
        sample = (f"{reps} repetitions of: attention of {len(head_ids)}/{Hq} query heads of 1/{cfg.layers} layers, all "
                  f"{B} sequences ({threads} thread{'s' if threads > 1 else ''}) + full {accept} acceptance (1 thread)"
                  + ("; step time extrapolated linearly to all heads and layers" if extrap else ""))
        return step_s, sample, extrap

    omp_s, omp_sample, extrap = leg(cores, 4.0e9, 10.0)
    one_s, one_sample, one_extrap = leg(1, 5.0e8, 6.0)
    return {"value": 1.0 / omp_s, "unit": "steps/s", "cores": cores, "kind": "oracle", "sample": omp_sample,
            "extrapolated": extrap, "nproc": nproc,
            "single_thread": {"value": 1.0 / one_s, "unit": "steps/s", "cores": 1, "sample": one_sample,
                              "extrapolated": one_extrap}}


if __name__ == "__main__":
    main()
