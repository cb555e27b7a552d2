"""Seeded synthetic inputs for tree verification, shared by tests, smoke and bench.

This package only *draws inputs* (tree shapes, Q/K/V, logits, draft tokens,
uniforms).  It holds none of the method's arithmetic: no mask construction, no
attention, no acceptance.  Both the GPU library and the CPU oracle are fed from
here; neither is imported here.

The inputs stand in for the shapes of the paper's workloads (Vicuna / LLaMA3
head geometry and vocabulary sizes, 60- and ~30-token draft trees built the
EAGLE-2 way, temperature 0 and 1); the paper's prompts, models and drafts are not
reproduced.
"""
from .configs import CONFIGS, VerifyConfig  # noqa: F401
from .generators import (  # noqa: F401
    GENERATOR_VERSION,
    gen_tree,
    gen_trees,
    gen_qkv,
    gen_logits,
    gen_draft_tokens,
    gen_uniforms,
    gen_candidates,
    gen_lm_head,
    gen_lm_head_exact,
    gen_feature_sampler,
    gen_draft_layer,
    gen_sampled_drafts,
    tree_depths,
    round_to_bf16,
    chain_tree,
)
