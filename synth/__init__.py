"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests/bench.

This package holds no arithmetic of the speculative-decoding method itself: it only
describes model shapes and draws random weights, contexts, page tables, cache contents,
logits and uniform numbers from seeds.
"""
from .inputs import (  # noqa: F401
    ModelCfg,
    TINY,
    MID,
    QWEN7B,
    QWEN32B,
    LLAMA70B,
    make_decoder_weights,
    make_drafter_weights,
    lognormal_contexts,
    uniform_contexts,
    random_block_table,
    fill_kv_pool,
    prompts,
    uniforms_u32,
    synthetic_logits,
    pages_needed,
)
