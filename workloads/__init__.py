"""Seeded synthetic inputs for the shared-prefix paged-KV attention path.

This module only *lays out data*: random bf16 tensors, block tables whose rows
alias the same physical prefix blocks, sequence lengths, and index lists for the
block copy operations.  It contains none of the method's arithmetic (no scores,
no softmax, no copies of KV rows) and is imported by both the tests of the CPU
oracle and the GPU binding's tests / benchmark, which otherwise share no code.

Shapes follow the serving structure the paper describes: an agent-template
prefix shared by every prompt, then graph context / notebook segments shared by
the branches of one query, then a private per-branch suffix (Sec. 5.1, 5.2),
with many concurrent branches per batch (Sec. 6.1).
"""
from .gen import (  # noqa: F401
    Geometry,
    Workload,
    ChurnStep,
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    config_seed,
    make_config,
    tiny_decode,
    llama8b_decode,
    qwen3_moe_decode,
    mixed_batch,
    short_turn_prefill,
    mixed_short_turns,
    prefill_on_prefix,
    tree_decode_70b,
    eviction_churn,
    churn_step,
    agent_trace,
    new_token_slots,
    custom_decode,
    custom_prefill,
    CONFIG_NAMES,
)
