"""Seeded synthetic inputs for the DDD draft-round tests and benchmark.

This package only *generates inputs* (weights, hidden states, target argmaxes,
workload configurations).  It contains none of the method's arithmetic: no
projection, no softmax, no top-k, no beam or tree logic.  Both the CPU oracle
tests and the GPU tests draw their inputs from here so that the two sides see
identical bits.
"""
from .inputs import (  # noqa: F401
    Workload,
    WORKLOADS,
    PAPER_MODES,
    paper_mode,
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    make_lm_head,
    make_plant_table,
    make_body_weights,
    make_prompt_context,
    make_random_tree,
    make_target_logits,
    mix64,
    stream_key,
    node_key,
    hidden_row,
    hidden_rows,
    root_hidden,
    ROOT_PARENT,
    target_argmax_for_tree,
)
