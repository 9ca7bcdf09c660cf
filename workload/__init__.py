"""Seeded synthetic inputs for the speculative-decoding step.

This package only *draws inputs* (weights, prompts, stop masks, tree shapes, planted drafts,
synthetic KV rows) and names the workload presets. It holds none of the method's arithmetic:
no model forward, no acceptance rule, no tree assembly. Both the CPU oracle's tests and the
HIP path's tests feed from it, so the two sides always see identical inputs.
"""
from .configs import ModelShape, Workload, PRESETS, preset
from .gen import (
    make_weights,
    zipf_prompt,
    frag_filled_labels,
    stop_set,
    pack_mask_words,
    default_tree,
    chain_tree,
    full_tree,
    synthetic_kv_rows,
    plant_drafts,
    round_to_bf16,
    SEEDS,
)

__all__ = [
    "ModelShape", "Workload", "PRESETS", "preset",
    "make_weights", "zipf_prompt", "frag_filled_labels", "stop_set", "pack_mask_words",
    "default_tree", "chain_tree", "full_tree", "synthetic_kv_rows", "plant_drafts",
    "round_to_bf16", "SEEDS",
]
