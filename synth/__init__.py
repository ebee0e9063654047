"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke run.

This package only *draws inputs* (token histories with planted repeats, random
model weights, random KV caches).  It holds none of the method's arithmetic:
no match search, no model forward, no acceptance rule.  Both the CPU oracle
and the HIP path are fed from here; neither is imported here.
"""
from .workloads import (  # noqa: F401
    ModelShape, TINY, LLAMA_1B, LLAMA_8B, QWEN_7B, LLAMA_70B, QWEN_72B, BASE_SEED, seed_for, model_weights_lazy,
    bf16_bits_to_f32, f32_to_bf16_bits,
    model_weights, random_kv,
    history_cfg1, history_cfg2, history_cfg3, history_cfg4, history_cfg5,
    planted_history, multiturn_replay, zipf_replay,
)
