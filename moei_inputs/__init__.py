"""Seeded synthetic inputs for the MoE decode-step hot path.

This module only *draws* inputs (weights, router matrices, EAMC traces, request
preference distributions, hidden states). It holds none of the method's
arithmetic: no routing, no matching, no priority scoring, no FFN.  Both the CPU
oracle's tests and the HIP path's tests/bench read their inputs from here so
that the two sides see bit-identical data; neither side's code lives here.

The paper evaluates on BIGBench / FLAN / MMLU / LongBench prompts with trained
checkpoints (Sec. 6, experiment setup).  None of those is available, so these
generators stand in for them and reproduce only the *structure* the paper
reports: per-request skewed expert reuse that evens out across requests
(Sec. 4.2), a few tens of activation groups per thousand sequences (Table 2),
EAMC sizes of 1K and 10K traces (App. B.1, runtime overhead).
"""
from .configs import Config, CONFIGS, get_config, BASE_SEED  # noqa: F401
from .gen import (  # noqa: F401
    stream,
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    store_dtype,
    to_store,
    store_to_f32,
    expert_weights,
    expert_bank,
    router_weights,
    cluster_preferences,
    trace_preferences,
    counts_from_preferences,
    eamc_traces,
    Request,
    make_request,
)
