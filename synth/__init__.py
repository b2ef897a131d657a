"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests/bench.

This package only *generates inputs* (model descriptions, weights, token ids, score
samples).  It contains none of the method's arithmetic: no norm, attention, softmax,
rank or classification code lives here, and it imports neither the oracle nor the
HIP binding.
"""
from .inputs import (  # noqa: F401
    ModelConfig,
    Workload,
    WORKLOADS,
    hash_uniform,
    make_weights,
    make_token_ids,
    lognormal_scores,
    stream_id,
)
