"""Seeded synthetic inputs shaped like the paper's long-context serving workloads.

This module only *makes inputs* (tensors a serving stack would hand to the library): a bf16
KV cache with planted heavy tokens, a speculative query block, a target->draft head map and
draft attention probabilities. It contains none of the method's steps (no aggregation, no
selection, no sparse attention) and is imported by tests and the benchmark, never by the
library or by the oracle.
"""
from .synth import (CONFIGS, Workload, WorkloadConfig, budget_tokens, default_head_map,
                    make_draft_layer, make_workload)

__all__ = ["CONFIGS", "Workload", "WorkloadConfig", "budget_tokens", "default_head_map",
           "make_draft_layer", "make_workload"]
