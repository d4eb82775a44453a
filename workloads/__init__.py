"""Seeded synthetic inputs for the batched speculative-decoding verify step.

This package serves both the CPU oracle and the HIP library with identical inputs.  It contains no
arithmetic of the method itself (no transformer, no accept/resample rule): only seeded random tensors,
their rounding onto the bf16 grid, and the shapes of the workloads.
"""
from .configs import ModelCfg, Workload, WORKLOADS, get_workload  # noqa: F401
from .gen import (Weights, prefix_tokens, synthetic_kv, private_lens, random_draft_q, perturbed_draft_q,  # noqa: F401
                  draw_tokens, to_bf16_grid)
from .philox import uniform24, philox4x32_10  # noqa: F401
