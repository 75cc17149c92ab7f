"""Seeded synthetic inputs for the DAS verify-step build.

This package holds none of the method's arithmetic.  It produces the inputs
both the CPU oracle and the HIP library consume: random-init weight blobs,
synthetic KV contents, context-length mixes, draft budgets, synthetic drafts
with controlled acceptance and keyed uniform streams.
"""
from .gen import (build, weight_count, weights_bf16, bf16_to_f32, f32_to_bf16,
                  kv_synth, uniforms, num_threads)
from .workloads import (ModelShape, Workload, MODELS, WORKLOADS, workload,
                        context_lengths, draft_budgets, max_budget, prompts, make_drafts,
                        expected_accept_len)
